"""Side-by-side driver for the parity tests: the HIP path (through the C ABI binding) and the
CPU oracle consume the same seeded inputs; every step is compared."""
from __future__ import annotations

import numpy as np
import torch

import paper_2505_13109_amd as fkv
from paper_2505_13109_amd import binding as B
import workloads as W
from oracle import freekv_oracle as O

TOL_OUT = 2e-3     # max relative error of attention outputs, per head: |d|_inf / |ref|_inf


def to_dev(bits: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == "fp16" else torch.bfloat16)


def rel_err_per_head(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    d = np.abs(got.astype(np.float64) - ref).max(axis=-1)
    return d / np.abs(ref).max(axis=-1)


def _diff(got, ref):
    if got.shape != ref.shape:
        return f"shapes {got.shape} vs {ref.shape}"
    bad = np.argwhere(got != ref)
    return f"{len(bad)} entries, first {[(tuple(i), float(got[tuple(i)]), float(ref[tuple(i)])) for i in bad[:4]]}"


class Pair:
    """One HIP context and the matching oracles for `layers` x `batch` of a workload."""

    def __init__(self, wl, layers, ctx=None, placement=None, tau=None, max_ctx=None, steps=None, recall_mode=0,
                 select_pooling="MeanS", corr_pooling="mean"):
        self.wl = wl
        self.layers = list(layers)
        self.n_ctx = wl.ctx if ctx is None else ctx
        self.steps = wl.steps if steps is None else steps
        self.placement = wl.placement if placement is None else placement
        self.tau = wl.tau if tau is None else tau
        p = wl.page_size
        self.max_ctx = max_ctx or ((self.n_ctx + self.steps + p - 1) // p) * p
        self.g = fkv.FreeKV(n_layers=len(self.layers), batch=wl.batch, n_q_heads=wl.n_q_heads,
                            n_kv_heads=wl.n_kv_heads, max_ctx=self.max_ctx, budget=wl.budget,
                            sink=wl.sink, window=wl.window, tau=self.tau, dtype=wl.dtype,
                            placement=self.placement, recall_mode=recall_mode,
                            select_pooling=select_pooling, corr_pooling=corr_pooling)
        self.q_pooled = select_pooling in ("MeanQ", "MaxQ")
        self.oracles = {}
        self.q, self.kd, self.vd = {}, {}, {}
        self.copy_stream = torch.cuda.Stream()
        for li, layer in enumerate(self.layers):
            Kb_all, Vb_all = [], []
            for r in range(wl.batch):
                (K, Kb), (V, Vb) = W.kv_prefix(wl, layer, r, self.n_ctx)
                o = O.FreeKVOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, p, wl.budget, wl.sink,
                                   wl.window, self.tau, self.max_ctx,
                                   select_pooling=select_pooling, corr_pooling=corr_pooling)
                o.load_prefix_bulk(K, V)
                self.oracles[(li, r)] = o
                Kb_all.append(Kb)
                Vb_all.append(Vb)
                self.q[(li, r)] = W.query_stream(wl, layer, r, self.steps)
                self.kd[(li, r)], self.vd[(li, r)] = W.kv_decode_tokens(wl, layer, r, self.steps)
            if self.n_ctx:
                self.g.load_prefix(li, to_dev(np.stack(Kb_all), wl.dtype), to_dev(np.stack(Vb_all), wl.dtype))
        torch.cuda.synchronize()
        self.out = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device="cuda")
        self.stats = dict(max_rel=0.0, flagged=0, heads=0, misses=0, picked=0)

    def step_inputs(self, li, t):
        wl = self.wl
        qb = np.stack([self.q[(li, r)][1][t] for r in range(wl.batch)])
        kb = np.stack([self.kd[(li, r)][1][t] for r in range(wl.batch)])
        vb = np.stack([self.vd[(li, r)][1][t] for r in range(wl.batch)])
        return to_dev(qb, wl.dtype), to_dev(kb, wl.dtype), to_dev(vb, wl.dtype)

    def check_summaries(self, li):
        wl = self.wl
        s = W.decode(self.g.debug_read(li, B.DBG_SUMMARIES), wl.dtype)
        for r in range(wl.batch):
            o = self.oracles[(li, r)]
            n_page = (o.L + wl.page_size - 1) // wl.page_size
            assert np.array_equal(s[r, :, 0, :n_page, :], o.kmax[:n_page].transpose(1, 0, 2)), "kmax"
            assert np.array_equal(s[r, :, 1, :n_page, :], o.kmin[:n_page].transpose(1, 0, 2)), "kmin"

    def step(self, li, t, check=True, deep=True):
        """One decode step of layer index li on both sides; returns the oracle results per request."""
        wl = self.wl
        q, k, v = self.step_inputs(li, t)
        self.g.decode_step(li, q, k, v, self.out, copy_stream=self.copy_stream)
        res = []
        for r in range(wl.batch):
            res.append(self.oracles[(li, r)].step(self.q[(li, r)][0][t], self.kd[(li, r)][0][t], self.vd[(li, r)][0][t]))
        if check:
            self.compare(li, t, res, self.read_step(li, deep), deep)
        return res

    def read_step(self, li, deep):
        """What the HIP side holds after decode step of layer index li (blocking reads)."""
        got = dict(ids=self.g.debug_read(li, B.DBG_ACTIVE_IDS),      # after commit the step's selection is ACTIVE
                   flags=self.g.debug_read(li, B.DBG_FLAGS), out=self.out.cpu().numpy())
        if deep:
            got.update(P=self.g.debug_read(li, B.DBG_WEIGHTS), score=self.g.debug_read(li, B.DBG_SCORES),
                       cosine=self.g.debug_read(li, B.DBG_COSINE))
        if self.placement == 1:
            got["miss"] = self.g.debug_read(li, B.DBG_MISS)
        return got

    def compare(self, li, t, res, got, deep):
        """HIP results `got` of one layer-step against the oracle's `res` (one per request)."""
        wl = self.wl
        for r in range(wl.batch):
            ref = res[r]
            gm = ref["geom"]
            if isinstance(gm, tuple):
                gm = O.Geometry(*gm)
            tag = f"layer {self.layers[li]} step {t} request {r} L {gm.L}"
            if deep and wl.k_pages > 0 and "P" in ref:      # with nothing selectable the library skips scoring altogether
                lo, hi = gm.cand_lo, gm.cand_lo + gm.n_cand
                # a pooled query has one row of weights per KV head, kept in the row of the group's first head
                Pg = got["P"][r, ::wl.n_q_heads // wl.n_kv_heads, lo:hi] if self.q_pooled else got["P"][r, :, lo:hi]
                assert np.array_equal(Pg, ref["P"]), f"page weights differ: {tag}: {_diff(Pg, ref['P'])}"
                assert np.array_equal(got["score"][r, :, lo:hi], ref["score"]), f"pooled scores differ: {tag}: {_diff(got['score'][r, :, lo:hi], ref['score'])}"
                if t > 0:
                    np.testing.assert_allclose(got["cosine"][r], ref["cosine"], rtol=0, atol=1e-12, err_msg=tag)
            assert np.array_equal(got["flags"][r], ref["flags"]), f"flags differ: {tag}: {got['flags'][r]} vs {ref['flags']}"
            assert np.array_equal(got["ids"][r], ref["new_ids"]), f"page ids differ: {tag}"
            err = rel_err_per_head(got["out"][r], ref["out"])
            assert err.max() <= TOL_OUT, f"attention output off by {err.max():.3e}: {tag}"
            self.stats["max_rel"] = max(self.stats["max_rel"], float(err.max()))
            self.stats["flagged"] += int(ref["flags"].sum())
            self.stats["heads"] += wl.n_kv_heads
            if self.placement == 1:
                for m in range(wl.n_kv_heads):
                    n = int(got["miss"][r, m, 0])
                    assert sorted(got["miss"][r, m, 1:1 + n].tolist()) == ref["miss"][m], f"miss list differs: {tag} head {m}"
                    self.stats["misses"] += n
                    self.stats["picked"] += int((ref["new_ids"][m] >= 0).sum())

    def check_nhd_export(self, li):
        """The NHD-layout pool of the ACTIVE selection equals the oracle's, byte for byte."""
        wl = self.wl
        n_slots = wl.budget // wl.page_size + 1
        pool = torch.full((wl.batch, n_slots, 2, wl.page_size, wl.n_kv_heads, wl.head_dim), 7.0,
                          dtype=self.g.torch_dtype, device="cuda")
        pages = torch.full((wl.batch, wl.n_kv_heads, n_slots), -7, dtype=torch.int32, device="cuda")
        self.g.export_nhd(li, pool, pages)
        got = W.decode(pool.view(torch.int16).cpu().numpy().view(np.uint16), wl.dtype)
        for r in range(wl.batch):
            o = self.oracles[(li, r)]
            ref_pool, ref_pages = o.export_nhd(o.active, n_slots)
            assert np.array_equal(pages.cpu().numpy()[r], ref_pages), f"slot pages differ: layer index {li} request {r}"
            assert np.array_equal(got[r], ref_pool), f"NHD pool differs: layer index {li} request {r}: {_diff(got[r], ref_pool)}"

    def check_cached_pages(self, li, r, m, where):
        """Bytes of the picked pages where the HIP side keeps them == the bytes appended (oracle's K, V)."""
        wl = self.wl
        o = self.oracles[(li, r)]
        p = wl.page_size
        for page in [int(j) for j in o.active[m] if j >= 0]:
            got = W.decode(self.g.debug_read_page(li, r, m, page, where), wl.dtype)
            assert np.array_equal(got[0], o.K[page * p:(page + 1) * p, m, :]), f"K bytes page {page}"
            assert np.array_equal(got[1], o.V[page * p:(page + 1) * p, m, :]), f"V bytes page {page}"

    def close(self):
        for li in range(len(self.layers)):
            self.g.health(li)            # no kernel gave up a bounded wait
        self.g.close()


class PoolPair(Pair):
    """Pair whose oracles live in worker processes (tests/oracle_pool.py): for the cases whose oracle
    state or oracle time is too big for one process.  Every (layer, request) unit generates its own
    inputs in its worker; the parent uploads the context bits the worker sends back and draws only the
    small per-step streams itself."""

    def __init__(self, wl, layers, pool, ctx=None, placement=None, tau=None, steps=None, keep_prefix=False):
        self.wl = wl
        self.layers = list(layers)
        self.pool = pool
        self.n_ctx = wl.ctx if ctx is None else ctx
        self.steps = wl.steps if steps is None else steps
        self.placement = wl.placement if placement is None else placement
        self.tau = wl.tau if tau is None else tau
        p = wl.page_size
        self.max_ctx = ((self.n_ctx + self.steps + p - 1) // p) * p
        self.q_pooled = False
        self.g = fkv.FreeKV(n_layers=len(self.layers), batch=wl.batch, n_q_heads=wl.n_q_heads,
                            n_kv_heads=wl.n_kv_heads, max_ctx=self.max_ctx, budget=wl.budget,
                            sink=wl.sink, window=wl.window, tau=self.tau, dtype=wl.dtype, placement=self.placement)
        self.copy_stream = torch.cuda.Stream()
        self.oracles = {}
        self.q, self.kd, self.vd = {}, {}, {}
        n_workers = len(pool.conns)
        units = [(li, r) for li in range(len(self.layers)) for r in range(wl.batch)]
        for i, (li, r) in enumerate(units):
            pool.load_async((id(self), li, r), i % n_workers, wl=wl, layer=self.layers[li], request=r, n_ctx=self.n_ctx,
                            steps=self.steps, tau=self.tau, max_ctx=self.max_ctx, select_pooling="MeanS",
                            corr_pooling="mean", want_bits=True, keep_prefix=keep_prefix)
        for li, layer in enumerate(self.layers):
            Kd = torch.empty((wl.batch, self.n_ctx, wl.n_kv_heads, wl.head_dim), dtype=torch.int16, device="cuda")
            Vd = torch.empty_like(Kd)
            for r in range(wl.batch):
                Kb, Vb = pool.load_result((id(self), li, r), True)
                Kd[r].copy_(torch.from_numpy(Kb.view(np.int16)))
                Vd[r].copy_(torch.from_numpy(Vb.view(np.int16)))
                del Kb, Vb
                self.q[(li, r)] = W.query_stream(wl, layer, r, self.steps)
                self.kd[(li, r)], self.vd[(li, r)] = W.kv_decode_tokens(wl, layer, r, self.steps)
            dt = torch.float16 if wl.dtype == "fp16" else torch.bfloat16
            self.g.load_prefix(li, Kd.view(dt), Vd.view(dt))
            torch.cuda.synchronize()
            del Kd, Vd
        self.out = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device="cuda")
        self.stats = dict(max_rel=0.0, flagged=0, heads=0, misses=0, picked=0)

    def key(self, li, r):
        return (id(self), li, r)

    def step_all_layers(self, t, deep=True):
        """Decode step t of every layer: the oracles work in their processes while the HIP side decodes."""
        wl = self.wl
        for li in range(len(self.layers)):
            for r in range(wl.batch):
                self.pool.steps_async(self.key(li, r), t, t + 1, 1 if deep else 0)
        got = []
        for li in range(len(self.layers)):
            q, k, v = self.step_inputs(li, t)
            self.g.decode_step(li, q, k, v, self.out, copy_stream=self.copy_stream)
            got.append(self.read_step(li, deep))
        for li in range(len(self.layers)):
            res = [self.pool.result(self.key(li, r))[0] for r in range(wl.batch)]
            self.compare(li, t, res, got[li], deep)

    def check_summaries(self, li):
        wl = self.wl
        s = W.decode(self.g.debug_read(li, B.DBG_SUMMARIES), wl.dtype)
        for r in range(wl.batch):
            kmax, kmin = self.pool.summaries(self.key(li, r))
            n_page = kmax.shape[0]
            assert np.array_equal(s[r, :, 0, :n_page, :], kmax.transpose(1, 0, 2)), "kmax"
            assert np.array_equal(s[r, :, 1, :n_page, :], kmin.transpose(1, 0, 2)), "kmin"
