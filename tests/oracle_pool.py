"""Worker processes that run the CPU oracle for the big parity cases.

The oracle is single-threaded NumPy; the (layer, request) units of a workload are independent, so
the full-size cases (80 layers of config 4, 32 requests x 2 layers of the batch-32 bench shape, the
32768 steps of config 5 cut into segments) are spread over the host cores.  The workers are
spawned (the parent has the GPU open; nothing here touches it), import only NumPy, the seeded
generators and the oracle, and answer over a pipe.  A unit generates its own inputs from the
workload's seeds, so the only bulk data that travels is the bit pattern of a context's K and V for
the parent to upload."""
from __future__ import annotations

import multiprocessing as mp
import os
import traceback

import numpy as np


def _compact(res, deep):
    g = res["geom"]
    out = dict(out=res["out"], new_ids=res["new_ids"], flags=res["flags"], miss=res["miss"], cosine=res["cosine"],
               geom=(g.L, g.n_full, g.r, g.n_sink, g.n_win, g.cand_lo, g.n_cand, g.k_eff))
    if deep:
        out["P"], out["score"] = res["P"], res["score"]
    return out


def _worker_main(conn):
    from threadpoolctl import threadpool_limits
    import workloads as W
    from oracle import freekv_oracle as O
    units = {}

    def make(u):
        wl = u["wl"]
        return O.FreeKVOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.page_size, wl.budget, wl.sink, wl.window,
                              u["tau"], u["max_ctx"], select_pooling=u["select_pooling"], corr_pooling=u["corr_pooling"])

    with threadpool_limits(limits=1):
        while True:
            msg = conn.recv()
            op = msg[0]
            if op == "close":
                break
            try:
                if op == "load":
                    _, key, u = msg
                    wl = u["wl"]
                    (K, Kb), (V, Vb) = W.kv_prefix(wl, u["layer"], u["request"], u["n_ctx"])
                    o = make(u)
                    o.load_prefix_bulk(K, V)
                    u["o"] = o
                    u["q"] = W.query_stream(wl, u["layer"], u["request"], u["steps"])[0]
                    (u["kd"], _), (u["vd"], _) = W.kv_decode_tokens(wl, u["layer"], u["request"], u["steps"])
                    u["prefix"] = (K, V) if u["keep_prefix"] else None
                    units[key] = u
                    conn.send(("ok", (Kb.shape, Vb.shape) if u["want_bits"] else None))
                    if u["want_bits"]:
                        conn.send_bytes(np.ascontiguousarray(Kb).data)
                        conn.send_bytes(np.ascontiguousarray(Vb).data)
                elif op == "resync":
                    # the state before decode step t0 is a function of the inputs alone: the tokens so far,
                    # q_{t0-1}, and Sel(q_{t0-1}), which every head has committed by the end of step t0-1
                    _, key, t0 = msg
                    u = units[key]
                    K, V = u["prefix"]
                    o = make(u)
                    o.load_prefix_bulk(np.concatenate([K, u["kd"][:t0 - 1]]), np.concatenate([V, u["vd"][:t0 - 1]]))
                    o.step(u["q"][t0 - 1], u["kd"][t0 - 1], u["vd"][t0 - 1])
                    u["o"] = o
                    conn.send(("ok", None))
                elif op == "steps":
                    _, key, t0, t1, deep_every = msg
                    u = units[key]
                    res = []
                    for t in range(t0, t1):
                        r = u["o"].step(u["q"][t], u["kd"][t], u["vd"][t])
                        res.append(_compact(r, deep_every > 0 and t % deep_every == 0))
                    conn.send(("ok", res))
                elif op == "summaries":
                    _, key = msg
                    o = units[key]["o"]
                    n_page = (o.L + o.p - 1) // o.p
                    conn.send(("ok", (o.kmax[:n_page], o.kmin[:n_page])))
                else:
                    conn.send(("err", f"unknown op {op}"))
            except Exception:                      # noqa: BLE001 - reported to the parent, which fails the test
                conn.send(("err", traceback.format_exc()))


class OraclePool:
    def __init__(self, n_workers=None):
        n = n_workers or max(1, min(16, os.cpu_count() or 1))
        ctx = mp.get_context("spawn")
        self.conns, self.procs = [], []
        for _ in range(n):
            a, b = ctx.Pipe()
            p = ctx.Process(target=_worker_main, args=(b,), daemon=True)
            p.start()
            b.close()
            self.conns.append(a)
            self.procs.append(p)
        self.where = {}          # unit key -> worker index
        self.pending = [[] for _ in range(n)]   # per worker: keys of the requests in flight, in order

    # -- plumbing -------------------------------------------------------------------------
    def _send(self, w, msg, tag):
        self.conns[w].send(msg)
        self.pending[w].append(tag)

    def _recv(self, w):
        status, payload = self.conns[w].recv()
        tag = self.pending[w].pop(0)
        if status != "ok":
            raise RuntimeError(f"oracle worker failed on {tag}:\n{payload}")
        return payload

    # -- operations -----------------------------------------------------------------------
    def load_async(self, key, worker, **unit):
        self.where[key] = worker
        self._send(worker, ("load", key, unit), ("load", key))

    def load_result(self, key, want_bits):
        """Blocks until the unit is built; returns (Kbits, Vbits) uint16 arrays if they were asked for."""
        w = self.where[key]
        shapes = self._recv(w)
        if not want_bits:
            return None
        Kb = np.frombuffer(self.conns[w].recv_bytes(), dtype=np.uint16).reshape(shapes[0])
        Vb = np.frombuffer(self.conns[w].recv_bytes(), dtype=np.uint16).reshape(shapes[1])
        return Kb, Vb

    def resync_async(self, key, t0):
        self._send(self.where[key], ("resync", key, t0), ("resync", key))

    def steps_async(self, key, t0, t1, deep_every=0):
        self._send(self.where[key], ("steps", key, t0, t1, deep_every), ("steps", key, t0))

    def result(self, key):
        return self._recv(self.where[key])

    def summaries(self, key):
        self._send(self.where[key], ("summaries", key), ("summaries", key))
        return self._recv(self.where[key])

    def close(self):
        for c in self.conns:
            try:
                c.send(("close",))
            except Exception:                      # noqa: BLE001
                pass
        for p in self.procs:
            p.join(timeout=10)
            if p.is_alive():
                p.kill()
