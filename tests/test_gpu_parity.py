"""Parity of the HIP path against the CPU oracle, through the C ABI, on a real MI355X.
Page ids, flags, page weights and pooled scores must agree bit for bit; attention
outputs within 2e-3 (max relative error per head)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import freekv_oracle as O

pytestmark = pytest.mark.gpu

def _pair(*a, **kw):
    from harness import Pair
    return Pair(*a, **kw)


@pytest.fixture(scope="module")
def oracle_pool():
    """Oracle worker processes for the full-size cases (one per host core, at most 16)."""
    from oracle_pool import OraclePool
    pool = OraclePool()
    yield pool
    pool.close()


def test_c1_every_step():
    """Config 1 as stated: fp16, 4096 tokens, budget 512, 64 steps, everything compared."""
    wl = W.get_workload("c1")
    pr = _pair(wl, [0])
    pr.check_summaries(0)
    for t in range(wl.steps):
        pr.step(0, t)
    pr.check_summaries(0)
    assert pr.stats["flagged"] == wl.n_kv_heads          # only the first step corrects at rho = 0.9, tau = 0.8
    print("c1", pr.stats)
    pr.close()


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_growing_context_ragged_geometry(dtype):
    """Context grows from 5 tokens through sink, window, first candidates (k_eff < k), page fills; G = 7."""
    wl = W.Workload("grow", 1, 2, 14, 2, dtype, 5, 256, 32, 64, 0.7, 330, 0.7, 0.714, 11, shift_every=100)
    pr = _pair(wl, [3])
    for t in range(wl.steps):
        pr.step(0, t)
        if t % 50 == 0:
            pr.check_summaries(0)
    assert 0 < pr.stats["flagged"] < pr.stats["heads"]
    print("grow", dtype, pr.stats)
    pr.close()


@pytest.mark.parametrize("placement", [0, 1])
def test_decoding_from_an_empty_context(placement):
    """Nothing loaded: the first decode step appends token 0 and attends over that one token; the context then grows
    through the open page, the first full pages, sink and window, the first page offloads (host pool) and the first
    candidates."""
    wl = W.Workload("empty", 1, 2, 6, 2, "bf16", 0, 192, 32, 64, 0.75, 200, 0.75, 0.66, 13, placement=placement)
    pr = _pair(wl, [1])
    for t in range(wl.steps):
        pr.step(0, t)
        if t in (0, 31, 32, 100, 199):
            pr.check_summaries(0)
    assert pr.stats["flagged"] > 0
    if placement == 1:
        torch.cuda.synchronize()
        pr.check_cached_pages(0, 1, 0, where=1)
    print("empty", placement, pr.stats)
    pr.close()


def test_budget_covering_context_is_dense_attention():
    wl = W.Workload("dense", 1, 1, 8, 2, "bf16", 700, 1024, 64, 64, 1.5, 40, 0.9, 0.436, 5)   # tau > 1: every step selects afresh
    pr = _pair(wl, [0])
    for t in range(wl.steps):
        res = pr.step(0, t)[0]
        o = pr.oracles[(0, 0)]
        assert res["geom"].k_eff == res["geom"].n_cand
        dense = O.dense_attention(pr.q[(0, 0)][0][t], o.K[:o.L], o.V[:o.L])
        got = pr.out.cpu().numpy()[0]
        from harness import rel_err_per_head
        assert rel_err_per_head(got, dense).max() <= 2e-3
    pr.close()


def test_groups_of_1_2_3_5_6_8():
    for G in (1, 2, 3, 5, 6, 8):
        wl = W.Workload(f"g{G}", 1, 1, 2 * G, 2, "bf16", 1500, 384, 64, 64, 0.8, 6, 0.8, 0.6, 20 + G)
        pr = _pair(wl, [0])
        for t in range(wl.steps):
            pr.step(0, t)
        pr.close()


def test_empty_window_no_sink_and_nothing_selectable():
    """W = 0 (a page becomes a candidate the moment it fills), S = 0, and budget = S + W (k = 0)."""
    for sink, window, budget in ((0, 0, 256), (64, 0, 256), (0, 64, 192), (64, 64, 128)):
        wl = W.Workload("edge", 1, 2, 8, 2, "bf16", 1000, budget, sink, window, 0.85, 70, 0.85, 0.527, 31)
        pr = _pair(wl, [0])
        for t in range(wl.steps):
            pr.step(0, t)
        pr.close()


def test_batch_of_three_in_hbm():
    wl = W.Workload("b3", 2, 3, 16, 4, "fp16", 5000, 1024, 128, 256, 0.8, 20, 0.8, 0.6, 77)
    pr = _pair(wl, [0, 1])
    for t in range(wl.steps):
        for li in range(2):
            pr.step(li, t)
    pr.close()


def test_primitives_and_call_order():
    import paper_2505_13109_amd as fkv
    from paper_2505_13109_amd import binding as B
    from harness import to_dev, rel_err_per_head
    wl = W.Workload("prim", 1, 1, 8, 2, "bf16", 2000, 512, 64, 64, 0.8, 4, 0.9, 0.436, 9)
    pr = _pair(wl, [0])
    g, o = pr.g, pr.oracles[(0, 0)]
    q, k, v = pr.step_inputs(0, 0)
    out = torch.empty((1, 8, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(fkv.FreeKVError):
        g.sparse_decode_attn(0, q, out, use=fkv.FKV_USE_PENDING)       # no selection yet
    with pytest.raises(fkv.FreeKVError):
        g.commit(0)
    with pytest.raises(fkv.FreeKVError):
        g.kv_append(5, k, v)                                           # layer out of range
    g.kv_append(0, k, v)
    o.append(pr.kd[(0, 0)][0][0], pr.vd[(0, 0)][0][0])
    flags = torch.zeros((1, 2), dtype=torch.uint8, device="cuda")
    ids = torch.zeros((1, 2, g.k), dtype=torch.int32, device="cuda")
    g.corr_check(0, q, flags)
    g.page_select(0, q, ids)
    ref_ids, _, _ = o.select(pr.q[(0, 0)][0][0])
    assert flags.cpu().numpy().all()                                   # no previous query
    assert np.array_equal(ids.cpu().numpy()[0], ref_ids)
    g.sparse_decode_attn(0, q, out, use=fkv.FKV_USE_PENDING)
    ref = o.attend(pr.q[(0, 0)][0][0], ref_ids)
    assert rel_err_per_head(out.cpu().numpy()[0], ref).max() <= 2e-3
    # ACTIVE is still empty: attention over sink + window + open page only
    g.sparse_decode_attn(0, q, out, use=fkv.FKV_USE_ACTIVE)
    ref = o.attend(pr.q[(0, 0)][0][0], np.full_like(ref_ids, -1))
    assert rel_err_per_head(out.cpu().numpy()[0], ref).max() <= 2e-3
    g.commit(0)
    assert g.context_len(0) == 2001
    # recomputing summaries from the stored keys changes nothing
    before = g.debug_read(0, B.DBG_SUMMARIES)
    g.page_summary_update(0, 0, (2001 + 31) // 32)
    assert np.array_equal(before, g.debug_read(0, B.DBG_SUMMARIES))
    # stored pages read back token-major equal what was appended
    got = W.decode(g.debug_read_page(0, 0, 1, 62, 0), "bf16")
    assert np.array_equal(got[0][:17], o.K[62 * 32:2001, 1, :]) and np.array_equal(got[1][:17], o.V[62 * 32:2001, 1, :])
    pr.close()


def test_top_k_ties_go_to_the_lower_page():
    """All keys identical -> all pooled scores equal -> the lowest candidate page ids are picked."""
    import paper_2505_13109_amd as fkv
    from harness import to_dev
    g = fkv.FreeKV(n_layers=1, batch=1, n_q_heads=4, n_kv_heads=1, max_ctx=2048, budget=256, sink=32,
                   window=32, tau=0.8, dtype="bf16")
    K = np.ones((1, 1600, 1, 128), dtype=np.float32)
    g.load_prefix(0, to_dev(W.encode(K, "bf16"), "bf16"), to_dev(W.encode(K, "bf16"), "bf16"))
    q = to_dev(W.encode(np.random.default_rng(0).standard_normal((1, 4, 128)).astype(np.float32), "bf16"), "bf16")
    ids = torch.zeros((1, 1, g.k), dtype=torch.int32, device="cuda")
    g.page_select(0, q, ids)
    assert ids.cpu().numpy()[0, 0].tolist() == list(range(1, 1 + g.k))
    g.close()


def test_c2_shape_two_layers_all_steps():
    """Config 2 at full size (32K context, bf16, budget 2048), the shape bench.py times: 2 of the 32
    layers, all 256 steps, every step compared (weights and scores on every 4th)."""
    wl = W.get_workload("c2")
    pr = _pair(wl, [0, 17])
    for t in range(wl.steps):
        for li in range(2):
            pr.step(li, t, deep=(t % 4 == 0))
        if t % 64 == 63:
            print("c2 step", t, pr.stats, flush=True)
    for li in range(2):
        assert pr.g.step_launches(li) == 1            # the one-launch layer kernel is what ran
        pr.check_summaries(li)
    pr.close()


def test_c2_shape_across_layers():
    """Config 2: 4 steps of all 32 layers in one context."""
    wl = W.get_workload("c2")
    layers = list(range(wl.n_layers))
    pr = _pair(wl, layers, steps=4)
    for t in range(4):
        for li in range(len(layers)):
            pr.step(li, t)
        print("c2 layers step", t, flush=True)
    pr.close()


def test_c4_shape_sampled_layers():
    """Config 4 at full size (64K context, G = 8, budget 4096): two of the 80 layers, all 128 steps."""
    wl = W.get_workload("c4")
    layers, steps = [41, 79], wl.steps
    pr = _pair(wl, layers, steps=steps)
    for t in range(steps):
        for li in range(len(layers)):
            pr.step(li, t, deep=(t % 4 == 0))
        if t % 16 == 15:
            print("c4 step", t, pr.stats, flush=True)
    pr.close()


def test_c4_every_layer_four_steps(oracle_pool):
    """Config 4 as stated in one context: all 80 layers (20 GiB of KV in HBM), 4 decode steps of every layer,
    everything compared (weights and scores on steps 0 and 3)."""
    from harness import PoolPair
    wl = W.get_workload("c4")
    pr = PoolPair(wl, range(wl.n_layers), oracle_pool, steps=4)
    print("c4 x 80: contexts loaded", flush=True)
    for t in range(4):
        pr.step_all_layers(t, deep=(t in (0, 3)))
        print("c4 x 80 step", t, pr.stats, flush=True)
    for li in (0, 39, 79):
        assert pr.g.step_launches(li) == 1
        pr.check_summaries(li)
    assert pr.stats["heads"] == 80 * 4 * wl.n_kv_heads
    pr.close()


def test_bench_saturated_shape_batch_32(oracle_pool):
    """The shape bench.py reports as `saturated_shape`, at size: the config-2 shape with 32 requests of 32K
    tokens, 2 layers, 4 steps, in the dispatch the bench times there (separate launches: scoring blocks that
    take several chunks of 4 passes, the selection in a launch of its own, one attention block per head)."""
    from harness import PoolPair
    wl = W.get_workload("c2").scaled(batch=32)
    pr = PoolPair(wl, [0, 17], oracle_pool, steps=4)
    print("batch 32: contexts loaded", flush=True)
    for t in range(4):
        pr.step_all_layers(t, deep=(t in (0, 3)))
        print("batch 32 step", t, pr.stats, flush=True)
    for li in range(2):
        assert pr.g.step_launches(li) == 3
    pr.close()


def test_c5_shape_long_generation():
    """Config 5 shape (G = 7, context grows from 2048, tau 0.9, rho 0.7, topic shifts), 1300 steps of one layer."""
    wl = W.get_workload("c5").scaled(shift_every=500)
    pr = _pair(wl, [13], steps=1300)
    for t in range(1300):
        pr.step(0, t, deep=(t % 16 == 0))
    assert pr.stats["flagged"] > 0.9 * pr.stats["heads"]
    print("c5", pr.stats)
    pr.close()


def test_c5_every_step_of_the_long_generation(oracle_pool):
    """Config 5 as stated, one layer: the HIP side decodes all 32768 steps in one run (context 2048 -> 34816)
    and EVERY step is compared (weights and scores on every 64th).  The oracle's steps are cut into segments
    that run side by side in worker processes: its state at the start of a segment follows from the inputs
    alone -- the tokens so far, q_{t-1}, and Sel(q_{t-1}), which every head has committed by the end of step
    t-1 -- so a fresh bulk load plus one step reproduces it."""
    from harness import PoolPair
    import paper_2505_13109_amd.binding as B
    wl = W.get_workload("c5")
    pool = oracle_pool
    n_seg = 2 * len(pool.conns)
    bounds = [round(i * wl.steps / n_seg) for i in range(n_seg + 1)]
    pr = PoolPair(wl, [13], pool, keep_prefix=True)          # its own unit serves segment 0
    keys = [pr.key(0, 0)]
    for s in range(1, n_seg):
        key = (id(pr), "segment", s)
        pool.load_async(key, s % len(pool.conns), wl=wl, layer=13, request=0, n_ctx=wl.ctx, steps=wl.steps, tau=wl.tau,
                        max_ctx=pr.max_ctx, select_pooling="MeanS", corr_pooling="mean", want_bits=False, keep_prefix=True)
        keys.append(key)
    for s in range(1, n_seg):
        pool.load_result(keys[s], False)
    for s in range(n_seg):                                    # per worker the answers come back in this order
        if s > 0:
            pool.resync_async(keys[s], bounds[s])
        pool.steps_async(keys[s], bounds[s], bounds[s + 1], 64)
    got = []
    for t in range(wl.steps):
        q, k, v = pr.step_inputs(0, t)
        pr.g.decode_step(0, q, k, v, pr.out, copy_stream=pr.copy_stream)
        got.append(pr.read_step(0, t % 64 == 0))
        if t % 4096 == 4095:
            print("c5 HIP step", t, flush=True)
    assert pr.g.context_len(0) == wl.ctx + wl.steps
    for s in range(n_seg):
        if s > 0:
            pool.result(keys[s])                              # the resync
        res = pool.result(keys[s])
        assert len(res) == bounds[s + 1] - bounds[s]
        for i, ref in enumerate(res):
            t = bounds[s] + i
            pr.compare(0, t, [ref], got[t], t % 64 == 0)
        print("c5 segment", s, bounds[s], bounds[s + 1], pr.stats, flush=True)
    assert pr.stats["heads"] == wl.steps * wl.n_kv_heads and pr.stats["flagged"] > 0.9 * pr.stats["heads"]
    pr.close()


def test_c3_full_context_one_layer_all_requests():
    """Config 3 as stated for one layer: 4 requests of 128K tokens in the pinned host pool, all 128 steps."""
    wl = W.get_workload("c3")
    pr = _pair(wl, [7])
    for t in range(wl.steps):
        pr.step(0, t, deep=(t % 8 == 0))
        if t % 16 == 15:
            print("c3 step", t, pr.stats, flush=True)
    # this size takes the separate launches: scan, selection with the recall plan, the corrected heads' gather, attention
    assert pr.g.step_launches(0) == 4
    torch.cuda.synchronize()
    for r in range(wl.batch):
        pr.check_cached_pages(0, r, r, where=2)
    assert pr.stats["misses"] > 0
    pr.close()


def test_c3_shape_host_pool_recall():
    """Config 3 shape with the KV pool in pinned host memory (scaled: 2 requests, 16K context, 2 layers).  At this size
    the layer-step is one launch on the compute stream: the selecting blocks make the recall plan and the attention
    blocks of a corrected head fetch its missing pages from the host pool themselves; the other heads' recall follows
    on the copy stream."""
    wl = W.get_workload("c3").scaled(batch=2, ctx=16384 - 40, steps=96)
    pr = _pair(wl, [0, 31], steps=96)
    for t in range(96):
        for li in range(2):
            pr.step(li, t)
            assert pr.g.step_launches(li) == 1
        if t % 24 == 23:
            torch.cuda.synchronize()
            for li in range(2):
                pr.check_cached_pages(li, 1, 3, where=1)     # host pool holds the appended bytes
                pr.check_cached_pages(li, 0, 5, where=2)     # recalled pages sit in their page-cache slots
    print("c3", pr.stats)
    assert pr.stats["misses"] > 0 and pr.stats["misses"] < pr.stats["picked"]
    pr.close()


def test_host_pool_recall_with_memcpy_per_unit():
    """The alternative recall engine (one hipMemcpyAsync per 16 KiB unit) gives the same results."""
    wl = W.get_workload("c3").scaled(batch=2, ctx=8192 - 11, steps=40)
    pr = _pair(wl, [5], steps=40, recall_mode=1)
    for t in range(40):
        pr.step(0, t)
    torch.cuda.synchronize()
    pr.check_cached_pages(0, 1, 2, where=2)
    assert pr.stats["misses"] > 0
    pr.close()


def test_recall_pages_with_a_callers_list():
    """fkv_recall_pages as a primitive of its own (Sec. 4.1 data plane, Sec. 4.2 recall unit): an arbitrary
    list of pages, first for a masked subset of the heads, then for all; the page-cache slots must hold the
    bytes that were appended (the oracle's K, V), ids that are no full page are dropped, pages the previous
    list already holds are not copied again, attention over the list matches the oracle, and a commit
    before every head was recalled is refused."""
    import paper_2505_13109_amd as fkv
    from paper_2505_13109_amd import binding as B
    from harness import rel_err_per_head
    wl = W.get_workload("c3").scaled(batch=2, ctx=6000 + 7, steps=4)
    pr = _pair(wl, [6], steps=4)
    g, k, n_kv = pr.g, pr.g.k, wl.n_kv_heads
    q, kn, vn = pr.step_inputs(0, 0)
    g.kv_append(0, kn, vn)
    for r in range(2):
        pr.oracles[(0, r)].append(pr.kd[(0, r)][0][0], pr.vd[(0, r)][0][0])
    n_full = (6000 + 8) // 32
    rng = np.random.default_rng(99)

    def draw(n_real):
        ids = np.full((2, n_kv, k), -1, dtype=np.int32)
        for r in range(2):
            for m in range(n_kv):
                ids[r, m, :n_real] = np.sort(rng.choice(np.arange(16, n_full - 16), n_real, replace=False))
        return ids

    def check_slots(ids, heads, where):
        torch.cuda.synchronize()
        for r, m in heads:
            o = pr.oracles[(0, r)]
            for page in [int(j) for j in ids[r, m] if j >= 0][::5]:
                got = W.decode(g.debug_read_page(0, r, m, page, where), wl.dtype)
                assert np.array_equal(got[0], o.K[page * 32:(page + 1) * 32, m, :]), (r, m, page)
                assert np.array_equal(got[1], o.V[page * 32:(page + 1) * 32, m, :]), (r, m, page)

    first = draw(k - 3)
    first[1, 2, k - 3] = n_full + 5                           # not a full page of this context: dropped
    mask = np.zeros((2, n_kv), dtype=np.uint8)
    mask[0, 1] = mask[1, 5] = mask[1, 2] = 1
    ids_dev = torch.from_numpy(first).cuda()
    g.recall_pages(0, ids_dev, torch.from_numpy(mask).cuda())
    clean = first.copy()
    clean[1, 2, k - 3] = -1
    assert np.array_equal(g.debug_read(0, B.DBG_PENDING_IDS), clean)
    assert (g.debug_read(0, B.DBG_MISS)[..., 0] == k - 3).all()       # cold cache: every page is a miss
    check_slots(clean, [(0, 1), (1, 5), (1, 2)], where=3)
    g.corr_check(0, q)
    with pytest.raises(fkv.FreeKVError, match="before every head"):
        g.commit(0)                                           # the masked recall filled three heads only
    g.recall_pages(0, None, None)                             # the pending list, every head
    check_slots(clean, [(r, m) for r in range(2) for m in range(n_kv)], where=3)
    out = torch.empty((2, wl.n_q_heads, 128), dtype=torch.float32, device="cuda")
    g.sparse_decode_attn(0, q, out, use=fkv.FKV_USE_PENDING)
    for r in range(2):
        ref = pr.oracles[(0, r)].attend(pr.q[(0, r)][0][0], clean[r])
        assert rel_err_per_head(out.cpu().numpy()[r], ref).max() <= 2e-3
    g.commit(0)
    # a second list sharing half its pages with the first: the shared ones keep their slots and are not copied
    second = draw(k)
    second[:, :, ::2] = np.where(clean[:, :, ::2] >= 0, clean[:, :, ::2], second[:, :, ::2])
    second = np.sort(second, axis=-1)
    for r in range(2):                                        # keep it distinct per head
        for m in range(n_kv):
            u = np.unique(second[r, m][second[r, m] >= 0])
            second[r, m] = -1
            second[r, m, :len(u)] = u
    g.recall_pages(0, torch.from_numpy(second).cuda(), None)
    miss = g.debug_read(0, B.DBG_MISS)
    for r in range(2):
        for m in range(n_kv):
            want = sorted(set(second[r, m][second[r, m] >= 0].tolist()) - set(clean[r, m][clean[r, m] >= 0].tolist()))
            assert sorted(miss[r, m, 1:1 + miss[r, m, 0]].tolist()) == want
    check_slots(second, [(r, m) for r in range(2) for m in range(n_kv)], where=3)
    check_slots(clean, [(0, 0), (1, 7)], where=2)             # the ACTIVE list's slots were not overwritten
    pr.close()


def test_commit_before_recall_is_refused_with_the_host_pool():
    wl = W.get_workload("c3").scaled(batch=1, ctx=4000, steps=2)
    import paper_2505_13109_amd as fkv
    pr = _pair(wl, [2], steps=2)
    q, kn, vn = pr.step_inputs(0, 0)
    pr.g.kv_append(0, kn, vn)
    pr.g.corr_check(0, q)
    pr.g.page_select(0, q)
    with pytest.raises(fkv.FreeKVError, match="before every head"):
        pr.g.commit(0)
    pr.g.recall_pending(0, fkv.FKV_HEADS_FLAGGED)
    with pytest.raises(fkv.FreeKVError, match="before every head"):
        pr.g.commit(0)
    pr.g.recall_pending(0, fkv.FKV_HEADS_UNFLAGGED)
    pr.g.commit(0)
    pr.close()


# ---------------------------------------------------------------- App. B.2 / B.3: the alternative poolings
VARIANTS = ["MaxS", "MeanQK", "MaxQK", "MeanQ", "MaxQ"]


@pytest.mark.parametrize("pooling", VARIANTS)
def test_selection_pooling_variants(pooling):
    """Each alternative group pooling of the selection, every step compared, G = 4 bf16 and G = 7 fp16."""
    for wl in (W.Workload("v4", 1, 1, 16, 4, "bf16", 6000, 512, 32, 64, 0.8, 24, 0.8, 0.6, 31, shift_every=9),
               W.Workload("v7", 1, 2, 14, 2, "fp16", 20, 256, 32, 64, 0.75, 200, 0.75, 0.7, 32, shift_every=60)):
        pr = _pair(wl, [1], select_pooling=pooling)
        for t in range(wl.steps):
            pr.step(0, t)
        assert 0 < pr.stats["flagged"] < pr.stats["heads"]
        print(pooling, wl.name, pr.stats)
        pr.close()


@pytest.mark.parametrize("pooling", ["max", "min"])
def test_correction_pooling_variants(pooling):
    """Max- and min-pooled query similarity decide the flags; both sides must flag the same heads."""
    wl = W.Workload("cp", 1, 1, 12, 3, "bf16", 3000, 512, 32, 64, 0.72, 120, 0.72, 0.7, 33, shift_every=40)
    counts = {}
    for cp in ("mean", pooling):
        pr = _pair(wl, [2], corr_pooling=cp)
        for t in range(wl.steps):
            pr.step(0, t, deep=(t % 8 == 0))
        counts[cp] = pr.stats["flagged"]
        assert 0 < counts[cp] < pr.stats["heads"]
        pr.close()
    # the largest similarity of a group is below tau less often than the mean, the smallest more often
    assert counts["max"] < counts["mean"] if pooling == "max" else counts["min"] > counts["mean"]
    print("corr pooling", counts)


@pytest.mark.parametrize("pooling", ["MeanS"] + VARIANTS)
def test_negative_page_weights_and_long_context_selection(pooling):
    """With all-negative queries a page of all-positive keys has a negative weight and one of all-negative
    keys a positive one; only 20 pages are of the second kind, so most of the k = 62 picks are decided
    among negative scores (the variants that rank raw weights).  150K tokens with G = 8 is past what
    the selection can stage in LDS next to its keys."""
    import paper_2505_13109_amd as fkv
    from harness import to_dev
    rng = np.random.default_rng(77)
    n_ctx, n_q, n_kv = 150000, 16, 2
    g = fkv.FreeKV(n_layers=1, batch=1, n_q_heads=n_q, n_kv_heads=n_kv, max_ctx=150016, budget=2048, sink=32,
                   window=32, tau=0.8, dtype="bf16", select_pooling=pooling)
    Kf = (np.abs(rng.standard_normal((n_ctx, n_kv, 128))) + 0.05).astype(np.float32)
    for page in rng.choice(np.arange(10, 4600), 20, replace=False):
        Kf[page * 32:(page + 1) * 32] *= -1.0
    Kb = W.encode(Kf, "bf16")
    K = W.decode(Kb, "bf16")
    o = O.FreeKVOracle(n_q, n_kv, 128, 32, 2048, 32, 32, 0.8, 150016, select_pooling=pooling)
    o.load_prefix_bulk(K, K)
    g.load_prefix(0, to_dev(Kb[None], "bf16"), to_dev(Kb[None], "bf16"))
    ids = torch.zeros((1, n_kv, g.k), dtype=torch.int32, device="cuda")
    for trial in range(3):
        qf = rng.standard_normal((n_q, 128))
        qb = W.encode((qf if trial == 0 else -np.abs(qf) - 0.01).astype(np.float32), "bf16")
        g.page_select(0, to_dev(qb[None], "bf16"), ids)
        ref_ids, P, score = o.select(W.decode(qb, "bf16"))
        if trial > 0 and pooling not in ("MeanS", "MaxS"):
            assert (score > 0).any() and ((score > 0).sum(axis=1) < g.k).all()    # negative scores get picked
        assert np.array_equal(ids.cpu().numpy()[0], ref_ids), (pooling, trial)
    g.close()


def test_nhd_export_of_the_attended_pages():
    """The hybrid layouts taken literally: the attended pages converted to an NHD pool, in HBM placement
    (growing context: empty slots, partial open page, fp16, G = 7) and from the recalled page cache of the
    host-pool placement (bf16, 2 requests)."""
    wl = W.Workload("nhd", 1, 1, 14, 2, "fp16", 5, 256, 32, 64, 0.7, 300, 0.7, 0.714, 41, shift_every=100)
    pr = _pair(wl, [0])
    for t in range(wl.steps):
        pr.step(0, t, deep=False)
        if t % 13 == 0 or t == wl.steps - 1:
            pr.check_nhd_export(0)
    pr.close()
    wl = W.get_workload("c3").scaled(batch=2, ctx=8192 - 3, steps=40)
    pr = _pair(wl, [9], steps=40)
    for t in range(40):
        pr.step(0, t, deep=False)
        if t % 8 == 7:
            pr.check_nhd_export(0)
    pr.close()


def test_streamed_recall_into_an_nhd_pool():
    """Sec. 4.2 "Streamed recall" taken literally: with an NHD pool attached, every recalled unit passes through
    the recall kernel's two staging buffers and lands converted in the pool (and unconverted in its page-cache
    slot), the pages already on the GPU are converted in place.  After every step the pool must equal the
    oracle's NHD pool of the selection the step committed, byte for byte; ids, flags and attention stay exact."""
    wl = W.get_workload("c3").scaled(batch=2, ctx=8192 - 3, steps=48)
    pr = _pair(wl, [9], steps=48)
    n_slots = wl.budget // wl.page_size + 1
    pool = torch.full((wl.batch, n_slots, 2, wl.page_size, wl.n_kv_heads, wl.head_dim), 7.0, dtype=pr.g.torch_dtype, device="cuda")
    pages = torch.full((wl.batch, wl.n_kv_heads, n_slots), -7, dtype=torch.int32, device="cuda")
    pr.g.attach_nhd_pool(pool, pages)
    for t in range(48):
        pr.step(0, t, deep=False)
        torch.cuda.synchronize()                           # the deferred recall on the copy stream included
        got = W.decode(pool.view(torch.int16).cpu().numpy().view(np.uint16), wl.dtype)
        for r in range(wl.batch):
            o = pr.oracles[(0, r)]
            ref_pool, ref_pages = o.export_nhd(o.active, n_slots)
            assert np.array_equal(pages.cpu().numpy()[r], ref_pages), f"slot pages differ: step {t} request {r}"
            assert np.array_equal(got[r], ref_pool), f"NHD pool differs: step {t} request {r}"
    assert pr.stats["misses"] > 100 and 0 < pr.stats["flagged"] < pr.stats["heads"]
    pr.g.attach_nhd_pool(None, None)
    pr.close()
    # growing context in fp16 with G = 5: empty slots, the first candidates, the first recalls
    wl = W.Workload("nhdgrow", 1, 2, 10, 2, "fp16", 40, 256, 32, 64, 0.75, 200, 0.75, 0.66, 83, placement=1, shift_every=70)
    pr = _pair(wl, [1])
    n_slots = wl.budget // wl.page_size + 1
    pool = torch.zeros((wl.batch, n_slots, 2, wl.page_size, wl.n_kv_heads, wl.head_dim), dtype=pr.g.torch_dtype, device="cuda")
    pages = torch.zeros((wl.batch, wl.n_kv_heads, n_slots), dtype=torch.int32, device="cuda")
    pr.g.attach_nhd_pool(pool, pages)
    for t in range(wl.steps):
        pr.step(0, t, deep=False)
        if t % 7 == 0 or t > wl.steps - 4:
            torch.cuda.synchronize()
            got = W.decode(pool.view(torch.int16).cpu().numpy().view(np.uint16), wl.dtype)
            for r in range(wl.batch):
                o = pr.oracles[(0, r)]
                ref_pool, ref_pages = o.export_nhd(o.active, n_slots)
                assert np.array_equal(pages.cpu().numpy()[r], ref_pages) and np.array_equal(got[r], ref_pool), (t, r)
    assert pr.stats["misses"] > 0
    pr.close()


def test_a_wait_that_runs_out_is_reported():
    """The bounded wait of a corrected head's attention: with the library's test hook on, the waves that
    attend picked pages wait for ids of an epoch that never comes.  Every kernel still ends; the failure
    shows on the data path (the outputs of the query groups are NaN) and fkv_health reports it once.
    With the hook off again the same context decodes normally."""
    import paper_2505_13109_amd as fkv
    from harness import to_dev
    g = fkv.FreeKV(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, max_ctx=4096, budget=512, sink=64,
                   window=64, tau=1.5, dtype="bf16")
    rng = np.random.default_rng(3)
    kv = to_dev(W.encode(rng.standard_normal((1, 3000, 2, 128)).astype(np.float32), "bf16"), "bf16")
    g.load_prefix(0, kv, kv)
    q = to_dev(W.encode(rng.standard_normal((1, 8, 128)).astype(np.float32), "bf16"), "bf16")
    kn = to_dev(W.encode(rng.standard_normal((1, 2, 128)).astype(np.float32), "bf16"), "bf16")
    out = torch.zeros((1, 8, 128), dtype=torch.float32, device="cuda")
    g.health(0)
    g.test_lose_selection(True)
    g.decode_step(0, q, kn, kn, out)
    g.test_lose_selection(False)
    assert g.step_launches(0) == 1
    with pytest.raises(fkv.FreeKVError, match="gave up waiting"):
        g.health(0)
    g.health(0)                                        # reported once, then clear
    assert torch.isnan(out).all()                      # both KV heads were corrected (tau > 1): every row is marked
    g.decode_step(0, q, kn, kn, out)
    g.health(0)
    assert torch.isfinite(out).all()
    g.close()


def test_a_wait_that_runs_out_with_the_host_pool_marks_the_layer():
    """The same with the KV in the host pool, where the waves that give up also leave page-cache slots unfilled:
    the step's outputs are NaN, the next step's too (the layer stays marked while the flag is up), fkv_health reports
    it once, and after a reload of the layer it decodes normally."""
    import paper_2505_13109_amd as fkv
    from harness import to_dev
    g = fkv.FreeKV(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, max_ctx=4096, budget=512, sink=64,
                   window=64, tau=1.5, dtype="bf16", placement=1)
    rng = np.random.default_rng(4)
    kv = to_dev(W.encode(rng.standard_normal((1, 3000, 2, 128)).astype(np.float32), "bf16"), "bf16")
    g.load_prefix(0, kv, kv)
    q = to_dev(W.encode(rng.standard_normal((1, 8, 128)).astype(np.float32), "bf16"), "bf16")
    kn = to_dev(W.encode(rng.standard_normal((1, 2, 128)).astype(np.float32), "bf16"), "bf16")
    out = torch.zeros((1, 8, 128), dtype=torch.float32, device="cuda")
    cs = torch.cuda.Stream()
    g.decode_step(0, q, kn, kn, out, copy_stream=cs)
    g.health(0)
    assert g.step_launches(0) == 1 and torch.isfinite(out).all()
    g.test_lose_selection(True)
    g.decode_step(0, q, kn, kn, out, copy_stream=cs)
    g.test_lose_selection(False)
    torch.cuda.synchronize()
    assert torch.isnan(out).all()
    out.zero_()
    g.decode_step(0, q, kn, kn, out, copy_stream=cs)   # no wait is lost here, but the flag is still up
    torch.cuda.synchronize()
    assert torch.isnan(out).all()
    with pytest.raises(fkv.FreeKVError, match="gave up waiting"):
        g.health(0)
    g.health(0)
    g.load_prefix(0, kv, kv)
    g.decode_step(0, q, kn, kn, out, copy_stream=cs)
    g.health(0)
    assert torch.isfinite(out).all()
    g.close()


def test_longest_supported_context():
    """max_ctx at its limit (491520 tokens, 15360 pages; G = 8): one more page is refused at creation, and
    a selection and a whole decode step over 15.3K candidate pages match the oracle."""
    import paper_2505_13109_amd as fkv
    from harness import to_dev, rel_err_per_head
    cfg = dict(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=1, budget=2048, sink=512, window=512, tau=0.8, dtype="bf16")
    with pytest.raises(fkv.FreeKVError):
        fkv.FreeKV(max_ctx=491520 + 32, **cfg)
    g = fkv.FreeKV(max_ctx=491520, **cfg)
    wl = W.Workload("max", 1, 1, 8, 1, "bf16", 491520 - 40, 2048, 512, 512, 0.8, 2, 0.9, 0.436, 51)
    (K, Kb), (V, Vb) = W.kv_prefix(wl, 0, 0)
    o = O.FreeKVOracle(8, 1, 128, 32, 2048, 512, 512, 0.8, 491520)
    o.load_prefix_bulk(K, V)
    g.load_prefix(0, to_dev(Kb[None], "bf16"), to_dev(Vb[None], "bf16"))
    q, qb = W.query_stream(wl, 0, 0)
    (kd, kdb), (vd, vdb) = W.kv_decode_tokens(wl, 0, 0)
    out = torch.empty((1, 8, 128), dtype=torch.float32, device="cuda")
    from paper_2505_13109_amd import binding as B
    for t in range(2):
        g.decode_step(0, to_dev(qb[t][None], "bf16"), to_dev(kdb[t][None], "bf16"), to_dev(vdb[t][None], "bf16"), out)
        ref = o.step(q[t], kd[t], vd[t])
        assert ref["geom"].n_cand > 15300
        assert np.array_equal(g.debug_read(0, B.DBG_ACTIVE_IDS)[0], ref["new_ids"]), t
        assert np.array_equal(g.debug_read(0, B.DBG_FLAGS)[0], ref["flags"]), t
        assert rel_err_per_head(out.cpu().numpy()[0], ref["out"]).max() <= 2e-3
    g.health(0)
    g.close()


def test_many_requests_take_the_bandwidth_bound_dispatch():
    """40 requests x 8 KV heads: past the size of the one-launch layer kernel, so the step runs as separate
    launches with the selection in a launch of its own and one attention block per head."""
    wl = W.Workload("many", 1, 40, 32, 8, "bf16", 3000, 512, 64, 64, 0.8, 6, 0.8, 0.6, 61)
    pr = _pair(wl, [0])
    for t in range(wl.steps):
        pr.step(0, t, deep=(t % 2 == 0))
    assert pr.g.step_launches(0) > 1
    assert 0 < pr.stats["flagged"] < pr.stats["heads"]
    print("many", pr.stats)
    pr.close()


def test_big_scan_blocks_take_several_chunks():
    """24 requests x 16 KV heads x 12K tokens: the scoring launch is past the size where a block takes
    several chunks of its head in turn (and 4 passes per chunk)."""
    wl = W.Workload("scan", 1, 24, 16, 16, "bf16", 12000, 1024, 64, 64, 0.8, 3, 0.8, 0.6, 71)
    pr = _pair(wl, [0])
    for t in range(wl.steps):
        pr.step(0, t)
    assert pr.g.step_launches(0) == 3        # scoring, selection, attention
    pr.close()


def test_pooling_variants_with_the_host_pool():
    """A selection variant together with max-pooled correction on the host-pool placement: the recall plan
    follows whatever the variant selects."""
    wl = W.get_workload("c3").scaled(batch=2, ctx=6000, steps=30)
    pr = _pair(wl, [3], steps=30, select_pooling="MaxQK", corr_pooling="min")
    for t in range(30):
        pr.step(0, t)
    assert pr.stats["misses"] > 0 and 0 < pr.stats["flagged"] < pr.stats["heads"]
    pr.close()


def test_host_pool_deferred_recall_shared_by_groups_of_layers():
    """Eleven layers with the KV in the host pool, one launch per layer-step.  The recall of the uncorrected heads
    (Sec. 3.2: off the critical path, for the next step) is kept back and submitted for several layers at once (a
    quarter of the layers: here two), so nothing is read back here until a whole decode step of all layers has been
    enqueued: first full steps (groups of two, the eleventh layer alone as the context's last), then steps over five
    layers only, where the fifth layer's recall stays on the list until the same layers step again, then an explicit
    fkv_flush before the copy stream is synchronised and the page cache inspected."""
    wl = W.get_workload("c3").scaled(batch=1, ctx=4096 - 9, steps=20)
    n_lay = 11
    pr = _pair(wl, list(range(0, 2 * n_lay, 2)), steps=20)

    def whole_step(t, layers):
        res, outs = {}, {}
        for li in layers:
            res[li] = pr.step(li, t, check=False)
            assert pr.g.step_launches(li) == 1
            outs[li] = pr.out.clone()                 # (device-side copy on the compute stream: no call into the library)
        return res, outs

    def compare(t, res, outs):
        for li in res:
            got = pr.read_step(li, deep=False)
            got["out"] = outs[li].cpu().numpy()
            pr.compare(li, t, res[li], got, False)

    t = 0
    for _ in range(10):
        res, outs = whole_step(t, range(n_lay))
        compare(t, res, outs)
        t += 1
    # five layers only, two steps without a read in between: the fifth layer's recall stays on the list until the same
    # layers step again (the other six layers rest: each layer's context is its own)
    from harness import rel_err_per_head, TOL_OUT
    res_a, outs_a = whole_step(t, range(5))
    t += 1
    res_b, outs_b = whole_step(t, range(5))
    compare(t, res_b, outs_b)
    t += 1
    for li in res_a:                                  # of the step before, only the outputs are still around
        assert rel_err_per_head(outs_a[li].cpu().numpy()[0], res_a[li][0]["out"]).max() <= TOL_OUT
    res, outs = whole_step(t, range(5))
    pr.g.flush()
    pr.copy_stream.synchronize()
    torch.cuda.current_stream().synchronize()
    compare(t, res, outs)
    for li in (0, 4):
        pr.check_cached_pages(li, 0, 3, where=2)
    assert pr.stats["misses"] > 0 and 0 < pr.stats["flagged"] < pr.stats["heads"]
    print("deferred groups", pr.stats)
    pr.close()


def test_host_pool_fp16_ragged_growth():
    """fp16, G = 5, two requests, host pool, context growing from 40 tokens through page fills (offloads),
    the first candidates and the first recalls."""
    wl = W.Workload("hostgrow", 1, 2, 10, 2, "fp16", 40, 256, 32, 64, 0.75, 260, 0.75, 0.66, 81, placement=1, shift_every=70)
    pr = _pair(wl, [4])
    for t in range(wl.steps):
        pr.step(0, t, deep=(t % 5 == 0))
        assert pr.g.step_launches(0) == 1
        if t % 64 == 63:
            torch.cuda.synchronize()
            pr.check_cached_pages(0, 1, 1, where=1)
            pr.check_cached_pages(0, 0, 0, where=2)
    assert pr.stats["misses"] > 0 and 0 < pr.stats["flagged"] < pr.stats["heads"]
    print("hostgrow", pr.stats)
    pr.close()


def test_a_seeded_sample_of_small_shapes():
    """Forty shapes drawn from a seeded generator: group size, heads, requests, budget / sink / window,
    context length, dtype, placement, pooling variants; 24 steps each, every step compared."""
    rng = np.random.default_rng(2025)
    for i in range(40):
        G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8]))
        n_kv = int(rng.choice([1, 2, 3, 4]))
        batch = int(rng.choice([1, 1, 2, 3]))
        sink = int(rng.choice([0, 32, 64, 128]))
        window = int(rng.choice([0, 32, 64, 96]))
        k = int(rng.choice([1, 2, 5, 9, 16]))
        ctx = int(rng.integers(1, 2600))
        dtype = str(rng.choice(["bf16", "fp16"]))
        placement = int(rng.choice([0, 0, 1]))
        sp = str(rng.choice(["MeanS", "MeanS", "MaxS", "MeanQK", "MaxQK", "MeanQ", "MaxQ"]))
        cp = str(rng.choice(["mean", "mean", "max", "min"]))
        tau = float(rng.choice([0.6, 0.75, 0.85]))
        wl = W.Workload(f"rand{i}", 1, batch, G * n_kv, n_kv, dtype, ctx, sink + window + 32 * k, sink, window, tau, 24,
                        0.8, 0.6, 300 + i, placement=placement, shift_every=11)
        tag = f"shape {i}: G {G} n_kv {n_kv} batch {batch} S {sink} W {window} k {k} ctx {ctx} {dtype} placement {placement} {sp}/{cp} tau {tau}"
        print(tag, flush=True)
        pr = _pair(wl, [i], select_pooling=sp, corr_pooling=cp)
        for t in range(wl.steps):
            pr.step(0, t)
        pr.close()


def test_selection_paths_of_the_separate_step_kernel():
    """The host-pool placement always takes the separate step kernel.  Candidate counts on both sides of its
    register / LDS-staging thresholds, for small and large groups, with the selection inside the scoring
    launch (few blocks) and in a launch of its own (many blocks)."""
    shapes = [  # (G, n_kv, batch, ctx): n_cand = ctx/32 - 4
        (8, 1, 1, 30000),     # 933 candidates, G > 4: in registers, 2 per thread
        (8, 1, 1, 50000),     # 1558 candidates, G > 4: staged in LDS
        (3, 2, 1, 50000),     # 1558 candidates, G <= 4: in registers, 4 per thread
        (4, 2, 2, 90000),     # 2808 candidates: staged in LDS, selection in its own launch
        (6, 2, 3, 20000),     # 621 candidates: 2 per thread
        (4, 2, 1, 200000),    # 6246 candidates: the selection of a head spread over 13 blocks (maxima, sums, short lists, merge)
        (7, 1, 2, 170000),    # 5308 candidates, G = 7, two requests: 11 blocks per head
    ]
    for i, (G, n_kv, batch, ctx) in enumerate(shapes):
        wl = W.Workload(f"sel{i}", 1, batch, G * n_kv, n_kv, "bf16", ctx, 1024, 64, 64, 0.8, 5, 0.8, 0.6, 400 + i, placement=1)
        print(wl.name, G, n_kv, batch, ctx, flush=True)
        pr = _pair(wl, [i])
        for t in range(wl.steps):
            pr.step(0, t)
        assert pr.stats["misses"] > 0
        pr.close()
