"""The attention entry point that allocates nothing (its split partials and counters live in a static
device array the library owns) against the ordinary one, through the C ABI: two calls in a row, the
second on a smaller input, then the first shape again -- the array keeps the previous call's contents,
so stale partials or counters would show.  Same kernels, same split: the outputs must be bit-equal,
and both stay within 2e-3 of the CPU oracle."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def _ready(wl, layer):
    """A context with one appended token, the correction test and the selection done (nothing committed)."""
    from harness import Pair
    pr = Pair(wl, [layer])
    q, k, v = pr.step_inputs(0, 0)
    pr.g.kv_append(0, k, v)
    pr.g.corr_check(0, q)
    pr.g.page_select(0, q)
    for r in range(wl.batch):
        pr.oracles[(0, r)].append(pr.kd[(0, r)][0][0], pr.vd[(0, r)][0][0])
    return pr, q


def _both(pr, q, use):
    import paper_2505_13109_amd as fkv
    wl = pr.wl
    ref = torch.full((wl.batch, wl.n_q_heads, 128), 7.0, dtype=torch.float32, device="cuda")
    got = torch.full_like(ref, -7.0)
    pr.g.sparse_decode_attn(0, q, ref, use=use)
    pr.g.sparse_decode_attn_static(0, q, got, use=use)
    torch.cuda.synchronize()
    assert torch.equal(got, ref), f"static-scratch attention differs from the arena one ({wl.name})"
    if use == fkv.FKV_USE_PENDING:
        from harness import rel_err_per_head
        for r in range(wl.batch):
            o = pr.oracles[(0, r)]
            ids, _, _ = o.select(pr.q[(0, r)][0][0])
            err = rel_err_per_head(got.cpu().numpy()[r], o.attend(pr.q[(0, r)][0][0], ids))
            assert err.max() <= 2e-3, (wl.name, float(err.max()))
    return got


def test_static_scratch_attention_matches_twice_in_a_row_second_call_smaller():
    import paper_2505_13109_amd as fkv
    big = W.Workload("na_big", 1, 2, 32, 8, "bf16", 9000, 1024, 128, 128, 0.8, 2, 0.8, 0.6, 901)
    small = W.Workload("na_small", 1, 1, 6, 2, "fp16", 1500, 256, 32, 64, 0.8, 2, 0.8, 0.6, 902)
    pa, qa = _ready(big, 0)
    pb, qb = _ready(small, 1)
    first = _both(pa, qa, fkv.FKV_USE_PENDING).clone()
    _both(pb, qb, fkv.FKV_USE_PENDING)                  # smaller input right behind the bigger one
    _both(pb, qb, fkv.FKV_USE_ACTIVE)                   # nothing picked yet: sink + window + open page only
    again = _both(pa, qa, fkv.FKV_USE_PENDING)          # and the first shape again on the used array
    assert torch.equal(first, again)
    pa.close()
    pb.close()


def test_static_scratch_refuses_a_shape_that_does_not_fit():
    """255 single-KV-head requests with G = 8 and 65 attended pages take two splits per head:
    255 x 2 x 8 x (128 + 2) floats plus the counters is just past the 2 MiB the library holds.  Refused with
    a message that names both sizes; the arena variant takes the same shape."""
    import paper_2505_13109_amd as fkv
    from harness import to_dev
    g = fkv.FreeKV(n_layers=1, batch=255, n_q_heads=8, n_kv_heads=1, max_ctx=2112, budget=2048, sink=512,
                   window=512, tau=0.8, dtype="bf16")
    rng = np.random.default_rng(5)
    kv = to_dev(W.encode(rng.standard_normal((255, 2100, 1, 128)).astype(np.float32), "bf16"), "bf16")
    g.load_prefix(0, kv, kv)
    q = to_dev(W.encode(rng.standard_normal((255, 8, 128)).astype(np.float32), "bf16"), "bf16")
    out = torch.zeros((255, 8, 128), dtype=torch.float32, device="cuda")
    g.sparse_decode_attn(0, q, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    with pytest.raises(fkv.FreeKVError, match="static scratch too small: this shape needs 2122752 bytes, the library holds 2097152"):
        g.sparse_decode_attn_static(0, q, out)
    g.close()
