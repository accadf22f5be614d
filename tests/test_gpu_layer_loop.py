"""The decoder layer stack around the retrieval loop (paper_2505_13109_amd/layer_loop.py) on a real MI355X:
a closed loop in which each layer's own projected, rotated q, k, v drive the retrieval step.  The oracle is
fed the very q, k, v the layer produced on the GPU (copied back bit for bit), one oracle per (layer,
request), and every layer-step is compared: page ids and flags exact, attention within 2e-3."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import freekv_oracle as O

pytestmark = pytest.mark.gpu


def _f32(t):
    """bf16 / fp16 device tensor -> float32 numpy, exact."""
    return t.float().cpu().numpy()


@pytest.mark.parametrize("placement", [0, 1])
def test_layers_own_qkv_drive_the_retrieval_loop(placement):
    import paper_2505_13109_amd as fkv
    from paper_2505_13109_amd.layer_loop import DecoderStack
    from harness import to_dev, rel_err_per_head
    n_layers, batch, n_q, n_kv, ctx, steps = 3, 2, 8, 2, 5000 - 9, 40
    wl = W.Workload("loop", n_layers, batch, n_q, n_kv, "bf16", ctx, 1024, 128, 128, 0.8, steps, 0.9, 0.436, 700, placement=placement)
    g = fkv.FreeKV(n_layers=n_layers, batch=batch, n_q_heads=n_q, n_kv_heads=n_kv, max_ctx=wl.max_ctx, budget=wl.budget,
                   sink=wl.sink, window=wl.window, tau=wl.tau, dtype="bf16", placement=placement)
    oracles = {}
    for layer in range(n_layers):
        Kb_all, Vb_all = [], []
        for r in range(batch):
            (K, Kb), (V, Vb) = W.kv_prefix(wl, layer, r)
            o = O.FreeKVOracle(n_q, n_kv, 128, 32, wl.budget, wl.sink, wl.window, wl.tau, wl.max_ctx)
            o.load_prefix_bulk(K, V)
            oracles[(layer, r)] = o
            Kb_all.append(Kb); Vb_all.append(Vb)
        g.load_prefix(layer, to_dev(np.stack(Kb_all), "bf16"), to_dev(np.stack(Vb_all), "bf16"))
    stack = DecoderStack(g, ffn_mult=2.0, copy_stream=torch.cuda.Stream())
    # hidden states: a step-correlated stream, so that some steps reuse and some correct
    gen = torch.Generator(device="cuda").manual_seed(5)
    state = torch.randn((batch, stack.hidden), generator=gen, device="cuda")
    flagged = heads = 0
    worst = 0.0
    for t in range(steps):
        rho = 0.2 if t % 9 == 8 else 0.97                      # now and then the hidden state jumps
        state = rho * state + (1 - rho * rho) ** 0.5 * torch.randn((batch, stack.hidden), generator=gen, device="cuda")
        y = stack.step(state.to(torch.bfloat16))
        torch.cuda.synchronize()
        assert torch.isfinite(y).all()
        for layer in range(n_layers):
            q, k, v = (_f32(x) for x in stack.last_qkv[layer])
            ids = g.debug_read(layer, fkv.binding.DBG_ACTIVE_IDS)
            # flags of a layer are overwritten by nothing until its next step
            flags = g.debug_read(layer, fkv.binding.DBG_FLAGS)
            out = stack.out[layer].cpu().numpy()
            for r in range(batch):
                ref = oracles[(layer, r)].step(q[r], k[r], v[r])
                tag = f"step {t} layer {layer} request {r}"
                assert np.array_equal(flags[r], ref["flags"]), tag
                assert np.array_equal(ids[r], ref["new_ids"]), tag
                err = rel_err_per_head(out[r], ref["out"]).max()
                assert err <= 2e-3, (tag, err)
                worst = max(worst, float(err))
                flagged += int(ref["flags"].sum()); heads += n_kv
    assert 0 < flagged < heads, (flagged, heads)           # both reuse and correction were exercised
    print("layer loop placement", placement, "flagged", flagged, "of", heads, "max rel err", worst)
    for layer in range(n_layers):
        g.health(layer)
    g.close()
