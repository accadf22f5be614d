"""A decoder layer stack around the retrieval loop (Sec. 3.2 "Speculative retrieval": selection and recall
overlap the rest of the layer -- attention output projection, FFN, the next layer's QKV projection).

The retrieval step itself is `fkv_decode_step` of the HIP library, unchanged.  Around it this module puts
what a Llama-shaped layer does for one token: RMSNorm, the QKV projection, rotary embedding, the output
projection and a SwiGLU FFN, as plain library GEMVs and elementwise PyTorch ops on the compute stream
(they are context for the loop -- something real for the deferred recall to hide behind and a closed loop in
which the layer's own q, k, v drive the selection -- not a tuned layer).  Weights are random (there are no
checkpoints here); the cached context of each layer is synthetic and loaded by the caller.

`step()` feeds one hidden state per request through all layers.  With `external_qkv` the loop's q, k, v are
taken from the caller (seeded synthetic streams with a set adjacent-step similarity) while the projections
still run and are dropped: that keeps a workload's reuse and correction statistics, which random weights
would not produce.
"""
from __future__ import annotations

import torch

from .binding import FreeKV


class DecoderStack:
    def __init__(self, fkv: FreeKV, *, ffn_mult: float = 3.5, seed: int = 7, rope_base: float = 500000.0,
                 copy_stream: torch.cuda.Stream | None = None):
        c = fkv.cfg
        self.fkv = fkv
        self.n_layers, self.batch = c.n_layers, c.batch
        self.n_q, self.n_kv, self.d = c.n_q_heads, c.n_kv_heads, c.head_dim
        self.hidden = self.n_q * self.d
        self.ffn = int(ffn_mult * self.hidden)
        self.dtype = fkv.torch_dtype
        dev = fkv.device
        g = torch.Generator(device=dev).manual_seed(seed)

        def mk(*shape, scale):
            return (torch.randn(*shape, generator=g, device=dev, dtype=torch.float32) * scale).to(self.dtype)

        qkv_out = (self.n_q + 2 * self.n_kv) * self.d
        s_in = self.hidden ** -0.5
        self.wqkv = [mk(self.hidden, qkv_out, scale=s_in) for _ in range(self.n_layers)]
        self.wo = [mk(self.hidden, self.hidden, scale=s_in) for _ in range(self.n_layers)]
        self.wgu = [mk(self.hidden, 2 * self.ffn, scale=s_in) for _ in range(self.n_layers)]
        self.wd = [mk(self.ffn, self.hidden, scale=self.ffn ** -0.5) for _ in range(self.n_layers)]
        self.inv_freq = (rope_base ** (-torch.arange(0, self.d, 2, device=dev, dtype=torch.float32) / self.d))
        self.out = torch.empty((self.n_layers, self.batch, self.n_q, self.d), dtype=torch.float32, device=dev)
        self.copy_stream = copy_stream
        self.last_qkv = [None] * self.n_layers       # what each layer fed to the loop at the last step (for tests)
        self.weight_bytes_per_layer = (self.hidden * qkv_out + self.hidden * self.hidden + 3 * self.hidden * self.ffn) * 2

    def _rms(self, x):
        return torch.nn.functional.rms_norm(x, (self.hidden,), eps=1e-5)

    def _rope(self, x, cos, sin):
        """x [batch, heads, d]; rotate pairs (i, i + d/2) by pos * inv_freq[i]."""
        a, b = x[..., : self.d // 2], x[..., self.d // 2:]
        return torch.cat([a * cos - b * sin, a * sin + b * cos], dim=-1)

    def step(self, x, external_qkv=None, stream=None):
        """x [batch, hidden] -> [batch, hidden].  external_qkv: per layer (q [batch,n_q,d], k, v [batch,n_kv,d])."""
        pos_cached, cos, sin = None, None, None
        for layer in range(self.n_layers):
            pos = self.fkv.context_len(layer)                   # position of the token being appended
            if pos != pos_cached:                               # (the layers of one model share it)
                ang = float(pos) * self.inv_freq
                cos, sin, pos_cached = ang.cos().to(self.dtype), ang.sin().to(self.dtype), pos
            qkv = (self._rms(x) @ self.wqkv[layer]).view(self.batch, self.n_q + 2 * self.n_kv, self.d)
            qk = self._rope(qkv[:, : self.n_q + self.n_kv], cos, sin)       # queries and keys in one go
            q, k = qk[:, : self.n_q].contiguous(), qk[:, self.n_q:].contiguous()
            v = qkv[:, self.n_q + self.n_kv:].contiguous()
            if external_qkv is not None:
                q, k, v = external_qkv[layer]
            self.last_qkv[layer] = (q, k, v)
            self.fkv.decode_step(layer, q, k, v, self.out[layer], stream=stream, copy_stream=self.copy_stream)
            x = x + self.out[layer].to(self.dtype).view(self.batch, self.hidden) @ self.wo[layer]
            gu = self._rms(x) @ self.wgu[layer]
            x = x + (torch.nn.functional.silu(gu[:, : self.ffn]) * gu[:, self.ffn:]) @ self.wd[layer]
        return x
