"""Device-side synthetic workloads at the sizes the benchmark times.

Input plumbing only (no method arithmetic): seeded torch generators fill the
query/key tensors directly in HBM, because the host generators of `synth` would
take minutes at these sizes.  Shapes and statistics follow the long-context
configuration: Llama-3-8B-shaped layers (32 query heads sharing 8 KV heads,
d = 128), 32768 prompt tokens per layer, bf16, N(0,1) values with a few
magnified "outlier" channels per KV head in the keys.
"""
from __future__ import annotations

import numpy as np
import torch

from . import synth


class LongContext:
    """Config "long context": layers x kv_heads heads stacked along the head axis."""

    def __init__(self, layers: int = 32, kv_heads: int = 8, q_per_kv: int = 4, n_tokens: int = 32768,
                 d: int = 128, r: int = 32, lam: float = 1e-3, bits: int = 2, group: int = 32, g: int = 32,
                 seed: int = 5000, device: str = "cuda:0", planted_rank: int = 0):
        self.layers, self.kv_heads, self.q_per_kv, self.n_tokens, self.d = layers, kv_heads, q_per_kv, n_tokens, d
        self.r, self.lam, self.bits, self.group, self.g = r, lam, bits, group, g
        self.heads = layers * kv_heads
        self.device = torch.device(device)
        gen = torch.Generator(device=self.device)
        gen.manual_seed(seed)
        hgen = synth.rng(seed)
        # keys [1, heads, n, d]
        self.k = torch.empty((1, self.heads, n_tokens, d), dtype=torch.bfloat16, device=self.device)
        oc = synth.outlier_channels(hgen, self.heads, d)
        for h0 in range(0, self.heads, kv_heads):
            x = torch.randn((kv_heads, n_tokens, d), generator=gen, device=self.device, dtype=torch.float32)
            fac = np.ones((kv_heads, 1, d), dtype=np.float32)
            for j in range(kv_heads):
                idx, f = oc[h0 + j]
                fac[j, 0, idx] = f
            x *= torch.from_numpy(fac).to(self.device)
            self.k[0, h0:h0 + kv_heads] = x.to(torch.bfloat16)
            del x
        # queries [heads * q_per_kv, n, d]
        self.q = torch.empty((self.heads * q_per_kv, n_tokens, d), dtype=torch.bfloat16, device=self.device)
        for h0 in range(0, self.heads * q_per_kv, 32):
            x = torch.randn((32, n_tokens, d), generator=gen, device=self.device, dtype=torch.float32)
            if planted_rank > 0:
                # amplify a shared random orthonormal set of directions per KV head
                for j in range(0, 32, q_per_kv):
                    B, _ = np.linalg.qr(hgen.standard_normal((d, planted_rank)))
                    gains = 4.0 * (0.85 ** np.arange(planted_rank))
                    Bt = torch.from_numpy(B.astype(np.float32)).to(self.device)
                    gt = torch.from_numpy(gains.astype(np.float32)).to(self.device)
                    blk = x[j:j + q_per_kv]
                    blk += ((blk @ Bt) * gt) @ Bt.T
            self.q[h0:h0 + 32] = x.to(torch.bfloat16)
            del x
        torch.cuda.synchronize(self.device)

    @property
    def n_keys(self) -> int:
        return self.heads * self.n_tokens

    def key_bytes(self) -> int:
        """Algorithmic bytes per key of the quantize pass: input row + packed codes + fp16 scale and zero."""
        return self.d * 2 + self.d * self.bits // 8 + 2 * 2 * (self.d // self.group)
