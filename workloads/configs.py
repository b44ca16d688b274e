"""Decoder shapes of the five workloads and the seeded weight recipe.

Matrices and the embedding are N(0, 0.02^2); RMSNorm gains are 1 + 0.02 N(0,1)
so that a dropped gain multiply changes the result.  For the bf16 shapes the
matrices are rounded once to bf16 (round-to-nearest-even) here, and both the
oracle and the GPU path consume those rounded values.  Gains stay fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import torch

from . import gen

SEED_BASE = 20240600


@dataclass(frozen=True)
class DecoderShape:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str            # "f32" | "bf16": storage type of matrices and of the KV pool
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    kv_block: int = 16
    window: int = 0       # > 0: banded attention over the last `window` positions; 0: all preceding positions

    def with_layers(self, n: int) -> "DecoderShape":
        return replace(self, n_layers=n, name=f"{self.name}-{n}L")

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * self.n_layers * (4 if self.dtype == "f32" else 2)

    @property
    def weight_bytes_per_step(self) -> int:
        """Bytes of weights one decode step must read: all layers, LM head, gains (not the embedding table)."""
        e = 4 if self.dtype == "f32" else 2
        d, f = self.d_model, self.d_ffn
        qkv = (self.n_heads + 2 * self.n_kv_heads) * self.head_dim * d
        per_layer = qkv + self.n_heads * self.head_dim * d + 3 * d * f
        return (per_layer * self.n_layers + self.vocab * d) * e + (2 * self.n_layers + 1) * d * 4


TINY = DecoderShape("tiny", 2, 256, 4, 4, 64, 688, 1024, "f32")
LLAMA7B = DecoderShape("7b", 32, 4096, 32, 32, 128, 11008, 32000, "bf16")
LLAMA13B = DecoderShape("13b", 40, 5120, 40, 40, 128, 13824, 32000, "bf16")
# grouped key/value heads (4 query heads per KV head) and a 4096-position attention band
MISTRAL7B = DecoderShape("7b-gqa", 32, 4096, 32, 8, 128, 14336, 32000, "bf16", window=4096)


def _matrix(seed, stream, rows, cols, shape: DecoderShape, device):
    w = gen.normal(seed, stream, (rows, cols), std=0.02, device=device)
    return w.to(torch.bfloat16) if shape.dtype == "bf16" else w


def make_weights(shape: DecoderShape, seed: int, device="cpu") -> dict:
    """All tensors of one decoder, generated on `device`.

    Layout (row-major, output row first, so one output is one contiguous dot product):
      embed, lm_head [vocab, d]; wqkv [(H + 2 Hkv) hd, d] (q rows, then k rows, then v rows);
      wo [d, H hd]; wgate_up [2 ffn, d] (gate rows, then up rows); wdown [d, ffn];
      attn_norm, ffn_norm, final_norm [d] fp32.
    """
    d, f, hd = shape.d_model, shape.d_ffn, shape.head_dim
    nq, nkv = shape.n_heads * hd, shape.n_kv_heads * hd
    w = {
        "embed": _matrix(seed, 1, shape.vocab, d, shape, device),
        "lm_head": _matrix(seed, 2, shape.vocab, d, shape, device),
        "final_norm": gen.normal(seed, 3, (d,), std=0.02, mean=1.0, device=device),
        "attn_norm": [], "wqkv": [], "wo": [], "ffn_norm": [], "wgate_up": [], "wdown": [],
    }
    for l in range(shape.n_layers):
        s = 16 * (l + 1)
        w["attn_norm"].append(gen.normal(seed, s + 0, (d,), std=0.02, mean=1.0, device=device))
        w["wqkv"].append(_matrix(seed, s + 1, nq + 2 * nkv, d, shape, device))
        w["wo"].append(_matrix(seed, s + 2, d, nq, shape, device))
        w["ffn_norm"].append(gen.normal(seed, s + 3, (d,), std=0.02, mean=1.0, device=device))
        w["wgate_up"].append(_matrix(seed, s + 4, 2 * f, d, shape, device))
        w["wdown"].append(_matrix(seed, s + 5, d, f, shape, device))
    return w


def weights_to(w: dict, device) -> dict:
    """Copy of a weight dict on another device (same values, same dtypes)."""
    out = {}
    for k, v in w.items():
        out[k] = [t.to(device) for t in v] if isinstance(v, list) else v.to(device)
    return out
