"""The attention entry point that allocates nothing (its chunk partials live in a device array built into the
library) against the entry point that takes a caller's scratch buffer: same kernels, so bit-equal outputs,
and both within the decode-attention tolerance of the oracle.  Two calls in a row share the array, the second
with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2406_00059_amd as ld
from helpers import device_pool
from test_kernels_gpu import _attention_case, _attn_tol, _oracle_attention, _run_attention

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _run_static(table, pool, q, lens, H, Hkv, hd, window=0):
    B = len(lens)
    ctx = torch.tensor(lens, dtype=torch.int32, device=DEV)
    slot = torch.arange(B, dtype=torch.int32, device=DEV)
    out = torch.full((B, H, hd), float("nan"), device=DEV)
    ld.ldk_paged_attention_static(q, H * hd, device_pool(pool), table.to(DEV), slot, ctx, max(lens), H, Hkv, hd, out,
                                  window=window)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("dtype,hd,H,Hkv,window", [("bf16", 128, 32, 32, 0), ("bf16", 128, 32, 8, 0), ("f32", 64, 4, 4, 0),
                                                   ("bf16", 128, 8, 2, 100)])
def test_static_scratch_attention_two_calls_second_smaller(dtype, hd, H, Hkv, window):
    big = [1, 2, 15, 16, 17, 63, 255, 256, 257, 300, 1025, 2500, 4096]
    small = [300, 17, 1]
    cases = []
    for seed, lens in ((31, big), (32, small)):
        table, pool, q = _attention_case(seed, lens, H, Hkv, hd, dtype)
        cases.append((table, pool, q, lens))
    # both calls on the built-in array first, back to back, then the reference runs
    got = [_run_static(t, p, q, lens, H, Hkv, hd, window) for t, p, q, lens in cases]
    for (t, p, q, lens), g in zip(cases, got):
        assert np.isfinite(g).all()
        same = _run_attention(t, p, q, lens, H, Hkv, hd, window=window)
        assert np.array_equal(g, same), "the built-in scratch array changed the result"
        ref = _oracle_attention(t, p, q, lens, Hkv, hd, window=window)
        assert np.max(np.abs(g - ref)) <= _attn_tol(dtype, hd, H, Hkv) * np.abs(ref).max() + 1e-6


def test_static_scratch_attention_refuses_what_does_not_fit():
    H, hd, T, ctx = 64, 128, 256, 16384
    assert ld.ldk_attention_scratch_bytes(T, H, H, hd, ctx) > ld.ldk_static_scratch_bytes()
    out = torch.zeros(T, H, hd, device=DEV)
    dummy = torch.zeros(16, dtype=torch.int32, device=DEV)
    rc = ld.ldk_paged_attention_static(out, H * hd, torch.zeros(16, dtype=torch.bfloat16, device=DEV), dummy.view(1, 16),
                                       dummy, dummy, ctx, H, H, hd, out, check=False)
    assert rc == ld.LD_E_RANGE and "exceed" in ld.ld_last_error()
    assert float(out.abs().max()) == 0.0
