"""Per-kernel parity on the GPU: every kernel-level entry point against the oracle's step functions
on the same seeded inputs, element by element, at sizes spanning several tiles and ragged tails."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2406_00059_amd as ld
from workloads import gen
from helpers import device_pool, logical_pool

pytestmark = pytest.mark.gpu
DEV = "cuda"


_silu = np.vectorize(oracle.silu, otypes=[np.float64])      # the oracle's activation, element by element


def _mat(seed, stream, n, k, dtype):
    w = gen.normal(seed, stream, (n, k), std=0.05)
    return w.bfloat16() if dtype == "bf16" else w


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T", [1, 2, 3, 4, 7, 8, 19])
def test_linear_store_add_and_fused_norm(dtype, T):
    N, K = 301, 688           # ragged row count, K not a multiple of 512
    W = _mat(1, 1, N, K, dtype); x = gen.normal(1, 2, (T, K)); g = gen.normal(1, 3, (K,), std=0.1, mean=1.0)
    y0 = gen.normal(1, 4, (T, N))
    Wh = oracle.to_host_matrix(W)
    Wd, xd, gd = W.to(DEV), x.to(DEV), g.to(DEV)
    y = torch.empty(T, N, device=DEV)
    ld.ldk_linear(Wd, xd, y, ld.LDK_STORE)
    ref = np.stack([oracle.matvec(Wh, x[t].numpy()) for t in range(T)])
    np.testing.assert_allclose(y.cpu().numpy(), ref, rtol=0, atol=2e-6 * np.abs(ref).max())
    y = y0.to(DEV).clone()
    ld.ldk_linear(Wd, xd, y, ld.LDK_ADD, g=gd, eps=1e-5)
    refn = np.stack([oracle.matvec(Wh, oracle.rmsnorm(x[t].numpy(), g.numpy(), 1e-5)) for t in range(T)])
    np.testing.assert_allclose(y.cpu().numpy(), y0.numpy() + refn, rtol=0, atol=3e-6 * np.abs(refn).max())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T", [1, 2, 3, 4, 5])
def test_linear_swiglu(dtype, T):
    F, K = 173, 256
    W = _mat(2, 1, 2 * F, K, dtype); x = gen.normal(2, 2, (T, K)); g = gen.normal(2, 3, (K,), std=0.1, mean=1.0)
    Wh = oracle.to_host_matrix(W)
    y = torch.empty(T, F, device=DEV)
    ld.ldk_linear(W.to(DEV), x.to(DEV), y, ld.LDK_SWIGLU, g=g.to(DEV), eps=1e-5)
    for t in range(T):
        gu = oracle.matvec(Wh, oracle.rmsnorm(x[t].numpy(), g.numpy(), 1e-5))
        ref = np.array([oracle.silu(gu[i]) * gu[F + i] for i in range(F)])
        np.testing.assert_allclose(y[t].cpu().numpy(), ref, rtol=0, atol=3e-6 * np.abs(ref).max())


def test_linear_full_7b_shapes_on_sampled_outputs():
    """The launch shapes of the 7B decode step (T = 1), checked on sampled output rows."""
    for N, K, epi in [(12288, 4096, ld.LDK_STORE), (4096, 11008, ld.LDK_ADD), (11008, 4096, ld.LDK_SWIGLU),
                      (32000, 4096, ld.LDK_STORE)]:
        rows = N * (2 if epi == ld.LDK_SWIGLU else 1)
        W = gen.normal(3, N, (rows, K), std=0.02, device=DEV).bfloat16()
        x = gen.normal(3, 7, (1, K), device=DEV)
        y = torch.zeros(1, N, device=DEV)
        ld.ldk_linear(W, x, y, epi)
        idx = gen.randint(3, 9, 0, N - 1, 48).tolist() + [0, N - 1]
        xh = x[0].cpu().numpy()
        for n in idx:
            a = oracle.matvec(oracle.to_host_matrix(W[n:n + 1]), xh)[0]
            if epi == ld.LDK_SWIGLU:
                a = oracle.silu(a) * oracle.matvec(oracle.to_host_matrix(W[N + n:N + n + 1]), xh)[0]
            assert abs(y[0, n].item() - a) <= 1e-5 * max(1.0, abs(a)) + 2e-6 * math.sqrt(K) * 0.02


def test_embed_and_rmsnorm_gather():
    E = _mat(4, 1, 50, 256, "bf16"); tok = torch.tensor([3, 49, 0, 3], dtype=torch.int32)
    x = torch.empty(4, 256, device=DEV)
    ld.ldk_embed(E.to(DEV), tok.to(DEV), x)
    assert torch.equal(x.cpu(), E.float()[tok.long()])
    g = gen.normal(4, 2, (256,), std=0.1, mean=1.0)
    idx = torch.tensor([2, 0], dtype=torch.int32)
    out = torch.empty(2, 256, device=DEV)
    ld.ldk_rmsnorm(x, g.to(DEV), out, 1e-5, row_idx=idx.to(DEV))
    for r, src in enumerate([2, 0]):
        ref = oracle.rmsnorm(x[src].cpu().numpy(), g.numpy(), 1e-5)
        np.testing.assert_allclose(out[r].cpu().numpy(), ref, rtol=2e-6, atol=1e-7)


@pytest.mark.parametrize("dtype,hd", [("f32", 64), ("bf16", 128)])
def test_rope_and_cache_append_values_and_block_indexing(dtype, hd):
    H, Hkv, T, nblk = 4, 2, 5, 9
    nqkv = (H + 2 * Hkv) * hd
    qkv = gen.normal(5, 1, (T, nqkv))
    pos = torch.tensor([0, 15, 16, 17, 4000], dtype=torch.int32)
    slot = torch.tensor([0, 1, 1, 1, 2], dtype=torch.int32)
    table = torch.full((3, 256), -1, dtype=torch.int32)
    table[0, 0] = 4; table[1, 0] = 7; table[1, 1] = 2; table[2, 4000 // 16] = 5
    pdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    pool = torch.full((nblk, 2, Hkv, 16, hd), 512.0, dtype=pdt, device=DEV)
    cs = torch.empty(T, hd // 2, 2, device=DEV)
    q = qkv.to(DEV).clone()
    ld.ldk_rope_table(pos.to(DEV), hd, 10000.0, cs)
    ld.ldk_rope_kv_write(q, cs, pos.to(DEV), slot.to(DEV), table.to(DEV), pool, H, Hkv, hd)
    q, pool_h = q.cpu().numpy(), logical_pool(pool).float().cpu().numpy().astype(np.float64)
    touched = np.zeros(pool_h.shape[:4], bool)
    for t in range(T):
        p = int(pos[t]); blk = int(table[slot[t], p // 16]); s = p % 16
        for h in range(H):
            ref = oracle.rope_head(qkv[t, h * hd:(h + 1) * hd].numpy(), p)
            np.testing.assert_allclose(q[t, h * hd:(h + 1) * hd], ref, rtol=0, atol=4e-7 * np.abs(ref).max() + 1e-7)
        for j in range(Hkv):
            k = oracle.rope_head(qkv[t, (H + j) * hd:(H + j + 1) * hd].numpy(), p)
            v = qkv[t, (H + Hkv + j) * hd:(H + Hkv + j + 1) * hd].double().numpy()
            if dtype == "bf16":
                np.testing.assert_array_equal(pool_h[blk, 1, j, s], oracle.round_bf16(v))      # v: exact rounding
                # k is rotated in fp32 before rounding: equal to the oracle's rounding up to one bf16 step
                kr = oracle.round_bf16(k)
                assert np.all(np.abs(pool_h[blk, 0, j, s] - kr) <= np.abs(kr) * 2.0 ** -7 + 1e-30)
                assert np.mean(pool_h[blk, 0, j, s] == kr) > 0.9
            else:
                np.testing.assert_array_equal(pool_h[blk, 1, j, s], v)
                np.testing.assert_allclose(pool_h[blk, 0, j, s], k, rtol=0, atol=4e-7 * np.abs(k).max())
            touched[blk, :, j, s] = True
    assert np.all(pool_h[~touched] == 512.0), "a write landed outside the (block, slot) the table names"
    assert touched.sum() == T * 2 * Hkv


def _attention_case(seed, lens, H, Hkv, hd, dtype, spare=5):
    B = len(lens)
    nb = [(n + 15) // 16 for n in lens]
    total = sum(nb) + spare
    perm = gen.permutation(seed, 1, total).tolist()
    table = torch.full((B, max(nb)), 0, dtype=torch.int32)
    it = iter(perm)
    for b in range(B):
        for j in range(nb[b]):
            table[b, j] = next(it)
    pdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    pool = gen.normal(seed, 2, (total, 2, Hkv, 16, hd), device=DEV).to(pdt)
    # slots past a sequence's last position were never written: they may hold anything, so they hold NaN here
    # (a masked probability of zero times NaN would still poison the output), and so do the blocks no table
    # entry names
    used = torch.zeros(total, dtype=torch.bool)
    for b in range(B):
        used[table[b, :nb[b]].long()] = True
        if lens[b] % 16:
            pool[table[b, nb[b] - 1], :, :, lens[b] % 16:, :] = float("nan")
    pool[(~used).to(DEV)] = float("nan")
    q = gen.normal(seed, 3, (B, H, hd), device=DEV)
    return table, pool, q


def _attn_tol(dtype, hd, H, Hkv):
    """Relative tolerance of decode attention: the scalar kernel computes in float32 (2e-6); grouped heads
    on a bf16 pool with head_dim 128 run on the matrix cores with q and the probabilities split into two
    bf16 terms, which leaves 2^-17 = 7.6e-6 per operand element (3e-5 with the accumulation)."""
    return 3e-5 if (dtype == "bf16" and hd == 128 and 2 <= H // Hkv <= 16) else 2e-6


def _run_attention(table, pool, q, lens, H, Hkv, hd, window=0):
    B = len(lens)
    ctx = torch.tensor(lens, dtype=torch.int32, device=DEV)
    slot = torch.arange(B, dtype=torch.int32, device=DEV)
    out = torch.empty(B, H, hd, device=DEV)
    scratch = torch.empty(ld.ldk_attention_scratch_bytes(B, H, Hkv, hd, max(lens), window), dtype=torch.uint8,
                          device=DEV)
    ld.ldk_paged_attention(q, H * hd, device_pool(pool), table.to(DEV), slot, ctx, max(lens), H, Hkv, hd, out,
                           scratch, window=window)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _oracle_attention(table, pool, q, lens, Hkv, hd, rows=None, window=0):
    ph = oracle.to_host_matrix(pool.reshape(pool.shape[0], -1))
    kp = ph.reshape(-1)
    vp = kp[Hkv * 16 * hd:]                      # V half of each block starts Hkv*16*hd elements later
    strides = (2 * Hkv * 16 * hd, 16 * hd, hd)
    qh = q.cpu().numpy()
    if rows is None:
        return oracle.paged_attention(qh, kp, vp, strides, table.numpy(), lens, Hkv, window=window)
    sel = np.array(rows)
    return oracle.paged_attention(qh[sel], kp, vp, strides, table.numpy()[sel], [lens[r] for r in rows], Hkv,
                                  window=window)


@pytest.mark.parametrize("dtype,hd,H,Hkv", [("bf16", 128, 4, 4), ("f32", 64, 4, 4), ("bf16", 128, 8, 2), ("f32", 128, 2, 1),
                                            ("bf16", 128, 16, 2), ("bf16", 64, 6, 2), ("bf16", 128, 32, 8)])
def test_paged_attention_edge_lengths(dtype, hd, H, Hkv):
    lens = [1, 2, 15, 16, 17, 63, 255, 256, 257, 300, 1025]
    table, pool, q = _attention_case(21, lens, H, Hkv, hd, dtype)
    got = _run_attention(table, pool, q, lens, H, Hkv, hd)
    ref = _oracle_attention(table, pool, q, lens, Hkv, hd)
    assert np.max(np.abs(got - ref)) <= _attn_tol(dtype, hd, H, Hkv) * np.abs(ref).max() + 1e-6
    # ctx = 1 returns V of the single cached token
    v0 = pool[table[0, 0], 1, :, 0, :].float().cpu().numpy()
    for h in range(H):
        np.testing.assert_allclose(got[0, h], v0[h // (H // Hkv)], rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("window", [1, 5, 16, 17, 100, 256, 4096])
@pytest.mark.parametrize("dtype,hd,H,Hkv", [("bf16", 128, 8, 2), ("f32", 64, 4, 4)])
def test_paged_attention_band(dtype, hd, H, Hkv, window):
    """Attention band: the row sees its last `window` positions only; bands that start inside a block, at a
    block boundary, that are longer than the context, and of a single position."""
    lens = [1, 2, 15, 16, 17, 63, 255, 256, 257, 300, 1025]
    table, pool, q = _attention_case(22, lens, H, Hkv, hd, dtype)
    got = _run_attention(table, pool, q, lens, H, Hkv, hd, window=window)
    ref = _oracle_attention(table, pool, q, lens, Hkv, hd, window=window)
    assert np.max(np.abs(got - ref)) <= _attn_tol(dtype, hd, H, Hkv) * np.abs(ref).max() + 1e-6
    if window == 1:      # the own value
        for b, n in enumerate(lens):
            v = pool[table[b, (n - 1) // 16], 1, :, (n - 1) % 16, :].float().cpu().numpy()
            for h in range(H):
                np.testing.assert_allclose(got[b, h], v[h // (H // Hkv)], rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("H,Hkv", [(32, 32), (32, 8)])
def test_paged_attention_scratch_sized_for_the_cap_serves_every_shorter_context(H, Hkv):
    """The chunking follows the launch's longest context; scratch sized once for the cap must do for all
    shorter ones (the chunk count is not monotonic in the context length)."""
    hd, cap = 128, 16384
    lens_all = [1, 100, 1030, 2052, 3074, 4103, 5125, 7169, 9220, 13315, 16384]
    table, pool, q = _attention_case(23, [cap], H, Hkv, hd, "bf16")
    dpool = device_pool(pool)
    for T in (1, 3, 8):
        scratch = torch.empty(ld.ldk_attention_scratch_bytes(T, H, Hkv, hd, cap, 0), dtype=torch.uint8, device=DEV)
        qq = q.expand(T, H, hd).contiguous()
        slot = torch.zeros(T, dtype=torch.int32, device=DEV)
        out = torch.empty(T, H, hd, device=DEV)
        for n in lens_all:
            ctx = torch.full((T,), n, dtype=torch.int32, device=DEV)
            ld.ldk_paged_attention(qq, H * hd, dpool, table.to(DEV), slot, ctx, n, H, Hkv, hd, out, scratch)
        torch.cuda.synchronize()
        ref = _oracle_attention(table, pool, q, [lens_all[-1]], Hkv, hd)
        assert np.max(np.abs(out[0].cpu().numpy() - ref[0])) <= 3e-5 * np.abs(ref).max() + 1e-6


def test_paged_attention_grouped_band_serving_shape_sampled():
    """Batch 32, 32 query heads on 8 KV heads, contexts uniform in [512, 8192], band of 4096 positions:
    sampled rows (the longest, the shortest, one just over the band) against the oracle."""
    lens = gen.randint(20240602, 1, 512, 8192, 32).tolist()
    lens[3] = 4097
    table, pool, q = _attention_case(20240602, lens, 32, 8, 128, "bf16")
    got = _run_attention(table, pool, q, lens, 32, 8, 128, window=4096)
    assert np.isfinite(got).all()
    rows = [3, 9, int(np.argmax(lens)), int(np.argmin(lens))]
    ref = _oracle_attention(table, pool, q, lens, 8, 128, rows=rows, window=4096)
    err = np.max(np.abs(got[rows] - ref)) / np.abs(ref).max()
    assert err <= 2e-5, err


def test_paged_attention_microbench_shape():
    """Batch 16, 32 heads x 128, contexts uniform in [256, 4096] (the benchmark's draw), permuted block table:
    every (sequence, head) output against the oracle."""
    lens = gen.randint(20240601, 1, 256, 4096, 16).tolist()
    table, pool, q = _attention_case(20240601, lens, 32, 32, 128, "bf16")
    got = _run_attention(table, pool, q, lens, 32, 32, 128)
    assert np.isfinite(got).all()
    rows = list(range(16))
    ref = _oracle_attention(table, pool, q, lens, 32, 128, rows=rows)
    err = np.max(np.abs(got[rows] - ref)) / np.abs(ref).max()
    assert err <= 2e-5, err


def test_argmax_ties_and_brute_force():
    V = 32000
    lg = gen.normal(6, 1, (5, V))
    lg[1, [31999, 12, 700]] = 50.0
    lg[2, :] = 1.5
    lg[3, V - 1] = 60.0
    out = torch.empty(5, dtype=torch.int32, device=DEV)
    ld.ldk_argmax(lg.to(DEV), out)
    ref = [oracle.argmax(lg[r].numpy()) for r in range(5)]
    assert out.cpu().tolist() == ref and ref[1] == 12 and ref[2] == 0 and ref[3] == V - 1


def test_sampling_kernel_draws_the_oracles_tokens():
    """Gumbel-max token choice: for every row the kernel's draw equals the oracle's for the same (seed,
    position); rows with temperature 0 are the plain argmax; over many positions the draws of a small
    vocabulary follow softmax(logits / T)."""
    V, R = 32000, 12
    lg = gen.normal(7, 1, (R, V)) * 3.0
    temps = [0.0, 0.3, 0.7, 1.0, 1.5, 2.0] * 2
    seeds = [int(x) for x in gen.randint(7, 2, 0, 2 ** 40, R).tolist()]
    seeds[3] = 2 ** 64 - 5                                   # a seed above 2^63: unsigned arithmetic
    pos = [0, 1, 17, 4095, 8191, 100000, 5, 6, 7, 8, 9, 10]
    out = torch.empty(R, dtype=torch.int32, device=DEV)
    seed_t = torch.tensor([s - 2 ** 64 if s >= 2 ** 63 else s for s in seeds], dtype=torch.int64, device=DEV)
    ld.ldk_sample(lg.to(DEV), torch.tensor(temps, device=DEV), seed_t, torch.tensor(pos, dtype=torch.int32, device=DEV), out)
    got = out.cpu().tolist()
    for r in range(R):
        ref = oracle.sample_gumbel(lg[r].numpy(), temps[r], seeds[r], pos[r]) if temps[r] > 0 else oracle.argmax(lg[r].numpy())
        assert got[r] == ref, (r, got[r], ref)
    assert len(set(got[1:6])) > 1                            # the noise does move the choice
    # frequencies on a small vocabulary
    small = torch.tensor([1.2, -0.3, 0.0, 2.5, 2.4, -4.0, 0.7, 1.9])
    n = 20000
    out = torch.empty(n, dtype=torch.int32, device=DEV)
    ld.ldk_sample(small.repeat(n, 1).to(DEV), torch.full((n,), 0.7, device=DEV), torch.full((n,), 777, dtype=torch.int64, device=DEV),
                  torch.arange(n, dtype=torch.int32, device=DEV), out)
    cnt = np.bincount(out.cpu().numpy(), minlength=8)
    p = np.exp(small.numpy() / 0.7); p /= p.sum()
    assert np.abs((cnt - n * p) / np.sqrt(n * p * (1 - p))).max() < 4.5
    ref = [oracle.sample_gumbel(small.numpy(), 0.7, 777, i) for i in range(2000)]
    assert out.cpu().tolist()[:2000] == ref


@pytest.mark.parametrize("dtype,hd,T", [("bf16", 128, 1), ("bf16", 128, 2), ("bf16", 128, 3), ("bf16", 128, 4), ("f32", 64, 1),
                                        ("bf16", 64, 1), ("bf16", 64, 4)])
def test_fused_qkv_projection_rope_cache_append(dtype, hd, T):
    """ldk_qkv_rope = RMSNorm + q/k/v projection + rotary embedding + cache append in one call
    (one fused kernel for a single bf16 row, a composition otherwise)."""
    H, Hkv, K, nblk = 6, 2, 1160, 7
    N = (H + 2 * Hkv) * hd
    W = _mat(8, 1, N, K, dtype); x = gen.normal(8, 2, (T, K)); g = gen.normal(8, 3, (K,), std=0.1, mean=1.0)
    pos = torch.tensor([37, 16, 95, 0][:T], dtype=torch.int32)
    slot = torch.tensor([1, 0, 1, 0][:T], dtype=torch.int32)
    table = torch.tensor([[3, 6, 0, 0, 0, 0], [5, 1, 4, 2, 0, 0]], dtype=torch.int32)   # logical -> physical
    pdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    pool = torch.full((nblk, 2, Hkv, 16, hd), 512.0, dtype=pdt, device=DEV)
    cs = torch.empty(T, hd // 2, 2, device=DEV)
    qkv = torch.zeros(T, N, device=DEV)
    ld.ldk_rope_table(pos.to(DEV), hd, 10000.0, cs)
    ld.ldk_qkv_rope(W.to(DEV), x.to(DEV), qkv, cs, pos.to(DEV), slot.to(DEV), table.to(DEV), pool, H, Hkv, hd,
                    g=g.to(DEV), eps=1e-5)
    qkv_h, pool_h = qkv.cpu().numpy(), logical_pool(pool).float().cpu().numpy().astype(np.float64)
    Wh = oracle.to_host_matrix(W)
    touched = np.zeros(pool_h.shape[:4], bool)
    for t in range(T):
        ref = oracle.matvec(Wh, oracle.rmsnorm(x[t].numpy(), g.numpy(), 1e-5))
        scale = np.abs(ref).max()
        p = int(pos[t]); blk = int(table[slot[t], p // 16]); s = p % 16
        for h in range(H):
            r = oracle.rope_head(ref[h * hd:(h + 1) * hd], p)
            np.testing.assert_allclose(qkv_h[t, h * hd:(h + 1) * hd], r, rtol=0, atol=4e-6 * scale)
        for j in range(Hkv):
            k = oracle.rope_head(ref[(H + j) * hd:(H + j + 1) * hd], p)
            v = ref[(H + Hkv + j) * hd:(H + Hkv + j + 1) * hd]
            tol = (2.0 ** -7 if dtype == "bf16" else 4e-6) * scale
            assert np.max(np.abs(pool_h[blk, 0, j, s] - k)) <= tol and np.max(np.abs(pool_h[blk, 1, j, s] - v)) <= tol
            if dtype == "bf16":
                assert np.mean(pool_h[blk, 0, j, s] == oracle.round_bf16(k)) > 0.9
                assert np.mean(pool_h[blk, 1, j, s] == oracle.round_bf16(v)) > 0.9
            touched[blk, :, j, s] = True
    assert np.all(pool_h[~touched] == 512.0) and touched.sum() == T * 2 * Hkv


@pytest.mark.parametrize("K", [4096, 5120, 8192, 11008, 13824])
@pytest.mark.parametrize("T", [2, 3, 4])
def test_linear_two_to_four_rows_every_row_length(T, K):
    """Decode batches of 2 .. 4 rows at the row lengths of the 7B and 13B shapes (model and FFN widths:
    8 to 27 K slabs of the small-batch matrix-core kernel), all three epilogues, ragged output counts."""
    N = 77
    W = _mat(12, K, 2 * N, K, "bf16"); x = gen.normal(12, 2, (T, K)); g = gen.normal(12, 3, (K,), std=0.1, mean=1.0)
    y0 = gen.normal(12, 4, (T, N))
    Wh = oracle.to_host_matrix(W)
    Wd, xd, gd = W.to(DEV), x.to(DEV), g.to(DEV)
    scratch = torch.empty(ld.ldk_linear_scratch_bytes(T, N, K, ld.LDK_SWIGLU), dtype=torch.uint8, device=DEV)
    gu = np.stack([oracle.matvec(Wh, oracle.rmsnorm(x[t].numpy(), g.numpy(), 1e-5)) for t in range(T)])
    y = torch.empty(T, N, device=DEV)
    ld.ldk_linear(Wd, xd, y, ld.LDK_SWIGLU, g=gd, eps=1e-5, scratch=scratch)
    ref = _silu(gu[:, :N]) * gu[:, N:]
    assert np.max(np.abs(y.cpu().numpy() - ref)) <= 2e-5 * np.abs(ref).max()
    y = y0.to(DEV).clone()
    ld.ldk_linear(Wd[:N], xd, y, ld.LDK_ADD, g=gd, eps=1e-5, scratch=scratch)
    assert np.max(np.abs(y.cpu().numpy() - (y0.numpy() + gu[:, :N]))) <= 2e-5 * np.abs(gu).max()
    plain = np.stack([oracle.matvec(Wh, x[t].numpy()) for t in range(T)])
    y = torch.empty(T, 2 * N, device=DEV)
    ld.ldk_linear(Wd, xd, y, ld.LDK_STORE, scratch=scratch)
    assert np.max(np.abs(y.cpu().numpy() - plain)) <= 2e-5 * np.abs(plain).max()


@pytest.mark.parametrize("T", [2, 5, 31, 32, 33, 41, 48, 49, 64, 100, 257, 300, 320, 321])
@pytest.mark.parametrize("epi", ["store", "add_norm", "swiglu_norm"])
def test_linear_matrix_core_path(T, epi):
    """bf16 matrices, several rows, K a multiple of 128, scratch given: the MFMA kernel with split
    (hi + lo) activations.  Ragged N (not a multiple of the 128-column tile) and ragged T (33, 41, 48: the
    small-batch kernel's second group of rows, full and ragged; 49: the first row count of the 64-row kernel)."""
    N, K = 333, 1152
    rows = 2 * N if epi == "swiglu_norm" else N
    W = _mat(9, 1, rows, K, "bf16"); x = gen.normal(9, 2, (T, K)); g = gen.normal(9, 3, (K,), std=0.1, mean=1.0)
    y0 = gen.normal(9, 4, (T, N))
    Wh = oracle.to_host_matrix(W)
    scratch = torch.empty(ld.ldk_linear_scratch_bytes(T, N, K, ld.LDK_SWIGLU), dtype=torch.uint8, device=DEV)
    y = y0.to(DEV).clone()
    if epi == "store":
        ld.ldk_linear(W.to(DEV), x.to(DEV), y, ld.LDK_STORE, scratch=scratch)
        ref = np.stack([oracle.matvec(Wh, x[t].numpy()) for t in range(T)])
    elif epi == "add_norm":
        ld.ldk_linear(W.to(DEV), x.to(DEV), y, ld.LDK_ADD, g=g.to(DEV), eps=1e-5, scratch=scratch)
        ref = y0.numpy() + np.stack([oracle.matvec(Wh, oracle.rmsnorm(x[t].numpy(), g.numpy(), 1e-5)) for t in range(T)])
    else:
        ld.ldk_linear(W.to(DEV), x.to(DEV), y, ld.LDK_SWIGLU, g=g.to(DEV), eps=1e-5, scratch=scratch)
        gu = np.stack([oracle.matvec(Wh, oracle.rmsnorm(x[t].numpy(), g.numpy(), 1e-5)) for t in range(T)])
        ref = _silu(gu[:, :N]) * gu[:, N:]
    err = np.max(np.abs(y.cpu().numpy() - ref)) / np.abs(ref).max()
    assert err <= 2e-5, err


@pytest.mark.parametrize("plan", ["2,128,1", "2,128,3", "2,256,1", "2,256,2", "4,256,1", "4,256,4"])
@pytest.mark.parametrize("epi", ["store", "add", "swiglu"])
def test_linear_big_tile_every_plan(plan, epi, monkeypatch):
    """The big-tile kernel picks its tile and split-K factor from a cost estimate; here every tile
    (128 x 128, 128 x 256, 256 x 256) is forced in turn, with and without split-K, on a shape that is ragged
    in tokens and in output columns, against the oracle on every output."""
    monkeypatch.setenv("LD_GEMM_BIG", plan)
    T, N, K = 333, 301, 1152
    rows = 2 * N if epi == "swiglu" else N
    W = _mat(11, 1, rows, K, "bf16"); x = gen.normal(11, 2, (T, K)); y0 = gen.normal(11, 4, (T, N))
    Wh = oracle.to_host_matrix(W)
    code = {"store": ld.LDK_STORE, "add": ld.LDK_ADD, "swiglu": ld.LDK_SWIGLU}[epi]
    scratch = torch.empty(ld.ldk_linear_scratch_bytes(T, N, K, code), dtype=torch.uint8, device=DEV)
    y = y0.to(DEV).clone()
    ld.ldk_linear(W.to(DEV), x.to(DEV), y, code, scratch=scratch)
    ref = np.stack([oracle.matvec(Wh, x[t].numpy()) for t in range(T)])
    if epi == "add":
        ref = y0.numpy() + ref
    elif epi == "swiglu":
        ref = _silu(ref[:, :N]) * ref[:, N:]
    err = np.max(np.abs(y.cpu().numpy() - ref)) / np.abs(ref).max()
    assert err <= 2e-5, err


def test_linear_matrix_core_7b_shapes_sampled():
    """Launch shapes of the batch-32 decode step, of a 256-row prefill chunk, of a mixed step (32 decode rows
    + four 256-row chunks) and of a 2048-row chunk beside 63 decode rows, sampled outputs.  The last two have
    a tail of 32 / 63 rows past the last full 256-row tile, which is cut off and computed by the small-batch
    kernels: the rows on both sides of the cut are among the samples.  768 rows: three row tiles, a grid of
    less than one round."""
    _sampled_linear_cases((32, 256, 768, 1056, 2111),
                          [(12288, 4096, ld.LDK_STORE), (4096, 11008, ld.LDK_ADD), (11008, 4096, ld.LDK_SWIGLU)])


def test_linear_matrix_core_13b_shapes_sampled():
    """The four layer matrices of the 13B shape (row lengths 5120 and 13824) at the row counts of its batch-64
    step: 63 decode rows beside a 2048-row chunk (2111), and 2112 (one more decode row, or a chunk behind a
    pending token); sampled outputs, the rows on both sides of the 256-row tile cut among them."""
    _sampled_linear_cases((2111, 2112), [(15360, 5120, ld.LDK_STORE), (5120, 5120, ld.LDK_ADD),
                                         (5120, 13824, ld.LDK_ADD), (13824, 5120, ld.LDK_SWIGLU)])


def _sampled_linear_cases(row_counts, matrices):
    for T in row_counts:
        for N, K, epi in matrices:
            rows = N * (2 if epi == ld.LDK_SWIGLU else 1)
            W = gen.normal(3, N, (rows, K), std=0.02, device=DEV).bfloat16()
            x = gen.normal(3, 7 + T, (T, K), device=DEV)
            y = torch.zeros(T, N, device=DEV)
            scratch = torch.empty(ld.ldk_linear_scratch_bytes(T, N, K, epi), dtype=torch.uint8, device=DEV)
            ld.ldk_linear(W, x, y, epi, scratch=scratch)
            ns = gen.randint(3, 9, 0, N - 1, 6).tolist() + [0, N - 1]
            ts = sorted(set(gen.randint(3, 10, 0, T - 1, 5).tolist() + [0, T - 1, max(T - T % 256 - 1, 0), min(T - T % 256, T - 1)]))
            xh = x.cpu().numpy(); yh = y.cpu().numpy()
            for n in ns:
                wr = oracle.to_host_matrix(W[n:n + 1]); wu = oracle.to_host_matrix(W[N + n:N + n + 1]) if epi == ld.LDK_SWIGLU else None
                for t in ts:
                    a = oracle.matvec(wr, xh[t])[0]
                    if wu is not None:
                        a = oracle.silu(a) * oracle.matvec(wu, xh[t])[0]
                    # two-term bf16 split of the activations: ~2^-17 per element, random-walk over K terms
                    assert abs(yh[t, n] - a) <= 1e-4 * max(1.0, abs(a)), (T, N, t, n, yh[t, n], a)


def test_linear_fp16_rows_sampled():
    """The form of the multi-row product that long prefill chunks take in the engine (ldk_linear_f16: activations
    rounded to fp16 in one term, bf16 matrix entries widened to fp16 exactly): sampled outputs against the oracle's
    dot product on the inputs rounded as the kernel rounds them (the 16-bit sum of the split image, then fp16; what
    remains is float32 accumulation: the two-term test's bound) and
    against the oracle on the exact inputs (the rounding itself: 2^-12 per term, random walk over K terms).  Row
    counts with a tail that keeps both terms (1056, 2111), with three and one row tiles, and one that stays on the
    small-batch kernel (32: bit-equal to ldk_linear).  With the matrix's fp16 image (ldk_weights_to_f16: equal to the
    bf16 values entry by entry, truncated toward zero below 2^-17 where fp16 has no bits left) the same call gives
    bit-equal results.  A value beyond the fp16 range in the input or in the matrix raises the flag."""
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    for T in (32, 256, 768, 1056, 2111):
        for N, K, epi in [(12288, 4096, ld.LDK_STORE), (4096, 11008, ld.LDK_ADD), (11008, 4096, ld.LDK_SWIGLU)]:
            rows = N * (2 if epi == ld.LDK_SWIGLU else 1)
            W = gen.normal(3, N, (rows, K), std=0.02, device=DEV).bfloat16()
            x = gen.normal(3, 7 + T, (T, K), device=DEV)
            y = torch.zeros(T, N, device=DEV); y2 = torch.zeros(T, N, device=DEV)
            scratch = torch.empty(ld.ldk_linear_scratch_bytes(T, N, K, epi), dtype=torch.uint8, device=DEV)
            flag.zero_()
            ld.ldk_linear_f16(W, x, y, flag, epi, scratch=scratch)
            assert int(flag.item()) == 0
            ld.ldk_linear(W, x, y2, epi, scratch=scratch)
            r = T % 256 if T > 256 and T % 256 <= 64 else 0       # tail rows: both terms in either form
            if T <= 64:
                assert torch.equal(y, y2)
            else:
                assert not torch.equal(y[:T - r], y2[:T - r])     # the single-term form did run
            Wh = torch.zeros(rows, K, dtype=torch.float16, device=DEV); y3 = torch.zeros(T, N, device=DEV)
            ld.ldk_weights_to_f16(W, Wh, flag)
            assert int(flag.item()) == 0
            wf, whf = W.float(), Wh.float()
            fits = wf.abs() >= 2.0 ** -17
            assert torch.equal(whf[fits], wf[fits])
            assert bool(((whf.abs() <= wf.abs()) & ((wf - whf).abs() < 2.0 ** -24) & (whf * wf >= 0))[~fits].all())
            ld.ldk_linear_f16(W, x, y3, flag, epi, scratch=scratch, W_f16=Wh)
            assert int(flag.item()) == 0 and torch.equal(y3, y)
            del Wh, wf, whf, fits, y3
            ns = gen.randint(3, 9, 0, N - 1, 6).tolist() + [0, N - 1]
            ts = sorted(set(gen.randint(3, 10, 0, T - 1, 5).tolist() + [0, T - 1, max(T - T % 256 - 1, 0), min(T - T % 256, T - 1)]))
            xh = x.cpu().numpy(); yh = y.cpu().numpy()
            # what the kernel rounds: the sum of the two bf16 terms of the split image (16 bits), not x itself
            xc = x.cpu(); hi = xc.bfloat16().float(); lo = (xc - hi).bfloat16().float()
            xr = (hi + lo).half().float().numpy()
            for n in ns:
                wr = oracle.to_host_matrix(W[n:n + 1]); wu = oracle.to_host_matrix(W[N + n:N + n + 1]) if epi == ld.LDK_SWIGLU else None
                for t in ts:
                    vals = []
                    for xin in (xh, xr):
                        a = oracle.matvec(wr, xin[t])[0]
                        if wu is not None:
                            a = oracle.silu(a) * oracle.matvec(wu, xin[t])[0]
                        vals.append(a)
                    exact, rounded = vals
                    assert abs(yh[t, n] - exact) <= 2e-3 * max(1.0, abs(exact)), (T, N, t, n, yh[t, n], exact)
                    if T > 64 and t < T - r:
                        assert abs(yh[t, n] - rounded) <= 1e-4 * max(1.0, abs(rounded)), (T, N, t, n, yh[t, n], rounded)
    # values beyond the fp16 range
    T, N, K = 300, 4096, 4096
    W = gen.normal(3, 1, (N, K), std=0.02, device=DEV).bfloat16()
    x = gen.normal(3, 2, (T, K), device=DEV)
    y = torch.zeros(T, N, device=DEV)
    scratch = torch.empty(ld.ldk_linear_scratch_bytes(T, N, K, ld.LDK_STORE), dtype=torch.uint8, device=DEV)
    xb = x.clone(); xb[17, 1234] = 7.0e4
    flag.zero_(); ld.ldk_linear_f16(W, xb, y, flag, scratch=scratch); assert int(flag.item()) == 1
    xb[17, 1234] = -6.5e4           # the largest fp16 magnitude is 65504
    flag.zero_(); ld.ldk_linear_f16(W, xb, y, flag, scratch=scratch); assert int(flag.item()) == 0
    Wb = W.clone(); Wb[4000, 4095] = 1.0e5
    flag.zero_(); ld.ldk_linear_f16(Wb, x, y, flag, scratch=scratch); assert int(flag.item()) == 1
    Wh = torch.zeros(N, K, dtype=torch.float16, device=DEV)
    flag.zero_(); ld.ldk_weights_to_f16(Wb, Wh, flag); assert int(flag.item()) == 1
    Wb[4000, 4095] = float("nan")
    flag.zero_(); ld.ldk_linear_f16(Wb, x, y, flag, scratch=scratch); assert int(flag.item()) == 1
    flag.zero_(); ld.ldk_weights_to_f16(Wb, Wh, flag); assert int(flag.item()) == 1
    Wb[4000, 4095] = -65504.0 * 0.75   # bf16 has no 65504; -49128 rounds to a bf16 within range
    flag.zero_(); ld.ldk_weights_to_f16(Wb, Wh, flag); assert int(flag.item()) == 0 and float(Wh[4000, 4095]) == float(Wb[4000, 4095])


def test_linear_fp16_image_13b_shapes_bit_equal():
    """The four layer matrices of the 13B shape at the row count of its batch-64 step (63 decode rows beside a
    2048-row chunk): the fp16 form gives the same bits whether the kernel widens the bf16 weights itself or reads
    the matrix's fp16 image, and differs from the two-term form (so it did run)."""
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    T = 2111
    for N, K, epi in [(15360, 5120, ld.LDK_STORE), (5120, 5120, ld.LDK_ADD), (5120, 13824, ld.LDK_ADD), (13824, 5120, ld.LDK_SWIGLU)]:
        rows = N * (2 if epi == ld.LDK_SWIGLU else 1)
        W = gen.normal(5, N, (rows, K), std=0.02, device=DEV).bfloat16()
        x = gen.normal(5, 7 + K, (T, K), device=DEV)
        y0 = gen.normal(5, 8, (T, N), device=DEV)                 # the residual that LDK_ADD adds to
        scratch = torch.empty(ld.ldk_linear_scratch_bytes(T, N, K, epi), dtype=torch.uint8, device=DEV)
        Wh = torch.zeros(rows, K, dtype=torch.float16, device=DEV)
        ld.ldk_weights_to_f16(W, Wh, flag)
        outs = []
        for img in (None, Wh):
            y = y0.clone()
            ld.ldk_linear_f16(W, x, y, flag, epi, scratch=scratch, W_f16=img)
            outs.append(y)
        y2 = y0.clone()
        ld.ldk_linear(W, x, y2, epi, scratch=scratch)
        assert int(flag.item()) == 0
        assert torch.equal(outs[0], outs[1]) and not torch.equal(outs[0], y2), (N, K, epi)
        assert float((outs[0] - y2).abs().max()) <= 2e-3 * max(1.0, float(y2.abs().max()))


@pytest.mark.parametrize("split", [False, True], ids=["whole", "kv-split"])
@pytest.mark.parametrize("window", [0, 40, 200])
@pytest.mark.parametrize("H,Hkv", [(4, 4), (8, 2)])
def test_prefill_attention_fp16_form(H, Hkv, window, split):
    """The form of chunk-prefill attention that the engine's long passes take (ldk_prefill_attention_f16: queries and
    probabilities as one fp16 term, keys and values widened to fp16 exactly): the segments of
    test_prefill_attention_segments, every row against the oracle's single-query attention.  What the form rounds
    is q (2^-12 per element of a 128-term score of a few units: ~1e-3 in the exponent's argument) and p (2^-12):
    bound 1e-3 of the largest output, thirty times the two-term bound and a third of what the cache's own bf16
    rounding of a key moves a score by.  A key or value beyond the fp16 range at a position the walk reads, or a
    query that is, raises the flag; the same values at positions no row sees do not."""
    hd = 128
    segs = [(37, 100), (0, 5), (1000, 300), (255, 1), (16, 32)]
    lens = [p + n for p, n in segs]
    table, pool, _ = _attention_case(31, lens, H, Hkv, hd, "bf16")
    T = sum(n for _, n in segs)
    q = gen.normal(31, 9, (T, H, hd), device=DEV)
    tiles, row_seq, row_pos, r = [], [], [], 0
    for s, (p0, n) in enumerate(segs):
        for off in range(0, n, 128):
            tiles.append([r + off, min(128, n - off), p0 + off, s])
        row_seq += [s] * n; row_pos += list(range(p0, p0 + n)); r += n
    tiles_d = torch.tensor(tiles, dtype=torch.int32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    scratch = torch.empty(ld.ldk_prefill_attention_scratch_bytes(), dtype=torch.uint8, device=DEV) if split else None

    def run(qq, pp):
        out = torch.zeros(T, H, hd, device=DEV)
        flag.zero_()
        ld.ldk_prefill_attention_f16(qq, H * hd, device_pool(pp), table.to(DEV), tiles_d, H, Hkv, hd, out, max(row_pos), flag,
                                     window=window, scratch=scratch)
        torch.cuda.synchronize()
        return out.cpu().numpy(), int(flag.item())

    got, f = run(q, pool)
    assert f == 0
    out2 = torch.zeros(T, H, hd, device=DEV)
    ld.ldk_prefill_attention(q, H * hd, device_pool(pool), table.to(DEV), tiles_d, H, Hkv, hd, out2, max(row_pos),
                             window=window, scratch=scratch)
    assert not np.array_equal(got, out2.cpu().numpy())      # the single-term form did run
    ph = oracle.to_host_matrix(pool.reshape(pool.shape[0], -1)).reshape(-1)
    ref = oracle.paged_attention(q.cpu().numpy(), ph, ph[Hkv * 16 * hd:], (2 * Hkv * 16 * hd, 16 * hd, hd),
                                 table.numpy()[row_seq], [p + 1 for p in row_pos], Hkv, window=window)
    err = np.max(np.abs(got - ref), axis=(1, 2)) / np.abs(ref).max()
    assert 3e-5 < err.max() <= 1e-3, (err.max(), int(err.argmax()), row_pos[int(err.argmax())])
    # out of range: the key of position 1100 of the third sequence (seen by its rows from 1100 on, inside every band)
    blk, slot = int(table[2, 1100 // 16]), 1100 % 16
    big = pool.clone(); big[blk, 0, Hkv - 1, slot, 5] = 7.0e4
    assert run(q, big)[1] == 1
    big = pool.clone(); big[blk, 1, 0, slot, 77] = -1.0e5
    assert run(q, big)[1] == 1
    # the last block of the second sequence (5 positions): slots 5..15 were never written and no row reads them as values;
    # its keys there are read and masked, so a key counts, a value slot beyond the tile is zeroed before it is looked at
    qb = q.clone(); qb[3, 1, 9] = 1.0e6
    assert run(qb, pool)[1] == 1


@pytest.mark.parametrize("split", [False, True], ids=["whole", "kv-split"])
@pytest.mark.parametrize("window", [0, 1, 40, 128, 200, 5000])
@pytest.mark.parametrize("H,Hkv", [(4, 4), (8, 2)])
def test_prefill_attention_segments(H, Hkv, window, split):
    """Chunk-prefill attention (matrix cores): segments of different sequences, a fresh prompt (position 0),
    an observation appended to a long context, a segment longer than one 128-row tile; causal inside
    the chunk; permuted block table; with and without an attention band (shorter than a wave's 32 rows,
    shorter and longer than a tile, longer than every context).  Every row against the oracle's
    single-query attention.  With scratch the KV range of a tile is split over several workgroups and merged
    (some shares are empty or wholly masked for some rows); without it every tile walks its whole range."""
    hd = 128
    segs = [(37, 100), (0, 5), (1000, 300), (255, 1), (16, 32)]          # (first position, rows) per sequence
    lens = [p + n for p, n in segs]
    table, pool, _ = _attention_case(31, lens, H, Hkv, hd, "bf16")
    T = sum(n for _, n in segs)
    q = gen.normal(31, 9, (T, H, hd), device=DEV)
    tiles, row_seq, row_pos, r = [], [], [], 0
    for s, (p0, n) in enumerate(segs):
        for off in range(0, n, 128):
            tiles.append([r + off, min(128, n - off), p0 + off, s])
        row_seq += [s] * n; row_pos += list(range(p0, p0 + n)); r += n
    out = torch.zeros(T, H, hd, device=DEV)
    scratch = torch.empty(ld.ldk_prefill_attention_scratch_bytes(), dtype=torch.uint8, device=DEV) if split else None
    ld.ldk_prefill_attention(q, H * hd, device_pool(pool), table.to(DEV), torch.tensor(tiles, dtype=torch.int32, device=DEV),
                             H, Hkv, hd, out, max(row_pos), window=window, scratch=scratch)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ph = oracle.to_host_matrix(pool.reshape(pool.shape[0], -1)).reshape(-1)
    ref = oracle.paged_attention(q.cpu().numpy(), ph, ph[Hkv * 16 * hd:], (2 * Hkv * 16 * hd, 16 * hd, hd),
                                 table.numpy()[row_seq], [p + 1 for p in row_pos], Hkv, window=window)
    err = np.max(np.abs(got - ref), axis=(1, 2)) / np.abs(ref).max()
    assert err.max() <= 3e-5, (err.max(), int(err.argmax()), row_pos[int(err.argmax())])
