"""Pins for the CPU oracle: closed forms, invariants, float64 library routines, brute force.

The paper prints no worked numeric example of the forward pass (section 2.1 defines attention in
prose only), so the oracle is pinned by what the mathematics fixes.  Each test is chosen so that a
plausible slip in oracle/ld_oracle.c (dropped gain or scale, eps outside the root, wrong RoPE pairing
or sign, transposed matrix, off-by-one context, wrong block/slot index, wrong tie-break) fails it.
"""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from workloads import gen, TINY, make_weights, SEED_BASE

RNG = np.random.default_rng(7)


# ------------------------------------------------------------------ RMSNorm

def test_rmsnorm_constant_vector_closed_form():
    d, c, eps = 256, 3.0, 1e-5
    g = (1 + 0.1 * RNG.standard_normal(d)).astype(np.float32)
    out = oracle.rmsnorm(np.full(d, c), g, eps)
    np.testing.assert_allclose(out, g.astype(np.float64) * c / math.sqrt(c * c + eps), rtol=1e-14)


def test_rmsnorm_unit_gain_mean_square():
    x = RNG.standard_normal(512) * 1e-2          # small x so that eps matters
    eps = 1e-5
    out = oracle.rmsnorm(x, np.ones(512, np.float32), eps)
    ms = np.mean(x * x)
    assert np.mean(out * out) == pytest.approx(ms / (ms + eps), rel=1e-12)


def test_rmsnorm_matches_library():
    x = torch.from_numpy(RNG.standard_normal(688)); g = torch.from_numpy(RNG.standard_normal(688)).float()
    ref = F.rms_norm(x, (688,), g.double(), eps=1e-5).numpy()
    np.testing.assert_allclose(oracle.rmsnorm(x.numpy(), g.numpy(), 1e-5), ref, rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------ RoPE

def test_rope_position_zero_is_identity_and_norm_preserved():
    u = RNG.standard_normal(128)
    np.testing.assert_array_equal(oracle.rope_head(u, 0), u)
    r = oracle.rope_head(u, 1234)
    half = 64
    np.testing.assert_allclose(r[:half] ** 2 + r[half:] ** 2, u[:half] ** 2 + u[half:] ** 2, rtol=1e-12)


def test_rope_pair_zero_is_plain_rotation_by_position():
    u = np.zeros(64); u[0] = 1.0                # pair 0 = (u[0], u[32]) has theta_0 = 1
    r = oracle.rope_head(u, 5)
    assert r[0] == pytest.approx(math.cos(5.0), abs=1e-15)
    assert r[32] == pytest.approx(math.sin(5.0), abs=1e-15)
    assert np.count_nonzero(r) == 2


def test_rope_matches_complex_multiplication():
    hd, pos, base = 128, 977, 10000.0
    u = RNG.standard_normal(hd)
    theta = torch.tensor([base ** (-2.0 * i / hd) for i in range(hd // 2)], dtype=torch.float64)
    z = torch.complex(torch.from_numpy(u[: hd // 2]), torch.from_numpy(u[hd // 2:]))
    w = z * torch.polar(torch.ones_like(theta), pos * theta)
    ref = np.concatenate([w.real.numpy(), w.imag.numpy()])
    np.testing.assert_allclose(oracle.rope_head(u, pos, base), ref, rtol=1e-12, atol=1e-14)


def test_rope_scores_depend_on_relative_position_only():
    q, k = RNG.standard_normal(64), RNG.standard_normal(64)
    a = oracle.rope_head(q, 40) @ oracle.rope_head(k, 17)
    b = oracle.rope_head(q, 40 + 300) @ oracle.rope_head(k, 17 + 300)
    assert a == pytest.approx(b, rel=1e-10)
    assert abs(a - oracle.rope_head(q, 41) @ oracle.rope_head(k, 17)) > 1e-6


# ------------------------------------------------------------------ softmax / attention

def test_softmax_sums_to_one_shift_invariant_and_matches_library():
    s = RNG.standard_normal(1000) * 5
    p = oracle.softmax(s)
    assert p.sum() == pytest.approx(1.0, abs=1e-14)
    np.testing.assert_allclose(oracle.softmax(s + 123.0), p, rtol=1e-11)
    np.testing.assert_allclose(p, torch.softmax(torch.from_numpy(s), 0).numpy(), rtol=1e-13)
    big = oracle.softmax(np.array([1e4, 0.0, -1e4]))     # max subtraction: no overflow
    np.testing.assert_allclose(big, [1.0, 0.0, 0.0], atol=1e-300)


def test_attention_single_token_returns_value_exactly():
    q, k, v = RNG.standard_normal(128), RNG.standard_normal((1, 128)), RNG.standard_normal((1, 128))
    np.testing.assert_array_equal(oracle.attention_contig(q, k, v), v[0])


def test_attention_equal_keys_gives_mean_of_values():
    q = RNG.standard_normal(64); k = np.tile(RNG.standard_normal(64), (37, 1)); v = RNG.standard_normal((37, 64))
    np.testing.assert_allclose(oracle.attention_contig(q, k, v), v.mean(0), rtol=1e-12, atol=1e-14)


def test_attention_dominant_key_selects_its_value():
    q = np.zeros(64); q[3] = 1.0
    k = np.zeros((9, 64)); k[5, 3] = 1e4
    v = RNG.standard_normal((9, 64))
    np.testing.assert_allclose(oracle.attention_contig(q, k, v), v[5], atol=1e-12)


def test_attention_is_invariant_to_permuting_key_value_pairs():
    q, k, v = RNG.standard_normal(128), RNG.standard_normal((50, 128)), RNG.standard_normal((50, 128))
    p = RNG.permutation(50)
    np.testing.assert_allclose(oracle.attention_contig(q, k[p], v[p]), oracle.attention_contig(q, k, v), rtol=1e-11)


def test_attention_matches_library_sdpa_including_scale():
    n, hd = 77, 128
    q, k, v = RNG.standard_normal(hd), RNG.standard_normal((n, hd)), RNG.standard_normal((n, hd))
    ref = F.scaled_dot_product_attention(torch.from_numpy(q)[None, None, None, :], torch.from_numpy(k)[None, None],
                                         torch.from_numpy(v)[None, None])[0, 0, 0].numpy()
    np.testing.assert_allclose(oracle.attention_contig(q, k, v), ref, rtol=1e-11, atol=1e-14)


def _paged_case(B, H, Hkv, hd, lens, bits):
    blk = 16
    nblk = [(n + blk - 1) // blk for n in lens]
    total = sum(nblk) + 3
    perm = gen.permutation(11, 5, total).numpy()
    table = np.full((B, max(nblk)), -1, np.int32)
    it = iter(perm)
    for b in range(B):
        for j in range(nblk[b]):
            table[b, j] = next(it)
    kf = gen.normal(11, 6, (total, Hkv, blk, hd)); vf = gen.normal(11, 7, (total, Hkv, blk, hd))
    if bits:
        kf, vf = kf.bfloat16(), vf.bfloat16()
    return table, kf, vf


@pytest.mark.parametrize("bits", [False, True])
def test_paged_attention_equals_contiguous_gather(bits):
    B, H, Hkv, hd = 3, 4, 2, 64
    lens = [1, 17, 48]
    table, kf, vf = _paged_case(B, H, Hkv, hd, lens, bits)
    q = RNG.standard_normal((B, H, hd))
    kp, vp = oracle.to_host_matrix(kf), oracle.to_host_matrix(vf)
    out = oracle.paged_attention(q, kp, vp, (Hkv * 16 * hd, 16 * hd, hd), table, lens, Hkv)
    kd, vd = kf.double().numpy(), vf.double().numpy()
    for b in range(B):
        for h in range(H):
            g = h // (H // Hkv)
            K = np.stack([kd[table[b, j // 16], g, j % 16] for j in range(lens[b])])
            V = np.stack([vd[table[b, j // 16], g, j % 16] for j in range(lens[b])])
            ref = torch.softmax(torch.from_numpy(K @ q[b, h]) / math.sqrt(hd), 0).numpy() @ V
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-11, atol=1e-14)


# ------------------------------------------------------------------ SwiGLU, matvec, rounding, argmax

def test_silu_identities():
    assert oracle.silu(0.0) == 0.0
    for z in (0.3, 2.0, 11.5):
        assert oracle.silu(z) - oracle.silu(-z) == pytest.approx(z, rel=1e-14)
    assert oracle.silu(1.0) == pytest.approx(F.silu(torch.tensor(1.0, dtype=torch.float64)).item(), rel=1e-15)


def test_matvec_matches_float64_matmul_and_is_not_transposed():
    w = RNG.standard_normal((37, 53)).astype(np.float32); x = RNG.standard_normal(53)
    np.testing.assert_allclose(oracle.matvec(w, x), w.astype(np.float64) @ x, rtol=1e-13, atol=1e-14)
    onehot = np.zeros((2, 53), np.float32); onehot[0, 7] = 1; onehot[1, 50] = 1
    np.testing.assert_array_equal(oracle.matvec(onehot, x), x[[7, 50]])


def test_matvec_reads_bf16_bit_patterns():
    w = torch.from_numpy(RNG.standard_normal((19, 64))).bfloat16(); x = RNG.standard_normal(64)
    np.testing.assert_allclose(oracle.matvec(oracle.to_host_matrix(w), x), w.double().numpy() @ x, rtol=1e-13)


def test_round_bf16_is_nearest_even_like_the_library_cast():
    x = torch.cat([torch.from_numpy(RNG.standard_normal(5000)).float() * 3,
                   torch.tensor([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.00390625, 0.0, -2.5, 3e-39])])
    ref = x.bfloat16().double().numpy()                 # float32 -> bf16 is RNE in torch
    np.testing.assert_array_equal(oracle.round_bf16(x.double().numpy()), ref)
    # ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.round_bf16(1.0 + 2 ** -8) == 1.0 and oracle.round_bf16(1.0 + 3 * 2 ** -8) == 1.0 + 2 ** -6
    # a double just above the tie must round up although its float32 image is the tie itself
    assert oracle.round_bf16(1.0 + 2 ** -8 + 2 ** -40) == 1.0 + 2 ** -7


def test_argmax_lowest_index_on_ties():
    x = RNG.standard_normal(1000)
    assert oracle.argmax(x) == int(np.argmax(x))
    x[[900, 17, 400]] = 99.0
    assert oracle.argmax(x) == 17


def test_counter_based_uniform_moments_range_and_independence_of_counters():
    u = np.array([oracle.uniform(12345, c) for c in range(40000)])
    assert u.min() > 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 4 * math.sqrt(1 / 12 / u.size)
    assert abs(u.var() - 1 / 12) < 0.002
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.02                       # neighbouring counters
    v = np.array([oracle.uniform(12346, c) for c in range(40000)])
    assert abs(np.corrcoef(u, v)[0, 1]) < 0.02                                # neighbouring seeds
    assert oracle.uniform(7, 99) == oracle.uniform(7, 99)
    assert set(np.round(u * 2 ** 23 - 0.5, 6) % 1) == {0.0}                   # the grid (k + 1/2) / 2^23


def test_gumbel_sampling_draws_from_the_softmax_at_the_given_temperature():
    """argmax(logits / T + Gumbel noise) is a draw from softmax(logits / T): the empirical frequencies over
    many positions (= independent counters) match within 4.5 standard deviations for every outcome; as
    T -> 0 the draw is the argmax; a draw is a pure function of (seed, position)."""
    lg = np.array([1.2, -0.3, 0.0, 2.5, 2.4, -4.0, 0.7, 1.9])
    for T in (0.7, 1.0, 2.0):
        p = np.exp(lg / T) / np.exp(lg / T).sum()
        n = 30000
        cnt = np.bincount([oracle.sample_gumbel(lg, T, 777, pos) for pos in range(n)], minlength=lg.size)
        z = (cnt - n * p) / np.sqrt(n * p * (1 - p))
        assert np.abs(z).max() < 4.5, (T, z)
    assert all(oracle.sample_gumbel(lg, 1e-4, 5, pos) == 3 for pos in range(500))
    a = [oracle.sample_gumbel(lg, 1.0, 5, pos) for pos in range(200)]
    assert a == [oracle.sample_gumbel(lg, 1.0, 5, pos) for pos in range(200)]
    assert a != [oracle.sample_gumbel(lg, 1.0, 6, pos) for pos in range(200)]


def test_gumbel_scores_are_what_the_sampler_maximises():
    """The diagnostic scores (logits / T + noise) name the sampler's token as their lowest-index maximum,
    reduce to logits / T plus a term that does not depend on the logits, and use the same uniforms."""
    rng = np.random.default_rng(5)
    for trial in range(50):
        n = int(rng.integers(2, 300)); T = float(rng.choice([0.3, 0.7, 1.0, 2.5]))
        seed = int(rng.integers(0, 2 ** 63)); pos = int(rng.integers(0, 5000))
        lg = rng.normal(size=n) * 3
        sc = oracle.gumbel_scores(lg, T, seed, pos)
        assert int(np.argmax(sc)) == oracle.sample_gumbel(lg, T, seed, pos)
        noise = sc - lg / T
        u = np.array([oracle.uniform(seed, pos * n + i) for i in range(n)])
        np.testing.assert_allclose(noise, -np.log(-np.log(u)), rtol=0, atol=1e-12)
        np.testing.assert_allclose(oracle.gumbel_scores(lg + 1.0, T, seed, pos) - sc, 1.0 / T, rtol=0, atol=1e-12)


def test_sequence_sampling_state(tiny_weights):
    """A sequence at temperature 0 is greedy whatever its seed; at temperature > 0 its emitted tokens are
    the sampler's draws on its own logits at the position the token will take."""
    shape, w = tiny_weights
    m = oracle.Model(shape, w)
    kv = oracle.KV(m, 8, 2, 4)
    tok = _prompt(20, shape.vocab, 110)
    (_, a), (_, b) = kv.alloc(0), kv.alloc(0)
    assert kv.set_sampling(a, 0.0, 99) == 0 and kv.set_sampling(b, 0.8, 4242) == 0 and kv.set_sampling(b, -1.0, 1) == oracle.E_INVAL
    rc, ta, lga = kv.prefill(a, tok)
    rc, tb, lgb = kv.prefill(b, tok)
    np.testing.assert_array_equal(lga, lgb)
    assert ta == int(np.argmax(lga)) and tb == oracle.sample_gumbel(lgb, 0.8, 4242, 20)
    for _ in range(5):
        rc, tb, lgb = kv.decode(b)
        assert tb == oracle.sample_gumbel(lgb, 0.8, 4242, kv.length(b))


# ------------------------------------------------------------------ block allocator (integer exact)

class _PyAlloc:
    """Brute-force model of the allocator policy: LIFO stack that first yields 0,1,2,..; blocks of a
    freed sequence are pushed back in reverse logical order."""

    def __init__(self, n):
        self.free = list(range(n - 1, -1, -1)); self.tab = {}

    def alloc(self, sid, reserve):
        self.tab[sid] = [self.free.pop() for _ in range((reserve + 15) // 16)]

    def grow(self, sid, n_tokens):
        while len(self.tab[sid]) * 16 < n_tokens:
            self.tab[sid].append(self.free.pop())

    def release(self, sid):
        for b in reversed(self.tab.pop(sid)):
            self.free.append(b)


def _toy_model(layers=1):
    shape = TINY.with_layers(layers)
    return shape, oracle.Model(shape, make_weights(shape, 99))


def test_allocator_matches_bruteforce_simulation():
    shape, m = _toy_model()
    kv = oracle.KV(m, 40, 4, 12); py = _PyAlloc(40)
    rc, a = kv.alloc(33); py.alloc(a, 33)
    rc, b = kv.alloc(0); py.alloc(b, 0)
    assert (a, b) == (0, 1)
    lens = {a: 0, b: 0}
    steps = [(a, 35), (b, 17), (a, 20), (b, 1), (b, 15), (a, 9)]
    for sid, n in steps:
        kvd = np.zeros((n, shape.n_layers, 2, shape.n_kv_heads, shape.head_dim))
        assert kv.inject(sid, kvd) == 0
        lens[sid] += n; py.grow(sid, lens[sid])
        assert kv.block_table(sid)[1].tolist() == py.tab[sid]
    kv.free(a); py.release(a)
    rc, c = kv.alloc(50); py.alloc(c, 50)
    assert c == a and kv.block_table(c)[1].tolist() == py.tab[c]
    assert kv.free_blocks() == len(py.free)
    # out of blocks: state unchanged, error reported
    before = kv.block_table(b)[1].tolist(), kv.free_blocks()
    assert kv.inject(b, np.zeros((16 * 60, 1, 2, 4, 64))) in (oracle.E_NOMEM, oracle.E_RANGE)
    assert (kv.block_table(b)[1].tolist(), kv.free_blocks()) == before


def test_block_and_slot_of_every_position():
    """Token j is found in logical block j // 16, slot j % 16, including positions 15, 16, 17."""
    shape, m = _toy_model()
    kv = oracle.KV(m, 8, 1, 8)
    rc, s = kv.alloc(0)
    for lb, pb in enumerate([5, 2, 7]):
        assert kv.map(s, lb, pb) == 0
    n = 40
    data = np.arange(n * 2 * 4 * 64, dtype=np.float64).reshape(n, 1, 2, 4, 64)
    assert kv.inject(s, data) == 0
    assert kv.block_table(s)[1].tolist() == [5, 2, 7]
    for pos in (0, 15, 16, 17, 31, 32, 39):
        for which in (0, 1):
            np.testing.assert_array_equal(kv.read(s, 0, which, 3, pos)[1], data[pos, 0, which, 3])


# ------------------------------------------------------------------ whole decoder

def _torch_forward_all(shape, w, tokens, kv_cast=None, kv_out=None):
    """Whole-sequence float64 forward with library routines (matmul, rms_norm, sdpa, silu, polar):
    a formulation with no KV cache and no per-token loop.  kv_cast: applied to the rotated keys and to the
    values before they are attended to (the cache's storage grid); kv_out: list that receives, per layer,
    (rotated keys, values) before the cast, [T, kv_heads, hd]."""
    T = len(tokens); d, H, Hk, hd = shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim
    W = lambda t: t.double()
    x = W(w["embed"])[torch.tensor(tokens)]
    pos = torch.arange(T, dtype=torch.float64)
    theta = shape.rope_base ** (-2.0 * torch.arange(hd // 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(T, hd // 2, dtype=torch.float64), pos[:, None] * theta[None, :])

    def rope(u):                                     # u [T, heads, hd]
        z = torch.complex(u[..., : hd // 2], u[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    for l in range(shape.n_layers):
        h = F.rms_norm(x, (d,), W(w["attn_norm"][l]), eps=shape.rms_eps)
        qkv = h @ W(w["wqkv"][l]).T
        q, k, v = qkv.split([H * hd, Hk * hd, Hk * hd], dim=-1)
        q, k, v = rope(q.view(T, H, hd)), rope(k.view(T, Hk, hd)), v.view(T, Hk, hd)
        if kv_out is not None:
            kv_out.append((k.clone(), v.clone()))
        if kv_cast is not None:
            k, v = kv_cast(k), kv_cast(v)
        k = k.repeat_interleave(H // Hk, dim=1); v = v.repeat_interleave(H // Hk, dim=1)
        if shape.window > 0:                         # band: key j visible to query i iff i - window < j <= i
            i = torch.arange(T)
            mask = (i[None, :] <= i[:, None]) & (i[None, :] > i[:, None] - shape.window)
            o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                               v.transpose(0, 1)[None], attn_mask=mask)[0]
        else:
            o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                               v.transpose(0, 1)[None], is_causal=True)[0]
        x = x + o.transpose(0, 1).reshape(T, H * hd) @ W(w["wo"][l]).T
        h = F.rms_norm(x, (d,), W(w["ffn_norm"][l]), eps=shape.rms_eps)
        gu = h @ W(w["wgate_up"][l]).T
        x = x + (F.silu(gu[:, : shape.d_ffn]) * gu[:, shape.d_ffn:]) @ W(w["wdown"][l]).T
    return (F.rms_norm(x, (d,), W(w["final_norm"]), eps=shape.rms_eps) @ W(w["lm_head"]).T).numpy()


def _prompt(n, vocab, stream=100):
    return gen.randint(SEED_BASE, stream, 0, vocab - 1, n).numpy().astype(np.int32)


def test_decoder_matches_float64_library_rederivation(tiny_weights):
    shape, w = tiny_weights
    tok = _prompt(40, shape.vocab)
    m = oracle.Model(shape, w, kv_round=0)
    got = m.forward_contig(tok)
    ref = _torch_forward_all(shape, w, tok.tolist())
    scale = np.abs(ref).max(axis=1, keepdims=True)
    assert np.max(np.abs(got - ref) / scale) < 1e-11
    assert (got.argmax(1) == ref.argmax(1)).all()


def test_decoder_gqa_and_bf16_weights_match_library_rederivation():
    from dataclasses import replace
    shape = replace(TINY, n_kv_heads=2, dtype="bf16", name="tiny-gqa")
    w = make_weights(shape, 5)
    tok = _prompt(21, shape.vocab, 101)
    got = oracle.Model(shape, w, kv_round=0).forward_contig(tok)
    ref = _torch_forward_all(shape, w, tok.tolist())
    assert np.max(np.abs(got - ref)) / np.abs(ref).max() < 1e-11


def test_cache_rounding_is_applied_to_rotated_keys_and_to_values_when_they_are_appended():
    """The cache's element type is part of its contract: with a bf16 cache a token's keys (after the rotary
    embedding) and values are rounded to bf16 once, when appended, and every later query sees the rounded
    rows.  Pinned on a bf16 shape against the whole-sequence re-derivation: (i) every cached row read back
    lies on the bf16 grid and within half a bf16 unit of the re-derivation's unrounded rotated key / value
    (rounding before the rotation leaves values off the grid; skipping the values or the keys fails the grid
    check), (ii) the logits equal the re-derivation's with the same rounding placed between the rotation and
    the attention, and differ from the unrounded ones."""
    from dataclasses import replace
    shape = replace(TINY, n_kv_heads=2, dtype="bf16", name="tiny-gqa-bf16")
    w = make_weights(shape, 7)
    tok = _prompt(37, shape.vocab, 103)
    m = oracle.Model(shape, w, kv_round=1)
    kv = oracle.KV(m, 4, 1, 4)
    rc, s = kv.alloc(0)
    rc, t0, lg0 = kv.prefill(s, tok[:20])           # two calls: rounding must not depend on the chunking
    rc, t1, lg1 = kv.prefill(s, tok[20:])           # feeds the pending token t0 first, then tok[20:]
    seq = tok[:20].tolist() + [t0] + tok[20:].tolist()
    cast = lambda t: torch.from_numpy(oracle.round_bf16(t.numpy()))
    rows = []
    ref = _torch_forward_all(shape, w, seq, kv_cast=cast, kv_out=rows)
    plain = _torch_forward_all(shape, w, seq)
    assert np.max(np.abs(lg1 - ref[-1])) / np.abs(ref[-1]).max() < 1e-11
    assert np.max(np.abs(lg0 - ref[19])) / np.abs(ref[19]).max() < 1e-11
    assert np.max(np.abs(lg1 - plain[-1])) / np.abs(plain[-1]).max() > 1e-6      # the rounding is not a no-op
    for l in range(shape.n_layers):
        for which in (0, 1):
            for h in range(shape.n_kv_heads):
                for pos in range(len(seq)):
                    got = kv.read(s, l, which, h, pos)[1]
                    want = rows[l][which][pos, h].numpy()
                    np.testing.assert_array_equal(oracle.round_bf16(got), got)     # on the bf16 grid
                    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) * (1 + 1e-9))   # half a unit of an 8-bit significand
                    assert np.any(got != want)


@pytest.mark.parametrize("window", [1, 7, 16, 33])
def test_banded_decoder_matches_library_rederivation_with_band_mask(window):
    """Attention band: the float64 whole-sequence re-derivation with an explicit boolean band mask."""
    from dataclasses import replace
    shape = replace(TINY, n_kv_heads=2, window=window, name="tiny-band")
    w = make_weights(shape, 6)
    tok = _prompt(40, shape.vocab, 102)
    got = oracle.Model(shape, w, kv_round=0).forward_contig(tok)
    ref = _torch_forward_all(shape, w, tok.tolist())
    assert np.max(np.abs(got - ref)) / np.abs(ref).max() < 1e-11


def test_band_at_least_as_long_as_the_sequence_changes_nothing_and_shorter_does(tiny_weights):
    from dataclasses import replace
    shape, w = tiny_weights
    tok = _prompt(24, shape.vocab, 103)
    full = oracle.Model(shape, w, kv_round=0).forward_contig(tok)
    same = oracle.Model(replace(shape, window=24), w, kv_round=0).forward_contig(tok)
    np.testing.assert_array_equal(same, full)
    short = oracle.Model(replace(shape, window=23), w, kv_round=0).forward_contig(tok)
    np.testing.assert_array_equal(short[:23], full[:23])     # the band first bites at position 23
    assert np.abs(short[23] - full[23]).max() > 1e-9


def test_band_of_one_makes_attention_return_the_own_value(tiny_weights):
    """window = 1: softmax over the own position only, so the attention output is the token's own
    value vector and every token's logits are those of a one-token sequence rotated to its position:
    with rotary embedding acting on q and k only, they do not depend on the position at all."""
    from dataclasses import replace
    shape, w = tiny_weights
    tok = _prompt(6, shape.vocab, 104)
    got = oracle.Model(replace(shape, window=1), w, kv_round=0).forward_contig(tok)
    m = oracle.Model(shape, w, kv_round=0)
    for i, t in enumerate(tok):
        np.testing.assert_allclose(got[i], m.forward_contig(np.array([t], np.int32))[0], rtol=1e-12, atol=1e-13)


def test_paged_attention_band_equals_attention_over_the_last_positions():
    B, H, Hkv, hd = 3, 4, 2, 64
    lens = [5, 17, 48]
    table, kf, vf = _paged_case(B, H, Hkv, hd, lens, False)
    q = RNG.standard_normal((B, H, hd))
    kp, vp = oracle.to_host_matrix(kf), oracle.to_host_matrix(vf)
    kd, vd = kf.double().numpy(), vf.double().numpy()
    for window in (1, 9, 16, 40, 48, 100):
        out = oracle.paged_attention(q, kp, vp, (Hkv * 16 * hd, 16 * hd, hd), table, lens, Hkv, window=window)
        for b in range(B):
            vis = range(max(0, lens[b] - window), lens[b])
            for h in range(H):
                g = h // (H // Hkv)
                K = np.stack([kd[table[b, j // 16], g, j % 16] for j in vis])
                V = np.stack([vd[table[b, j // 16], g, j % 16] for j in vis])
                ref = torch.softmax(torch.from_numpy(K @ q[b, h]) / math.sqrt(hd), 0).numpy() @ V
                np.testing.assert_allclose(out[b, h], ref, rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("window", [0, 19])
def test_paged_equals_contiguous_and_rounds_follow_the_concatenation(tiny_weights, window):
    """Paged cache == contiguous cache bitwise, and a multi-round run (prefill, decode, append an
    observation, continue) produces at every call the logits of the concatenated sequence
    prompt ++ generated ++ observation (section 2.2 step (g)), the pending token being fed first.
    Also with an attention band shorter than the sequence (the band spans block boundaries)."""
    from dataclasses import replace
    shape, w = tiny_weights
    shape = replace(shape, window=window)
    tok = _prompt(37, shape.vocab)
    m = oracle.Model(shape, w)                 # cache rounded to fp32 for the fp32 shape
    kv = oracle.KV(m, 16, 3, 8)
    rc, s = kv.alloc(0)
    for lb, pb in enumerate([9, 3, 14, 0, 5]):
        kv.map(s, lb, pb)
    seq, calls = list(tok), []                 # calls: (index of the position whose logits were returned, logits)
    rc, t, lg = kv.prefill(s, tok); assert rc == 0
    calls.append((len(seq) - 1, lg, t))
    for _ in range(3):
        seq.append(t)
        rc, t, lg = kv.decode(s); assert rc == 0
        calls.append((len(seq) - 1, lg, t))
    obs = _prompt(20, shape.vocab, 102)
    seq.append(t); seq.extend(obs.tolist())
    rc, t, lg = kv.prefill(s, obs); assert rc == 0
    calls.append((len(seq) - 1, lg, t))
    seq.append(t)
    rc, t, lg = kv.decode(s); assert rc == 0
    calls.append((len(seq) - 1, lg, t))
    assert kv.length(s) == len(seq)
    ref = m.forward_contig(np.array(seq, np.int32))
    for idx, lg, t in calls:
        assert np.array_equal(lg, ref[idx])
        assert t == int(np.argmax(ref[idx]))
    assert kv.block_table(s)[1].tolist() == [9, 3, 14, 0, 5]
    # decode without a pending token and stepping a stopped sequence are state errors
    rc, s2 = kv.alloc(0)
    assert kv.decode(s2)[0] == oracle.E_STATE
    kv.stop(s); assert kv.decode(s)[0] == oracle.E_STATE
    assert kv.prefill(s2, np.array([shape.vocab], np.int32))[0] == oracle.E_RANGE


def test_swap_out_and_in_keeps_the_sequence_and_follows_the_allocator(tiny_weights):
    """KV retention (section 2.2): a sequence swapped out and back continues bit-identically to a twin that
    stayed in the pool, also when its blocks were taken by another sequence meanwhile (so it comes back on
    different physical blocks); the store holds exactly the rows the cache held; blocks return to the free
    list in the order a free would return them; a swapped-out sequence cannot be stepped; a swap-in without
    enough free blocks fails and changes nothing."""
    shape, w = tiny_weights
    m = oracle.Model(shape, w)
    tok = _prompt(37, shape.vocab, 105)
    kv, twin = oracle.KV(m, 8, 3, 6), oracle.KV(m, 8, 3, 6)
    (_, s), (_, s2) = kv.alloc(0), twin.alloc(0)
    for k in (kv, twin):
        assert k.prefill(0, tok)[0] == 0
        for _ in range(2):
            assert k.decode(0)[0] == 0
    assert kv.block_table(s)[1].tolist() == [0, 1, 2] and kv.free_blocks() == 5
    rows = {(l, wh, h, p): kv.read(s, l, wh, h, p)[1] for l in (0, 1) for wh in (0, 1) for h in (0, 3) for p in (0, 15, 16, 38)}
    rc, store = kv.swap_out(s)
    assert rc == 0 and kv.free_blocks() == 8 and kv.length(s) == 39 and kv.block_table(s)[1].tolist() == []
    st = store.reshape(3, shape.n_layers, 2, shape.n_kv_heads, 16, shape.head_dim)
    for (l, wh, h, p), row in rows.items():
        np.testing.assert_array_equal(st[p // 16, l, wh, h, p % 16], row)
    assert kv.decode(s)[0] == oracle.E_STATE and kv.prefill(s, tok[:2])[0] == oracle.E_STATE
    assert kv.swap_out(s)[0] == oracle.E_STATE
    # the freed blocks come back in logical order to the next taker
    rc, other = kv.alloc(6 * 16)
    assert kv.block_table(other)[1].tolist() == [0, 1, 2, 3, 4, 5] and kv.free_blocks() == 2
    assert kv.swap_in(s, store) == oracle.E_NOMEM and kv.free_blocks() == 2 and kv.decode(s)[0] == oracle.E_STATE
    kv.free(other)
    rc, filler = kv.alloc(2 * 16)                      # takes blocks 0, 1: the sequence returns on 2, 3, 4
    assert kv.swap_in(s, store) == 0 and kv.block_table(s)[1].tolist() == [2, 3, 4]
    assert kv.swap_in(s, store) == oracle.E_STATE
    for _ in range(12):                                # crosses into a new block on both sides
        (rc_a, t_a, lg_a), (rc_b, t_b, lg_b) = kv.decode(s), twin.decode(s2)
        assert rc_a == rc_b == 0 and t_a == t_b
        np.testing.assert_array_equal(lg_a, lg_b)


def test_fork_shares_full_blocks_and_equals_recomputing_the_prefix(tiny_weights):
    """Prefix sharing: a child forked from the first n positions of a parent continues exactly like a
    sequence that was fed the same prefix from scratch (a cached row depends on the tokens before it only);
    full blocks are shared by reference, a partly filled last block is copied; a shared block returns to the
    free list only when its last holder lets go; the parent's later appends and its death do not touch the
    child."""
    shape, w = tiny_weights
    m = oracle.Model(shape, w)
    prefix, tail_a, tail_b = _prompt(40, shape.vocab, 106), _prompt(9, shape.vocab, 107), _prompt(5, shape.vocab, 108)
    kv, ref = oracle.KV(m, 12, 4, 6), oracle.KV(m, 12, 4, 6)
    rc, parent = kv.alloc(0)
    assert kv.prefill(parent, np.concatenate([prefix, tail_a]))[0] == 0          # 49 positions: blocks 0..3
    assert kv.block_table(parent)[1].tolist() == [0, 1, 2, 3]
    # fork inside a block: 2 full blocks shared, the third copied into block 4
    rc, child = kv.fork(parent, 40)
    assert rc == 0 and kv.block_table(child)[1].tolist() == [0, 1, 4] and kv.length(child) == 40 and kv.free_blocks() == 7
    # fork at a block boundary: nothing copied, nothing popped
    rc, child2 = kv.fork(parent, 32)
    assert rc == 0 and kv.block_table(child2)[1].tolist() == [0, 1] and kv.free_blocks() == 7
    assert kv.fork(parent, 50)[0] == oracle.E_INVAL and kv.decode(child)[0] == oracle.E_STATE   # no pending token
    # the parent goes on and then dies; its own blocks are recycled and overwritten by a stranger
    for _ in range(20):
        kv.decode(parent)
    kv.free(parent)
    assert kv.free_blocks() == 6 + 3                       # it had grown into block 5; 2, 3, 5 came back, 0, 1 are still held
    rc, stranger = kv.alloc(0)
    kv.prefill(stranger, _prompt(48, shape.vocab, 109))
    # the child against a from-scratch sequence with the same tokens
    rc, solo = ref.alloc(0)
    rc_a, t_a, lg_a = kv.prefill(child, tail_b)
    rc_b, t_b, lg_b = ref.prefill(solo, np.concatenate([prefix, tail_b]))
    assert rc_a == rc_b == 0 and t_a == t_b
    np.testing.assert_array_equal(lg_a, lg_b)
    for _ in range(10):
        (rc_a, t_a, lg_a), (rc_b, t_b, lg_b) = kv.decode(child), ref.decode(solo)
        assert t_a == t_b
        np.testing.assert_array_equal(lg_a, lg_b)
    # last holders: child2 still pins blocks 0, 1 after the child is gone; then they return, last logical first
    kv.free(child); kv.free(stranger)
    assert kv.free_blocks() == 10
    kv.free(child2)
    assert kv.free_blocks() == 12
    rc, again = kv.alloc(32)
    assert kv.block_table(again)[1].tolist() == [0, 1]
    # no block for the copied tail: the fork fails and changes nothing
    small = oracle.KV(m, 3, 2, 6)
    rc, p2 = small.alloc(0); small.prefill(p2, prefix)
    assert small.free_blocks() == 0 and small.fork(p2, 33)[0] == oracle.E_NOMEM and small.fork(p2, 32)[0] == 0


def test_trim_releases_exactly_the_blocks_below_the_band_and_changes_no_output(tiny_weights):
    """Sliding-window memory: with a band of W positions, trimming after every step gives up exactly the
    blocks whose 16 positions all lie below n - W + 1 (brute force over positions), the sequence then holds
    ceil(n/16) - floor(max(0, n-W+1)/16) blocks, and tokens and logits are bitwise those of a twin that
    never trims -- also after a stranger has overwritten the released blocks.  Without a band nothing is
    released."""
    shape, w = tiny_weights
    W = 21
    banded = replace(shape, window=W)
    m = oracle.Model(banded, w)
    kv, ref = oracle.KV(m, 12, 3, 10), oracle.KV(m, 12, 3, 10)
    (_, s), (_, r) = kv.alloc(0), ref.alloc(0)
    tk = _prompt(50, shape.vocab, 120)
    assert kv.prefill(s, tk)[1] == ref.prefill(r, tk)[1]
    rc, n_rel = kv.trim(s)
    n = 50
    assert rc == 0 and n_rel == (n - W + 1) // 16 == 1 and kv.block_table(s)[1].tolist() == [-1, 1, 2, 3]
    assert kv.trim(s) == (0, 0)                                  # nothing more to give
    rc, stranger = kv.alloc(0)
    assert kv.prefill(stranger, _prompt(16, shape.vocab, 121))[0] == 0 and kv.block_table(stranger)[1].tolist() == [0]
    for step in range(60):
        (rc_a, t_a, lg_a), (rc_b, t_b, lg_b) = kv.decode(s), ref.decode(r)
        assert rc_a == rc_b == 0 and t_a == t_b
        np.testing.assert_array_equal(lg_a, lg_b)
        n += 1
        rc, n_rel = kv.trim(s)
        tab = kv.block_table(s)[1].tolist()
        visible_from = n - W + 1                                  # lowest position the next query sees
        for blk, phys in enumerate(tab):
            all_below = all(p < visible_from for p in range(16 * blk, 16 * blk + 16))
            assert (phys == -1) == all_below, (step, blk)
        assert sum(p >= 0 for p in tab) == -(-n // 16) - max(0, n - W + 1) // 16
    # the untrimmed twin holds every block of its 110 positions
    assert ref.free_blocks() == 12 - 7 and kv.free_blocks() == 12 - 1 - 2
    # an observation chunk after trimming: its rows see back to n - W + 1, all of which is still there
    obs = _prompt(30, shape.vocab, 122)
    (rc_a, t_a, lg_a), (rc_b, t_b, lg_b) = kv.prefill(s, obs), ref.prefill(r, obs)
    assert t_a == t_b
    np.testing.assert_array_equal(lg_a, lg_b)
    # no band: nothing is released
    kv0 = oracle.KV(oracle.Model(shape, w), 12, 1, 10)
    rc, s0 = kv0.alloc(0)
    kv0.prefill(s0, tk)
    assert kv0.trim(s0) == (0, 0) and kv0.free_blocks() == 12 - 4


def test_trim_with_shared_blocks_swap_and_fork(tiny_weights):
    """A shared block returns to the free list only when its last holder trims it; a trimmed sequence swaps
    out and in (only the blocks it still holds travel) and goes on unchanged; a fork below what the parent
    has released is refused, one inside the band shares only the blocks that are left."""
    shape, w = tiny_weights
    banded = replace(shape, window=20)
    m = oracle.Model(banded, w)
    kv, ref = oracle.KV(m, 16, 4, 10), oracle.KV(m, 16, 4, 10)
    (_, p), (_, r) = kv.alloc(0), ref.alloc(0)
    tk = _prompt(70, shape.vocab, 123)
    kv.prefill(p, tk); ref.prefill(r, tk)                          # blocks 0..4
    rc, child = kv.fork(p, 64)                                     # shares blocks 0..3
    assert rc == 0 and kv.free_blocks() == 16 - 5
    assert kv.trim(p) == (0, 3) and kv.free_blocks() == 16 - 5     # 70 - 20 + 1 = 51: blocks 0, 1, 2 go, still held by the child
    assert kv.trim(child) == (0, 2) and kv.free_blocks() == 16 - 5 + 2   # 64 - 20 + 1 = 45: blocks 0, 1; block 2 still held
    assert kv.block_table(child)[1].tolist() == [-1, -1, 2, 3]
    kv.free(child)
    assert kv.free_blocks() == 16 - 2                              # the parent holds 3 and 4
    # forks from the trimmed parent
    assert kv.fork(p, 40)[0] == oracle.E_STATE                     # would need block 1
    rc, c2 = kv.fork(p, 68)                                        # 68 - 20 + 1 = 49 -> block 3 on: shares block 3, copies the tail
    assert rc == 0 and kv.block_table(c2)[1].tolist()[:4] == [-1, -1, -1, 3]
    rc, r2 = ref.fork(r, 68)
    suf = _prompt(7, shape.vocab, 124)
    (rc_a, t_a, lg_a), (rc_b, t_b, lg_b) = kv.prefill(c2, suf), ref.prefill(r2, suf)
    assert rc_a == rc_b == 0 and t_a == t_b
    np.testing.assert_array_equal(lg_a, lg_b)
    # swap the trimmed parent out and in
    held = kv.free_blocks()
    rc, store = kv.swap_out(p)
    assert rc == 0 and kv.trim(p)[0] == oracle.E_STATE
    # block 3 was shared with the fork and stays with it; the parent comes back on two blocks of its own
    assert kv.swap_in(p, store) == 0 and kv.free_blocks() == held - 1 and kv.block_table(p)[1].tolist()[:3] == [-1, -1, -1]
    for _ in range(25):
        (rc_a, t_a, lg_a), (rc_b, t_b, lg_b) = kv.decode(p), ref.decode(r)
        assert t_a == t_b
        np.testing.assert_array_equal(lg_a, lg_b)
        kv.trim(p)


def test_wo_and_wdown_zero_make_every_layer_the_identity(tiny_weights):
    shape, w = tiny_weights
    w0 = dict(w)
    w0["wo"] = [torch.zeros_like(t) for t in w["wo"]]; w0["wdown"] = [torch.zeros_like(t) for t in w["wdown"]]
    tok = _prompt(6, shape.vocab)
    got = oracle.Model(shape, w0, kv_round=0).forward_contig(tok)
    E, Wl, g = w["embed"].double().numpy(), w["lm_head"].double().numpy(), w["final_norm"].double().numpy()
    for p, t in enumerate(tok):
        x = E[t]
        ref = Wl @ (x / np.sqrt(np.mean(x * x) + shape.rms_eps) * g)
        np.testing.assert_allclose(got[p], ref, rtol=1e-12, atol=1e-15)


def test_golden_tiny_tokens_are_reproduced_by_the_oracle():
    """The stored greedy tokens of workload 0 (written by tests/golden/make_tiny_tokens.py from the oracle)
    still come out of the oracle: guards the fixture and the generator against silent drift."""
    import json, os, importlib.util
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_tiny_tokens", os.path.join(here, "make_tiny_tokens.py"))
    mod = importlib.util.module_from_spec(spec); spec.loader.exec_module(mod)
    stored = json.load(open(os.path.join(here, "tiny_fp32_tokens.json")))
    fresh = mod.compute()
    assert fresh["tokens"] == stored["tokens"] and fresh["prompt"] == stored["prompt"]
    assert fresh["block_table"] == stored["block_table"] == [0, 1, 2, 3, 4, 5]
    assert len(set(stored["tokens"])) >= 4         # not a constant sequence
