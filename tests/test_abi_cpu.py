"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host logic
(block allocator, sequence state machine, argument validation) behaves as the header states and as
the oracle's allocator does (integer-exact).  No kernel is launched here."""
import ctypes as C
import glob
import os
import re

import numpy as np
import pytest

import oracle
import paper_2406_00059_amd as ld
from workloads import TINY, gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 1 << 20     # an aligned non-null "device address" that is never dereferenced on the CPU


def _declared():
    names = []
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        src = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names += re.findall(r"\b(ldk?_[a-z0-9_]+)\s*\(", src)
    return sorted(set(n for n in names if n not in ("ld_token_cb",)))


def test_library_exports_every_declared_symbol():
    L = ld.lib()
    decl = _declared()
    assert len(decl) >= 25
    for name in decl:
        assert hasattr(L, name), f"{name} declared in include/ but not exported"
    assert set(decl) == set(ld.binding.EXPORTS)


def _cfg(**over):
    base = dict(n_layers=2, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                rms_eps=1e-5, rope_base=10000.0, dtype=ld.LD_F32, kv_block=16, max_chunk=256, window=0)
    base.update(over)
    return ld.ld_model_config(**base)


def _weights(L=2):
    tab = (C.c_void_p * L)(*[FAKE] * L)
    p = C.cast(tab, C.POINTER(C.c_void_p))
    w = ld.ld_weights(FAKE, FAKE, FAKE, p, p, p, p, p, p)
    w._keep = tab
    return w


def _model(**over):
    return ld.ld_model_create(_cfg(**over), _weights())


def _kv(m, n_blocks=40, max_tokens=64, max_seqs=4, max_blocks=12):
    ws = ld.ld_workspace_bytes(m, max_tokens, max_seqs, max_blocks)
    assert ws > 0
    return ld.ld_kv_create(m, FAKE, n_blocks, FAKE, ws, max_tokens, max_seqs, max_blocks)


@pytest.mark.parametrize("bad", [dict(head_dim=48), dict(kv_block=32), dict(n_kv_heads=3), dict(d_model=250),
                                 dict(dtype=7), dict(vocab=0), dict(rms_eps=0.0), dict(window=-1)])
def test_model_create_rejects_bad_shapes(bad):
    with pytest.raises(ld.LdError) as e:
        _model(**bad)
    assert e.value.status == ld.LD_E_INVAL and ld.ld_last_error()


def test_pool_size_formula():
    m = _model()
    # [layer][block][2][kv_head][16][hd] float32
    assert ld.ld_kv_bytes(m, 10) == 2 * 10 * 2 * 4 * 16 * 64 * 4
    m2 = _model(dtype=ld.LD_BF16, n_kv_heads=2)
    assert ld.ld_kv_bytes(m2, 3) == 2 * 3 * 2 * 2 * 16 * 64 * 2
    with pytest.raises(ld.LdError):
        ld.ld_kv_create(m, FAKE, 4, FAKE, 16, 8, 2, 2)            # workspace too small
    with pytest.raises(ld.LdError):
        ld.ld_kv_create(m, FAKE + 8, 4, FAKE, 1 << 40, 8, 2, 2)   # misaligned pool


def test_f16_image_size_and_argument_checks():
    """Two bytes per layer-matrix entry for bf16 models, nothing for float32 ones; too small or misaligned a buffer
    is refused before any device memory is touched, and detaching needs no device."""
    m = _model(dtype=ld.LD_BF16, n_kv_heads=2)
    per_layer = (4 + 2 * 2) * 64 * 256 + 4 * 64 * 256 + 3 * 688 * 256
    assert ld.ld_model_f16_image_bytes(m) == 2 * 2 * per_layer
    assert ld.ld_model_f16_image_bytes(_model()) == 0

    def attach(model, ptr, nbytes):
        ok = C.c_int32(7)
        return ld.lib().ld_model_attach_f16_image(model, C.c_void_p(ptr), nbytes, None, C.byref(ok)), ok.value

    need = ld.ld_model_f16_image_bytes(m)
    assert attach(m, FAKE, need) == (ld.LD_E_INVAL, 0)            # the 256 bytes behind the image are missing
    assert attach(m, FAKE + 8, need + 256) == (ld.LD_E_INVAL, 0)  # misaligned
    assert attach(_model(), FAKE, 1 << 30) == (ld.LD_E_INVAL, 0)  # float32 model
    assert attach(m, None, 0) == (ld.LD_OK, 0)                    # detach


def test_allocator_matches_oracle_allocator_bit_exact():
    """Random alloc / map / grow / free traffic: block tables and free counts equal the oracle's."""
    from workloads import make_weights
    shape = TINY.with_layers(1)
    om = oracle.Model(shape, make_weights(shape, 3))
    okv = oracle.KV(om, 48, 5, 10)
    m = _model(n_layers=1)
    kv = _kv(m, n_blocks=48, max_seqs=5, max_blocks=10)
    r = gen.randint(77, 1, 0, 1 << 30, 400).numpy()
    live, lens = [], {}
    zero = lambda n: np.zeros((n, 1, 2, 4, 64))
    for step in range(100):
        op = r[4 * step] % 4
        if op == 0 or not live:
            res = int(r[4 * step + 1] % 40)
            rc_o, s_o = okv.alloc(res)
            rc_g, s_g = ld.ld_kv_alloc(kv, res, check=False)
            assert rc_o == rc_g
            if rc_o == 0:
                assert s_o == s_g
                live.append(s_o); lens[s_o] = 0
        elif op == 1:
            s = live[r[4 * step + 1] % len(live)]
            n = int(r[4 * step + 2] % 50)
            rc_o = okv.inject(s, zero(n))
            rc_g = ld.ld_kv_assume(kv, s, n, -1, check=False)
            assert rc_o == rc_g, (step, rc_o, rc_g)
        elif op == 2:
            s = live[r[4 * step + 1] % len(live)]
            lb, pb = int(r[4 * step + 2] % 10), int(r[4 * step + 3] % 48)
            assert okv.map(s, lb, pb) == ld.ld_kv_map(kv, s, lb, pb, check=False)
        else:
            s = live.pop(r[4 * step + 1] % len(live))
            assert okv.free(s) == 0 and ld.ld_kv_free(kv, s) == 0
        assert okv.free_blocks() == ld.ld_kv_free_blocks(kv)
        for s in live:
            assert okv.block_table(s)[1].tolist() == ld.ld_kv_block_table(kv, s).tolist()
            assert okv.length(s) == ld.ld_kv_len(kv, s)
    assert step == 99


def test_first_pops_are_0_1_2_and_free_returns_blocks_in_logical_order():
    m = _model()
    kv = _kv(m)
    a = ld.ld_kv_alloc(kv, 33)
    b = ld.ld_kv_alloc(kv, 16)
    assert ld.ld_kv_block_table(kv, a).tolist() == [0, 1, 2] and ld.ld_kv_block_table(kv, b).tolist() == [3]
    ld.ld_kv_free(kv, a)
    c = ld.ld_kv_alloc(kv, 48)
    assert c == a and ld.ld_kv_block_table(kv, c).tolist() == [0, 1, 2]


def test_state_errors_leave_state_unchanged():
    m = _model()
    kv = _kv(m, n_blocks=3, max_tokens=64, max_seqs=2, max_blocks=8)
    s = ld.ld_kv_alloc(kv, 0)
    # decode with no pending token
    rc, _ = ld.ld_decode_step(kv, [s], stream=0, check=False)
    assert rc == ld.LD_E_STATE and "pending" in ld.ld_last_error()
    # token id out of range, bad handle, duplicate sequence
    assert ld.ld_prefill(kv, s, [5, 1024], stream=0, check=False)[0] == ld.LD_E_RANGE
    assert ld.ld_prefill(kv, 1, [5], stream=0, check=False)[0] == ld.LD_E_INVAL
    ld.ld_kv_assume(kv, s, 5, pending=7)
    assert ld.ld_decode_step(kv, [s, s], stream=0, check=False)[0] == ld.LD_E_INVAL
    # out of blocks: 3 blocks = 48 tokens; prefill of 60 must fail without touching anything
    before = (ld.ld_kv_block_table(kv, s).tolist(), ld.ld_kv_free_blocks(kv), ld.ld_kv_len(kv, s))
    assert ld.ld_prefill(kv, s, list(range(60)), stream=0, check=False)[0] == ld.LD_E_NOMEM
    assert (ld.ld_kv_block_table(kv, s).tolist(), ld.ld_kv_free_blocks(kv), ld.ld_kv_len(kv, s)) == before
    # more rows than the workspace was sized for
    kv2 = _kv(m, n_blocks=30, max_tokens=8, max_seqs=2, max_blocks=8)
    s2 = ld.ld_kv_alloc(kv2, 0)
    t = np.arange(20, dtype=np.int32)
    rc, _ = ld.ld_step_mixed(kv2, [], [s2], [t], stream=0, check=False)
    assert rc == ld.LD_E_RANGE
    # context beyond max_blocks_per_seq
    assert ld.ld_kv_assume(kv2, s2, 16 * 8 + 1, check=False) == ld.LD_E_RANGE
    # double free
    assert ld.ld_kv_free(kv2, s2) == 0 and ld.ld_kv_free(kv2, s2, check=False) == ld.LD_E_INVAL


def test_decode_run_rejects_bad_calls_before_touching_anything():
    m = _model()
    kv = _kv(m, n_blocks=3, max_tokens=64, max_seqs=2, max_blocks=2)
    s = ld.ld_kv_alloc(kv, 0)
    assert ld.ld_decode_run(kv, [s], 4, stream=0, check=False) == (ld.LD_E_STATE, 0)        # nothing pending
    ld.ld_kv_assume(kv, s, 5, pending=7)
    assert ld.ld_decode_run(kv, [s, s], 4, stream=0, check=False)[0] == ld.LD_E_INVAL      # listed twice
    assert ld.ld_decode_run(kv, [s, 1], 4, stream=0, check=False)[0] == ld.LD_E_INVAL      # dead handle
    assert ld.ld_decode_run(kv, [s], -1, stream=0, check=False)[0] == ld.LD_E_INVAL
    assert ld.ld_decode_run(kv, [s], 0, stream=0) == (ld.LD_OK, 0)                          # no step asked for
    # the very first step cannot get its block: the error itself comes back, nothing moved
    kv2 = _kv(m, n_blocks=2, max_tokens=64, max_seqs=2, max_blocks=4)
    a, b = ld.ld_kv_alloc(kv2, 0), ld.ld_kv_alloc(kv2, 0)
    ld.ld_kv_assume(kv2, a, 16, pending=7)
    ld.ld_kv_assume(kv2, b, 5, pending=7)
    assert ld.ld_kv_free_blocks(kv2) == 0
    assert ld.ld_decode_run(kv2, [a], 4, stream=0, check=False) == (ld.LD_E_NOMEM, 0)
    assert ld.ld_kv_len(kv2, a) == 16 and ld.ld_kv_block_table(kv2, a).tolist() == [0]


def test_swap_state_machine_without_cached_tokens():
    """Swap-out / swap-in of a sequence that holds reserved blocks but no tokens moves no data, so the
    state machine and the allocator effects can be checked without a GPU: blocks go back as a free would
    return them, the handle stays, the sequence refuses work until swapped in, errors change nothing."""
    m = _model()
    kv = _kv(m, n_blocks=6, max_tokens=16, max_seqs=3, max_blocks=6)
    a = ld.ld_kv_alloc(kv, 40)                       # blocks 0, 1, 2 reserved, no token cached
    assert ld.ld_kv_swap_bytes(kv, a) == 0 and ld.ld_kv_free_blocks(kv) == 3
    assert ld.ld_kv_swap_in(kv, a, None, stream=0, check=False) == ld.LD_E_STATE      # not swapped out
    assert ld.ld_kv_swap_out(kv, a, None, stream=0) == 0
    assert ld.ld_kv_free_blocks(kv) == 6 and ld.ld_kv_block_table(kv, a).tolist() == [] and ld.ld_kv_len(kv, a) == 0
    assert ld.ld_kv_swap_out(kv, a, None, stream=0, check=False) == ld.LD_E_STATE
    assert ld.ld_kv_assume(kv, a, 5, check=False) == ld.LD_E_STATE
    assert ld.ld_kv_map(kv, a, 0, 4, check=False) == ld.LD_E_STATE
    assert ld.ld_prefill(kv, a, [1, 2], stream=0, check=False)[0] == ld.LD_E_STATE and "swapped" in ld.ld_last_error()
    b = ld.ld_kv_alloc(kv, 48)                       # the freed blocks come back in logical order
    assert b != a and ld.ld_kv_block_table(kv, b).tolist() == [0, 1, 2]
    assert ld.ld_kv_swap_in(kv, a, None, stream=0) == 0 and ld.ld_kv_block_table(kv, a).tolist() == []
    ld.ld_kv_assume(kv, a, 20, pending=3)            # usable again: takes blocks 3, 4
    assert ld.ld_kv_block_table(kv, a).tolist() == [3, 4] and ld.ld_kv_swap_bytes(kv, a) == 2 * 2 * (2 * 4 * 16 * 64 * 4)
    assert ld.ld_kv_free(kv, a) == 0 and ld.ld_kv_free_blocks(kv) == 3


def test_fork_at_block_boundaries_shares_blocks_by_holder_count():
    """Prefix sharing without a GPU (a fork at a block boundary copies nothing): shared blocks appear in
    both tables, return to the free list only with their last holder, last logical block first."""
    m = _model()
    kv = _kv(m, n_blocks=8, max_tokens=16, max_seqs=4, max_blocks=6)
    p = ld.ld_kv_alloc(kv, 0)
    ld.ld_kv_assume(kv, p, 50, pending=1)                               # blocks 0..3
    c1 = ld.ld_kv_fork(kv, p, 32, stream=0)
    c2 = ld.ld_kv_fork(kv, p, 48, stream=0)
    assert (c1, c2) == (1, 2) and ld.ld_kv_block_table(kv, c1).tolist() == [0, 1]
    assert ld.ld_kv_block_table(kv, c2).tolist() == [0, 1, 2] and ld.ld_kv_free_blocks(kv) == 4
    assert ld.ld_kv_len(kv, c1) == 32 and ld.ld_kv_len(kv, c2) == 48
    assert ld.ld_kv_fork(kv, p, 51, stream=0, check=False) == ld.LD_E_INVAL
    assert ld.ld_decode_step(kv, [c1], stream=0, check=False)[0] == ld.LD_E_STATE     # a child has no pending token
    ld.ld_kv_free(kv, p)
    assert ld.ld_kv_free_blocks(kv) == 5                                # only block 3 came back
    ld.ld_kv_assume(kv, c1, 16, pending=2)                              # c1 grows into a block of its own
    assert ld.ld_kv_block_table(kv, c1).tolist() == [0, 1, 3]
    ld.ld_kv_free(kv, c2)
    assert ld.ld_kv_free_blocks(kv) == 5                                # block 2 back, 0 and 1 still held by c1
    ld.ld_kv_free(kv, c1)
    assert ld.ld_kv_free_blocks(kv) == 8
    again = ld.ld_kv_alloc(kv, 48)
    assert ld.ld_kv_block_table(kv, again).tolist() == [0, 1, 3]        # LIFO: c1's blocks, logical order
    # a swapped-out parent cannot be forked
    ld.ld_kv_swap_out(kv, again, None, stream=0)
    assert ld.ld_kv_fork(kv, again, 0, stream=0, check=False) == ld.LD_E_STATE


def test_trim_follows_the_oracle_allocator_bit_exact():
    """Sliding-window memory without a GPU: a seeded schedule of growing, trimming, forking at block
    boundaries and freeing, run on the oracle's allocator and the library's side by side: released counts,
    status codes, block tables (released entries read -1) and free counts are identical at every step."""
    from dataclasses import replace
    from workloads import make_weights
    W = 37
    shape = replace(TINY, window=W)
    om = oracle.Model(shape, make_weights(TINY, 3))
    okv = oracle.KV(om, 24, 4, 12)
    m = _model(window=W, n_layers=shape.n_layers, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim)
    kv = _kv(m, n_blocks=24, max_tokens=16, max_seqs=4, max_blocks=12)
    rng = np.random.default_rng(5)
    live = []
    zeros = lambda n: np.zeros((n, shape.n_layers, 2, shape.n_kv_heads, shape.head_dim))
    counts = {}
    for it in range(300):
        op = str(rng.choice(["new"] * (len(live) < 4) + ["grow", "grow", "trim", "trim", "fork"] * bool(live) + ["free"] * (len(live) > 1)))
        if op == "new":
            rc, so = okv.alloc(0); sg = ld.ld_kv_alloc(kv, 0)
            assert rc == 0 and so == sg
            live.append(sg)
        elif op == "grow":
            s = int(rng.choice(live)); n = int(rng.integers(1, 40))
            rc_o = okv.inject(s, zeros(n), pending=1)
            rc_g = ld.ld_kv_assume(kv, s, n, pending=1, check=False)
            assert rc_o == rc_g, (it, rc_o, rc_g)
        elif op == "trim":
            s = int(rng.choice(live))
            rc_o, n_o = okv.trim(s)
            n_g = ld.ld_kv_trim(kv, s)
            assert rc_o == 0 and n_o == n_g, (it, n_o, n_g)
            counts["released"] = counts.get("released", 0) + n_o
        elif op == "fork":
            if len(live) == 4:
                continue
            p_ = int(rng.choice(live))
            n = 16 * int(rng.integers(0, ld.ld_kv_len(kv, p_) // 16 + 1))
            rc_o, co = okv.fork(p_, n)
            cg = ld.ld_kv_fork(kv, p_, n, stream=0, check=False)
            assert (rc_o == 0 and co == cg) or (rc_o != 0 and cg == rc_o), (it, rc_o, co, cg)
            if rc_o == 0:
                live.append(cg)
            else:
                counts["fork_refused"] = counts.get("fork_refused", 0) + 1
        else:
            s = int(rng.choice(live))
            assert okv.free(s) == 0 and ld.ld_kv_free(kv, s) == 0
            live.remove(s)
        counts[op] = counts.get(op, 0) + 1
        assert ld.ld_kv_free_blocks(kv) == okv.free_blocks(), (it, op)
        for s in live:
            assert ld.ld_kv_block_table(kv, s).tolist() == okv.block_table(s)[1].tolist(), (it, op, s)
    assert counts["released"] > 10 and counts.get("fork_refused", 0) > 0, counts
    # a swapped-out sequence cannot be trimmed (one without cached tokens swaps without a copy)
    for s in live:
        ld.ld_kv_free(kv, s)
    e = ld.ld_kv_alloc(kv, 32)
    ld.ld_kv_swap_out(kv, e, None, stream=0)
    assert ld.ld_kv_trim(kv, e, check=False) == ld.LD_E_STATE


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more exits with a message instead of a number."""
    import subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and not r.stdout.strip().startswith("{")
