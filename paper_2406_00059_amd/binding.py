"""ctypes binding of libld.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libld.so")

LD_OK, LD_E_INVAL, LD_E_NOMEM, LD_E_STATE, LD_E_HIP, LD_E_RANGE = 0, -1, -2, -3, -4, -5
LD_CB_CONTINUE, LD_CB_ABORT, LD_CB_PAUSE = 0, 1, 2
LD_F32, LD_BF16 = 0, 1
LDK_STORE, LDK_ADD, LDK_SWIGLU = 0, 1, 2

__all__ = [
    "LD_OK", "LD_E_INVAL", "LD_E_NOMEM", "LD_E_STATE", "LD_E_HIP", "LD_E_RANGE", "LD_F32", "LD_BF16",
    "LD_CB_CONTINUE", "LD_CB_ABORT", "LD_CB_PAUSE",
    "LDK_STORE", "LDK_ADD", "LDK_SWIGLU", "LIB_PATH", "lib", "LdError", "ld_model_config", "ld_weights",
    "ld_token_cb", "ld_model_create", "ld_model_destroy", "ld_model_f16_image_bytes", "ld_model_attach_f16_image", "ld_kv_bytes", "ld_workspace_bytes", "ld_kv_create",
    "ld_kv_destroy", "ld_kv_alloc", "ld_kv_map", "ld_kv_free", "ld_kv_block_table", "ld_kv_len",
    "ld_kv_free_blocks", "ld_kv_assume", "ld_kv_swap_bytes", "ld_kv_swap_out", "ld_kv_swap_in", "ld_kv_fork", "ld_kv_trim", "ld_kv_set_sampling", "ld_prefill", "ld_decode_step", "ld_decode_run", "ld_step_mixed", "ld_last_error", "ld_kv_profile", "ld_kv_profile_read", "ld_profile", "LD_PROF_NAMES",
    "ldk_embed", "ldk_rmsnorm", "ldk_linear", "ldk_linear_f16", "ldk_weights_to_f16", "ldk_prefill_attention_f16", "ldk_linear_scratch_bytes", "ldk_rope_table", "ldk_rope_kv_write", "ldk_qkv_rope",
    "ldk_attention_scratch_bytes", "ldk_paged_attention", "ldk_static_scratch_bytes", "ldk_paged_attention_static",
    "ldk_prefill_attention_scratch_bytes",
    "ldk_prefill_attention", "ldk_argmax", "ldk_sample", "Model", "KV",
]


class LdError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"libld status {status}: {text}")
        self.status = status


class ld_model_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("dtype", C.c_int32), ("kv_block", C.c_int32), ("max_chunk", C.c_int32), ("window", C.c_int32)]


class ld_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("wgate_up", C.POINTER(C.c_void_p)), ("wdown", C.POINTER(C.c_void_p))]


LD_PROF_NAMES = ("qkv", "rope_kv", "attention", "wo", "gate_up", "down", "lm_head", "other")


class ld_profile(C.Structure):
    _fields_ = [("ms", C.c_double * 8), ("launches", C.c_int64 * 8)]


ld_token_cb = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int32, C.c_int32, C.c_int32)

_lib = None
_i32p, _f32p, _vp = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_void_p

_SIGS = {
    "ld_model_create": (C.c_int, [C.POINTER(ld_model_config), C.POINTER(ld_weights), C.POINTER(_vp)]),
    "ld_model_destroy": (None, [_vp]),
    "ld_model_f16_image_bytes": (C.c_size_t, [_vp]),
    "ld_model_attach_f16_image": (C.c_int, [_vp, _vp, C.c_size_t, _vp, _i32p]),
    "ld_kv_bytes": (C.c_size_t, [_vp, C.c_int64]),
    "ld_workspace_bytes": (C.c_size_t, [_vp, C.c_int32, C.c_int32, C.c_int32]),
    "ld_kv_create": (C.c_int, [_vp, _vp, C.c_int64, _vp, C.c_size_t, C.c_int32, C.c_int32, C.c_int32, C.POINTER(_vp)]),
    "ld_kv_destroy": (None, [_vp]),
    "ld_kv_alloc": (C.c_int, [_vp, C.c_int64, _i32p]),
    "ld_kv_map": (C.c_int, [_vp, C.c_int32, C.c_int32, C.c_int32]),
    "ld_kv_free": (C.c_int, [_vp, C.c_int32]),
    "ld_kv_block_table": (C.c_int, [_vp, C.c_int32, _i32p, C.c_int32, _i32p]),
    "ld_kv_len": (C.c_int64, [_vp, C.c_int32]),
    "ld_kv_free_blocks": (C.c_int64, [_vp]),
    "ld_kv_assume": (C.c_int, [_vp, C.c_int32, C.c_int64, C.c_int32]),
    "ld_kv_set_sampling": (C.c_int, [_vp, C.c_int32, C.c_float, C.c_uint64]),
    "ldk_sample": (C.c_int, [_vp, C.c_int32, C.c_int32, _vp, _vp, _vp, _vp, _vp]),
    "ld_kv_fork": (C.c_int, [_vp, C.c_int32, C.c_int64, _vp, C.POINTER(C.c_int32)]),
    "ld_kv_swap_bytes": (C.c_size_t, [_vp, C.c_int32]),
    "ld_kv_swap_out": (C.c_int, [_vp, C.c_int32, _vp, C.c_size_t, _vp]),
    "ld_kv_swap_in": (C.c_int, [_vp, C.c_int32, _vp, C.c_size_t, _vp]),
    "ld_prefill": (C.c_int, [_vp, C.c_int32, _i32p, C.c_int32, _vp, ld_token_cb, _vp, _f32p]),
    "ld_kv_trim": (C.c_int, [_vp, C.c_int32, _i32p]),
    "ld_decode_step": (C.c_int, [_vp, _i32p, C.c_int32, _vp, ld_token_cb, _vp, _f32p]),
    "ld_decode_run": (C.c_int, [_vp, _i32p, C.c_int32, C.c_int32, _vp, ld_token_cb, _vp, _i32p]),
    "ld_step_mixed": (C.c_int, [_vp, _i32p, C.c_int32, _i32p, C.POINTER(_i32p), _i32p, C.c_int32, _vp,
                                ld_token_cb, _vp, _f32p]),
    "ld_kv_profile": (C.c_int, [_vp, C.c_int32]),
    "ld_kv_profile_read": (C.c_int, [_vp, _vp]),
    "ld_last_error": (C.c_char_p, []),
    "ldk_embed": (C.c_int, [_vp, C.c_int32, _vp, C.c_int32, C.c_int32, _vp, _vp]),
    "ldk_rmsnorm": (C.c_int, [_vp, _vp, _vp, C.c_int32, C.c_int32, C.c_float, _vp, _vp]),
    "ldk_linear_scratch_bytes": (C.c_size_t, [C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "ldk_linear": (C.c_int, [_vp, C.c_int32, _vp, _vp, C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp,
                             C.c_size_t, _vp]),
    "ldk_linear_f16": (C.c_int, [_vp, _vp, _vp, _vp, C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp,
                                C.c_size_t, _vp, _vp]),
    "ldk_weights_to_f16": (C.c_int, [_vp, C.c_int64, _vp, _vp, _vp]),
    "ldk_rope_table": (C.c_int, [_vp, C.c_int32, C.c_int32, C.c_float, _vp, _vp]),
    "ldk_rope_kv_write": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.c_int32, _vp, C.c_int32, C.c_int32, C.c_int32,
                                    C.c_int32, C.c_int32, _vp]),
    "ldk_qkv_rope": (C.c_int, [_vp, C.c_int32, _vp, _vp, C.c_float, _vp, _vp, _vp, _vp, _vp, C.c_int32, _vp,
                               C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, C.c_size_t, _vp]),
    "ldk_attention_scratch_bytes": (C.c_size_t, [C.c_int32] * 6),
    "ldk_paged_attention": (C.c_int, [_vp, C.c_int32, _vp, C.c_int32, _vp, C.c_int32, _vp, _vp, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp, C.c_size_t,
                                      _vp]),
    "ldk_static_scratch_bytes": (C.c_size_t, []),
    "ldk_paged_attention_static": (C.c_int, [_vp, C.c_int32, _vp, C.c_int32, _vp, C.c_int32, _vp, _vp, C.c_int32,
                                             C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp]),
    "ldk_prefill_attention_scratch_bytes": (C.c_size_t, []),
    "ldk_prefill_attention": (C.c_int, [_vp, C.c_int32, _vp, C.c_int32, _vp, C.c_int32, _vp, C.c_int32, C.c_int32,
                                        C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp, C.c_size_t, _vp]),
    "ldk_prefill_attention_f16": (C.c_int, [_vp, C.c_int32, _vp, C.c_int32, _vp, C.c_int32, _vp, C.c_int32, C.c_int32,
                                            C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp, C.c_size_t, _vp, _vp]),
    "ldk_argmax": (C.c_int, [_vp, C.c_int32, C.c_int32, _vp, _vp]),
}
EXPORTS = tuple(_SIGS)


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2406_00059_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2406_00059_amd/build.py` "
                              "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def ld_last_error() -> str:
    return lib().ld_last_error().decode()


def _check(rc, raise_on_error=True):
    if rc != LD_OK and raise_on_error:
        raise LdError(rc, ld_last_error())
    return rc


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return t.data_ptr()
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return int(t)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_i32p)


# ------------------------------------------------------------------ model / cache objects

def ld_model_create(cfg: ld_model_config, w: ld_weights):
    h = _vp()
    _check(lib().ld_model_create(C.byref(cfg), C.byref(w), C.byref(h)))
    return h


def ld_model_destroy(m):
    lib().ld_model_destroy(m)


def ld_model_f16_image_bytes(m):
    return lib().ld_model_f16_image_bytes(m)


def ld_model_attach_f16_image(m, buf, stream=None):
    """Returns True when the layer matrices lie within the fp16 range (the image is then in use)."""
    ok = C.c_int32(0)
    _check(lib().ld_model_attach_f16_image(m, _ptr(buf), _nbytes(buf), _stream(stream), C.byref(ok)))
    return bool(ok.value)


def ld_kv_bytes(m, n_blocks):
    return lib().ld_kv_bytes(m, n_blocks)


def ld_workspace_bytes(m, max_tokens, max_seqs, max_blocks_per_seq):
    return lib().ld_workspace_bytes(m, max_tokens, max_seqs, max_blocks_per_seq)


def ld_kv_create(m, pool, n_blocks, ws, ws_bytes, max_tokens, max_seqs, max_blocks_per_seq):
    h = _vp()
    _check(lib().ld_kv_create(m, _ptr(pool), n_blocks, _ptr(ws), ws_bytes, max_tokens, max_seqs,
                              max_blocks_per_seq, C.byref(h)))
    return h


def ld_kv_destroy(kv):
    lib().ld_kv_destroy(kv)


def ld_kv_alloc(kv, reserve_tokens=0, check=True):
    s = C.c_int32(-1)
    rc = _check(lib().ld_kv_alloc(kv, reserve_tokens, C.byref(s)), check)
    return s.value if check else (rc, s.value)


def ld_kv_map(kv, seq, logical, physical, check=True):
    return _check(lib().ld_kv_map(kv, seq, logical, physical), check)


def ld_kv_free(kv, seq, check=True):
    return _check(lib().ld_kv_free(kv, seq), check)


def ld_kv_block_table(kv, seq, cap=1 << 16):
    out = np.empty(cap, dtype=np.int32); n = C.c_int32(0)
    _check(lib().ld_kv_block_table(kv, seq, out.ctypes.data_as(_i32p), cap, C.byref(n)))
    return out[:n.value].copy()


def ld_kv_len(kv, seq):
    return lib().ld_kv_len(kv, seq)


def ld_kv_free_blocks(kv):
    return lib().ld_kv_free_blocks(kv)


def ld_kv_assume(kv, seq, n_tokens, pending=-1, check=True):
    return _check(lib().ld_kv_assume(kv, seq, n_tokens, pending), check)


def ld_kv_set_sampling(kv, seq, temperature, seed, check=True):
    return _check(lib().ld_kv_set_sampling(kv, seq, temperature, seed), check)


def ldk_sample(logits, temperature, seed, pos, out, stream=None):
    """temperature float32 [R], seed int64 [R] (bit pattern of the unsigned seed), pos int32 [R], on the device."""
    R, V = logits.shape
    _check(lib().ldk_sample(_ptr(logits), R, V, _ptr(temperature), _ptr(seed), _ptr(pos), _ptr(out), _stream(stream)))


def ld_kv_fork(kv, parent, n_tokens, stream=None, check=True):
    """-> handle of the child (or the status code when check=False and the call failed)."""
    out = C.c_int32(-1)
    rc = _check(lib().ld_kv_fork(kv, parent, n_tokens, _stream(stream), C.byref(out)), check)
    return out.value if rc == LD_OK else rc


def ld_kv_swap_bytes(kv, seq):
    return lib().ld_kv_swap_bytes(kv, seq)


def ld_kv_swap_out(kv, seq, host_buf, stream=None, check=True):
    """host_buf: a CPU uint8 tensor (pinned for an asynchronous copy) of at least ld_kv_swap_bytes bytes."""
    return _check(lib().ld_kv_swap_out(kv, seq, _ptr(host_buf), _nbytes(host_buf), _stream(stream)), check)


def ld_kv_swap_in(kv, seq, host_buf, stream=None, check=True):
    return _check(lib().ld_kv_swap_in(kv, seq, _ptr(host_buf), _nbytes(host_buf), _stream(stream)), check)


def _cb(callback):
    """Wrap a Python callable (seq, token, pos) as an ld_token_cb (or a null one): LD_CB_PAUSE passes through,
    any other truthy value stops the sequence."""
    if callback is None:
        return C.cast(None, ld_token_cb)
    def call(user, seq, tok, pos):
        r = callback(seq, tok, pos)
        return LD_CB_PAUSE if r is not True and r == LD_CB_PAUSE else (LD_CB_ABORT if r else LD_CB_CONTINUE)
    return ld_token_cb(call)


def _logits_buf(want, rows, vocab):
    if not want:
        return None, None
    a = np.empty((rows, vocab), dtype=np.float32)
    return a, a.ctypes.data_as(_f32p)


def ld_prefill(kv, seq, tokens, stream=None, callback=None, logits_vocab=0, check=True):
    """Returns (status, logits[vocab] or None).  The emitted token reaches `callback(seq, token, pos)`."""
    tok, tp = _i32(tokens)
    lg, lp = _logits_buf(logits_vocab, 1, logits_vocab)
    cb = _cb(callback)
    rc = _check(lib().ld_prefill(kv, seq, tp, tok.size, _stream(stream), cb, None, lp), check)
    return rc, (lg[0] if lg is not None else None)


def ld_decode_step(kv, seqs, stream=None, callback=None, logits_vocab=0, check=True):
    """Returns (status, logits[n_seqs, vocab] or None)."""
    s, sp = _i32(seqs)
    lg, lp = _logits_buf(logits_vocab, s.size, logits_vocab)
    cb = _cb(callback)
    rc = _check(lib().ld_decode_step(kv, sp, s.size, _stream(stream), cb, None, lp), check)
    return rc, lg


def ld_kv_trim(kv, seq, check=True):
    """Returns the number of blocks released (or the status if it failed and check is False)."""
    n = C.c_int32(0)
    rc = _check(lib().ld_kv_trim(kv, seq, C.byref(n)), check)
    return n.value if rc == LD_OK else rc


def ld_decode_run(kv, seqs, max_steps, stream=None, callback=None, check=True):
    """Returns (status, steps done)."""
    s, sp = _i32(seqs)
    cb = _cb(callback)
    done = C.c_int32(0)
    rc = _check(lib().ld_decode_run(kv, sp, s.size, max_steps, _stream(stream), cb, None, C.byref(done)), check)
    return rc, done.value


def ld_step_mixed(kv, dec, pf, pf_tokens, stream=None, callback=None, logits_vocab=0, check=True):
    """dec: decoding sequences; pf: prefilling sequences with their token arrays pf_tokens[i]."""
    d, dp = _i32(dec)
    p, pp = _i32(pf)
    arrs = [np.ascontiguousarray(t, dtype=np.int32) for t in pf_tokens]
    ptrs = (_i32p * max(len(arrs), 1))(*[a.ctypes.data_as(_i32p) for a in arrs])
    n, np_ = _i32([a.size for a in arrs])
    lg, lp = _logits_buf(logits_vocab, d.size + p.size, logits_vocab)
    cb = _cb(callback)
    rc = _check(lib().ld_step_mixed(kv, dp, d.size, pp, ptrs, np_, p.size, _stream(stream), cb, None, lp), check)
    return rc, lg


def ld_kv_profile(kv, enable):
    _check(lib().ld_kv_profile(kv, 1 if enable else 0))


def ld_kv_profile_read(kv):
    """{category: (total ms, launches)}"""
    p = ld_profile()
    _check(lib().ld_kv_profile_read(kv, C.addressof(p)))
    return {n: (p.ms[i], p.launches[i]) for i, n in enumerate(LD_PROF_NAMES)}


# ------------------------------------------------------------------ kernel-level calls (device tensors)

def _dt(dtype):
    return LD_BF16 if dtype in (torch.bfloat16, LD_BF16, "bf16") else LD_F32


def ldk_embed(embed, tok, x, stream=None):
    T, d = x.shape
    _check(lib().ldk_embed(_ptr(embed), _dt(embed.dtype), _ptr(tok), T, d, _ptr(x), _stream(stream)))


def ldk_rmsnorm(x, g, out, eps, row_idx=None, stream=None):
    R, d = out.shape
    _check(lib().ldk_rmsnorm(_ptr(x), _ptr(g), _ptr(row_idx), R, d, eps, _ptr(out), _stream(stream)))


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def ldk_linear_scratch_bytes(T, N, K, epilogue=LDK_STORE):
    return lib().ldk_linear_scratch_bytes(T, N, K, epilogue)


def ldk_linear(W, x, y, epilogue=LDK_STORE, g=None, eps=0.0, scratch=None, stream=None):
    T, K = x.shape
    N = y.shape[1]
    _check(lib().ldk_linear(_ptr(W), _dt(W.dtype), _ptr(x), _ptr(g), eps, T, N, K, epilogue, _ptr(y),
                            _ptr(scratch), _nbytes(scratch), _stream(stream)))


def ldk_linear_f16(W, x, y, overflow, epilogue=LDK_STORE, g=None, eps=0.0, scratch=None, stream=None, W_f16=None):
    T, K = x.shape
    N = y.shape[1]
    _check(lib().ldk_linear_f16(_ptr(W), _ptr(W_f16), _ptr(x), _ptr(g), eps, T, N, K, epilogue, _ptr(y), _ptr(scratch),
                                _nbytes(scratch), _ptr(overflow), _stream(stream)))


def ldk_weights_to_f16(W, out, overflow, stream=None):
    _check(lib().ldk_weights_to_f16(_ptr(W), W.numel(), _ptr(out), _ptr(overflow), _stream(stream)))


def ldk_rope_table(pos, hd, rope_base, cos_sin, stream=None):
    _check(lib().ldk_rope_table(_ptr(pos), pos.numel(), hd, rope_base, _ptr(cos_sin), _stream(stream)))


def ldk_rope_kv_write(qkv, cos_sin, pos, seq_slot, table, pool_layer, H, Hkv, hd, stream=None):
    _check(lib().ldk_rope_kv_write(_ptr(qkv), _ptr(cos_sin), _ptr(pos), _ptr(seq_slot), _ptr(table),
                                   table.shape[1], _ptr(pool_layer), _dt(pool_layer.dtype), qkv.shape[0], H, Hkv,
                                   hd, _stream(stream)))


def ldk_qkv_rope(W, x, qkv, cos_sin, pos, seq_slot, table, pool_layer, H, Hkv, hd, g=None, eps=0.0, scratch=None,
                 stream=None):
    T, K = x.shape
    _check(lib().ldk_qkv_rope(_ptr(W), _dt(W.dtype), _ptr(x), _ptr(g), eps, _ptr(qkv), _ptr(cos_sin), _ptr(pos),
                              _ptr(seq_slot), _ptr(table), table.shape[1], _ptr(pool_layer), T, K, H, Hkv, hd,
                              _ptr(scratch), _nbytes(scratch), _stream(stream)))


def ldk_attention_scratch_bytes(T, H, Hkv, hd, max_ctx, window=0):
    return lib().ldk_attention_scratch_bytes(T, H, Hkv, hd, max_ctx, window)


def ldk_paged_attention(q, q_stride, pool_layer, table, seq_slot, ctx_len, max_ctx, H, Hkv, hd, out, scratch,
                        window=0, stream=None):
    _check(lib().ldk_paged_attention(_ptr(q), q_stride, _ptr(pool_layer), _dt(pool_layer.dtype), _ptr(table),
                                     table.shape[1], _ptr(seq_slot), _ptr(ctx_len), max_ctx, out.shape[0], H, Hkv,
                                     hd, window, _ptr(out), _ptr(scratch), scratch.numel() * scratch.element_size(),
                                     _stream(stream)))


def ldk_static_scratch_bytes():
    return lib().ldk_static_scratch_bytes()


def ldk_paged_attention_static(q, q_stride, pool_layer, table, seq_slot, ctx_len, max_ctx, H, Hkv, hd, out, window=0,
                               stream=None, check=True):
    """ldk_paged_attention without a scratch argument (the library's built-in device array holds the partials)."""
    return _check(lib().ldk_paged_attention_static(_ptr(q), q_stride, _ptr(pool_layer), _dt(pool_layer.dtype),
                                                   _ptr(table), table.shape[1], _ptr(seq_slot), _ptr(ctx_len), max_ctx,
                                                   out.shape[0], H, Hkv, hd, window, _ptr(out), _stream(stream)), check)


def ldk_prefill_attention_scratch_bytes():
    return lib().ldk_prefill_attention_scratch_bytes()


def ldk_prefill_attention(q, q_stride, pool_layer, table, tiles, H, Hkv, hd, out, max_pos, window=0, scratch=None,
                          stream=None):
    _check(lib().ldk_prefill_attention(_ptr(q), q_stride, _ptr(pool_layer), _dt(pool_layer.dtype), _ptr(table),
                                       table.shape[1], _ptr(tiles), tiles.shape[0], H, Hkv, hd, window, max_pos,
                                       _ptr(out), _ptr(scratch) if scratch is not None else None,
                                       scratch.numel() * scratch.element_size() if scratch is not None else 0,
                                       _stream(stream)))


def ldk_prefill_attention_f16(q, q_stride, pool_layer, table, tiles, H, Hkv, hd, out, max_pos, overflow, window=0,
                              scratch=None, stream=None):
    _check(lib().ldk_prefill_attention_f16(_ptr(q), q_stride, _ptr(pool_layer), _dt(pool_layer.dtype), _ptr(table),
                                           table.shape[1], _ptr(tiles), tiles.shape[0], H, Hkv, hd, window, max_pos,
                                           _ptr(out), _ptr(scratch) if scratch is not None else None,
                                           scratch.numel() * scratch.element_size() if scratch is not None else 0,
                                           _ptr(overflow), _stream(stream)))


def ldk_argmax(logits, out, stream=None):
    R, V = logits.shape
    _check(lib().ldk_argmax(_ptr(logits), R, V, _ptr(out), _stream(stream)))


# ------------------------------------------------------------------ owners of handles + device memory

class Model:
    """Keeps the weight tensors alive and owns the ld_model handle."""

    def __init__(self, shape, weights, max_chunk=256):
        self.shape, self.weights = shape, weights
        L = shape.n_layers
        self.cfg = ld_model_config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                                   shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_base,
                                   LD_BF16 if shape.dtype == "bf16" else LD_F32, shape.kv_block, max_chunk,
                                   getattr(shape, "window", 0))
        self._tabs = {k: (C.c_void_p * max(L, 1))(*[t.data_ptr() for t in weights[k]])
                      for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "wgate_up", "wdown")}
        self.w = ld_weights(weights["embed"].data_ptr(), weights["lm_head"].data_ptr(),
                            weights["final_norm"].data_ptr(),
                            *[C.cast(self._tabs[k], C.POINTER(C.c_void_p)) for k in
                              ("attn_norm", "wqkv", "wo", "ffn_norm", "wgate_up", "wdown")])
        self.h = ld_model_create(self.cfg, self.w)
        self.f16_image = None

    def attach_f16_image(self, stream=None):
        """Allocates (torch, device memory) and attaches the fp16 copy of the layer matrices; True if it is in use."""
        n = ld_model_f16_image_bytes(self.h)
        if n == 0:
            return False
        self.f16_image = torch.empty(n + 256, dtype=torch.uint8, device=self.weights["wqkv"][0].device)
        ok = ld_model_attach_f16_image(self.h, self.f16_image, stream)
        if not ok:
            self.detach_f16_image()
        return ok

    def detach_f16_image(self):
        _check(lib().ld_model_attach_f16_image(self.h, None, 0, None, None))
        self.f16_image = None

    def close(self):
        if self.h:
            ld_model_destroy(self.h); self.h = None
        self.f16_image = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class KV:
    """Allocates pool + workspace with torch (device memory only) and owns the ld_kv handle."""

    def __init__(self, model: Model, n_blocks, max_tokens, max_seqs, max_blocks_per_seq, device="cuda", pool=None):
        self.model = model
        self.n_blocks, self.max_blocks = n_blocks, max_blocks_per_seq
        sh = model.shape
        pdtype = torch.bfloat16 if sh.dtype == "bf16" else torch.float32
        nbytes = ld_kv_bytes(model.h, n_blocks)
        # [layer][block][K|V][kv_head][16 * head_dim]: a head's keys are [slot][head_dim], its values are
        # stored transposed, [head_dim][slot] (the tensor's last two dimensions only size the memory)
        self.pool = pool if pool is not None else torch.zeros(
            (sh.n_layers, n_blocks, 2, sh.n_kv_heads, sh.kv_block, sh.head_dim), dtype=pdtype, device=device)
        assert self.pool.numel() * self.pool.element_size() == nbytes
        self.ws_bytes = ld_workspace_bytes(model.h, max_tokens, max_seqs, max_blocks_per_seq)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        self.h = ld_kv_create(model.h, self.pool, n_blocks, self.ws, self.ws_bytes, max_tokens, max_seqs,
                              max_blocks_per_seq)

    def close(self):
        if self.h:
            ld_kv_destroy(self.h); self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
