"""ctypes front end of the CPU oracle (oracle/ld_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import build, LIB

_lib = None

OK, E_INVAL, E_NOMEM, E_STATE, E_RANGE = 0, -1, -2, -3, -5


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", C.c_double), ("rope_base", C.c_double),
                ("wdtype", C.c_int32), ("kv_round", C.c_int32), ("kv_block", C.c_int32), ("window", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("wgate_up", C.POINTER(C.c_void_p)), ("wdown", C.POINTER(C.c_void_p))]


def lib():
    global _lib
    if _lib is None:
        path = build(force=False)
        L = C.CDLL(path)
        dp, ip, vp = C.POINTER(C.c_double), C.POINTER(C.c_int32), C.c_void_p
        L.orc_round_bf16.restype = C.c_double; L.orc_round_bf16.argtypes = [C.c_double]
        L.orc_silu.restype = C.c_double; L.orc_silu.argtypes = [C.c_double]
        L.orc_rmsnorm.argtypes = [dp, C.POINTER(C.c_float), C.c_int32, C.c_double, dp]
        L.orc_rope_head.argtypes = [dp, C.c_int32, C.c_int64, C.c_double]
        L.orc_matvec.argtypes = [vp, C.c_int32, C.c_int64, C.c_int64, dp, dp]
        L.orc_softmax.argtypes = [dp, C.c_int64]
        L.orc_argmax.restype = C.c_int32; L.orc_argmax.argtypes = [dp, C.c_int64]
        L.orc_attention_contig.argtypes = [dp, dp, dp, C.c_int64, C.c_int32, dp]
        L.orc_paged_attention.argtypes = [dp, vp, vp, C.c_int32, C.c_int64, C.c_int64, C.c_int64,
                                          ip, C.c_int32, ip, C.c_int32, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_int32, C.c_int32, dp]
        L.orc_model_create.restype = vp; L.orc_model_create.argtypes = [C.POINTER(Config), C.POINTER(Weights)]
        L.orc_model_destroy.argtypes = [vp]
        L.orc_forward_contig.restype = C.c_int32; L.orc_forward_contig.argtypes = [vp, ip, C.c_int64, dp]
        L.orc_kv_create.restype = vp; L.orc_kv_create.argtypes = [vp, C.c_int64, C.c_int32, C.c_int32]
        L.orc_kv_destroy.argtypes = [vp]
        L.orc_kv_alloc.restype = C.c_int32; L.orc_kv_alloc.argtypes = [vp, C.c_int64, ip]
        L.orc_kv_map.restype = C.c_int32; L.orc_kv_map.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32]
        L.orc_kv_free.restype = C.c_int32; L.orc_kv_free.argtypes = [vp, C.c_int32]
        L.orc_kv_block_table.restype = C.c_int32
        L.orc_kv_block_table.argtypes = [vp, C.c_int32, ip, C.c_int32, ip]
        L.orc_kv_free_blocks.restype = C.c_int64; L.orc_kv_free_blocks.argtypes = [vp]
        L.orc_kv_len.restype = C.c_int64; L.orc_kv_len.argtypes = [vp, C.c_int32]
        L.orc_kv_inject.restype = C.c_int32; L.orc_kv_inject.argtypes = [vp, C.c_int32, dp, C.c_int64, C.c_int32]
        L.orc_kv_read.restype = C.c_int32
        L.orc_kv_read.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64, dp]
        L.orc_prefill.restype = C.c_int32; L.orc_prefill.argtypes = [vp, C.c_int32, ip, C.c_int64, dp, ip]
        L.orc_decode.restype = C.c_int32; L.orc_decode.argtypes = [vp, C.c_int32, dp, ip]
        L.orc_seq_stop.restype = C.c_int32; L.orc_seq_stop.argtypes = [vp, C.c_int32]
        L.orc_uniform.restype = C.c_double; L.orc_uniform.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_sample_gumbel.restype = C.c_int32
        L.orc_sample_gumbel.argtypes = [dp, C.c_int64, C.c_double, C.c_uint64, C.c_int64]
        L.orc_gumbel_scores.restype = None
        L.orc_gumbel_scores.argtypes = [dp, C.c_int64, C.c_double, C.c_uint64, C.c_int64, dp]
        L.orc_seq_set_sampling.restype = C.c_int32
        L.orc_seq_set_sampling.argtypes = [vp, C.c_int32, C.c_double, C.c_uint64]
        L.orc_kv_fork.restype = C.c_int32; L.orc_kv_fork.argtypes = [vp, C.c_int32, C.c_int64, ip]
        L.orc_kv_trim.restype = C.c_int32; L.orc_kv_trim.argtypes = [vp, C.c_int32, ip]
        L.orc_kv_swap_doubles.restype = C.c_int64; L.orc_kv_swap_doubles.argtypes = [vp, C.c_int32]
        L.orc_kv_swap_out.restype = C.c_int32; L.orc_kv_swap_out.argtypes = [vp, C.c_int32, dp]
        L.orc_kv_swap_in.restype = C.c_int32; L.orc_kv_swap_in.argtypes = [vp, C.c_int32, dp]
        _lib = L
    return _lib


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ------------------------------------------------------------------ step functions

def round_bf16(x):
    return np.vectorize(lib().orc_round_bf16, otypes=[np.float64])(np.asarray(x, dtype=np.float64))


def rmsnorm(x, g, eps):
    x = _f64(x); g = np.ascontiguousarray(g, dtype=np.float32); out = np.empty_like(x)
    lib().orc_rmsnorm(_dp(x), g.ctypes.data_as(C.POINTER(C.c_float)), x.size, eps, _dp(out))
    return out


def rope_head(u, pos, base=10000.0):
    u = _f64(u).copy()
    lib().orc_rope_head(_dp(u), u.size, int(pos), base)
    return u


def softmax(s):
    s = _f64(s).copy()
    lib().orc_softmax(_dp(s), s.size)
    return s


def silu(z):
    return lib().orc_silu(float(z))


def argmax(x):
    x = _f64(x)
    return int(lib().orc_argmax(_dp(x), x.size))


def _wptr(w):
    """(pointer, wdtype) of a matrix held as float32 or as bf16 bit patterns (uint16 / int16)."""
    if w.dtype == np.float32:
        return w.ctypes.data, 0
    if w.dtype in (np.uint16, np.int16):
        return w.ctypes.data, 1
    raise TypeError(f"matrix dtype {w.dtype}: want float32 or uint16 bf16 bits")


def matvec(w, x):
    w = np.ascontiguousarray(w); x = _f64(x)
    p, dt = _wptr(w)
    y = np.empty(w.shape[0], dtype=np.float64)
    lib().orc_matvec(p, dt, w.shape[0], w.shape[1], _dp(x), _dp(y))
    return y


def uniform(seed, counter):
    return lib().orc_uniform(seed, counter)


def sample_gumbel(logits, temperature, seed, pos):
    x = _f64(logits)
    return lib().orc_sample_gumbel(_dp(x), x.size, temperature, seed, pos)


def gumbel_scores(logits, temperature, seed, pos):
    """The perturbed scores sample_gumbel takes the argmax of (near-tie diagnosis in the tests)."""
    x = _f64(logits); out = np.empty_like(x)
    lib().orc_gumbel_scores(_dp(x), x.size, temperature, seed, pos, _dp(out))
    return out


def attention_contig(q, K, V):
    q, K, V = _f64(q), _f64(K), _f64(V)
    out = np.empty_like(q)
    lib().orc_attention_contig(_dp(q), _dp(K), _dp(V), K.shape[0], K.shape[1], _dp(out))
    return out


def paged_attention(q, kpool, vpool, strides, block_table, ctx_len, n_kv_heads, kv_block=16, window=0):
    """q [B,H,hd]; pools float32 or uint16 (bf16 bits); strides = (block, head, slot) in elements;
    window > 0: the query (at position ctx_len - 1) sees the last `window` positions only."""
    q = _f64(q); B, H, hd = q.shape
    kp, dt = _wptr(kpool); vp, dt2 = _wptr(vpool)
    assert dt == dt2
    bt = np.ascontiguousarray(block_table, dtype=np.int32); cl = np.ascontiguousarray(ctx_len, dtype=np.int32)
    out = np.empty_like(q)
    lib().orc_paged_attention(_dp(q), kp, vp, dt, strides[0], strides[1], strides[2], _ip(bt), bt.shape[1],
                              _ip(cl), B, H, n_kv_heads, hd, kv_block, window, _dp(out))
    return out


# ------------------------------------------------------------------ model + paged cache

def to_host_matrix(t):
    """torch tensor (float32 or bfloat16, any device) -> numpy float32 / uint16 bit patterns."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.to(torch.float32).numpy()


class Model:
    """Decoder weights + configuration as the oracle sees them (host arrays, borrowed)."""

    def __init__(self, shape, weights, kv_round=None):
        L = shape.n_layers
        self.shape = shape
        self._keep = {k: ([to_host_matrix(t) for t in v] if isinstance(v, list) else to_host_matrix(v))
                      for k, v in weights.items()}
        k = self._keep
        wdtype = 1 if shape.dtype == "bf16" else 0
        if kv_round is None:
            kv_round = 1 if shape.dtype == "bf16" else 2
        self.cfg = Config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                          shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_base, wdtype, kv_round,
                          shape.kv_block, shape.window)
        arr = lambda name: (C.c_void_p * max(L, 1))(*[a.ctypes.data for a in k[name]])
        self._arrs = {n: arr(n) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "wgate_up", "wdown")}
        self.w = Weights(k["embed"].ctypes.data, k["lm_head"].ctypes.data, k["final_norm"].ctypes.data,
                         *[C.cast(self._arrs[n], C.POINTER(C.c_void_p)) for n in
                           ("attn_norm", "wqkv", "wo", "ffn_norm", "wgate_up", "wdown")])
        self.h = lib().orc_model_create(C.byref(self.cfg), C.byref(self.w))
        if not self.h:
            raise ValueError("orc_model_create rejected the configuration")

    def forward_contig(self, tokens):
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        out = np.empty((tok.size, self.shape.vocab), dtype=np.float64)
        rc = lib().orc_forward_contig(self.h, _ip(tok), tok.size, _dp(out))
        if rc:
            raise RuntimeError(f"orc_forward_contig: {rc}")
        return out

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_model_destroy(self.h); self.h = None


class KV:
    """Paged cache + sequence states (allocator policy of the boundary)."""

    def __init__(self, model, n_blocks, max_seqs, max_blocks_per_seq):
        self.model = model
        self.h = lib().orc_kv_create(model.h, n_blocks, max_seqs, max_blocks_per_seq)
        if not self.h:
            raise MemoryError("orc_kv_create")

    def alloc(self, reserve_tokens=0):
        s = C.c_int32(-1)
        rc = lib().orc_kv_alloc(self.h, reserve_tokens, C.byref(s))
        return rc, s.value

    def map(self, seq, logical, physical):
        return lib().orc_kv_map(self.h, seq, logical, physical)

    def free(self, seq):
        return lib().orc_kv_free(self.h, seq)

    def block_table(self, seq, cap=1 << 16):
        out = np.empty(cap, dtype=np.int32); n = C.c_int32(0)
        rc = lib().orc_kv_block_table(self.h, seq, _ip(out), cap, C.byref(n))
        return rc, out[:n.value].copy()

    def free_blocks(self):
        return lib().orc_kv_free_blocks(self.h)

    def length(self, seq):
        return lib().orc_kv_len(self.h, seq)

    def inject(self, seq, kvdata, pending=-1):
        kvdata = _f64(kvdata)
        return lib().orc_kv_inject(self.h, seq, _dp(kvdata), kvdata.shape[0], pending)

    def read(self, seq, layer, which, kvh, pos):
        out = np.empty(self.model.shape.head_dim, dtype=np.float64)
        rc = lib().orc_kv_read(self.h, seq, layer, which, kvh, pos, _dp(out))
        return rc, out

    def prefill(self, seq, tokens, want_logits=True):
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        lg = np.empty(self.model.shape.vocab, dtype=np.float64) if want_logits else None
        nxt = C.c_int32(-1)
        rc = lib().orc_prefill(self.h, seq, _ip(tok), tok.size, _dp(lg) if want_logits else None, C.byref(nxt))
        return rc, nxt.value, lg

    def decode(self, seq, want_logits=True):
        lg = np.empty(self.model.shape.vocab, dtype=np.float64) if want_logits else None
        nxt = C.c_int32(-1)
        rc = lib().orc_decode(self.h, seq, _dp(lg) if want_logits else None, C.byref(nxt))
        return rc, nxt.value, lg

    def stop(self, seq):
        return lib().orc_seq_stop(self.h, seq)

    def set_sampling(self, seq, temperature, seed):
        return lib().orc_seq_set_sampling(self.h, seq, temperature, seed)

    def fork(self, parent, n_tokens):
        s = C.c_int32(-1)
        rc = lib().orc_kv_fork(self.h, parent, n_tokens, C.byref(s))
        return rc, s.value

    def trim(self, seq):
        """-> (rc, blocks released): gives up the blocks below the attention band."""
        n = C.c_int32(0)
        rc = lib().orc_kv_trim(self.h, seq, C.byref(n))
        return rc, n.value

    def swap_out(self, seq):
        """-> (rc, store): the sequence's keys/values as a float64 array, its blocks back on the free list."""
        n = lib().orc_kv_swap_doubles(self.h, seq)
        if n < 0:
            return E_INVAL, None
        store = np.empty(max(n, 1), dtype=np.float64)
        rc = lib().orc_kv_swap_out(self.h, seq, _dp(store))
        return rc, store

    def swap_in(self, seq, store):
        return lib().orc_kv_swap_in(self.h, seq, _dp(np.ascontiguousarray(store, dtype=np.float64)))

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_kv_destroy(self.h); self.h = None
