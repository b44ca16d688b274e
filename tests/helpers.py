"""Shared set-up for the GPU parity tests: the same seeded weights handed to the oracle and to libld."""
import numpy as np
import torch

import oracle
import paper_2406_00059_amd as ld
from workloads import make_weights, gen
from workloads.configs import weights_to


def rel_err(got, ref):
    """Row-wise max-norm relative error: ||g - o||_inf / ||o||_inf."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


class Pair:
    """One decoder, twice: oracle (host) and libld (device), plus one paged cache on each side."""

    def __init__(self, shape, seed, n_blocks, max_tokens, max_seqs, max_blocks, max_chunk=256, kv_round=None,
                 gen_device="cpu"):
        self.shape = shape
        w = make_weights(shape, seed, device=gen_device)
        self.omodel = oracle.Model(shape, w, kv_round=kv_round)
        self.okv = oracle.KV(self.omodel, n_blocks, max_seqs, max_blocks)
        self.gmodel = ld.Model(shape, weights_to(w, "cuda"), max_chunk=max_chunk)
        self.gkv = ld.KV(self.gmodel, n_blocks, max_tokens, max_seqs, max_blocks)
        self.gkv.pool.fill_(float("nan"))       # a caller's pool is uninitialised memory: every slot not yet written is NaN
        self.V = shape.vocab

    def alloc(self, reserve=0):
        rc, so = self.okv.alloc(reserve)
        sg = ld.ld_kv_alloc(self.gkv.h, reserve)
        assert rc == 0 and so == sg
        return sg

    def tables_equal(self, s):
        return self.okv.block_table(s)[1].tolist() == ld.ld_kv_block_table(self.gkv.h, s).tolist()


def prompt(seed, stream, n, vocab):
    return gen.randint(seed, stream, 0, vocab - 1, n).numpy().astype(np.int32)


class Tokens:
    """Callback sink: records (seq, token, pos) in call order."""

    def __init__(self, stop_at=None):
        self.log, self.stop_at = [], stop_at

    def __call__(self, seq, tok, pos):
        self.log.append((seq, tok, pos))
        return self.stop_at is not None and len(self.log) >= self.stop_at

    def last(self, n=1):
        return [t for _, t, _ in self.log[-n:]]


def device_pool(logical):
    """KV blocks [..., K|V, kv_head, slot, hd] (the indexing the oracle uses) -> the memory image the
    library reads: the keys as they are, the values of a head transposed to [hd][slot].  Same shape
    and bytes; the last two dimensions of the value half then only size the memory."""
    out = logical.clone()
    v = logical[..., 1, :, :, :]
    out[..., 1, :, :, :] = v.transpose(-1, -2).reshape(v.shape)
    return out


def logical_pool(dev):
    """Inverse of device_pool: a pool the library wrote -> [..., K|V, kv_head, slot, hd]."""
    out = dev.clone()
    v = dev[..., 1, :, :, :]
    out[..., 1, :, :, :] = v.reshape(*v.shape[:-2], v.shape[-1], v.shape[-2]).transpose(-1, -2)
    return out
