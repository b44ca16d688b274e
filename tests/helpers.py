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
                 gen_device="cpu", models=None):
        self.shape = shape
        if models is None:          # models: (oracle.Model, ld.Model) built once by the caller and shared by several pairs
            w = make_weights(shape, seed, device=gen_device)
            models = (oracle.Model(shape, w, kv_round=kv_round), ld.Model(shape, weights_to(w, "cuda"), max_chunk=max_chunk))
        self.omodel, self.gmodel = models
        self.okv = oracle.KV(self.omodel, n_blocks, max_seqs, max_blocks)
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


class NearTies:
    """The rule for a token that differs from the oracle's.

    If the library's logits are within E of the oracle's in every element, the token it picks (greedy: the
    maximum of its own logits) can differ from the oracle's only when the oracle's own scores of the two
    candidates are closer than 2 E: score_o[t_o] - score_o[t_g] <= 2 E.  With a temperature T the scores are
    logits / T + noise, the same noise on both sides up to its float32 evaluation (|g| <= 16.7, a few units
    in the last place: 5e-6), so the bound becomes 2 (E / T + 5e-6).  E is the measured maximum absolute
    logits error of the row in question (for rows whose logits the call does not return, the largest error
    measured so far in the same test).  A mismatch inside the bound is a near-tie: it is logged and the
    caller re-synchronises; one outside fails."""

    C, NOISE = 2.0, 5e-6

    def __init__(self):
        self.cases, self.max_abs = [], 0.0

    def measured(self, lg, lg_o):
        e = float(np.max(np.abs(np.asarray(lg, np.float64) - lg_o)))
        self.max_abs = max(self.max_abs, e)
        return e

    def check(self, where, lg_o, t_o, t_g, err_abs=None, temperature=0.0, seed=0, pos=0):
        scores = np.asarray(lg_o, np.float64) if temperature == 0 else oracle.gumbel_scores(lg_o, temperature, seed, pos)
        assert int(np.argmax(scores)) == t_o
        e = self.max_abs if err_abs is None else err_abs
        gap = float(scores[t_o] - scores[t_g])
        bound = self.C * (e / (temperature or 1.0) + (self.NOISE if temperature else 0.0))
        case = dict(where=where, oracle_token=int(t_o), library_token=int(t_g), gap=gap, bound=bound,
                    gap_rel=gap / float(np.abs(lg_o).max()), temperature=temperature,
                    row_error="measured" if err_abs is not None else "largest so far")
        self.cases.append(case)
        print("near-tie:", case)
        assert 0.0 <= gap <= bound, f"token mismatch beyond a near-tie: {case}"
        return case
