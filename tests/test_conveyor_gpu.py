"""The tool-aware serving loop over the real engine on the GPU: tokens equal the oracle's for the same
sequence of prefills and decodes, equal between baseline and partial execution (same LLM output in both
modes, section 4.1), and the measured latencies obey Eq. (2)."""
import time

import numpy as np
import pytest

import oracle
import paper_2406_00059_amd as ld
from oracle import latency_model as lm
from paper_2406_00059_amd import conveyor as cv
from workloads import TINY
from helpers import Pair, prompt

pytestmark = pytest.mark.gpu


def _requests(tool_s):
    obs = prompt(31, 9, 48, TINY.vocab).tolist()
    return [cv.Request(prompt=prompt(31, k, 40, TINY.vocab).tolist(),
                       rounds=[cv.Round(48, cv.SyntheticTool(tool_s, obs, pieces_to_start=1)),
                               cv.Round(32, cv.SyntheticTool(tool_s, obs[:20], pieces_to_start=2)),
                               cv.Round(16, None)]) for k in range(3)]


def test_rounds_with_tools_match_oracle_and_bounds():
    P = Pair(TINY, 31, n_blocks=64, max_tokens=64, max_seqs=3, max_blocks=16)
    runs = {}
    for partial in (False, True):
        reqs = cv.serve(cv.LdEngine(ld, P.gkv.h), _requests(0.03), partial=partial)
        runs[partial] = reqs
    t0 = time.perf_counter()                      # start-up cost of a tool process from this (large) parent
    cv.ToolProcess(cv.SyntheticTool(0.0, [1]), [[1]]).wait()
    slack = 0.08 + 2 * (time.perf_counter() - t0)
    for b, p in zip(runs[False], runs[True]):
        assert b.tokens == p.tokens and len(p.tokens) == 96
        assert lm.l_best(p.g, p.t) - 1e-3 <= p.latency <= lm.l_old(p.g, p.t) + slack
        assert p.latency == pytest.approx(lm.l_new(p.g, p.t, p.s), abs=slack)
    assert sum(p.latency for p in runs[True]) < sum(b.latency for b in runs[False])
    # the same call sequence through the oracle, one request at a time
    for k, r in enumerate(runs[True]):
        rc, s = P.okv.alloc(0)
        ref, feed = [], r.prompt
        for rd in r.rounds:
            rc, t, _ = P.okv.prefill(s, np.array(feed, np.int32), want_logits=False); ref.append(t)
            for _ in range(rd.n_tokens - 1):
                rc, t, _ = P.okv.decode(s, want_logits=False); ref.append(t)
            feed = rd.tool.observation if rd.tool else None
        assert ref == r.tokens, k
        P.okv.free(s)


def test_swapping_the_cache_during_tool_waits_changes_nothing():
    """Baseline mode (every round waits for its tool) with the cache swapped to host memory during each
    wait: the tokens are those of the
    run that keeps the cache resident, every wait was a swap, and all blocks are free at the end."""
    P = Pair(TINY, 31, n_blocks=64, max_tokens=64, max_seqs=3, max_blocks=16)
    keep = cv.serve(cv.LdEngine(ld, P.gkv.h), _requests(0.03), partial=False)
    swap = cv.serve(cv.LdEngine(ld, P.gkv.h), _requests(0.03), partial=False, retention="swap")
    for a, b in zip(keep, swap):
        assert a.tokens == b.tokens and b.retained == ["swap", "swap"] and a.retained == ["keep", "keep"]
    assert ld.ld_kv_free_blocks(P.gkv.h) == 64


def test_shared_prompt_prefix_on_the_engine():
    """Three requests whose prompts share their first 24 tokens: the prefix is prefilled once and forked;
    the tokens equal those of the oracle replaying the same calls (fork included), and all blocks are free
    afterwards."""
    P = Pair(TINY, 31, n_blocks=64, max_tokens=64, max_seqs=4, max_blocks=16)
    head = prompt(31, 50, 24, TINY.vocab).tolist()
    obs = prompt(31, 51, 20, TINY.vocab).tolist()
    reqs = [cv.Request(prompt=head + prompt(31, 60 + k, 10 + k, TINY.vocab).tolist(),
                       rounds=[cv.Round(24, cv.SyntheticTool(0.01, obs, pieces_to_start=1)), cv.Round(8, None)])
            for k in range(3)]
    cv.serve(cv.LdEngine(ld, P.gkv.h), reqs, shared_prefix=24)
    assert ld.ld_kv_free_blocks(P.gkv.h) == 64
    rc, tmpl = P.okv.alloc(0)
    P.okv.prefill(tmpl, np.array(head, np.int32), want_logits=False)
    for r in reqs:
        rc, s = P.okv.fork(tmpl, 24)
        ref, feed = [], r.prompt[24:]
        for rd in r.rounds:
            rc, t, _ = P.okv.prefill(s, np.array(feed, np.int32), want_logits=False); ref.append(t)
            for _ in range(rd.n_tokens - 1):
                rc, t, _ = P.okv.decode(s, want_logits=False); ref.append(t)
            feed = rd.tool.observation if rd.tool else None
        assert ref == r.tokens
        P.okv.free(s)


def test_trimming_below_the_attention_band_changes_nothing():
    """A banded model served with and without sliding-window memory: the same tokens, and with trimming the
    pool's low-water mark of free blocks is higher (the sequences hold only their bands)."""
    from dataclasses import replace
    shape = replace(TINY, window=24, name="tiny-band")
    P = Pair(shape, 32, n_blocks=64, max_tokens=64, max_seqs=3, max_blocks=16)

    class Watch(cv.LdEngine):
        low = 10 ** 9
        def decode(self, seqs):
            self.low = min(self.low, ld.ld_kv_free_blocks(self.kv))
            return super().decode(seqs)

    plain, trimmed = Watch(ld, P.gkv.h), Watch(ld, P.gkv.h)
    a = cv.serve(plain, _requests(0.0), partial=False)
    b = cv.serve(trimmed, _requests(0.0), partial=False, trim=True)
    assert [r.tokens for r in a] == [r.tokens for r in b] and all(len(r.tokens) == 96 for r in b)
    assert trimmed.low > plain.low and ld.ld_kv_free_blocks(P.gkv.h) == 64
