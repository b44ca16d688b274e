"""Host-side tool-aware serving loop (paper sections 3.2-3.4) without a GPU: parser, plugin interface, tool
processes, scheduler in baseline and partial-execution mode over a stand-in engine, and the latency bounds of
Eq. (1) and Eq. (2)."""
import random
import time

import pytest

from oracle import latency_model as lm
from paper_2406_00059_amd import conveyor as cv
from fake_engine import FakeEngine


def test_latency_model_bounds_and_best_case_curve():
    rng = random.Random(3)
    for _ in range(200):
        n = rng.randint(1, 4)
        g = [rng.uniform(0.01, 2.0) for _ in range(n + 1)]
        t = [rng.uniform(0.0, 3.0) for _ in range(n)]
        s = [rng.uniform(0.0, gi) for gi in g[:-1]]
        assert lm.l_best(g, t) <= lm.l_new(g, t, s) + 1e-12 <= lm.l_old(g, t) + 1e-12      # Eq. (2)
        assert lm.l_new(g, t, [0.0] * n) == pytest.approx(lm.l_best(g, t))                 # started at once
        assert lm.l_new(g, t, g[:-1]) == pytest.approx(lm.l_old(g, t))                     # started at the end
    # one round, no trailing generation: the best-case improvement is r = t/g for r <= 1 and 1/r for r >= 1
    for r in (0.1, 0.5, 1.0, 2.0, 10.0):
        assert lm.best_improvement([1.0, 0.0], [r]) == pytest.approx(min(r, 1.0 / r))


def test_stream_parser_emits_pieces_at_their_delimiter():
    p = cv.StreamParser(lambda tok, i: tok == 0)
    out = [p.feed(t) for t in [5, 6, 0, 7, 0, 0, 8]]
    assert out == [[], [], [[5, 6]], [], [[7]], [[]], []]
    assert p.flush() == [[5, 6], [7], [], [8]]


def test_plugin_start_condition():
    t = cv.SyntheticTool(0.0, [1, 2], pieces_to_start=2)
    assert not t.can_start([[1]]) and t.can_start([[1], [2]])
    whole = cv.SyntheticTool(0.0, [1], pieces_to_start=None)
    assert not whole.can_start([[1], [2], [3]])


def test_tool_process_round_trip():
    tp = cv.ToolProcess(cv.SyntheticTool(0.05, [9, 8, 7]), [[1, 2]])
    assert tp.poll() is None
    obs, secs = tp.wait()
    assert obs == [9, 8, 7] and 0.04 <= secs < 0.5


def _requests(tool_s):
    obs = list(range(100, 140))
    return [cv.Request(prompt=list(range(10 + k, 42 + k)),
                       rounds=[cv.Round(40, cv.SyntheticTool(tool_s, obs, pieces_to_start=1)),
                               cv.Round(24, cv.SyntheticTool(tool_s / 2, obs[:16], pieces_to_start=2)),
                               cv.Round(16, None)]) for k in range(2)]


@pytest.mark.parametrize("tool_s", [0.03, 0.12])
def test_partial_execution_keeps_tokens_and_obeys_the_bounds(tool_s):
    base = cv.serve(FakeEngine(), _requests(tool_s), partial=False)
    part = cv.serve(FakeEngine(), _requests(tool_s), partial=True)
    # process start, pipe, polling granularity: forking is slow when the parent has large libraries mapped
    # (the whole suite in one process), so the start-up cost of a tool process is measured, not assumed
    t0 = time.perf_counter()
    cv.ToolProcess(cv.SyntheticTool(0.0, [1]), [[1]]).wait()
    slack = 0.06 + 2 * (time.perf_counter() - t0)
    for b, p in zip(base, part):
        assert b.tokens == p.tokens and len(p.tokens) == 80          # same LLM output in both modes
        assert len(p.g) == 3 and len(p.t) == 2 and len(p.s) == 2
        # baseline: tools start when their round ends; partial: after the first delimiter(s)
        assert all(abs(si - gi) < 0.02 for si, gi in zip(b.s, b.g))
        assert all(si < 0.8 * gi for si, gi in zip(p.s, p.g))       # 8 of 40 and 16 of 24 tokens in
        # measured latencies against the model evaluated on the measured g, t, s
        assert b.latency == pytest.approx(lm.l_old(b.g, b.t), abs=slack)
        assert p.latency == pytest.approx(lm.l_new(p.g, p.t, p.s), abs=slack)
        assert lm.l_best(p.g, p.t) - 1e-3 <= p.latency <= lm.l_old(p.g, p.t) + slack
    assert sum(p.latency for p in part) < sum(b.latency for b in base)


def test_retention_choice_thresholds():
    """choose_retention by wasted byte-seconds: keep for short waits, swap once the wait exceeds the copy
    out and the copy back, discard when recomputing is cheaper than both; closed-form crossing points."""
    kw = dict(kv_bytes_per_token=512 * 1024, swap_bytes_per_s=50e9, prefill_tokens_per_s=16000.0)
    ctx = 2048
    M = ctx * kw["kv_bytes_per_token"]
    t_copy = M / kw["swap_bytes_per_s"]                 # 21.5 ms one way
    t_recompute = ctx / kw["prefill_tokens_per_s"]      # 128 ms
    assert 2 * t_copy < t_recompute
    assert cv.choose_retention(ctx, 0.5 * t_copy, **kw) == "keep"          # the copy out does not even fit
    assert cv.choose_retention(ctx, 1.9 * t_copy, **kw) == "keep"          # cheaper to hold than to move twice
    assert cv.choose_retention(ctx, 2.0 * t_copy, **kw) == "keep"          # tie -> keep
    assert cv.choose_retention(ctx, 2.1 * t_copy, **kw) == "swap"
    assert cv.choose_retention(ctx, 100.0, **kw) == "swap"
    slow = dict(kw, swap_bytes_per_s=1e9)               # a slow link: recomputing beats swapping
    assert cv.choose_retention(ctx, 0.9 * t_recompute, **slow) == "keep"
    assert cv.choose_retention(ctx, 1.1 * t_recompute, **slow) == "discard"
    assert cv.choose_retention(ctx, 100.0, **slow) == "discard"


@pytest.mark.parametrize("retention", ["keep", "swap", "discard", "auto"])
def test_retention_modes_do_not_change_the_output(retention):
    """Baseline mode with a long tool (every round waits): whatever happens to the cache during the wait,
    the tokens are those of the run that keeps it; every wait records what was done."""
    ref = cv.serve(FakeEngine(), _requests(0.05), partial=False)
    eng = FakeEngine()
    kw = {}
    if retention == "auto":   # 50 ms tools against a 2 x 1 ms copy and a 100 ms recompute -> swap
        kw = dict(predict_tool_s=lambda plugin: plugin.duration_s,
                  rates=dict(kv_bytes_per_token=1e6, swap_bytes_per_s=50e9, prefill_tokens_per_s=500.0))
    got = cv.serve(eng, _requests(0.05), partial=False, retention=retention, **kw)
    for r, g in zip(ref, got):
        assert r.tokens == g.tokens
        assert g.retained == [("swap" if retention == "auto" else retention)] * 2
    assert not eng.swapped and not eng.hist            # everything swapped back in and freed


def test_shared_prompt_prefix_is_prefilled_once_and_changes_nothing():
    def reqs():
        head = list(range(500, 524))
        return [cv.Request(prompt=head + list(range(10 + k, 20 + k)),
                           rounds=[cv.Round(24, cv.SyntheticTool(0.02, [7, 8, 9], pieces_to_start=1)), cv.Round(8, None)])
                for k in range(3)]
    ref = cv.serve(FakeEngine(), reqs())
    eng = FakeEngine()
    got = cv.serve(eng, reqs(), shared_prefix=24)
    assert [r.tokens for r in ref] == [g.tokens for g in got] and not eng.hist
    with pytest.raises(AssertionError):
        cv.serve(FakeEngine(), reqs(), shared_prefix=30)        # the prompts differ from token 24 on


class _Stuck(cv.ToolPlugin):
    def run(self, pieces):
        time.sleep(60)
        return [1]


def test_a_tool_that_never_answers_is_killed_and_only_its_request_fails():
    """Two requests; the first one's tool hangs.  With a time-out the tool's process is killed, that request ends
    as failed with its sequence freed, and the other request completes with the tokens it has without the
    neighbour."""
    def reqs(stuck):
        tool = _Stuck() if stuck else cv.SyntheticTool(0.01, [4, 5, 6])
        return [cv.Request(prompt=[1, 2, 3], rounds=[cv.Round(6, tool), cv.Round(5)]),
                cv.Request(prompt=[7, 8], rounds=[cv.Round(7, cv.SyntheticTool(0.02, [9])), cv.Round(4)])]
    ref = cv.serve(FakeEngine(), reqs(False))
    eng = FakeEngine()
    t0 = time.perf_counter()
    got = cv.serve(eng, reqs(True), tool_timeout_s=0.3)
    assert time.perf_counter() - t0 < 5.0
    assert got[0].failed and "time-out" in got[0].failed and len(got[0].tokens) == 6
    assert got[1].failed is None and got[1].tokens == ref[1].tokens
    assert eng.hist == {}                                   # every sequence was freed, the failed one's too
