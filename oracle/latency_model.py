"""Closed-form latency model of tool partial execution (paper section 3.4).  TEST INFRASTRUCTURE ONLY.

g[i]: token-generation time of round i (prefill + decode), i = 0..n (the last entry is the final round, which
invokes no tool); t[i]: tool time of round i, i = 0..n-1; s[i]: time into round i at which the tool starts.
"""


def l_old(g, t):
    """No partial execution: every tool runs after its round, L_old = sum (g_i + t_i) + g_{n+1}."""
    assert len(g) == len(t) + 1
    return sum(g[:-1]) + sum(t) + g[-1]


def l_best(g, t):
    """Generation and tool fully overlapped: the lower bound of Eq. (2)."""
    assert len(g) == len(t) + 1
    return sum(max(gi, ti) for gi, ti in zip(g[:-1], t)) + g[-1]


def l_new(g, t, s):
    """A tool started s_i into its round finishes at s_i + t_i; the next round starts when both the
    round's generation and the tool are done: L_i = max(g_i, s_i + t_i)  (Eq. (1) with its two extremes
    s_i = 0 and s_i = g_i)."""
    assert len(g) == len(t) + 1 == len(s) + 1
    return sum(max(gi, si + ti) for gi, ti, si in zip(g[:-1], t, s)) + g[-1]


def best_improvement(g, t):
    """Relative latency improvement of the best case, L_old / L_best - 1."""
    return l_old(g, t) / l_best(g, t) - 1.0
