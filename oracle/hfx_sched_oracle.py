"""Oracle for the step-composition closed forms (HFX Section 3.3.1).

TEST INFRASTRUCTURE ONLY (imported by tests/ alone).  Shares no code with the library.

Nothing here uses the simplified bound of Eq. (3).  The token budget is found from the
definitions the paper gives before simplifying them: E_p = a + b*n, the slack of one decode
iteration TPOT - E_d, k = E_p / slack iterations until maturity, maturity = E_p + k*E_d, and the
worst-case condition maturity + E_p <= TTFT.  All arithmetic is exact (fractions.Fraction built
from the binary doubles), so "largest n that satisfies the condition" has one answer.
"""
from __future__ import annotations

from fractions import Fraction


def _f(x) -> Fraction:
    return Fraction(x)


def e_p(a, b, n) -> Fraction:
    """Linear prefill-latency model adopted in Section 3.3.1."""
    return _f(a) + _f(b) * n


def maturity(ep, tpot, e_d):
    """(k, maturity time): k decode iterations each save TPOT - E_d; together they must save E_p."""
    slack = _f(tpot) - _f(e_d)
    assert slack > 0
    k = _f(ep) / slack
    return k, _f(ep) + k * _f(e_d)


def admissible(n, ttft, tpot, a, b, e_d) -> bool:
    """Worst case of Section 3.3.1: a request arriving right after the dispatch waits for the
    maturity time and then for a prefill batch of its own."""
    if _f(tpot) - _f(e_d) <= 0:
        return False
    ep = e_p(a, b, n)
    _, m = maturity(ep, tpot, e_d)
    return m + ep <= _f(ttft)


def token_budget(ttft, tpot, a, b, e_d, hi=1 << 62) -> int:
    """Largest integer n >= 0 with admissible(n); 0 if none.  Bisection on the definition
    (the condition is monotone in n because b > 0)."""
    if not admissible(0, ttft, tpot, a, b, e_d):
        return 0
    lo = 0
    if admissible(hi, ttft, tpot, a, b, e_d):
        return hi
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if admissible(mid, ttft, tpot, a, b, e_d):
            lo = mid
        else:
            hi = mid
    return lo


def compose(ttft, tpot, a, b, e_d, running_ctx, prompt_len, urgency=None, mixed=False):
    """The four dispatching steps for a single instance; returns (admitted, kind, q_len, ctx_len,
    budget, n_token)."""
    budget = token_budget(ttft, tpot, a, b, e_d)
    order = list(range(len(prompt_len)))
    if urgency is not None:
        order.sort(key=lambda i: urgency[i])      # Python's sort is stable: ties keep queue order
    left, admitted, chosen = budget, [0] * len(prompt_len), []
    for i in order:
        if prompt_len[i] <= left:
            admitted[i] = 1
            chosen.append(i)
            left -= prompt_len[i]
    kind, q_len, ctx_len = [], [], []
    if mixed or not chosen:
        for c in running_ctx:
            kind.append(0); q_len.append(1); ctx_len.append(c + 1)
    for i in chosen:
        kind.append(1); q_len.append(prompt_len[i]); ctx_len.append(prompt_len[i])
    return admitted, kind, q_len, ctx_len, budget, budget - left
