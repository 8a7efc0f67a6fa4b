"""TEST INFRASTRUCTURE ONLY -- oracle for the MA-GC checkpoint-interval planner.

The paper's App. C memory model (the four-term sum M = M_L-ckpt + M_S-ckpt + M_grid + M_state):
    M(l, s) = (L*S/l) * C_Lckpt + (L*S/s) * C_Sckpt + l*s * C_grid + s * C_state
with L layers, S tokens, l / s the checkpoint intervals along the layer / sequence axis.
With every constant 1 and C_state 0 it is the model of Sec. 3.3 (M = LS/l + LS/s + l s).

The planner is an exhaustive search over the admissible integer grid, written out:
    l in [1, L];  s in the multiples of `s_multiple` inside [s_multiple, S] when
    S >= s_multiple (Sec. 4: s is kept a multiple of 256 once S >= 256), else s in [1, S].
Reading taken where the paper is silent: ties go to the larger s, then the smaller l; with a
budget, among the plans that fit the one with least recomputation (largest s, then largest l)
is returned.  `integer_counts` switches L/l and S/s to ceil(L/l) and ceil(S/s) (the number
of checkpoints actually stored); the default is the paper's real-valued quotient.
"""
from __future__ import annotations

import math
from fractions import Fraction


def memory_terms(L, S, l, s, C_L, C_S, C_grid, C_state, integer_counts=False):
    """Exact rational values of the four terms (no floating point)."""
    if integer_counts:
        nl, ns = Fraction(math.ceil(Fraction(L, l))), Fraction(math.ceil(Fraction(S, s)))
    else:
        nl, ns = Fraction(L, l), Fraction(S, s)
    return (nl * S * C_L, L * ns * C_S, Fraction(l * s * C_grid), Fraction(s * C_state))


def candidates_s(S, s_multiple):
    if s_multiple > 1 and S >= s_multiple:
        return list(range(s_multiple, S + 1, s_multiple))
    return list(range(1, S + 1))


def plan(L, S, C_L, C_S, C_grid, C_state, s_multiple=256, budget=0, integer_counts=False):
    """Returns dict(l, s, terms=(M_L, M_S, M_grid, M_state), total, fits)."""
    best = None
    best_fit = None
    for l in range(1, L + 1):
        for s in candidates_s(S, s_multiple):
            t = memory_terms(L, S, l, s, C_L, C_S, C_grid, C_state, integer_counts)
            tot = sum(t)
            key = (tot, -s, l)
            if best is None or key < best[0]:
                best = (key, l, s, t, tot)
            if budget > 0 and tot <= budget:
                kf = (-s, -l)
                if best_fit is None or kf < best_fit[0]:
                    best_fit = (kf, l, s, t, tot)
    if budget > 0 and best_fit is not None:
        _, l, s, t, tot = best_fit
        return {"l": l, "s": s, "terms": t, "total": tot, "fits": True}
    _, l, s, t, tot = best
    return {"l": l, "s": s, "terms": t, "total": tot, "fits": budget <= 0}
