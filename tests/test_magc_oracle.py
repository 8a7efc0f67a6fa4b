"""Pins for the checkpoint-interval planner oracle (paper Sec. 3.3 and App. C)."""
import math
import os
from fractions import Fraction

import pytest

from oracle import magc_ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "memory_constants_table.txt")


def read_table():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, d, nl, cl, cs, cg, ct = line.split()
            rows[name] = dict(d_model=int(d), n_layers=int(nl), C_L=int(cl), C_S=int(cs), C_grid=int(cg), C_state=int(ct))
    return rows


def test_unweighted_model_critical_point():
    # Sec. 3.3: with all constants 1 the interior optimum is l = s = (LS)^(1/3), M* = 3 (LS)^(2/3).
    # L*S = 2^18 with L = S = 512 lies in the interior regime (L <= S^2 and S <= L^2): l = s = 64.
    p = magc_ref.plan(512, 512, 1, 1, 1, 0, s_multiple=1)
    assert (p["l"], p["s"]) == (64, 64)
    assert p["total"] == 3 * 64 * 64 == 3 * round((512 * 512) ** (2 / 3))


def test_unweighted_model_layer_boundary_branch():
    # Sec. 3.3, regime L^2 <= S: optimum sits on l = L, where M = S + L (S/s + s) >= S + 2 L sqrt(S),
    # with equality at s = sqrt(S).
    L, S = 4, 1024
    p = magc_ref.plan(L, S, 1, 1, 1, 0, s_multiple=1)
    assert (p["l"], p["s"]) == (L, 32)
    assert p["total"] == S + 2 * L * 32


def test_unweighted_model_sequence_boundary_branch():
    # regime S^2 <= L: optimum on s = S with l = sqrt(L), M = L + 2 S sqrt(L)
    L, S = 1024, 4
    p = magc_ref.plan(L, S, 1, 1, 1, 0, s_multiple=1)
    assert (p["l"], p["s"]) == (32, S)
    assert p["total"] == L + 2 * S * 32


@pytest.mark.parametrize("L,S", [(8, 8), (3, 100), (100, 3), (16, 64), (7, 49)])
def test_unweighted_optimum_respects_regime_bounds(L, S):
    p = magc_ref.plan(L, S, 1, 1, 1, 0, s_multiple=1)
    m = float(p["total"])
    # the integer optimum can never beat the continuous bounds of each regime
    if L * L <= S:
        assert m >= S + 2 * L * math.sqrt(S) - 1e-9 or p["l"] < L
    if S * S <= L:
        assert m >= L + 2 * S * math.sqrt(L) - 1e-9 or p["s"] < S
    assert m >= 3 * (L * S) ** (2 / 3) - 1e-9 or p["l"] == L or p["s"] == S
    # and it is a true minimum of the four-term sum over the grid
    for l in range(1, L + 1):
        for s in range(1, S + 1):
            assert Fraction(L * S, l) + Fraction(L * S, s) + l * s >= p["total"]


def test_constants_table_decodes_to_mamba2_shapes():
    # The printed constants are consistent with a Mamba-2 block of d_inner = 2 d_model, heads of 64
    # channels, 128 states, one B/C group and a width-4 convolution; this pins H, P, N of the layer
    # shapes used by the synthetic configs (2.7b: H = 80, P = 64, N = 128).
    for name, r in read_table().items():
        d_inner = 2 * r["d_model"]
        H, P, N, G = d_inner // 64, 64, 128, 1
        conv_dim = d_inner + 2 * G * N
        assert r["C_L"] == r["d_model"]
        assert r["C_S"] == H * P * N + 3 * conv_dim, name
        assert r["C_state"] == H * P * N + conv_dim, name
        assert r["C_grid"] == (2 * d_inner + 2 * G * N + H) + d_inner, name
    assert 2 * read_table()["Mamba-2-2.7b"]["d_model"] // 64 == 80


def test_weighted_model_rule_of_256_and_first_order_conditions():
    r = read_table()["Mamba-2-2.7b"]
    L = r["n_layers"]
    for n in (14, 16, 19):
        S = 2 ** n
        p = magc_ref.plan(L, S, r["C_L"], r["C_S"], r["C_grid"], r["C_state"], s_multiple=256)
        assert p["s"] % 256 == 0 and 1 <= p["l"] <= L
        # near the real-valued stationary point: dM/dl = 0 -> l = sqrt(L S C_L / (s C_grid));
        # dM/ds = 0 -> s = sqrt(L S C_S / (l C_grid + C_state))
        l_star = math.sqrt(L * S * r["C_L"] / (p["s"] * r["C_grid"]))
        s_star = math.sqrt(L * S * r["C_S"] / (p["l"] * r["C_grid"] + r["C_state"]))
        assert abs(p["l"] - l_star) <= 1.0 or p["l"] == L
        assert abs(p["s"] - s_star) <= 256
    # short sequences: s is unconstrained below 256 tokens
    p = magc_ref.plan(4, 100, 1, 1, 1, 0, s_multiple=256)
    assert p["s"] == 10 and p["l"] == 4


def test_budget_mode_prefers_least_recompute():
    L, S = 8, 4096
    free = magc_ref.plan(L, S, 10, 1000, 10, 5, s_multiple=256)
    big = magc_ref.plan(L, S, 10, 1000, 10, 5, s_multiple=256, budget=10 ** 12)
    assert big["fits"] and (big["l"], big["s"]) == (L, S)
    tight = magc_ref.plan(L, S, 10, 1000, 10, 5, s_multiple=256, budget=int(free["total"]) - 1)
    assert not tight["fits"] and (tight["l"], tight["s"]) == (free["l"], free["s"])
    mid = magc_ref.plan(L, S, 10, 1000, 10, 5, s_multiple=256, budget=int(free["total"] * 1.2))
    assert mid["fits"] and mid["total"] <= free["total"] * 1.2 and mid["s"] >= free["s"]


def test_integer_counts_variant():
    t = magc_ref.memory_terms(10, 1000, 3, 256, 1, 1, 1, 1, integer_counts=True)
    assert t[0] == 4 * 1000 and t[1] == 10 * 4
    t = magc_ref.memory_terms(10, 1000, 3, 256, 1, 1, 1, 1)
    assert t[0] == Fraction(10000, 3) and t[1] == Fraction(10000, 256)
