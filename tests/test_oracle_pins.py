"""Pins for the fp64 oracle: every check here compares it with something that is not itself --
a different formula (the quadratic dual form), closed forms, algebraic identities, finite
differences -- chosen so that a dropped term, a wrong sign or index, or a transposed operand
anywhere in oracle/ssd_oracle.c fails at least one of them.  (Paper Sec. 3.1, Eq. 1.)"""
import numpy as np
import pytest

from oracle import ssd_ref


def draw(seed, Bt=2, L=12, H=4, P=3, G=2, N=5, states=True, dt_lo=0.05, dt_hi=0.6):
    r = np.random.default_rng(seed)
    d = dict(
        x=r.standard_normal((Bt, L, H, P)), dt=r.uniform(dt_lo, dt_hi, (Bt, L, H)),
        A=-np.exp(r.uniform(0, np.log(4.0), H)), B=r.standard_normal((Bt, L, G, N)),
        C=r.standard_normal((Bt, L, G, N)), D=r.standard_normal(H),
        dy=r.standard_normal((Bt, L, H, P)))
    if states:
        d["init_state"] = r.standard_normal((Bt, H, P, N))
        d["dfinal_state"] = r.standard_normal((Bt, H, P, N))
    else:
        d["init_state"] = None
        d["dfinal_state"] = None
    return d


def fwd(d, **kw):
    return ssd_ref.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["init_state"], **kw)


def bwd(d, **kw):
    return ssd_ref.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], d["init_state"],
                           d["dfinal_state"], **kw)


def dual_form(d):
    """y and final state from the O(L^2) 'attention-like' expansion of the recurrence:
    y_t = sum_{s<=t} (C_t.B_s) exp(sum_{r=s+1..t} a_r) dt_s x_s + D x_t + exp(sum_{r<=t} a_r) C_t h_init."""
    x, dt, A, Bm, Cm, D = d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"]
    Bt, L, H, P = x.shape
    G, N = Bm.shape[2:]
    y = np.zeros_like(x)
    fin = np.zeros((Bt, H, P, N))
    for b in range(Bt):
        for h in range(H):
            g = h // (H // G)
            a = dt[b, :, h] * A[h]
            h0 = np.zeros((P, N)) if d["init_state"] is None else d["init_state"][b, h]
            for t in range(L):
                acc = D[h] * x[b, t, h] + np.exp(a[: t + 1].sum()) * (h0 @ Cm[b, t, g])
                for s in range(t + 1):
                    acc = acc + (Cm[b, t, g] @ Bm[b, s, g]) * np.exp(a[s + 1: t + 1].sum()) * dt[b, s, h] * x[b, s, h]
                y[b, t, h] = acc
            f = np.exp(a.sum()) * h0
            for s in range(L):
                f = f + np.exp(a[s + 1:].sum()) * dt[b, s, h] * np.outer(x[b, s, h], Bm[b, s, g])
            fin[b, h] = f
    return y, fin


def close(a, b, tol=1e-12):
    scale = max(1.0, float(np.max(np.abs(b))))
    assert float(np.max(np.abs(a - b))) <= tol * scale, float(np.max(np.abs(a - b)))


@pytest.mark.parametrize("seed,states", [(0, True), (1, False)])
def test_forward_matches_quadratic_dual_form(seed, states):
    d = draw(seed, states=states)
    r = fwd(d)
    y, fin = dual_form(d)
    close(r["y"], y)
    close(r["final_state"], fin)


def test_zero_A_is_a_prefix_sum():
    d = draw(2)
    d["A"] = np.zeros_like(d["A"])
    r = fwd(d)
    Bt, L, H, P = d["x"].shape
    G = d["B"].shape[2]
    for b in range(Bt):
        for h in range(H):
            g = h // (H // G)
            X = d["x"][b, :, h]                                  # [L, P]
            S = np.tril(d["C"][b, :, g] @ d["B"][b, :, g].T)     # causal scores
            Y = S @ (d["dt"][b, :, h, None] * X) + d["D"][h] * X + d["C"][b, :, g] @ d["init_state"][b, h].T
            close(r["y"][b, :, h], Y)
            fin = d["init_state"][b, h] + np.einsum("t,tp,tn->pn", d["dt"][b, :, h], X, d["B"][b, :, g])
            close(r["final_state"][b, h], fin)


def test_single_token_closed_form():
    d = draw(3, L=1)
    r = fwd(d)
    g = bwd(d)
    Bt, _, H, P = d["x"].shape
    G = d["B"].shape[2]
    for b in range(Bt):
        for h in range(H):
            gi = h // (H // G)
            x, dt, A, Bv, Cv, D = d["x"][b, 0, h], d["dt"][b, 0, h], d["A"][h], d["B"][b, 0, gi], d["C"][b, 0, gi], d["D"][h]
            h0, dy, dfin = d["init_state"][b, h], d["dy"][b, 0, h], d["dfinal_state"][b, h]
            al = np.exp(dt * A)
            close(r["y"][b, 0, h], (Cv @ Bv) * dt * x + D * x + al * (h0 @ Cv))
            close(r["final_state"][b, h], al * h0 + dt * np.outer(x, Bv))
            lam = dfin + np.outer(dy, Cv)
            close(g["dx"][b, 0, h], dt * (lam @ Bv) + D * dy)
            close(g["ddt"][b, 0, h], A * al * np.sum(lam * h0) + x @ lam @ Bv)
            close(g["dinit_state"][b, h], al * lam)


def test_geometric_series_pins_the_decay():
    # constant dt, B = C = 1, x = 1, zero initial state: y_t[p] = N dt (1 - alpha^{t+1}) / (1 - alpha) + D
    Bt, L, H, P, G, N = 1, 40, 2, 2, 1, 3
    dt0, A = 0.3, np.array([-0.7, -2.0])
    d = dict(x=np.ones((Bt, L, H, P)), dt=np.full((Bt, L, H), dt0), A=A, B=np.ones((Bt, L, G, N)),
             C=np.ones((Bt, L, G, N)), D=np.array([0.25, -1.5]), init_state=None)
    r = fwd(d)
    t = np.arange(L)
    for h in range(H):
        al = np.exp(dt0 * A[h])
        want = N * dt0 * (1 - al ** (t + 1)) / (1 - al) + d["D"][h]
        close(r["y"][0, :, h, 0], want)
        close(r["y"][0, :, h, 1], want)
        close(r["final_state"][0, h], np.full((P, N), dt0 * (1 - al ** L) / (1 - al)))


def test_linearity_in_x_B_C():
    d = draw(4, states=False)
    e = draw(5, states=False)
    for key in ("x", "B", "C"):
        d1, d2, d3 = dict(d), dict(d), dict(d)
        d2[key] = e[key]
        d3[key] = 2.0 * d[key] - 3.0 * e[key]
        if key != "x":  # the D*x skip is linear in x only
            for q in (d1, d2, d3):
                q["D"] = np.zeros_like(d["D"])
        close(fwd(d3)["y"], 2.0 * fwd(d1)["y"] - 3.0 * fwd(d2)["y"])


def test_time_concatenation_and_boundary_states():
    d = draw(6, L=24)
    full = fwd(d, segment=8)
    assert full["boundary_states"].shape == (2, 3, 4, 3, 5)
    close(full["boundary_states"][:, 0], d["init_state"])
    state = d["init_state"]
    ys = []
    for k in range(3):
        sl = slice(8 * k, 8 * k + 8)
        close(full["boundary_states"][:, k], state)
        part = ssd_ref.ssd_fwd(d["x"][:, sl], d["dt"][:, sl], d["A"], d["B"][:, sl], d["C"][:, sl], d["D"], state)
        ys.append(part["y"])
        state = part["final_state"]
    close(np.concatenate(ys, axis=1), full["y"])
    close(state, full["final_state"])


def test_groups_and_head_group_map():
    d = draw(7, H=6, G=3)
    r1 = fwd(d)
    r2 = fwd(d, head_group=[0, 0, 1, 1, 2, 2])
    close(r1["y"], r2["y"], 0.0)
    # a head subset with an explicit map equals the same heads of the full run
    hs = [1, 4, 5]
    sub = ssd_ref.ssd_fwd(d["x"][:, :, hs], d["dt"][:, :, hs], d["A"][hs], d["B"], d["C"], d["D"][hs],
                          d["init_state"][:, hs], head_group=[0, 2, 2])
    close(sub["y"], r1["y"][:, :, hs], 0.0)


def loss(d):
    r = fwd(d)
    out = float(np.sum(d["dy"] * r["y"]))
    if d["dfinal_state"] is not None:
        out += float(np.sum(d["dfinal_state"] * r["final_state"]))
    return out


GRAD_OF = {"x": "dx", "dt": "ddt", "A": "dA", "B": "dB", "C": "dC", "D": "dD", "init_state": "dinit_state"}


@pytest.mark.parametrize("seed", [10, 11])
def test_gradients_by_central_finite_differences(seed):
    d = draw(seed)
    g = bwd(d, ckpt_every=5)      # 12 tokens, blocks of 5: exercises the ragged last block
    rng = np.random.default_rng(seed + 100)
    for key, gk in GRAD_OF.items():
        # directional derivative along a random direction
        v = rng.standard_normal(d[key].shape)
        eps = 1e-6
        dp, dm = dict(d), dict(d)
        dp[key] = d[key] + eps * v
        dm[key] = d[key] - eps * v
        fd = (loss(dp) - loss(dm)) / (2 * eps)
        an = float(np.sum(g[gk] * v))
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (key, fd, an)
        # and a few single entries, so that a permuted gradient is caught too
        flat = d[key].reshape(-1)
        for idx in rng.choice(flat.size, size=min(4, flat.size), replace=False):
            dp, dm = dict(d), dict(d)
            e = np.zeros(flat.size)
            e[idx] = eps
            dp[key] = d[key] + e.reshape(d[key].shape)
            dm[key] = d[key] - e.reshape(d[key].shape)
            fd = (loss(dp) - loss(dm)) / (2 * eps)
            an = float(g[gk].reshape(-1)[idx])
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (key, idx, fd, an)


def test_adjoint_identities():
    # y is linear in x (with D), in B, in C and in the initial state when the others are fixed:
    # <dy, y(v)> + <dfinal, final(v)> = <grad_v, v> exactly (no step size involved).
    d = draw(12)
    g = bwd(d)
    base = dict(d)
    zero_x = dict(d, x=np.zeros_like(d["x"]))
    zero_h = dict(d, init_state=np.zeros_like(d["init_state"]))
    # in (x, init) jointly linear: loss(x, h0) = <dx, x> + <dinit, h0>
    lhs = loss(base)
    rhs = float(np.sum(g["dx"] * d["x"]) + np.sum(g["dinit_state"] * d["init_state"]))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    # linear in B once the initial state is zero and D = 0
    q = dict(zero_h, D=np.zeros_like(d["D"]))
    gq = bwd(q)
    assert abs(loss(q) - float(np.sum(gq["dB"] * q["B"]))) <= 1e-12 * max(1.0, abs(loss(q)))
    # linear in C once D = 0 and dfinal = 0
    q = dict(d, D=np.zeros_like(d["D"]), dfinal_state=None)
    gq = bwd(q)
    assert abs(loss(q) - float(np.sum(gq["dC"] * q["C"]))) <= 1e-12 * max(1.0, abs(loss(q)))
    # with x = 0 only the initial state feeds the outputs
    gq = bwd(zero_x)
    assert abs(loss(zero_x) - float(np.sum(gq["dinit_state"] * d["init_state"]))) <= 1e-12 * max(1.0, abs(loss(zero_x)))
    # dD is the plain inner product of dy and x
    close(g["dD"], np.einsum("blhp,blhp->h", d["dy"], d["x"]))


def test_decay_gradient_identity():
    # From lambda_t - alpha_{t+1} lambda_{t+1} = dy_t (x) C_t one gets, with yhat = y - D x and
    # dxhat = dx - D dy:  da_t = sum_{t' >= t} [dy_t'.yhat_t' - x_t'.dxhat_t'] + <dfinal, h_final>,
    # then ddt_t = A da_t + x_t.dxhat_t / dt_t and dA = sum_t dt_t da_t.
    d = draw(13)
    r, g = fwd(d), bwd(d)
    D = d["D"][None, None, :, None]
    yhat = r["y"] - D * d["x"]
    dxhat = g["dx"] - D * d["dy"]
    term = np.sum(d["dy"] * yhat - d["x"] * dxhat, axis=-1)              # [Bt, L, H]
    tail = np.einsum("bhpn,bhpn->bh", d["dfinal_state"], r["final_state"])
    da = np.flip(np.cumsum(np.flip(term, 1), 1), 1) + tail[:, None, :]
    ddt = d["A"][None, None] * da + np.sum(d["x"] * dxhat, -1) / d["dt"]
    close(g["ddt"], ddt, 1e-11)
    close(g["dA"], np.einsum("blh,blh->h", d["dt"], da), 1e-11)


def test_backward_is_independent_of_recompute_block():
    d = draw(14, L=20)
    g1, g2, g3 = bwd(d, ckpt_every=1), bwd(d, ckpt_every=7), bwd(d, ckpt_every=64)
    for k in g1:
        close(g1[k], g2[k], 1e-14)
        close(g1[k], g3[k], 1e-14)


def test_segmented_backward_equals_full_backward():
    # The Markov property behind the sequence-axis checkpoints (paper Sec. 3.2): restarting a
    # segment from its stored entering state, and handing the state adjoint to the segment on its
    # left, reproduces the gradients of the unsegmented run.
    d = draw(15, L=24)
    full = bwd(d)
    f = fwd(d, segment=8)
    carry = d["dfinal_state"]
    acc = {k: np.zeros_like(v) for k, v in full.items() if k in ("dA", "dD")}
    parts = {"dx": [], "ddt": [], "dB": [], "dC": []}
    for k in (2, 1, 0):
        sl = slice(8 * k, 8 * k + 8)
        gk = ssd_ref.ssd_bwd(d["x"][:, sl], d["dt"][:, sl], d["A"], d["B"][:, sl], d["C"][:, sl], d["D"],
                             d["dy"][:, sl], f["boundary_states"][:, k], carry)
        carry = gk["dinit_state"]
        for n in parts:
            parts[n].insert(0, gk[n])
        acc["dA"] += gk["dA"]
        acc["dD"] += gk["dD"]
    for n in parts:
        close(np.concatenate(parts[n], axis=1), full[n])
    close(acc["dA"], full["dA"])
    close(acc["dD"], full["dD"])
    close(carry, full["dinit_state"])


def test_stack_gradients_and_cell_order():
    # two residual layers: finite differences through the stack, and the segment-major cell
    # order (paper Alg. 1: sequence outer, layers inner) equals the layer-major order.
    rng = np.random.default_rng(21)
    Bt, L, H, P, G, N = 1, 12, 2, 3, 1, 4
    layers = []
    for j in range(3):
        d = draw(30 + j, Bt=Bt, L=L, H=H, P=P, G=G, N=N, states=False)
        layers.append({k: d[k] for k in ("dt", "A", "B", "C", "D")})
    x0 = rng.standard_normal((Bt, L, H, P))
    dout = rng.standard_normal((Bt, L, H, P))
    f = ssd_ref.stack_fwd(x0, layers, segment=4)
    b = ssd_ref.stack_bwd(f["xs"], layers, dout)

    def stack_loss(x_in, lays):
        return float(np.sum(dout * ssd_ref.stack_fwd(x_in, lays)["out"]))

    v = rng.standard_normal(x0.shape)
    eps = 1e-6
    fd = (stack_loss(x0 + eps * v, layers) - stack_loss(x0 - eps * v, layers)) / (2 * eps)
    assert abs(fd - float(np.sum(b["dx0"] * v))) <= 1e-6 * max(1.0, abs(fd))
    for j in range(3):
        for key, gk in (("dt", "ddt"), ("A", "dA"), ("B", "dB"), ("C", "dC"), ("D", "dD")):
            v = rng.standard_normal(layers[j][key].shape)
            lp = [dict(q) for q in layers]
            lm = [dict(q) for q in layers]
            lp[j][key] = layers[j][key] + eps * v
            lm[j][key] = layers[j][key] - eps * v
            fd = (stack_loss(x0, lp) - stack_loss(x0, lm)) / (2 * eps)
            an = float(np.sum(b["grads"][j][gk] * v))
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (j, key, fd, an)
    # segment-major order: for each segment run all layers, carrying per-layer states
    states = [np.zeros((Bt, H, P, N)) for _ in layers]
    outs = []
    for k in range(3):
        sl = slice(4 * k, 4 * k + 4)
        x = x0[:, sl]
        for j, lay in enumerate(layers):
            close(f["boundary_states"][j][:, k], states[j])
            r = ssd_ref.ssd_fwd(x, lay["dt"][:, sl], lay["A"], lay["B"][:, sl], lay["C"][:, sl], lay["D"], states[j])
            states[j] = r["final_state"]
            x = x + r["y"]
        outs.append(x)
    close(np.concatenate(outs, axis=1), f["out"])
    # heads never mix (dt, B, C are inputs, not projections of x): a head subset stands alone
    sub_layers = [dict(q, dt=q["dt"][:, :, [1]], A=q["A"][[1]], D=q["D"][[1]]) for q in layers]
    fs = ssd_ref.stack_fwd(x0[:, :, [1]], sub_layers, head_group=[0])
    close(fs["out"], f["out"][:, :, [1]], 0.0)


def test_packed_sequences_equal_separate_runs():
    """reset[b, t] = 1 starts a new sequence at token t: the packed run must give, piece by piece, what
    separate runs of the pieces give (each from a zero state; the first piece from init_state), in the
    forward pass and in every gradient.  The pieces are checked with the plain (unpacked) entry points."""
    d = draw(21, Bt=2, L=14, H=4, P=3, G=2, N=5)
    cuts = [[0, 5, 6, 14], [0, 9, 14]]        # piece boundaries per batch row (a one-token piece included)
    reset = np.zeros((2, 14), dtype=np.uint8)
    for b, cs in enumerate(cuts):
        for c in cs[1:-1]:
            reset[b, c] = 1
    f = fwd(d, reset=reset)
    g = bwd(d, reset=reset)
    dA, dD = np.zeros(4), np.zeros(4)
    for b, cs in enumerate(cuts):
        for i in range(len(cs) - 1):
            lo, hi = cs[i], cs[i + 1]
            first, last = i == 0, i == len(cs) - 2
            piece = {k: d[k][b:b + 1, lo:hi] for k in ("x", "dt", "B", "C", "dy")}
            piece.update(A=d["A"], D=d["D"], init_state=d["init_state"][b:b + 1] if first else None,
                         dfinal_state=d["dfinal_state"][b:b + 1] if last else None)
            fp, gp = fwd(piece), bwd(piece)
            close(f["y"][b:b + 1, lo:hi], fp["y"])
            for k in ("dx", "ddt", "dB", "dC"):
                close(g[k][b:b + 1, lo:hi], gp[k])
            dA += gp["dA"]
            dD += gp["dD"]
            if last:
                close(f["final_state"][b:b + 1], fp["final_state"])
            if first:
                close(g["dinit_state"][b:b + 1], gp["dinit_state"])
    close(g["dA"], dA)
    close(g["dD"], dD)
    # a reset at token 0 discards the initial state
    r0 = np.zeros((2, 14), dtype=np.uint8)
    r0[:, 0] = 1
    d0 = dict(d, init_state=None)
    close(fwd(d, reset=r0)["y"], fwd(d0)["y"])
    assert float(np.max(np.abs(bwd(d, reset=r0)["dinit_state"]))) == 0.0
