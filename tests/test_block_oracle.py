"""Pins of the block oracle (CPU).  Its pieces are pinned in their own files; here the composition:
central differences through the whole block, and the law that makes sequence checkpoints exact
(a sequence cut in two, the second part restarted from the first part's two states)."""
import numpy as np

from oracle import block_ref

H, P, G, N, DM = 2, 4, 1, 3, 5


def draw(seed, L=9):
    r = np.random.default_rng(seed)
    d_inner, conv_dim, d_in = block_ref.dims(None, H, P, G, N)
    p = dict(W_in=r.standard_normal((d_in, DM)) * 0.5, conv_w=r.standard_normal((conv_dim, 4)) * 0.5,
             conv_b=r.standard_normal(conv_dim) * 0.3, dt_bias=r.standard_normal(H) * 0.3 - 1.0,
             A=-np.exp(r.uniform(0.0, 1.5, H)), D=r.standard_normal(H), norm_w=1.0 + 0.3 * r.standard_normal(d_inner),
             W_out=r.standard_normal((DM, d_inner)) * 0.5)
    return dict(u=r.standard_normal((L, DM)), p=p, dout=r.standard_normal((L, DM)),
                conv_state=r.standard_normal((3, conv_dim)), ssm_state=r.standard_normal((H, P, N)),
                dconv_state=r.standard_normal((3, conv_dim)), dssm_state=r.standard_normal((H, P, N)))


def close(a, b, tol):
    assert float(np.max(np.abs(np.asarray(a) - np.asarray(b)))) <= tol * max(1.0, float(np.max(np.abs(b))))


def loss(d, u=None, p=None, conv_state=None, ssm_state=None):
    f = block_ref.block_fwd(d["u"] if u is None else u, d["p"] if p is None else p, H, P, G, N, 1e-3,
                            d["conv_state"] if conv_state is None else conv_state,
                            d["ssm_state"] if ssm_state is None else ssm_state)
    return float(np.sum(f["out"] * d["dout"]) + np.sum(f["conv_state"] * d["dconv_state"]) + np.sum(f["ssm_state"] * d["dssm_state"]))


def numgrad(fn, a, h=1e-6):
    g = np.zeros_like(a)
    for idx in np.ndindex(*a.shape):
        p, m = a.copy(), a.copy()
        p[idx] += h
        m[idx] -= h
        g[idx] = (fn(p) - fn(m)) / (2 * h)
    return g


def test_gradients_of_the_whole_block_match_central_differences():
    d = draw(0)
    g = block_ref.block_bwd(d["u"], d["p"], H, P, G, N, d["dout"], 1e-3, d["conv_state"], d["ssm_state"],
                            d["dconv_state"], d["dssm_state"])
    close(g["du"], numgrad(lambda a: loss(d, u=a), d["u"]), 2e-7)
    close(g["dconv_state_in"], numgrad(lambda a: loss(d, conv_state=a), d["conv_state"]), 2e-7)
    close(g["dssm_state_in"], numgrad(lambda a: loss(d, ssm_state=a), d["ssm_state"]), 2e-7)
    for key, name in (("W_in", "dW_in"), ("conv_w", "dconv_w"), ("conv_b", "dconv_b"), ("dt_bias", "ddt_bias"), ("A", "dA"),
                      ("D", "dD"), ("norm_w", "dnorm_w"), ("W_out", "dW_out")):
        close(g[name], numgrad(lambda a: loss(d, p={**d["p"], key: a}), d["p"][key]), 2e-7)


def test_a_sequence_cut_in_two_and_restarted_from_both_states_is_the_whole_sequence():
    d = draw(1, L=11)
    whole = block_ref.block_fwd(d["u"], d["p"], H, P, G, N, 1e-5, d["conv_state"], d["ssm_state"])
    gw = block_ref.block_bwd(d["u"], d["p"], H, P, G, N, d["dout"], 1e-5, d["conv_state"], d["ssm_state"],
                             d["dconv_state"], d["dssm_state"])
    for cut in (2, 6):
        a = block_ref.block_fwd(d["u"][:cut], d["p"], H, P, G, N, 1e-5, d["conv_state"], d["ssm_state"])
        b = block_ref.block_fwd(d["u"][cut:], d["p"], H, P, G, N, 1e-5, a["conv_state"], a["ssm_state"])
        close(np.concatenate([a["out"], b["out"]]), whole["out"], 1e-12)
        close(b["ssm_state"], whole["ssm_state"], 1e-12)
        close(b["conv_state"], whole["conv_state"], 1e-12)
        # backward right to left: the state adjoints travel left, parameter gradients add up
        gb = block_ref.block_bwd(d["u"][cut:], d["p"], H, P, G, N, d["dout"][cut:], 1e-5, a["conv_state"], a["ssm_state"],
                                 d["dconv_state"], d["dssm_state"])
        ga = block_ref.block_bwd(d["u"][:cut], d["p"], H, P, G, N, d["dout"][:cut], 1e-5, d["conv_state"], d["ssm_state"],
                                 gb["dconv_state_in"], gb["dssm_state_in"])
        close(np.concatenate([ga["du"], gb["du"]]), gw["du"], 1e-11)
        for k in ("dW_in", "dconv_w", "dconv_b", "ddt_bias", "dA", "dD", "dnorm_w", "dW_out"):
            close(ga[k] + gb[k], gw[k], 1e-11)
        close(ga["dssm_state_in"], gw["dssm_state_in"], 1e-11)
        close(ga["dconv_state_in"], gw["dconv_state_in"], 1e-11)


def test_stack_of_blocks_gradients_match_central_differences():
    d0, d1 = draw(5, L=6), draw(6, L=6)
    layers = [d0["p"], d1["p"]]
    x0, dout = d0["u"], d0["dout"]
    f = block_ref.stack_fwd(x0, layers, H, P, G, N, 1e-3)
    b = block_ref.stack_bwd(f["xs"], layers, H, P, G, N, dout, 1e-3)
    L = lambda x=None, lay=None: float(np.sum(block_ref.stack_fwd(x0 if x is None else x, layers if lay is None else lay, H, P, G, N, 1e-3)["out"] * dout))
    close(b["dx0"], numgrad(lambda a: L(x=a), x0), 2e-7)
    for j in range(2):
        for key, name in (("W_in", "dW_in"), ("conv_b", "dconv_b"), ("A", "dA"), ("norm_w", "dnorm_w"), ("W_out", "dW_out")):
            def with_param(a, j=j, key=key):
                lay = [dict(p) for p in layers]
                lay[j][key] = a
                return L(lay=lay)
            close(b["grads"][j][name], numgrad(with_param, layers[j][key]), 2e-7)


def test_with_the_pre_norm_gradients_still_match_central_differences():
    d = draw(7)
    r = np.random.default_rng(70)
    d["p"]["pre_norm_w"] = 1.0 + 0.3 * r.standard_normal(DM)
    g = block_ref.block_bwd(d["u"], d["p"], H, P, G, N, d["dout"], 1e-3, d["conv_state"], d["ssm_state"],
                            d["dconv_state"], d["dssm_state"])
    close(g["du"], numgrad(lambda a: loss(d, u=a), d["u"]), 2e-7)
    for key, name in (("pre_norm_w", "dpre_norm_w"), ("W_in", "dW_in"), ("conv_w", "dconv_w"), ("norm_w", "dnorm_w")):
        close(g[name], numgrad(lambda a: loss(d, p={**d["p"], key: a}), d["p"][key]), 2e-7)
    # the normalised input does not see the scale of u (eps = 0): neither does anything behind it
    f1 = block_ref.block_fwd(d["u"], d["p"], H, P, G, N, 0.0)
    f2 = block_ref.block_fwd(13.0 * d["u"], d["p"], H, P, G, N, 0.0)
    close(f2["out"], f1["out"], 1e-12)
    # a two-layer pre-norm residual stack
    d1 = draw(8)
    d1["p"]["pre_norm_w"] = 1.0 + 0.3 * r.standard_normal(DM)
    layers, x0, dout = [d["p"], d1["p"]], d["u"], d["dout"]
    f = block_ref.stack_fwd(x0, layers, H, P, G, N, 1e-3)
    b = block_ref.stack_bwd(f["xs"], layers, H, P, G, N, dout, 1e-3)
    L = lambda x=None, lay=None: float(np.sum(block_ref.stack_fwd(x0 if x is None else x, layers if lay is None else lay, H, P, G, N, 1e-3)["out"] * dout))
    close(b["dx0"], numgrad(lambda a: L(x=a), x0), 2e-7)
    for j in range(2):
        def with_param(a, j=j):
            lay = [dict(p) for p in layers]
            lay[j]["pre_norm_w"] = a
            return L(lay=lay)
        close(b["grads"][j]["dpre_norm_w"], numgrad(with_param, layers[j]["pre_norm_w"]), 2e-7)


def test_a_stack_continued_from_the_states_of_every_layer_is_the_whole_sequence():
    d0, d1, d2 = draw(11, L=10), draw(12, L=10), draw(13, L=10)
    layers, x0 = [d0["p"], d1["p"], d2["p"]], d0["u"]
    whole = block_ref.stack_fwd(x0, layers, H, P, G, N)
    outs, cs, ss, t = [], None, None, 0
    for n in (4, 1, 1, 4):      # a prompt, two single tokens, the rest
        f = block_ref.stack_fwd(x0[t:t + n], layers, H, P, G, N, conv_states=cs, ssm_states=ss)
        outs.append(f["out"])
        cs, ss, t = f["conv_states"], f["ssm_states"], t + n
    close(np.concatenate(outs), whole["out"], 1e-12)
    for j in range(3):
        close(ss[j], whole["ssm_states"][j], 1e-12)
        close(cs[j], whole["conv_states"][j], 1e-12)
