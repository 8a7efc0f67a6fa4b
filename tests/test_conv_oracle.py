"""Pins of the convolution oracle (CPU): against the library routine it must reduce to, against finite
differences, and the composition law that makes checkpointing its state exact."""
import numpy as np
import torch

from oracle import conv_ref


def draw(seed, Bt=2, L=11, C=5, state=True):
    r = np.random.default_rng(seed)
    return dict(u=r.standard_normal((Bt, L, C)), w=r.standard_normal((C, 4)), bias=r.standard_normal(C),
                state_in=r.standard_normal((Bt, 3, C)) if state else None, dout=r.standard_normal((Bt, L, C)),
                dstate_out=r.standard_normal((Bt, 3, C)))


def close(a, b, tol=1e-12):
    assert float(np.max(np.abs(np.asarray(a) - np.asarray(b)))) <= tol * max(1.0, float(np.max(np.abs(b))))


def test_forward_is_the_depthwise_causal_convolution_of_the_library_followed_by_silu():
    d = draw(0, state=False)
    u = torch.from_numpy(d["u"]).permute(0, 2, 1)                      # [Bt, C, L]
    w = torch.from_numpy(d["w"]).unsqueeze(1)                          # [C, 1, 4]: tap 3 multiplies the current token
    pre = torch.nn.functional.conv1d(u, w, torch.from_numpy(d["bias"]), padding=3, groups=5)[..., :11]
    want = torch.nn.functional.silu(pre).permute(0, 2, 1).numpy()
    close(conv_ref.conv1d_silu_fwd(d["u"], d["w"], d["bias"])["out"], want)


def test_a_segment_restarted_from_its_state_continues_the_sequence():
    d = draw(1)
    full = conv_ref.conv1d_silu_fwd(d["u"], d["w"], d["bias"], d["state_in"])
    for cut in (1, 2, 3, 7):                                           # including pieces shorter than the kernel
        a = conv_ref.conv1d_silu_fwd(d["u"][:, :cut], d["w"], d["bias"], d["state_in"])
        b = conv_ref.conv1d_silu_fwd(d["u"][:, cut:], d["w"], d["bias"], a["state_out"])
        close(np.concatenate([a["out"], b["out"]], axis=1), full["out"])
        close(b["state_out"], full["state_out"])
    empty = conv_ref.conv1d_silu_fwd(d["u"][:, :0], d["w"], d["bias"], d["state_in"])
    close(empty["state_out"], d["state_in"])


def test_gradients_by_central_finite_differences_and_across_a_cut():
    d = draw(2, L=6, C=3)

    def loss(u, w, bias, state_in):
        f = conv_ref.conv1d_silu_fwd(u, w, bias, state_in)
        return float(np.sum(f["out"] * d["dout"]) + np.sum(f["state_out"] * d["dstate_out"]))

    g = conv_ref.conv1d_silu_bwd(d["u"], d["w"], d["bias"], d["state_in"], d["dout"], d["dstate_out"])
    eps = 1e-6
    for name, key in (("u", "du"), ("w", "dw"), ("bias", "dbias"), ("state_in", "dstate_in")):
        base = {k: d[k].copy() for k in ("u", "w", "bias", "state_in")}
        num = np.zeros_like(base[name])
        it = np.nditer(base[name], flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            hi = {k: v.copy() for k, v in base.items()}
            lo = {k: v.copy() for k, v in base.items()}
            hi[name][i] += eps
            lo[name][i] -= eps
            num[i] = (loss(**hi) - loss(**lo)) / (2 * eps)
        close(g[key], num, 1e-7)
    # reverse mode through a cut: the right piece hands dstate_in to the left piece as its dstate_out
    cut = 2
    left = conv_ref.conv1d_silu_fwd(d["u"][:, :cut], d["w"], d["bias"], d["state_in"])
    gr = conv_ref.conv1d_silu_bwd(d["u"][:, cut:], d["w"], d["bias"], left["state_out"], d["dout"][:, cut:], d["dstate_out"])
    gl = conv_ref.conv1d_silu_bwd(d["u"][:, :cut], d["w"], d["bias"], d["state_in"], d["dout"][:, :cut], gr["dstate_in"])
    close(np.concatenate([gl["du"], gr["du"]], axis=1), g["du"])
    close(gl["dw"] + gr["dw"], g["dw"])
    close(gl["dbias"] + gr["dbias"], g["dbias"])
    close(gl["dstate_in"], g["dstate_in"])
