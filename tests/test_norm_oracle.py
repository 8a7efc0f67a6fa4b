"""Pins of the gated RMS normalisation oracle (CPU): against the library's own rms_norm and silu, against
finite differences, and the invariants that scale-free normalisation fixes."""
import numpy as np
import torch

from oracle import norm_ref


def draw(seed, T=7, C=12):
    r = np.random.default_rng(seed)
    return dict(y=r.standard_normal((T, C)), z=r.standard_normal((T, C)), w=r.standard_normal(C),
                dout=r.standard_normal((T, C)))


def close(a, b, tol=1e-12):
    assert float(np.max(np.abs(np.asarray(a) - np.asarray(b)))) <= tol * max(1.0, float(np.max(np.abs(b))))


def test_forward_and_gradients_are_the_library_rms_norm_of_the_gated_input():
    for ngroups in (1, 3):
        d = draw(0)
        y, z, w = (torch.from_numpy(d[k]).requires_grad_() for k in ("y", "z", "w"))
        g = y * torch.nn.functional.silu(z)
        gs = 12 // ngroups
        out = torch.nn.functional.rms_norm(g.reshape(7, ngroups, gs), (gs,), eps=1e-5).reshape(7, 12) * w
        (out * torch.from_numpy(d["dout"])).sum().backward()
        close(norm_ref.gated_rmsnorm_fwd(d["y"], d["z"], d["w"], 1e-5, ngroups), out.detach().numpy())
        got = norm_ref.gated_rmsnorm_bwd(d["y"], d["z"], d["w"], d["dout"], 1e-5, ngroups)
        close(got["dy"], y.grad.numpy())
        close(got["dz"], z.grad.numpy())
        close(got["dw"], w.grad.numpy())


def test_gradients_match_central_differences():
    d = draw(1, T=3, C=8)
    loss = lambda **kw: float(np.sum(norm_ref.gated_rmsnorm_fwd(**{**{k: d[k] for k in ("y", "z", "w")}, **kw}, eps=1e-3, ngroups=2) * d["dout"]))
    got = norm_ref.gated_rmsnorm_bwd(d["y"], d["z"], d["w"], d["dout"], 1e-3, 2)
    h = 1e-6
    for name, key in (("y", "dy"), ("z", "dz"), ("w", "dw")):
        num = np.zeros_like(d[name])
        for idx in np.ndindex(*d[name].shape):
            p, m = d[name].copy(), d[name].copy()
            p[idx] += h
            m[idx] -= h
            num[idx] = (loss(**{name: p}) - loss(**{name: m})) / (2 * h)
        close(got[key], num, 1e-7)


def test_scale_invariance_unit_rms_and_orthogonality():
    d = draw(2)
    one = np.ones(12)
    out = norm_ref.gated_rmsnorm_fwd(d["y"], d["z"], one, 0.0, 3)
    close(np.mean(out.reshape(7, 3, 4) ** 2, axis=2), np.ones((7, 3)))                 # unit RMS per group
    close(norm_ref.gated_rmsnorm_fwd(37.0 * d["y"], d["z"], one, 0.0, 3), out)         # y -> c y changes nothing
    # hence the gradient with respect to y is orthogonal to y within every group (Euler's theorem, degree 0)
    g = norm_ref.gated_rmsnorm_bwd(d["y"], d["z"], d["w"], d["dout"], 0.0, 3)
    close(np.sum((g["dy"] * d["y"]).reshape(7, 3, 4), axis=2), np.zeros((7, 3)), 1e-12)
    # a closed form: one channel per group, eps = 0: out = sign(y z) w whatever the magnitudes
    t = norm_ref.gated_rmsnorm_fwd(d["y"], d["z"], d["w"], 0.0, 12)
    close(t, np.sign(d["y"] * d["z"]) * d["w"])


def test_without_a_gate_it_is_the_library_rms_norm():
    d = draw(3)
    y, w = (torch.from_numpy(d[k]).requires_grad_() for k in ("y", "w"))
    out = torch.nn.functional.rms_norm(y, (12,), weight=w, eps=1e-5)
    (out * torch.from_numpy(d["dout"])).sum().backward()
    close(norm_ref.gated_rmsnorm_fwd(d["y"], None, d["w"], 1e-5, 1), out.detach().numpy())
    got = norm_ref.gated_rmsnorm_bwd(d["y"], None, d["w"], d["dout"], 1e-5, 1)
    close(got["dy"], y.grad.numpy())
    close(got["dw"], w.grad.numpy())
    assert got["dz"] is None
    # and the gated form with a gate whose silu is one (z * sigmoid(z) = 1 at z = 1.2784645...) gives the same
    z1 = np.full_like(d["y"], 1.2784645427610738)
    close(norm_ref.gated_rmsnorm_fwd(d["y"], z1, d["w"], 1e-5, 1), out.detach().numpy(), 1e-9)
