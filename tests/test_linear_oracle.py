"""Pins of the projection oracle (CPU): the sums written out element by element, the library's own
linear layer under autograd, and the identity weight."""
import numpy as np
import torch

from oracle import linear_ref


def draw(seed, T=5, I=4, O=3):
    r = np.random.default_rng(seed)
    return r.standard_normal((T, I)), r.standard_normal((O, I)), r.standard_normal((T, O))


def close(a, b, tol=1e-12):
    assert float(np.max(np.abs(np.asarray(a) - np.asarray(b)))) <= tol * max(1.0, float(np.max(np.abs(b))))


def test_sums_written_out():
    x, w, dout = draw(0)
    out = linear_ref.linear_fwd(x, w)
    g = linear_ref.linear_bwd(x, w, dout)
    for t in range(5):
        for o in range(3):
            close(out[t, o], sum(x[t, i] * w[o, i] for i in range(4)))
    for t in range(5):
        for i in range(4):
            close(g["dx"][t, i], sum(dout[t, o] * w[o, i] for o in range(3)))
    for o in range(3):
        for i in range(4):
            close(g["dw"][o, i], sum(dout[t, o] * x[t, i] for t in range(5)))


def test_against_the_library_layer_under_autograd():
    x, w, dout = draw(1, 7, 6, 9)
    xt, wt = torch.from_numpy(x).requires_grad_(), torch.from_numpy(w).requires_grad_()
    out = torch.nn.functional.linear(xt, wt)
    (out * torch.from_numpy(dout)).sum().backward()
    close(linear_ref.linear_fwd(x, w), out.detach().numpy())
    g = linear_ref.linear_bwd(x, w, dout)
    close(g["dx"], xt.grad.numpy())
    close(g["dw"], wt.grad.numpy())


def test_identity_weight_copies_and_a_transposed_operand_would_show():
    x, _, _ = draw(2, 4, 3, 3)
    close(linear_ref.linear_fwd(x, np.eye(3)), x)
    w = np.array([[0.0, 1.0, 0.0], [0.0, 0.0, 1.0], [1.0, 0.0, 0.0]])   # out[:, o] = x[:, perm[o]]
    close(linear_ref.linear_fwd(x, w), x[:, [1, 2, 0]])
    close(linear_ref.linear_bwd(x, w, x)["dx"], x[:, [2, 0, 1]])
