"""Pins of the pointwise-operator oracle against things other than itself:
torch fp64 autograd of composed primitives, closed forms, finite differences
and the group properties of the rotation.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import ref_pointwise as rp


def rng_arrays(seed, *shapes):
    r = np.random.default_rng(seed)
    return [r.standard_normal(s) for s in shapes]


def test_rmsnorm_against_torch_autograd():
    T, C, eps = 7, 48, 1e-5
    x, w, dy = rng_arrays(0, (T, C), (C,), (T, C))
    xt, wt = torch.tensor(x, requires_grad=True), torch.tensor(w, requires_grad=True)
    yt = xt * torch.rsqrt((xt * xt).mean(dim=1, keepdim=True) + eps) * wt
    (yt * torch.tensor(dy)).sum().backward()
    y, rstd = rp.rmsnorm_fwd(x, w, eps)
    dx, dw = rp.rmsnorm_bwd(x, w, dy, eps)
    assert np.abs(y - yt.detach().numpy()).max() < 1e-13
    assert np.abs(dx - xt.grad.numpy()).max() < 1e-12
    assert np.abs(dw - wt.grad.numpy()).max() < 1e-12
    if hasattr(torch.nn.functional, "rms_norm"):  # the library routine, where this torch has it
        yl = torch.nn.functional.rms_norm(torch.tensor(x), (C,), torch.tensor(w), eps)
        assert np.abs(y - yl.numpy()).max() < 1e-13


def test_rmsnorm_closed_forms():
    C, eps = 64, 1e-6
    # a constant row c gives w * sign(c) / sqrt(1 + eps/c^2); scaling a row leaves y unchanged when eps = 0
    w = np.linspace(0.5, 2.0, C)
    x = np.full((1, C), -3.0)
    y, rstd = rp.rmsnorm_fwd(x, w, eps)
    assert np.allclose(y[0], -w / np.sqrt(1.0 + eps / 9.0), rtol=0, atol=1e-15)
    assert np.isclose(rstd[0], 1.0 / np.sqrt(9.0 + eps))
    x = rng_arrays(1, (3, C))[0]
    y1, _ = rp.rmsnorm_fwd(x, w, 0.0)
    y2, _ = rp.rmsnorm_fwd(5.0 * x, w, 0.0)
    assert np.abs(y1 - y2).max() < 1e-14
    assert np.allclose(np.mean((y1 / w) ** 2, axis=1), 1.0)     # unit RMS before the weight
    # with eps = 0 the gradient is orthogonal to x (y does not change along x)
    dy = rng_arrays(2, (3, C))[0]
    dx, _ = rp.rmsnorm_bwd(x, w, dy, 0.0)
    assert np.abs(np.sum(dx * x, axis=1)).max() < 1e-12


def test_rmsnorm_finite_differences():
    T, C, eps, h = 3, 16, 1e-5, 1e-6
    x, w, dy = rng_arrays(3, (T, C), (C,), (T, C))
    dx, dw = rp.rmsnorm_bwd(x, w, dy, eps)
    L = lambda x_, w_: float(np.sum(rp.rmsnorm_fwd(x_, w_, eps)[0] * dy))
    for (t, c) in [(0, 0), (1, 7), (2, 15)]:
        e = np.zeros_like(x); e[t, c] = h
        assert abs((L(x + e, w) - L(x - e, w)) / (2 * h) - dx[t, c]) < 1e-7
    for c in (0, 5, 15):
        e = np.zeros_like(w); e[c] = h
        assert abs((L(x, w + e) - L(x, w - e)) / (2 * h) - dw[c]) < 1e-7


def test_rope_properties():
    T, H, D = 9, 3, 16
    x = rng_arrays(4, (T, H, D))[0]
    pos = np.arange(100, 100 + T)
    a = rp.rope_angles(pos, D)
    assert a.shape == (T, D // 2) and np.isclose(a[3, 0], 103.0) and np.isclose(a[0, D // 2 - 1], 100.0 * 10000.0 ** (-(D - 2) / D))
    y = rp.rope(x, np.cos(a), np.sin(a))
    # position 0 (angle 0) is the identity
    z = np.zeros((T, D // 2))
    assert np.array_equal(rp.rope(x, np.cos(z), np.sin(z)), x)
    # a rotation: pair norms preserved, conjugate undoes it, angles add
    h = D // 2
    assert np.allclose(y[..., :h] ** 2 + y[..., h:] ** 2, x[..., :h] ** 2 + x[..., h:] ** 2)
    assert np.abs(rp.rope(y, np.cos(a), np.sin(a), conjugate=True) - x).max() < 1e-13
    b = rp.rope_angles(np.arange(7, 7 + T), D)
    assert np.abs(rp.rope(y, np.cos(b), np.sin(b)) - rp.rope(x, np.cos(a + b), np.sin(a + b))).max() < 1e-12
    # brute force on one pair
    t, hh, i = 4, 1, 5
    c, s = np.cos(a[t, i]), np.sin(a[t, i])
    assert np.isclose(y[t, hh, i], x[t, hh, i] * c - x[t, hh, i + h] * s)
    assert np.isclose(y[t, hh, i + h], x[t, hh, i + h] * c + x[t, hh, i] * s)
    # the score q.k depends on the position difference only
    q, k = rng_arrays(5, (1, 1, D), (1, 1, D))
    def score(pq, pk):
        aq, ak = rp.rope_angles(np.array([pq]), D), rp.rope_angles(np.array([pk]), D)
        return float(np.sum(rp.rope(q, np.cos(aq), np.sin(aq)) * rp.rope(k, np.cos(ak), np.sin(ak))))
    assert abs(score(10, 3) - score(1007, 1000)) < 1e-9


def test_rope_gradient_is_the_conjugate_rotation():
    T, H, D = 5, 2, 8
    x, dy = rng_arrays(6, (T, H, D), (T, H, D))
    a = rp.rope_angles(np.arange(T) * 17, D)
    cos, sin = np.cos(a), np.sin(a)
    xt = torch.tensor(x, requires_grad=True)
    h = D // 2
    c, s = torch.tensor(cos)[:, None, :], torch.tensor(sin)[:, None, :]
    yt = torch.cat([xt[..., :h] * c - xt[..., h:] * s, xt[..., h:] * c + xt[..., :h] * s], dim=-1)
    (yt * torch.tensor(dy)).sum().backward()
    assert np.abs(rp.rope(x, cos, sin) - yt.detach().numpy()).max() < 1e-14
    assert np.abs(rp.rope(dy, cos, sin, conjugate=True) - xt.grad.numpy()).max() < 1e-14


def test_swiglu_against_torch_and_closed_forms():
    g, u, dy = rng_arrays(7, (6, 40), (6, 40), (6, 40))
    g *= 3.0
    gt, ut = torch.tensor(g, requires_grad=True), torch.tensor(u, requires_grad=True)
    yt = torch.nn.functional.silu(gt) * ut
    (yt * torch.tensor(dy)).sum().backward()
    y = rp.swiglu_fwd(g, u)
    dg, du = rp.swiglu_bwd(g, u, dy)
    assert np.abs(y - yt.detach().numpy()).max() < 1e-14
    assert np.abs(dg - gt.grad.numpy()).max() < 1e-13
    assert np.abs(du - ut.grad.numpy()).max() < 1e-14
    # g = 0 gives y = 0, dg = dy*u/2, du = 0; large g gives y -> g*u; large negative g gives y -> 0
    z = np.zeros((1, 4)); uu = np.array([[1.0, -2.0, 3.0, 0.5]]); dd = np.ones((1, 4))
    assert np.array_equal(rp.swiglu_fwd(z, uu), z)
    dg0, du0 = rp.swiglu_bwd(z, uu, dd)
    assert np.allclose(dg0, uu / 2) and np.array_equal(du0, z)
    assert np.allclose(rp.swiglu_fwd(np.full((1, 4), 40.0), uu), 40.0 * uu)
    assert np.abs(rp.swiglu_fwd(np.full((1, 4), -40.0), uu)).max() < 1e-15
    # finite differences of dg
    h = 1e-6
    L = lambda g_: float(np.sum(rp.swiglu_fwd(g_, u) * dy))
    for (i, j) in [(0, 0), (3, 17), (5, 39)]:
        e = np.zeros_like(g); e[i, j] = h
        assert abs((L(g + e) - L(g - e)) / (2 * h) - dg[i, j]) < 1e-7
