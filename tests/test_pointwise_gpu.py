"""Parity of the HIP pointwise operators (RMS norm, rotary embedding, SwiGLU
gate; forward and backward) with the fp64 oracle, element by element.

Tolerance (derived from the arithmetic): the kernels evaluate in fp32 and round
the result to bf16 once, so an output element may differ from the exact value by
half a bf16 ulp (2^-9 relative) plus fp32 evaluation noise; the bar is 2^-8
relative plus an absolute floor for cancelling sums, stated per test."""
import numpy as np
import pytest
import torch

from oracle import ref_numpy as rn
from oracle import ref_pointwise as rp
from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import synth
from gpu_util import dev_bf16, host_f64

pytestmark = pytest.mark.gpu

REL = 2.0 ** -8


def bits(seed, shape, scale=1.0):
    return synth.normal_bf16(np.random.default_rng([seed, 0xB17]), shape, scale)


def close(got, ref, floor, what):
    err = np.abs(got - ref)
    bound = REL * np.abs(ref) + floor
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} elements off, worst {float((err - bound).max()):.3e} over the bar"
    return float((err / (np.abs(ref) + floor)).max())


@pytest.mark.parametrize("T,C", [(1, 8), (5, 64), (37, 520), (130, 4096), (9, 8192), (1030, 1024)])
def test_rmsnorm_matches_oracle(T, C):
    eps = 1e-5
    xb, wb, dyb = bits(T + C, (T, C), 1.5), bits(1, (C,)), bits(2, (T, C))
    x, w, dy = dev_bf16(xb), dev_bf16(wb), dev_bf16(dyb)
    y, rstd = sp.sp_rmsnorm_fwd(x, w, eps)
    dx, dw = sp.sp_rmsnorm_bwd(x, w, rstd, dy)
    dx2, dw2 = sp.sp_rmsnorm_bwd(x, w, rstd, dy)
    torch.cuda.synchronize()
    xf, wf, dyf = rn.widen_bf16(xb), rn.widen_bf16(wb), rn.widen_bf16(dyb)
    y_r, rstd_r = rp.rmsnorm_fwd(xf, wf, eps)
    dx_r, dw_r = rp.rmsnorm_bwd(xf, wf, dyf, eps)
    assert np.abs(rstd.cpu().numpy() / rstd_r - 1.0).max() <= 1e-5      # fp32 sum of C squares and one rsqrt
    close(host_f64(y), y_r, 1e-30, "y")
    # dx is a difference of two terms of similar size: the floor scales with the terms, not with the result
    floor_dx = 4e-6 * (np.abs(dyf * wf * rstd_r[:, None]) + np.abs(xf) * np.abs(np.sum(dyf * wf * xf, axis=1) * rstd_r ** 3 / C)[:, None])
    close(host_f64(dx), dx_r, floor_dx, "dx")
    floor_dw = 4e-6 * np.sum(np.abs(dyf * xf * rstd_r[:, None]), axis=0)  # fp32 accumulation over T rows
    close(host_f64(dw), dw_r, floor_dw, "dw")
    assert torch.equal(dw.view(torch.int16), dw2.view(torch.int16)) and torch.equal(dx.view(torch.int16), dx2.view(torch.int16))


@pytest.mark.parametrize("T,H,D", [(1, 1, 16), (7, 3, 64), (300, 8, 128), (33, 5, 128)])
def test_rope_matches_oracle_and_is_a_rotation(T, H, D):
    xb = bits(T * H, (T, H, D))
    pos = np.arange(T) * 977 + 5                      # positions up to ~3e5: large angles
    ang = rp.rope_angles(pos, D)
    cos32, sin32 = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    x = dev_bf16(xb)
    cs, sn = torch.from_numpy(cos32).cuda(), torch.from_numpy(sin32).cuda()
    y = sp.sp_rope(x, cs, sn)
    yc = sp.sp_rope(x, cs, sn, conjugate=True)
    torch.cuda.synchronize()
    xf = rn.widen_bf16(xb)
    # the tables the kernel sees are the fp32-rounded ones: the oracle takes the same values
    c64, s64 = cos32.astype(np.float64), sin32.astype(np.float64)
    floor = 4e-7 * (np.abs(xf) + np.abs(np.roll(xf, D // 2, axis=-1)))
    close(host_f64(y), rp.rope(xf, c64, s64), floor, "rope")
    close(host_f64(yc), rp.rope(xf, c64, s64, conjugate=True), floor, "rope conjugate")
    # in place: same bits as out of place
    z = x.clone()
    sp.sp_rope(z, cs, sn, out=z)
    torch.cuda.synchronize()
    assert torch.equal(z.view(torch.int16), y.view(torch.int16))


@pytest.mark.parametrize("shape", [(1, 8), (3, 40), (257, 1000), (64, 14336)])
def test_swiglu_matches_oracle(shape):
    gb, ub, dyb = bits(11, shape, 2.5), bits(12, shape), bits(13, shape)
    g, u, dy = dev_bf16(gb), dev_bf16(ub), dev_bf16(dyb)
    y = sp.sp_swiglu_fwd(g, u)
    dg, du = sp.sp_swiglu_bwd(g, u, dy)
    torch.cuda.synchronize()
    gf, uf, dyf = rn.widen_bf16(gb), rn.widen_bf16(ub), rn.widen_bf16(dyb)
    dg_r, du_r = rp.swiglu_bwd(gf, uf, dyf)
    # hardware exp2 and reciprocal are good to about one fp32 ulp each: a few 1e-7 relative on the sigmoid;
    # dg's factor 1 + g(1 - s) can cancel, hence its floor in terms of |dy u s g|
    sig = 1.0 / (1.0 + np.exp(-gf))
    close(host_f64(y), rp.swiglu_fwd(gf, uf), 1e-30, "y")
    close(host_f64(dg), dg_r, 4e-6 * np.abs(dyf * uf * sig) * (1.0 + np.abs(gf)), "dg")
    close(host_f64(du), du_r, 1e-30, "du")


def test_pointwise_llama_shard_shapes():
    """The shapes of one device's shard of the 8B-shaped layer at 128K tokens over 8 devices (16384 tokens):
    model dim 4096, 32 query heads of 128, MLP width 14336; sampled rows against the oracle."""
    T, C, H, D, F = 16384, 4096, 32, 128, 14336
    g = torch.Generator(device="cuda").manual_seed(9)
    mk = lambda *s: torch.randn(s, device="cuda", generator=g).to(torch.bfloat16)
    rows = np.unique(np.concatenate([[0, 1, T - 1], np.random.default_rng(3).integers(0, T, 29)]))
    ridx = torch.from_numpy(rows).cuda()
    f64 = lambda t: host_f64(t)
    x, w, dy = mk(T, C), mk(C), mk(T, C)
    y, rstd = sp.sp_rmsnorm_fwd(x, w, 1e-5)
    dx, dw = sp.sp_rmsnorm_bwd(x, w, rstd, dy)
    y_r, _ = rp.rmsnorm_fwd(f64(x[ridx]), f64(w), 1e-5)
    dx_r, _ = rp.rmsnorm_bwd(f64(x[ridx]), f64(w), f64(dy[ridx]), 1e-5)
    close(f64(y[ridx]), y_r, 1e-30, "y")
    close(f64(dx[ridx]), dx_r, 1e-4, "dx")
    # dw needs every row: fp64 on the host in blocks
    xs, dys, rs_ = f64(x), f64(dy), rstd.double().cpu().numpy()
    dw_r = np.einsum("tc,tc,t->c", dys, xs, rs_)
    close(f64(dw), dw_r, 4e-6 * np.einsum("tc,tc,t->c", np.abs(dys), np.abs(xs), rs_), "dw")
    del xs, dys
    q = mk(T, H, D)
    ang = rp.rope_angles(np.arange(T) + 7 * T, D)   # this device's slice of the positions
    cs, sn = torch.from_numpy(np.cos(ang).astype(np.float32)).cuda(), torch.from_numpy(np.sin(ang).astype(np.float32)).cuda()
    r = sp.sp_rope(q, cs, sn)
    qf = f64(q[ridx])
    close(f64(r[ridx]), rp.rope(qf, cs[ridx].double().cpu().numpy(), sn[ridx].double().cpu().numpy()),
          4e-7 * (np.abs(qf) + np.abs(np.roll(qf, D // 2, axis=-1))), "rope")
    back = sp.sp_rope(r, cs, sn, conjugate=True)
    assert (back.float() - q.float()).abs().max().item() <= 2.0 ** -6 * q.float().abs().max().item()  # two bf16 roundings
    gt, ut, dyt = mk(T, F) * 2, mk(T, F), mk(T, F)
    yy = sp.sp_swiglu_fwd(gt, ut)
    dg, du = sp.sp_swiglu_bwd(gt, ut, dyt)
    torch.cuda.synchronize()
    gf, uf, df = f64(gt[ridx]), f64(ut[ridx]), f64(dyt[ridx])
    dg_r, du_r = rp.swiglu_bwd(gf, uf, df)
    close(f64(yy[ridx]), rp.swiglu_fwd(gf, uf), 1e-30, "swiglu y")
    close(f64(dg[ridx]), dg_r, 4e-6 * np.abs(df * uf) * (1.0 + np.abs(gf)), "swiglu dg")
    close(f64(du[ridx]), du_r, 1e-30, "swiglu du")
