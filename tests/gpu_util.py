"""Helpers for the GPU parity tests: move seeded bf16 bit patterns to the
device and results back, and compare against the fp64 oracle."""
import numpy as np
import torch

from oracle import ref_numpy as rn

# Parity bars (stated by the build's target): O max-abs, gradients relative L2.
O_MAX_ABS = 1e-2
GRAD_REL_L2 = 2e-2
# LSE is fp32 end to end (fp32 MFMA accumulation of exact bf16 products, fp32
# exp2/log2): errors are ~1e-6 relative to |s| <= ~20 plus the hardware
# transcendental error (~1 ulp) accumulated over a row.
LSE_MAX_ABS = 2e-4


def progress(msg: str):
    """A line into the run's output folder (test_progress.log) and stderr: a long CPU oracle pass says how far it is."""
    import os, sys, time
    d = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    try:
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "test_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass
    print(msg, file=sys.stderr, flush=True)


def guarded(shape, dtype, pad_elems: int = 4096):
    """A device tensor of `shape` carved from the middle of a larger buffer whose margins hold a canary
    pattern; returns (tensor, check) where check() asserts that both margins are untouched."""
    n = 1
    for x in shape:
        n *= int(x)
    item = torch.empty((), dtype=dtype).element_size()
    pad = (pad_elems * item + 255) // 256 * 256 // item  # keep the payload 256-byte aligned
    buf = torch.empty(n + 2 * pad, dtype=dtype, device="cuda")
    raw = buf.view(torch.uint8)
    raw.fill_(0xA5)
    t = buf[pad:pad + n].view(*shape)

    def check(what=""):
        torch.cuda.synchronize()
        lo, hi = raw[:pad * item], raw[(pad + n) * item:]
        assert bool((lo == 0xA5).all()), f"{what}: bytes in front of the buffer were overwritten"
        assert bool((hi == 0xA5).all()), f"{what}: bytes behind the buffer were overwritten"

    return t, check


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return rn.widen_bf16(host_bits(t))
    return t.detach().cpu().numpy().astype(np.float64)


def rel_l2(got: np.ndarray, ref: np.ndarray) -> float:
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((got - ref).ravel()))
    return num / den if den > 0 else num


# Per-row gradient bar, beside the tensor-wide norm (which a few entirely wrong rows among 10^5 would pass):
# every vector along the head dim (one key position of dK/dV, one query row of dQ, per head) must be within
#   ||got - ref|| <= ROW_REL * ||ref|| + abs_floor.
# Relative part: the result is rounded to bf16 once (<= 2^-9 per element, so <= 2^-9 of the row's norm); P and
# dS are rounded to bf16 before the second contraction, relative 2^-9 per term with random signs, which over
# the terms of a row adds about 2^-9 of the row's norm again.  A few times 2^-9 = 2e-3: observed rows sit at
# 2e-3..8e-3; 5e-2 leaves an order of magnitude over that and is still 20x below "this row is wrong".
# Absolute part: Delta_i = dO_i.O_i comes from the bf16 O a training step has, not from the exact one.  The
# rounding of O (uniform within half an ulp, rms 2^-9/sqrt(3) relative) puts an error of rms
#   sd = 2^-9/sqrt(3) * sqrt(D) * rms(dO) * rms(O)          (0.013 for D = 128, unit-variance rows)
# on Delta_i, which enters dQ_i as scale * dDelta_i * sum_j P_ij k_j whatever the size of dQ_i itself, and dK_j
# likewise through sum_i P_ij dDelta_i q_i.  Where P sits on one or two keys (the first rows of a sequence,
# peaked inputs) that is scale * dDelta_i * ||k||, and dQ_i itself is small by cancellation.  delta_floor()
# = 8 sd * scale * max||k|| covers the worst of ~10^5 rows with margin: 0.12 for unit-variance inputs, D = 128,
# scale 1/sqrt(D); observed worst rows 0.03 there, 0.38 with Q, K x4 (floor 0.47), 0.84 at scale 1 (floor 1.3).
# dV does not depend on Delta: callers that know which tensor they hold pass abs_floor = 0 for it.
ROW_REL = 5e-2
DELTA_FLOOR_UNIT = 0.12


def delta_floor(scale: float, D: int, rms_do: float, rms_v: float, max_norm: float) -> float:
    return 8.0 * (2.0 ** -9 / np.sqrt(3.0)) * np.sqrt(D) * rms_do * rms_v * scale * max_norm


def grad_err(got: np.ndarray, ref: np.ndarray, what="", abs_floor: float = DELTA_FLOOR_UNIT) -> float:
    """Tensor-wide relative L2 (returned; the caller holds it to GRAD_REL_L2) and the per-row bar (asserted)."""
    if ref.ndim >= 2 and ref.shape[-1] >= 16:
        e = np.linalg.norm(got - ref, axis=-1)
        r = np.linalg.norm(ref, axis=-1)
        bound = ROW_REL * r + abs_floor + 1e-4  # the constant covers rows that are exactly zero
        bad = e > bound
        if bad.any():
            idx = np.argwhere(bad)
            w = tuple(idx[np.argmax((e - bound)[bad])])
            raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} rows off; worst at {w}: "
                                 f"err {e[w]:.3e}, ref norm {r[w]:.3e}, bound {bound[w]:.3e}")
    return rel_l2(got, ref)


def check_o(o_gpu: np.ndarray, o_ref: np.ndarray, what="", big_from: float = 4.0):
    """max-abs bar on O; where |O| >= 4 a bf16 store alone can exceed the bar
    (half an ulp is 2^-6), so those elements are held to one bf16 ulp of the
    oracle instead, and are reported.  `big_from` = 2 is for peaked softmax rows
    only (the dynamic-range cases): there O is close to single V rows, |O| in [2, 4)
    is common, and the store's half ulp (2^-7 = 7.8e-3) plus the bf16 rounding of
    two or three dominant weights (2^-9 |v| each) passes 1e-2 on a few elements of
    any kernel that stores bf16."""
    err = np.abs(o_gpu - o_ref)
    big = np.abs(o_ref) >= big_from
    if big.any():
        ulp = 2.0 ** (np.floor(np.log2(np.abs(o_ref[big]))) - 7)
        assert np.all(err[big] <= ulp), f"{what}: large-|O| elements off by more than one bf16 ulp"
        err = np.where(big, 0.0, err)
    assert err.max() <= O_MAX_ABS, f"{what}: O max-abs {err.max():.3e} > {O_MAX_ABS}"
    return float(err.max())
