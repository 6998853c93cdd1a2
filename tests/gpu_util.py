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
    """A line into gpurun_out/test_progress.log (and stderr): a long CPU oracle pass says how far it is."""
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
#   ||got - ref|| <= ROW_REL * ||ref|| + ROW_FLOOR * rms_rows(||ref||).
# Where it comes from: the result is rounded to bf16 once (<= 2^-9 per element, so <= 2^-9 of the row's norm);
# P and dS are rounded to bf16 before the second contraction, relative 2^-9 per term with random signs, which
# over the n terms of a row adds about 2^-9 of the row's norm again (the terms of a gradient row do not cancel
# to far below their own size); Delta comes from the bf16 O (relative 2^-9 on a sum over D).  Together a few
# times 2^-9 = 2e-3: observed rows sit at 2e-3..8e-3.  5e-2 leaves one order of magnitude over that and is
# still 20x below "this row is wrong" (relative error 1).  The floor covers rows that are zero or nearly so by
# cancellation (dQ of row 0 is exactly 0; dK of the last key): their error scales with the terms, not the sum.
ROW_REL = 5e-2
ROW_FLOOR = 5e-3


def grad_err(got: np.ndarray, ref: np.ndarray, what="") -> float:
    """Tensor-wide relative L2 (returned; the caller holds it to GRAD_REL_L2) and the per-row bar (asserted)."""
    if ref.ndim >= 2 and ref.shape[-1] >= 16:
        e = np.linalg.norm(got - ref, axis=-1)
        r = np.linalg.norm(ref, axis=-1)
        rms = float(np.sqrt(np.mean(r * r))) if r.size else 0.0
        bound = ROW_REL * r + ROW_FLOOR * rms + 1e-4  # the constant covers tensors that are zero altogether
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
