"""Helpers of the GPU parity tests: run the HIP library through its C ABI and the CPU oracle on the
same seeded inputs, and the error measures both are compared with."""
import numpy as np

from oracle import rwkvq_oracle as orc
from paper_2505_03803_amd import binding as B

TOL = 2e-3   # bar on outputs: max relative error, binary32 accumulate, fp16/bf16 I/O


def torch_():
    import torch
    return torch


def to_dev_bits(bits: np.ndarray):
    torch = torch_()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def gpu_dequant(dm, w_dtype=B.F32):
    out = B.dequant(dm, w_dtype)
    torch_().cuda.synchronize()
    a = out.cpu().numpy()
    return a if w_dtype == B.F32 else a.view(np.uint16)


def gpu_gemm(dm, x_bits, x_dtype, y_dtype=B.F32):
    M = x_bits.shape[0]
    y = B.gemm(dm, to_dev_bits(x_bits), M, B.DTYPES[x_dtype], y_dtype)
    torch_().cuda.synchronize()
    a = y.cpu().numpy()
    return a.astype(np.float64) if y_dtype == B.F32 else a.view(np.uint16)


def err_g1(y, ref):
    """max |y - ref| / max |ref|  (one denominator per matrix)."""
    return float(np.abs(y - ref).max() / np.abs(ref).max())


def err_g2(y, ref):
    """max over outputs of |y - ref| / max(|ref|, rms(ref)): element-wise relative error with
    outputs smaller than the root mean square measured against the root mean square."""
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float((np.abs(y - ref) / np.maximum(np.abs(ref), rms)).max())


def check_outputs(y, mat, x_bits, x_dtype, fed=None, tight=None):
    """The output bar.  G1 against the oracle with exact binary32 weights; G2 against the oracle fed
    the weight rounding the kernel declares (`fed` = None, 'f16' or 'bf16'); both in binary64 sums."""
    x = orc.widen(x_bits, x_dtype)
    exact = orc.linear(mat, x, "f64")
    g1 = err_g1(y, exact)
    asfed = exact if fed is None else orc.linear(mat, x, "f64", weight_round=fed)
    g2 = err_g2(y, asfed)
    assert g1 <= TOL, f"G1 {g1}"
    assert g2 <= TOL, f"G2 {g2}"
    if tight is not None:
        assert g2 <= tight, f"as-fed error {g2} above the expected binary32 accumulation error {tight}"
    return g1, g2
