"""ctypes binding of librwkvq.so: the same entry points as include/rwkvq.h, argument marshalling
only.  PyTorch supplies device memory (tensors) and the stream; every computation runs in the
library's HIP kernels.  There is no fallback: if the library cannot be loaded this module raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_double, c_int, c_int32, c_longlong, c_size_t, c_void_p
from dataclasses import dataclass
from typing import Optional, Sequence

from . import build as _build

OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_ALIGN, ERR_DEVICE = range(6)
F16, BF16, F32 = 0, 1, 2
VQ, SQ = 0, 1
CANONICAL, NATIVE = 0, 1
DTYPES = {"f16": F16, "bf16": BF16, "f32": F32}

EXPORTS = ["rwkvq_version", "rwkvq_status_string", "rwkvq_sq_prepack", "rwkvq_vq_prepack",
           "rwkvq_sq_dequant", "rwkvq_vq_dequant", "rwkvq_sq_gemm", "rwkvq_vq_gemm",
           "rwkvq_linear_dispatch", "rwkvq_proxy_workspace_bytes", "rwkvq_proxy", "rwkvq_sq_encode",
           "rwkvq_vq_assign", "rwkvq_clip_mean", "rwkvq_mu_codebook", "rwkvq_token_shift_mix", "rwkvq_linear_dispatch_mixed",
           "rwkvq_wkv", "rwkvq_relu2", "rwkvq_sigmoid_gate", "rwkvq_linear_dispatch_post", "rwkvq_linear_dispatch_plan", "rwkvq_rkv_wkv", "rwkvq_proxy_static",
           "rwkvq_set_option", "rwkvq_get_option", "rwkvq_proxy_workspace_size"]


class rwkvq_mix_input(Structure):
    _fields_ = [("x", c_void_p), ("x_prev", c_void_p), ("indices", c_void_p), ("codebook", c_void_p),
                ("kbits", c_int32), ("reserved", c_int32)]


class rwkvq_post_mix(Structure):
    _fields_ = [("indices", c_void_p), ("codebook", c_void_p), ("out", c_void_p), ("kbits", c_int32), ("reserved", c_int32)]


class rwkvq_post_op(Structure):
    _fields_ = [("op", c_int32), ("n_mix", c_int32), ("gate", c_void_p), ("x_prev", c_void_p), ("mix", rwkvq_post_mix * 4)]


POST_NONE, POST_RELU2, POST_SIGMOID_GATE = 0, 1, 2


class rwkvq_matrix(Structure):
    _fields_ = [("kind", c_int32), ("layout", c_int32), ("N", c_int32), ("K", c_int32),
                ("bits", c_int32), ("group", c_int32),
                ("vdim", c_int32), ("kbits", c_int32), ("block_rows", c_int32), ("block_cols", c_int32),
                ("codes", c_void_p), ("scales", c_void_p), ("zeros", c_void_p), ("codebooks", c_void_p)]


class RwkvqError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"rwkvq status {status}: {status_string(status)}")


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load librwkvq.so (compiling it with hipcc only if no built library exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        # The tensors and streams passed in come from PyTorch's HIP runtime: load it first, so
        # that the library binds to that copy of the runtime and not to a second one of its own
        # (kernels launched through another copy on torch's streams fail with a launch error).
        import torch  # noqa: F401
        L = ctypes.CDLL(_build.LIB)
        L.rwkvq_version.restype = c_int
        L.rwkvq_version.argtypes = []
        L.rwkvq_status_string.restype = c_char_p
        L.rwkvq_status_string.argtypes = [c_int]
        L.rwkvq_set_option.restype = c_int
        L.rwkvq_set_option.argtypes = [c_int, c_int]
        L.rwkvq_get_option.restype = c_int
        L.rwkvq_get_option.argtypes = [c_int, POINTER(c_int)]
        L.rwkvq_sq_prepack.restype = c_int
        L.rwkvq_sq_prepack.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p,
                                       c_void_p, c_void_p]
        L.rwkvq_vq_prepack.restype = c_int
        L.rwkvq_vq_prepack.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p]
        L.rwkvq_sq_dequant.restype = c_int
        L.rwkvq_sq_dequant.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int,
                                       c_void_p, c_int, c_void_p]
        L.rwkvq_vq_dequant.restype = c_int
        L.rwkvq_vq_dequant.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_int,
                                       c_void_p, c_int, c_void_p]
        L.rwkvq_sq_gemm.restype = c_int
        L.rwkvq_sq_gemm.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_int, c_int,
                                    c_int, c_int, c_int, c_int, c_int, c_void_p]
        L.rwkvq_vq_gemm.restype = c_int
        L.rwkvq_vq_gemm.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_int, c_int, c_int,
                                    c_int, c_int, c_int, c_int, c_int, c_int, c_void_p]
        L.rwkvq_linear_dispatch.restype = c_int
        L.rwkvq_linear_dispatch.argtypes = [POINTER(rwkvq_matrix), POINTER(c_void_p), POINTER(c_void_p),
                                            c_int, c_int, c_int, c_int, c_void_p]
        L.rwkvq_proxy_workspace_bytes.restype = c_size_t
        L.rwkvq_proxy_workspace_bytes.argtypes = [c_int]
        L.rwkvq_proxy_workspace_size.restype = c_size_t
        L.rwkvq_proxy_workspace_size.argtypes = [POINTER(c_int), POINTER(c_int), c_int, c_int]
        L.rwkvq_proxy.restype = c_int
        L.rwkvq_proxy.argtypes = [POINTER(c_void_p), POINTER(c_int), POINTER(c_int), c_int, c_int, c_int,
                                  c_double, c_double, c_void_p, c_void_p, c_void_p, c_void_p]
        L.rwkvq_proxy_static.restype = c_int
        L.rwkvq_proxy_static.argtypes = [POINTER(c_void_p), POINTER(c_int), POINTER(c_int), c_int, c_int, c_int,
                                         c_double, c_double, c_void_p, c_void_p, c_void_p]
        L.rwkvq_sq_encode.restype = c_int
        L.rwkvq_sq_encode.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                      c_void_p]
        L.rwkvq_vq_assign.restype = c_int
        L.rwkvq_vq_assign.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int,
                                      c_void_p, c_void_p]
        L.rwkvq_clip_mean.restype = c_int
        L.rwkvq_clip_mean.argtypes = [c_void_p, c_int, c_int, c_int, c_double, c_void_p, c_void_p]
        L.rwkvq_mu_codebook.restype = c_int
        L.rwkvq_mu_codebook.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p,
                                        c_void_p]
        L.rwkvq_token_shift_mix.restype = c_int
        L.rwkvq_token_shift_mix.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p, c_void_p, c_int, c_int,
                                            c_void_p, c_void_p]
        L.rwkvq_linear_dispatch_mixed.restype = c_int
        L.rwkvq_linear_dispatch_mixed.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_void_p]
        L.rwkvq_linear_dispatch_post.restype = c_int
        L.rwkvq_linear_dispatch_post.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int,
                                                 c_void_p]
        L.rwkvq_linear_dispatch_plan.restype = c_int
        L.rwkvq_linear_dispatch_plan.argtypes = [c_void_p, c_int, c_int, c_void_p]
        L.rwkvq_rkv_wkv.restype = c_int
        L.rwkvq_rkv_wkv.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int,
                                    c_void_p]
        L.rwkvq_wkv.restype = c_int
        L.rwkvq_wkv.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                c_void_p, c_void_p]
        L.rwkvq_relu2.restype = c_int
        L.rwkvq_relu2.argtypes = [c_void_p, c_int, c_longlong, c_void_p, c_void_p]
        L.rwkvq_sigmoid_gate.restype = c_int
        L.rwkvq_sigmoid_gate.argtypes = [c_void_p, c_void_p, c_int, c_longlong, c_void_p, c_void_p]
        _lib = L
    return _lib


(OPT_SMALL_BATCH_PATH, OPT_PREFILL_TILE_ROWS, OPT_STREAM_WIDE_GBPS, OPT_STREAM_NARROW_GBPS, OPT_STREAM_WIDE_MIN_US,
 OPT_STREAM_NARROW_MIN_US, OPT_MFMA_KSTEP_NS, OPT_STREAM_TWO_PASS_MIN_WGS, OPT_STREAM_SPLIT_MAX_WORK,
 OPT_SPLIT_GRID_2D) = range(10)
SMALL_BATCH_AUTO, SMALL_BATCH_STREAM, SMALL_BATCH_MATRIX_CORES = 0, 1, 2


def rwkvq_set_option(option: int, value: int, check=True):
    st = lib().rwkvq_set_option(option, value)
    return _check(st) if check else st


def rwkvq_get_option(option: int) -> int:
    v = c_int(0)
    _check(lib().rwkvq_get_option(option, ctypes.byref(v)))
    return int(v.value)


def status_string(status: int) -> str:
    return lib().rwkvq_status_string(status).decode()


def version() -> int:
    return int(lib().rwkvq_version())


def _check(st: int) -> None:
    if st != OK:
        raise RwkvqError(st)


def _ptr(t) -> Optional[int]:
    """Device address of a tensor (or pass through ints / None)."""
    if t is None or isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    return stream if isinstance(stream, int) else stream.cuda_stream


# ---- raw entry points (names as in the header); `check=False` returns the status instead --------

def rwkvq_sq_prepack(codes, scales, zeros, N, K, bits, group, codes_native, sz_native, stream=None,
                     check=True):
    st = lib().rwkvq_sq_prepack(_ptr(codes), _ptr(scales), _ptr(zeros), N, K, bits, group,
                                _ptr(codes_native), _ptr(sz_native), _stream(stream))
    return _check(st) if check else st


def rwkvq_vq_prepack(indices, N, K, vdim, kbits, indices_native, stream=None, check=True):
    st = lib().rwkvq_vq_prepack(_ptr(indices), N, K, vdim, kbits, _ptr(indices_native), _stream(stream))
    return _check(st) if check else st


def rwkvq_sq_dequant(codes, scales, zeros, layout, N, K, bits, group, w_out, w_dtype, stream=None,
                     check=True):
    st = lib().rwkvq_sq_dequant(_ptr(codes), _ptr(scales), _ptr(zeros), layout, N, K, bits, group,
                                _ptr(w_out), w_dtype, _stream(stream))
    return _check(st) if check else st


def rwkvq_vq_dequant(indices, codebooks, layout, N, K, vdim, kbits, block_rows, block_cols, w_out,
                     w_dtype, stream=None, check=True):
    st = lib().rwkvq_vq_dequant(_ptr(indices), _ptr(codebooks), layout, N, K, vdim, kbits, block_rows,
                                block_cols, _ptr(w_out), w_dtype, _stream(stream))
    return _check(st) if check else st


def rwkvq_sq_gemm(codes, scales, zeros, layout, x, y, M, N, K, bits, group, x_dtype, y_dtype,
                  stream=None, check=True):
    st = lib().rwkvq_sq_gemm(_ptr(codes), _ptr(scales), _ptr(zeros), layout, _ptr(x), _ptr(y), M, N, K,
                             bits, group, x_dtype, y_dtype, _stream(stream))
    return _check(st) if check else st


def rwkvq_vq_gemm(indices, codebooks, layout, x, y, M, N, K, vdim, kbits, block_rows, block_cols,
                  x_dtype, y_dtype, stream=None, check=True):
    st = lib().rwkvq_vq_gemm(_ptr(indices), _ptr(codebooks), layout, _ptr(x), _ptr(y), M, N, K, vdim,
                             kbits, block_rows, block_cols, x_dtype, y_dtype, _stream(stream))
    return _check(st) if check else st


def rwkvq_proxy_workspace_bytes(n_mats: int) -> int:
    return int(lib().rwkvq_proxy_workspace_bytes(n_mats))


class ProxyTable:
    """Host arrays for rwkvq_proxy (device pointers and shapes of the matrices), reusable."""

    def __init__(self, ws: Sequence, shapes: Sequence):
        n = len(ws)
        assert len(shapes) == n
        self.n = n
        self.ws = (c_void_p * n)(*[_ptr(w) for w in ws])
        self.Ns = (c_int * n)(*[int(s[0]) for s in shapes])
        self.Ks = (c_int * n)(*[int(s[1]) for s in shapes])


def rwkvq_proxy(table: ProxyTable, w_dtype, terms, tau_c, tau_f, workspace, proxies, phi, stream=None,
                check=True):
    st = lib().rwkvq_proxy(table.ws, table.Ns, table.Ks, table.n, w_dtype, terms, tau_c, tau_f,
                           _ptr(workspace), _ptr(proxies), _ptr(phi), _stream(stream))
    return _check(st) if check else st


def rwkvq_proxy_static(table: ProxyTable, w_dtype, terms, tau_c, tau_f, proxies, phi, stream=None, check=True):
    st = lib().rwkvq_proxy_static(table.ws, table.Ns, table.Ks, table.n, w_dtype, terms, tau_c, tau_f,
                                  _ptr(proxies), _ptr(phi), _stream(stream))
    return _check(st) if check else st


def rwkvq_sq_encode(w, w_dtype, N, K, bits, group, codes, scales, zeros, stream=None, check=True):
    st = lib().rwkvq_sq_encode(_ptr(w), w_dtype, N, K, bits, group, _ptr(codes), _ptr(scales), _ptr(zeros),
                               _stream(stream))
    return _check(st) if check else st


def rwkvq_vq_assign(w, w_dtype, codebooks, N, K, vdim, kbits, block_rows, block_cols, indices, stream=None,
                    check=True):
    st = lib().rwkvq_vq_assign(_ptr(w), w_dtype, _ptr(codebooks), N, K, vdim, kbits, block_rows, block_cols,
                               _ptr(indices), _stream(stream))
    return _check(st) if check else st


def rwkvq_clip_mean(x, x_dtype, n_samples, n, percentile, xbar, stream=None, check=True):
    st = lib().rwkvq_clip_mean(_ptr(x), x_dtype, n_samples, n, float(percentile), _ptr(xbar), _stream(stream))
    return _check(st) if check else st


def _ptr_array(items):
    return (c_void_p * len(items))(*[_ptr(t) for t in items])


def rwkvq_mu_codebook(mus, xbars, n_elems, mu_dtype, kbits, iters, codebooks, indices, stream=None, check=True):
    """mus, xbars, codebooks, indices: sequences of device tensors (one per weight tensor)."""
    n = len(mus)
    st = lib().rwkvq_mu_codebook(_ptr_array(mus), _ptr_array(xbars), (c_int * n)(*[int(v) for v in n_elems]), n,
                                 mu_dtype, kbits, iters, _ptr_array(codebooks), _ptr_array(indices), _stream(stream))
    return _check(st) if check else st


class MixTable:
    """Host arrays for rwkvq_token_shift_mix (indices, codebooks and outputs of the projections)."""

    def __init__(self, indices: Sequence, codebooks: Sequence, outs: Sequence):
        assert len(indices) == len(codebooks) == len(outs)
        self.n = len(indices)
        self.idx, self.cb, self.out = _ptr_array(indices), _ptr_array(codebooks), _ptr_array(outs)
        self.keep = (indices, codebooks, outs)


def rwkvq_token_shift_mix(x, x_prev, x_dtype, M, d, table: MixTable, kbits, stream=None, check=True):
    st = lib().rwkvq_token_shift_mix(_ptr(x), _ptr(x_prev), x_dtype, M, d, table.idx, table.cb, kbits, table.n,
                                     table.out, _stream(stream))
    return _check(st) if check else st


class MixedDispatchTable:
    """Host arrays for rwkvq_linear_dispatch_mixed: per matrix its descriptor, (x, x_prev, indices,
    codebook, kbits) of the mix in front of it, and the output."""

    def __init__(self, descs: Sequence, mixes: Sequence, ys: Sequence):
        n = len(descs)
        assert len(mixes) == n and len(ys) == n
        self.n = n
        self.mats = (rwkvq_matrix * n)(*descs)
        self.mixes = (rwkvq_mix_input * n)(*[rwkvq_mix_input(_ptr(x), _ptr(xp), _ptr(ix), _ptr(cb), int(kb), 0)
                                             for x, xp, ix, cb, kb in mixes])
        self.ys = _ptr_array(ys)
        self.keep = (mixes, ys)


def rwkvq_linear_dispatch_mixed(table: MixedDispatchTable, x_dtype, y_dtype, stream=None, check=True):
    st = lib().rwkvq_linear_dispatch_mixed(table.mats, table.mixes, table.ys, table.n, x_dtype, y_dtype, _stream(stream))
    return _check(st) if check else st


class DispatchTable:
    """Host arrays for rwkvq_linear_dispatch, built once and reusable across calls."""

    def __init__(self, descs: Sequence[rwkvq_matrix], xs: Sequence, ys: Sequence):
        n = len(descs)
        assert len(xs) == n and len(ys) == n
        self.n = n
        self.mats = (rwkvq_matrix * n)(*descs)
        self.xs = (c_void_p * n)(*[_ptr(x) for x in xs])
        self.ys = (c_void_p * n)(*[_ptr(y) for y in ys])


def rwkvq_linear_dispatch(table: DispatchTable, M, x_dtype, y_dtype, stream=None, check=True):
    st = lib().rwkvq_linear_dispatch(table.mats, table.xs, table.ys, table.n, M, x_dtype, y_dtype,
                                     _stream(stream))
    return _check(st) if check else st


# ---- device-side holder of one matrix (memory plumbing for tests, smoke and bench) ---------------

@dataclass
class DeviceMatrix:
    kind: int
    layout: int
    N: int
    K: int
    kbits: int
    codes: object                 # torch tensors on the GPU
    scales: object = None
    zeros: object = None
    codebooks: object = None
    packed_bytes: int = 0

    def desc(self) -> rwkvq_matrix:
        d = rwkvq_matrix()
        d.kind, d.layout, d.N, d.K = self.kind, self.layout, self.N, self.K
        d.bits, d.group = 3, 128
        d.vdim, d.kbits, d.block_rows, d.block_cols = 2, self.kbits, 256, 256
        d.codes = _ptr(self.codes)
        d.scales = _ptr(self.scales)
        d.zeros = _ptr(self.zeros)
        d.codebooks = _ptr(self.codebooks)
        return d


def upload(mat, native: bool = True, device: str = "cuda:0") -> DeviceMatrix:
    """Copy a canonical-layout matrix record (fields kind, N, K, kbits, codes, scales, zeros,
    codebooks as numpy arrays) to the GPU; with native=True also run the library's prepack and
    keep only the native buffers."""
    import numpy as np
    import torch

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int32 if a.dtype == np.uint32 else np.int16)).to(device)

    codes = dev(mat.codes)
    if mat.kind == "sq":
        scales, zeros = dev(mat.scales), dev(mat.zeros)
        if not native:
            return DeviceMatrix(SQ, CANONICAL, mat.N, mat.K, 0, codes, scales, zeros, None, mat.packed_bytes)
        cn = torch.empty_like(codes)
        sz = torch.empty(scales.numel() * 2, dtype=torch.int16, device=device)
        rwkvq_sq_prepack(codes, scales, zeros, mat.N, mat.K, 3, 128, cn, sz)
        torch.cuda.synchronize()
        return DeviceMatrix(SQ, NATIVE, mat.N, mat.K, 0, cn, sz, None, None, mat.packed_bytes)
    cb = dev(mat.codebooks)
    if not native:
        return DeviceMatrix(VQ, CANONICAL, mat.N, mat.K, mat.kbits, codes, None, None, cb, mat.packed_bytes)
    cn = torch.empty_like(codes)
    rwkvq_vq_prepack(codes, mat.N, mat.K, 2, mat.kbits, cn)
    torch.cuda.synchronize()
    return DeviceMatrix(VQ, NATIVE, mat.N, mat.K, mat.kbits, cn, None, None, cb, mat.packed_bytes)


def dequant(dm: DeviceMatrix, w_dtype: int = F32, stream=None):
    """Dense Deq(W) [N, K] on the GPU as a torch tensor (float32, or int16 bit patterns)."""
    import torch
    out = torch.empty((dm.N, dm.K), dtype=torch.float32 if w_dtype == F32 else torch.int16,
                      device=dm.codes.device)
    if dm.kind == SQ:
        rwkvq_sq_dequant(dm.codes, dm.scales, dm.zeros, dm.layout, dm.N, dm.K, 3, 128, out, w_dtype, stream)
    else:
        rwkvq_vq_dequant(dm.codes, dm.codebooks, dm.layout, dm.N, dm.K, 2, dm.kbits, 256, 256, out, w_dtype,
                         stream)
    return out


def gemm(dm: DeviceMatrix, x, M: int, x_dtype: int, y_dtype: int = F32, stream=None):
    """y [M, N] = x [M, K] Deq(W)^T through rwkvq_sq_gemm / rwkvq_vq_gemm; x is an int16 tensor
    of fp16 / bf16 bit patterns on the GPU."""
    import torch
    y = torch.empty((M, dm.N), dtype=torch.float32 if y_dtype == F32 else torch.int16, device=x.device)
    if dm.kind == SQ:
        rwkvq_sq_gemm(dm.codes, dm.scales, dm.zeros, dm.layout, x, y, M, dm.N, dm.K, 3, 128, x_dtype,
                      y_dtype, stream)
    else:
        rwkvq_vq_gemm(dm.codes, dm.codebooks, dm.layout, x, y, M, dm.N, dm.K, 2, dm.kbits, 256, 256,
                      x_dtype, y_dtype, stream)
    return y


def rwkvq_proxy_workspace_size(table: "ProxyTable", w_dtype: int) -> int:
    return int(lib().rwkvq_proxy_workspace_size(table.Ns, table.Ks, table.n, w_dtype))


def proxy(ws, w_dtype: int, terms: int = 5, tau_c: float = 1.5, tau_f: float = 50.0, stream=None):
    """[(P_c, P_f, phi)] of dense weight matrices through one rwkvq_proxy call; ws is a list of 2-D
    tensors on the GPU (int16 bit patterns of fp16 / bf16 values, or float32).  Synchronises to read
    the results back."""
    import torch
    dev = ws[0].device
    table = ProxyTable(ws, [tuple(w.shape) for w in ws])
    workspace = torch.empty((rwkvq_proxy_workspace_size(table, w_dtype) + 3) // 4, dtype=torch.int32, device=dev)
    out = torch.empty(2 * table.n, dtype=torch.float64, device=dev)
    flag = torch.empty(table.n + 3, dtype=torch.int32, device=dev)
    rwkvq_proxy(table, w_dtype, terms, tau_c, tau_f, workspace, out, flag, stream)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    f = flag.cpu().numpy()
    return [(float(o[2 * i]), float(o[2 * i + 1]), int(f[i])) for i in range(table.n)]


def sq_encode(w, w_dtype: int, stream=None) -> DeviceMatrix:
    """Round-to-nearest SQ of a dense [N][K] tensor on the GPU (int16 bit patterns or float32) ->
    canonical-layout DeviceMatrix."""
    import torch
    N, K = w.shape
    codes = torch.empty((N, 3 * K // 32), dtype=torch.int32, device=w.device)
    scales = torch.empty((N, K // 128), dtype=torch.int16, device=w.device)
    zeros = torch.empty((N, K // 128), dtype=torch.int16, device=w.device)
    rwkvq_sq_encode(w, w_dtype, N, K, 3, 128, codes, scales, zeros, stream)
    return DeviceMatrix(SQ, CANONICAL, N, K, 0, codes, scales, zeros, None, codes.numel() * 4 + scales.numel() * 4)


def vq_assign(w, w_dtype: int, codebooks, kbits: int, stream=None) -> DeviceMatrix:
    """Nearest-entry VQ assignment of a dense [N][K] tensor against given codebooks (int16 fp16 bit
    patterns, [N/256][K/256][2^kbits][2]) -> canonical-layout DeviceMatrix."""
    import torch
    N, K = w.shape
    idx = torch.empty((N, K // 2 * kbits // 32), dtype=torch.int32, device=w.device)
    rwkvq_vq_assign(w, w_dtype, codebooks, N, K, 2, kbits, 256, 256, idx, stream)
    return DeviceMatrix(VQ, CANONICAL, N, K, kbits, idx, None, None, codebooks, idx.numel() * 4 + codebooks.numel() * 2)


def rwkvq_wkv(r, k, v, x_dtype, M, d, w, u, state, out, stream=None, check=True):
    st = lib().rwkvq_wkv(_ptr(r), _ptr(k), _ptr(v), x_dtype, M, d, _ptr(w), _ptr(u), _ptr(state), _ptr(out),
                         _stream(stream))
    return _check(st) if check else st


def rwkvq_relu2(x, x_dtype, n, out, stream=None, check=True):
    st = lib().rwkvq_relu2(_ptr(x), x_dtype, n, _ptr(out), _stream(stream))
    return _check(st) if check else st


def rwkvq_sigmoid_gate(r, y, x_dtype, n, out, stream=None, check=True):
    st = lib().rwkvq_sigmoid_gate(_ptr(r), _ptr(y), x_dtype, n, _ptr(out), _stream(stream))
    return _check(st) if check else st


def _post_op(p) -> rwkvq_post_op:
    """(op, gate) or (op, gate, x_prev, [(indices, codebook, kbits, out), ...]) -> rwkvq_post_op."""
    o = rwkvq_post_op()
    o.op, o.gate = int(p[0]), _ptr(p[1])
    if len(p) > 2 and p[3]:
        o.x_prev, o.n_mix = _ptr(p[2]), len(p[3])
        for q, (ix, cb, kb, out) in enumerate(p[3]):
            o.mix[q] = rwkvq_post_mix(_ptr(ix), _ptr(cb), _ptr(out), int(kb), 0)
    return o


class PostDispatchTable:
    """Host arrays for rwkvq_linear_dispatch_post: descriptors, inputs (xs: device tensors, or mixes:
    (x, x_prev, indices, codebook, kbits) per matrix), posts: (op, gate tensor or None) per matrix, or
    (op, gate, x_prev, [(indices, codebook, kbits, out), ...]) to have the output also stored as mixes."""

    def __init__(self, descs: Sequence, xs: Optional[Sequence], mixes: Optional[Sequence], posts: Sequence, ys: Sequence):
        n = len(descs)
        assert len(posts) == n and len(ys) == n and (xs is None or len(xs) == n) and (mixes is None or len(mixes) == n)
        self.n = n
        self.mats = (rwkvq_matrix * n)(*descs)
        self.xs = _ptr_array(xs) if xs is not None else None
        self.mixes = None if mixes is None else (rwkvq_mix_input * n)(
            *[rwkvq_mix_input(_ptr(x), _ptr(xp), _ptr(ix), _ptr(cb), int(kb), 0) for x, xp, ix, cb, kb in mixes])
        self.posts = (rwkvq_post_op * n)(*[_post_op(p) for p in posts])
        self.ys = _ptr_array(ys)
        self.keep = (xs, mixes, posts, ys)


def rwkvq_linear_dispatch_post(table: PostDispatchTable, x_dtype, y_dtype, stream=None, check=True):
    st = lib().rwkvq_linear_dispatch_post(table.mats, table.xs, table.mixes, table.posts, table.ys, table.n, x_dtype,
                                          y_dtype, _stream(stream))
    return _check(st) if check else st


PATH_REFERENCE, PATH_STREAM, PATH_STREAM_PASSES, PATH_MATRIX_CORES = 0, 1, 2, 3


def rwkvq_linear_dispatch_plan(descs: Sequence, M: int, check=True):
    """The path (PATH_*) each matrix of a dispatch call with these descriptors and this M would take."""
    n = len(descs)
    mats = (rwkvq_matrix * n)(*descs)
    paths = (c_int32 * n)()
    st = lib().rwkvq_linear_dispatch_plan(mats, n, M, paths)
    if check:
        _check(st)
        return list(paths)
    return st


class RkvWkvTable:
    """Host arrays for rwkvq_rkv_wkv: the descriptors of r, k, v, their inputs and outputs."""

    def __init__(self, descs: Sequence, xs: Sequence, ys: Sequence):
        assert len(descs) == 3 and len(xs) == 3 and len(ys) == 3
        self.mats = (rwkvq_matrix * 3)(*descs)
        self.xs = _ptr_array(xs)
        self.ys = _ptr_array(ys)
        self.keep = (xs, ys)


def rwkvq_rkv_wkv(table: RkvWkvTable, w, u, state, out, x_dtype, y_dtype, stream=None, check=True):
    st = lib().rwkvq_rkv_wkv(table.mats, table.xs, table.ys, _ptr(w), _ptr(u), _ptr(state), _ptr(out), x_dtype, y_dtype,
                             _stream(stream))
    return _check(st) if check else st
