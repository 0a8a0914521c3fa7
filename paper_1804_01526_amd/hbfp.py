"""Thin ctypes binding of ``libhbfp.so``: same names as the C ABI, argument marshalling only.

PyTorch supplies device memory (``tensor.data_ptr()``) and the HIP stream; every
step of the path runs in the library's kernels.  There is no CPU fallback: if the
library has not been built, importing this module fails.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhbfp.so")

OK, ERR_ARG, ERR_FORMAT, ERR_LAYOUT, ERR_RANGE, ERR_LAUNCH, ERR_WORKSPACE = 0, -1, -2, -3, -4, -5, -6
RNE, STOCHASTIC = 0, 1
HINT_HEAVY_TAILS = 1


class HbfpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class Format(ctypes.Structure):
    """hbfp_format: how a source matrix is cut into exponent blocks."""
    _fields_ = [("mant_bits", ctypes.c_int32), ("rounding", ctypes.c_int32),
                ("block_rows", ctypes.c_int64), ("block_cols", ctypes.c_int64), ("seed", ctypes.c_uint64),
                ("k_slot", ctypes.c_int64)]


class Conv2d(ctypes.Structure):
    """hbfp_conv2d: NHWC input, filter r x s, zero padding and strides."""
    _fields_ = [("n", ctypes.c_int64), ("h", ctypes.c_int64), ("w", ctypes.c_int64), ("c", ctypes.c_int64),
                ("r", ctypes.c_int32), ("s", ctypes.c_int32), ("pad_h", ctypes.c_int32), ("pad_w", ctypes.c_int32),
                ("stride_h", ctypes.c_int32), ("stride_w", ctypes.c_int32), ("c_block", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]

    def out_hw(self):
        return ((self.h + 2 * self.pad_h - self.r) // self.stride_h + 1, (self.w + 2 * self.pad_w - self.s) // self.stride_w + 1)


class EncodeJob(ctypes.Structure):
    """hbfp_encode_job: one source of hbfp_encode_packed_batch."""
    _fields_ = [("src", ctypes.c_void_p), ("ld", ctypes.c_int64), ("n", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("outs", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("packed_bytes", ctypes.c_void_p)]


class TensorDesc(ctypes.Structure):
    """hbfp_tensor: an encoded operand (layout in include/hbfp.h)."""
    _fields_ = [("mant", ctypes.c_void_p), ("exps", ctypes.c_void_p),
                ("rows", ctypes.c_int64), ("kdim", ctypes.c_int64), ("kblock", ctypes.c_int64),
                ("kblock_pad", ctypes.c_int64), ("nblk", ctypes.c_int64), ("kpad", ctypes.c_int64),
                ("exp_ld", ctypes.c_int64), ("rblock", ctypes.c_int64), ("kshare", ctypes.c_int64),
                ("src_rows", ctypes.c_int64), ("src_cols", ctypes.c_int64),
                ("contract_axis", ctypes.c_int32), ("mant_bits", ctypes.c_int32),
                ("rounding", ctypes.c_int32), ("hints", ctypes.c_int32),
                ("seed", ctypes.c_uint64), ("mant_bytes", ctypes.c_uint64), ("exp_bytes", ctypes.c_uint64)]


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    F, T = ctypes.POINTER(Format), ctypes.POINTER(TensorDesc)
    lib.hbfp_version.restype = i32
    lib.hbfp_status_string.restype = ctypes.c_char_p
    lib.hbfp_status_string.argtypes = [i32]
    lib.hbfp_plan.argtypes = [F, i64, i64, i32, T]
    lib.hbfp_sizes.argtypes = [F, i64, i64, i32, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(i64)]
    lib.hbfp_sizes.restype = i32
    lib.hbfp_encode_workspace.argtypes = [T, ctypes.POINTER(sz)]
    lib.hbfp_encode.argtypes = [vp, i64, i64, i64, i32, F, T, vp, sz, vp]
    lib.hbfp_encode_static.argtypes = [vp, i64, i64, i64, i32, F, T, vp]
    lib.hbfp_encode_static_limit.restype = sz
    lib.hbfp_encode_static_limit.argtypes = []
    lib.hbfp_decode.argtypes = [T, vp, i64, vp]
    lib.hbfp_encode_im2col.argtypes = [vp, ctypes.POINTER(Conv2d), T, vp, sz, vp]
    lib.hbfp_encode_im2col_workspace.argtypes = [ctypes.POINTER(Conv2d), T, ctypes.POINTER(sz)]
    lib.hbfp_encode_im2col_workspace.restype = i32
    lib.hbfp_gemm_conv2d_workspace.argtypes = [T, ctypes.POINTER(Conv2d), T, ctypes.POINTER(sz)]
    lib.hbfp_gemm_conv2d_workspace.restype = i32
    lib.hbfp_gemm_conv2d.argtypes = [T, ctypes.POINTER(Conv2d), T, vp, i64, ctypes.c_float, vp, sz, vp]
    lib.hbfp_gemm_conv2d.restype = i32
    lib.hbfp_gemm_conv2d_bfp_workspace.argtypes = [T, ctypes.POINTER(Conv2d), T, T, ctypes.POINTER(sz)]
    lib.hbfp_gemm_conv2d_bfp_workspace.restype = i32
    lib.hbfp_gemm_conv2d_bfp.argtypes = [T, ctypes.POINTER(Conv2d), T, T, i32, vp, sz, vp]
    lib.hbfp_gemm_conv2d_bfp.restype = i32
    lib.hbfp_gemm_conv2d_dgrad_workspace.argtypes = [T, ctypes.POINTER(Conv2d), T, ctypes.POINTER(sz)]
    lib.hbfp_gemm_conv2d_dgrad_workspace.restype = i32
    lib.hbfp_gemm_conv2d_dgrad.argtypes = [T, ctypes.POINTER(Conv2d), T, vp, i64, ctypes.c_float, vp, sz, vp]
    lib.hbfp_gemm_conv2d_dgrad.restype = i32
    lib.hbfp_gemm_workspace.argtypes = [T, T, ctypes.POINTER(sz)]
    lib.hbfp_gemm.argtypes = [T, T, vp, i64, ctypes.c_float, vp, sz, vp]
    lib.hbfp_gemm_select_workspace.argtypes = [T, T, i32, ctypes.POINTER(sz)]
    lib.hbfp_gemm_select.argtypes = [T, T, vp, i64, ctypes.c_float, i32, vp, sz, vp]
    lib.hbfp_gemm_batch_workspace.argtypes = [i32, ctypes.POINTER(T), ctypes.POINTER(T), i32, ctypes.POINTER(sz)]
    lib.hbfp_gemm_batch.argtypes = [i32, ctypes.POINTER(T), ctypes.POINTER(T), ctypes.POINTER(vp), ctypes.POINTER(i64),
                                    ctypes.c_float, i32, vp, sz, vp]
    lib.hbfp_gemm_bfp_workspace.argtypes = [T, T, T, i32, ctypes.POINTER(sz)]
    lib.hbfp_gemm_bfp.argtypes = [T, T, T, i32, i32, vp, sz, vp]
    lib.hbfp_pack_bytes.argtypes = [T, ctypes.POINTER(sz)]
    lib.hbfp_pack.argtypes = [T, vp, sz, vp]
    lib.hbfp_gemm_packed_workspace.argtypes = [T, T, ctypes.POINTER(sz)]
    lib.hbfp_gemm_packed.argtypes = [T, vp, T, vp, vp, i64, ctypes.c_float, vp, sz, vp]
    lib.hbfp_gemm_packed_batch_workspace.argtypes = [i32, ctypes.POINTER(T), ctypes.POINTER(T), ctypes.POINTER(sz)]
    lib.hbfp_gemm_packed_batch.argtypes = [i32, ctypes.POINTER(T), ctypes.POINTER(vp), ctypes.POINTER(T), ctypes.POINTER(vp),
                                           ctypes.POINTER(vp), ctypes.POINTER(i64), ctypes.c_float, vp, sz, vp]
    lib.hbfp_gemm_partials.argtypes = [T, T, vp, vp, sz, vp]
    lib.hbfp_gemm_partials_window.argtypes = [T, T, i64, i64, i64, i64, vp, vp, sz, vp]
    lib.hbfp_gemm_f32_workspace.argtypes = [i32, i32, i64, i64, i64, F, F, ctypes.POINTER(sz)]
    lib.hbfp_gemm_f32.argtypes = [i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, F, F, vp, sz, vp]
    lib.hbfp_encode_multi_workspace.argtypes = [i32, ctypes.POINTER(T), ctypes.POINTER(sz)]
    lib.hbfp_encode_multi.argtypes = [vp, i64, i32, ctypes.POINTER(T), vp, sz, vp]
    lib.hbfp_encode_packed_workspace.argtypes = [i32, ctypes.POINTER(T), ctypes.POINTER(sz)]
    lib.hbfp_encode_packed.argtypes = [vp, i64, i32, ctypes.POINTER(T), ctypes.POINTER(vp), ctypes.POINTER(sz), vp, sz, vp]
    lib.hbfp_encode_packed_batch_workspace.argtypes = [i32, ctypes.POINTER(EncodeJob), ctypes.POINTER(sz)]
    lib.hbfp_encode_packed_batch.argtypes = [i32, ctypes.POINTER(EncodeJob), vp, sz, vp]
    lib.hbfp_probe_matrix_rate.argtypes = [i32, vp, i32, i32, vp, vp, vp]
    lib.hbfp_probe_matrix_rate.restype = i32
    lib.hbfp_weight_update_workspace.argtypes = [T, T, T, ctypes.POINTER(sz)]
    lib.hbfp_weight_update.argtypes = [T, vp, i64, ctypes.c_float, T, T, vp, sz, vp]
    for name in ("hbfp_gemm_batch_workspace", "hbfp_gemm_batch", "hbfp_gemm_bfp_workspace", "hbfp_gemm_bfp", "hbfp_encode_im2col", "hbfp_encode_multi_workspace", "hbfp_encode_multi", "hbfp_encode_packed_workspace", "hbfp_encode_packed", "hbfp_encode_packed_batch_workspace", "hbfp_encode_packed_batch", "hbfp_weight_update_workspace", "hbfp_weight_update", "hbfp_plan", "hbfp_encode_workspace", "hbfp_encode", "hbfp_encode_static", "hbfp_decode", "hbfp_gemm_workspace",
                 "hbfp_gemm", "hbfp_gemm_select_workspace", "hbfp_gemm_select", "hbfp_pack_bytes", "hbfp_pack",
                 "hbfp_gemm_packed_workspace", "hbfp_gemm_packed", "hbfp_gemm_packed_batch_workspace", "hbfp_gemm_packed_batch", "hbfp_gemm_partials", "hbfp_gemm_partials_window", "hbfp_gemm_f32_workspace",
                 "hbfp_gemm_f32"):
        getattr(lib, name).restype = i32
    return lib


_lib = _load()


def library_path() -> str:
    return _LIB_PATH


def version() -> int:
    return int(_lib.hbfp_version())


def status_string(status: int) -> str:
    return _lib.hbfp_status_string(status).decode()


def _check(rc: int, where: str):
    if rc != OK:
        raise HbfpError(rc, where)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_ptr(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def make_format(mant_bits: int, block_rows: int, block_cols: int, rounding: int = RNE, seed: int = 0,
                k_slot: int = 0) -> Format:
    return Format(mant_bits, rounding, block_rows, block_cols, seed, k_slot)


# ---------------------------------------------------------------------------- C ABI, one to one
def plan(fmt: Format, rows: int, cols: int, contract_axis: int) -> TensorDesc:
    d = TensorDesc()
    _check(_lib.hbfp_plan(ctypes.byref(fmt), rows, cols, contract_axis, ctypes.byref(d)), "hbfp_plan")
    return d


def sizes(fmt: Format, rows: int, cols: int, contract_axis: int):
    """hbfp_sizes: (mantissa bytes, exponent bytes, stored contraction length) of the operand a conversion produces."""
    mb, eb, kp = ctypes.c_size_t(0), ctypes.c_size_t(0), ctypes.c_int64(0)
    _check(_lib.hbfp_sizes(ctypes.byref(fmt), rows, cols, contract_axis, ctypes.byref(mb), ctypes.byref(eb), ctypes.byref(kp)), "hbfp_sizes")
    return int(mb.value), int(eb.value), int(kp.value)


def encode_workspace(desc: TensorDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_encode_workspace(ctypes.byref(desc), ctypes.byref(n)), "hbfp_encode_workspace")
    return int(n.value)


def gemm_workspace(a: TensorDesc, b: TensorDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_gemm_workspace(ctypes.byref(a), ctypes.byref(b), ctypes.byref(n)), "hbfp_gemm_workspace")
    return int(n.value)


def gemm_f32_workspace(trans_a: int, trans_b: int, M: int, N: int, K: int, fa: Format, fb: Format) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_gemm_f32_workspace(trans_a, trans_b, M, N, K, ctypes.byref(fa), ctypes.byref(fb),
                                        ctypes.byref(n)), "hbfp_gemm_f32_workspace")
    return int(n.value)


@dataclass
class BfpTensor:
    """An encoded operand: the descriptor plus the torch buffers that back its two pointers."""
    desc: TensorDesc
    mant: torch.Tensor   # int8 / int16 [rows, kpad]
    exps: torch.Tensor   # uint8 [rows, exp_ld]


def alloc(fmt: Format, rows: int, cols: int, contract_axis: int, device="cuda") -> BfpTensor:
    d = plan(fmt, rows, cols, contract_axis)
    dt = torch.int8 if d.mant_bits <= 8 else torch.int16
    mant = torch.empty((d.rows, d.kpad), dtype=dt, device=device)
    exps = torch.empty((d.rows, d.exp_ld), dtype=torch.uint8, device=device)
    d.mant, d.exps = mant.data_ptr(), exps.data_ptr()
    return BfpTensor(d, mant, exps)


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return workspace
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return workspace


def encode(src: torch.Tensor, contract_axis: int, fmt: Format, out: Optional[BfpTensor] = None,
           workspace: Optional[torch.Tensor] = None, stream=None) -> BfpTensor:
    """hbfp_encode on a 2-D FP32 device tensor (row stride = its leading dimension)."""
    assert src.is_cuda and src.dtype == torch.float32 and src.dim() == 2 and src.stride(1) == 1
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else max(src.stride(0), cols)
    if out is None:
        out = alloc(fmt, rows, cols, contract_axis, src.device)
    workspace = _workspace(encode_workspace(out.desc), src.device, workspace)
    _check(_lib.hbfp_encode(_dev_ptr(src), rows, cols, ld, contract_axis, ctypes.byref(fmt), ctypes.byref(out.desc),
                            _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                            _stream_ptr(stream)), "hbfp_encode")
    return out


def encode_static_limit() -> int:
    return int(_lib.hbfp_encode_static_limit())


def encode_static(src: torch.Tensor, contract_axis: int, fmt: Format, out: BfpTensor, stream=None) -> BfpTensor:
    """hbfp_encode_static: hbfp_encode whose scratch is a fixed array inside the library (nothing is allocated;
    `out` comes from ``alloc``)."""
    assert src.is_cuda and src.dtype == torch.float32 and src.dim() == 2 and src.stride(1) == 1
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else max(src.stride(0), cols)
    _check(_lib.hbfp_encode_static(_dev_ptr(src), rows, cols, ld, contract_axis, ctypes.byref(fmt), ctypes.byref(out.desc),
                                   _stream_ptr(stream)), "hbfp_encode_static")
    return out


def decode(t: BfpTensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((t.desc.src_rows, t.desc.src_cols), dtype=torch.float32, device=t.mant.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.stride(1) == 1
    _check(_lib.hbfp_decode(ctypes.byref(t.desc), _dev_ptr(out), out.stride(0), _stream_ptr(stream)), "hbfp_decode")
    return out


KERNEL_AUTO, KERNEL_INT8, KERNEL_SCALED, KERNEL_INT8_WIDE, KERNEL_FP16, KERNEL_BF16, KERNEL_FP16_PLANES = 0, 1, 2, 3, 4, 5, 6


def gemm_select_workspace(a: TensorDesc, b: TensorDesc, kernel: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_gemm_select_workspace(ctypes.byref(a), ctypes.byref(b), kernel, ctypes.byref(n)),
           "hbfp_gemm_select_workspace")
    return n.value


def gemm(a: BfpTensor, b: BfpTensor, out: Optional[torch.Tensor] = None, beta: float = 0.0,
         workspace: Optional[torch.Tensor] = None, stream=None, kernel: int = KERNEL_AUTO) -> torch.Tensor:
    """C[M,N] (+)= A . B^T over k (both operands k-contiguous); `kernel` as in hbfp_gemm_select."""
    if out is None:
        out = torch.empty((a.desc.rows, b.desc.rows), dtype=torch.float32, device=a.mant.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.stride(1) == 1
    workspace = _workspace(gemm_select_workspace(a.desc, b.desc, kernel), out.device, workspace)
    _check(_lib.hbfp_gemm_select(ctypes.byref(a.desc), ctypes.byref(b.desc), _dev_ptr(out), out.stride(0), beta, kernel,
                                 _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                                 _stream_ptr(stream)), "hbfp_gemm_select")
    return out


def gemm_batch_workspace(pairs, kernel: int = KERNEL_AUTO) -> int:
    """pairs: sequence of (A, B), each a BfpTensor or a TensorDesc."""
    n = ctypes.c_size_t(0)
    a, b = _desc_array([p[0] for p in pairs]), _desc_array([p[1] for p in pairs])
    _check(_lib.hbfp_gemm_batch_workspace(len(pairs), a, b, kernel, ctypes.byref(n)), "hbfp_gemm_batch_workspace")
    return int(n.value)


def gemm_batch(pairs, outs, beta: float = 0.0, kernel: int = KERNEL_AUTO, workspace: Optional[torch.Tensor] = None, stream=None):
    """hbfp_gemm_batch: outs[i] (+)= A[i] . B[i]^T for up to 4 independent products in one call."""
    n = len(pairs)
    a, b = _desc_array([p[0] for p in pairs]), _desc_array([p[1] for p in pairs])
    for o in outs:
        assert o.is_cuda and o.dtype == torch.float32 and o.stride(1) == 1
    c = (ctypes.c_void_p * n)(*[o.data_ptr() for o in outs])
    ld = (ctypes.c_int64 * n)(*[o.stride(0) for o in outs])
    workspace = _workspace(gemm_batch_workspace(pairs, kernel), outs[0].device, workspace)
    _check(_lib.hbfp_gemm_batch(n, a, b, c, ld, beta, kernel, _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                                _stream_ptr(stream)), "hbfp_gemm_batch")
    return outs


def gemm_bfp_workspace(a: TensorDesc, b: TensorDesc, out: TensorDesc, kernel: int = KERNEL_AUTO) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_gemm_bfp_workspace(ctypes.byref(a), ctypes.byref(b), ctypes.byref(out), kernel, ctypes.byref(n)),
           "hbfp_gemm_bfp_workspace")
    return int(n.value)


def gemm_bfp(a: BfpTensor, b: BfpTensor, fmt: Format, contract_axis: int = 1, relu: bool = False, kernel: int = KERNEL_AUTO,
             out: Optional[BfpTensor] = None, workspace: Optional[torch.Tensor] = None, stream=None) -> BfpTensor:
    """hbfp_gemm_bfp: encode(relu?(A . B^T)) as an operand in format `fmt` (the next product's input)."""
    if out is None:
        out = alloc(fmt, a.desc.rows, b.desc.rows, contract_axis, a.mant.device)
    workspace = _workspace(gemm_bfp_workspace(a.desc, b.desc, out.desc, kernel), a.mant.device, workspace)
    _check(_lib.hbfp_gemm_bfp(ctypes.byref(a.desc), ctypes.byref(b.desc), ctypes.byref(out.desc), int(relu), kernel,
                              _dev_ptr(workspace), 0 if workspace is None else workspace.numel(), _stream_ptr(stream)),
           "hbfp_gemm_bfp")
    return out


def pack_bytes(desc: TensorDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_pack_bytes(ctypes.byref(desc), ctypes.byref(n)), "hbfp_pack_bytes")
    return int(n.value)


def pack(t: BfpTensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Limb planes of an encoded operand for gemm_packed (opaque bytes; pack again after encoding again)."""
    n = pack_bytes(t.desc)
    if out is None:
        out = torch.empty(n, dtype=torch.uint8, device=t.mant.device)
    _check(_lib.hbfp_pack(ctypes.byref(t.desc), _dev_ptr(out), out.numel(), _stream_ptr(stream)), "hbfp_pack")
    return out


def gemm_packed_workspace(a: TensorDesc, b: TensorDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_gemm_packed_workspace(ctypes.byref(a), ctypes.byref(b), ctypes.byref(n)), "hbfp_gemm_packed_workspace")
    return int(n.value)


def gemm_packed(a: BfpTensor, packed_a: torch.Tensor, b: BfpTensor, packed_b: torch.Tensor,
                out: Optional[torch.Tensor] = None, beta: float = 0.0, workspace: Optional[torch.Tensor] = None,
                stream=None) -> torch.Tensor:
    """C[M,N] (+)= A . B^T on the block-scaled kernel from operands packed beforehand."""
    if out is None:
        out = torch.empty((a.desc.rows, b.desc.rows), dtype=torch.float32, device=a.mant.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.stride(1) == 1
    workspace = _workspace(gemm_packed_workspace(a.desc, b.desc), out.device, workspace)
    _check(_lib.hbfp_gemm_packed(ctypes.byref(a.desc), _dev_ptr(packed_a), ctypes.byref(b.desc), _dev_ptr(packed_b),
                                 _dev_ptr(out), out.stride(0), beta, _dev_ptr(workspace),
                                 0 if workspace is None else workspace.numel(), _stream_ptr(stream)), "hbfp_gemm_packed")
    return out


def gemm_packed_batch_workspace(pairs) -> int:
    """pairs: sequence of (A, B), each a BfpTensor or a TensorDesc."""
    n = ctypes.c_size_t(0)
    a, b = _desc_array([p[0] for p in pairs]), _desc_array([p[1] for p in pairs])
    _check(_lib.hbfp_gemm_packed_batch_workspace(len(pairs), a, b, ctypes.byref(n)), "hbfp_gemm_packed_batch_workspace")
    return int(n.value)


def gemm_packed_batch(products, outs, beta: float = 0.0, workspace: Optional[torch.Tensor] = None, stream=None):
    """hbfp_gemm_packed_batch: outs[i] (+)= A[i] . B[i]^T; products: sequence of (A, packed A, B, packed B)."""
    n = len(products)
    a, b = _desc_array([p[0] for p in products]), _desc_array([p[2] for p in products])
    pa = (ctypes.c_void_p * n)(*[p[1].data_ptr() for p in products])
    pb = (ctypes.c_void_p * n)(*[p[3].data_ptr() for p in products])
    for o in outs:
        assert o.is_cuda and o.dtype == torch.float32 and o.stride(1) == 1
    c = (ctypes.c_void_p * n)(*[o.data_ptr() for o in outs])
    ld = (ctypes.c_int64 * n)(*[o.stride(0) for o in outs])
    workspace = _workspace(gemm_packed_batch_workspace([(p[0], p[2]) for p in products]), outs[0].device, workspace)
    _check(_lib.hbfp_gemm_packed_batch(n, a, pa, b, pb, c, ld, beta, _dev_ptr(workspace),
                                       0 if workspace is None else workspace.numel(), _stream_ptr(stream)), "hbfp_gemm_packed_batch")
    return outs


def gemm_partials(a: BfpTensor, b: BfpTensor, workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    P = torch.empty((a.desc.rows, b.desc.rows, a.desc.nblk), dtype=torch.int32, device=a.mant.device)
    workspace = _workspace(gemm_select_workspace(a.desc, b.desc, KERNEL_INT8), P.device, workspace)
    _check(_lib.hbfp_gemm_partials(ctypes.byref(a.desc), ctypes.byref(b.desc), _dev_ptr(P), _dev_ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream_ptr(stream)),
           "hbfp_gemm_partials")
    return P


def gemm_partials_window(a: BfpTensor, b: BfpTensor, row0: int, rows: int, col0: int, cols: int,
                          workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """hbfp_gemm_partials_window: the integer block sums of rows row0.. x columns col0.. of the product only."""
    P = torch.empty((rows, cols, a.desc.nblk), dtype=torch.int32, device=a.mant.device)
    workspace = _workspace(gemm_select_workspace(a.desc, b.desc, KERNEL_INT8), P.device, workspace)
    _check(_lib.hbfp_gemm_partials_window(ctypes.byref(a.desc), ctypes.byref(b.desc), row0, rows, col0, cols, _dev_ptr(P),
                                          _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                                          _stream_ptr(stream)), "hbfp_gemm_partials_window")
    return P


def gemm_f32(trans_a: int, trans_b: int, A: torch.Tensor, B: torch.Tensor, fa: Format, fb: Format,
             out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """C = op(A) op(B): encode both operands along the contraction axis, then the BFP product."""
    assert A.is_cuda and B.is_cuda and A.dtype == B.dtype == torch.float32
    assert A.stride(1) == 1 and B.stride(1) == 1
    M, K = (A.shape[1], A.shape[0]) if trans_a else A.shape
    N = B.shape[0] if trans_b else B.shape[1]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    workspace = _workspace(gemm_f32_workspace(trans_a, trans_b, M, N, K, fa, fb), A.device, workspace)
    _check(_lib.hbfp_gemm_f32(trans_a, trans_b, M, N, K, _dev_ptr(A), A.stride(0), _dev_ptr(B), B.stride(0),
                              _dev_ptr(out), out.stride(0), ctypes.byref(fa), ctypes.byref(fb),
                              _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                              _stream_ptr(stream)), "hbfp_gemm_f32")
    return out


def _desc_ref(t: Optional[BfpTensor]):
    return None if t is None else ctypes.byref(t.desc)


def weight_update_workspace(wide: BfpTensor, narrow_a: Optional[BfpTensor] = None,
                            narrow_b: Optional[BfpTensor] = None) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_weight_update_workspace(ctypes.byref(wide.desc), _desc_ref(narrow_a), _desc_ref(narrow_b),
                                             ctypes.byref(n)), "hbfp_weight_update_workspace")
    return int(n.value)


def weight_update(wide: BfpTensor, delta: torch.Tensor, alpha: float, narrow_a: Optional[BfpTensor] = None,
                  narrow_b: Optional[BfpTensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """hbfp_weight_update: wide <- encode(fma(alpha, delta, value(wide))), and the same FP32 result into the narrow tensors."""
    assert delta.is_cuda and delta.dtype == torch.float32 and delta.dim() == 2 and delta.stride(1) == 1
    workspace = _workspace(weight_update_workspace(wide, narrow_a, narrow_b), delta.device, workspace)
    _check(_lib.hbfp_weight_update(ctypes.byref(wide.desc), _dev_ptr(delta), delta.stride(0), alpha,
                                   _desc_ref(narrow_a), _desc_ref(narrow_b), _dev_ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream_ptr(stream)),
           "hbfp_weight_update")
    return workspace


def _desc_array(outs):
    arr = (ctypes.POINTER(TensorDesc) * len(outs))()
    for i, t in enumerate(outs):
        arr[i] = ctypes.pointer(t.desc if hasattr(t, "desc") else t)     # BfpTensor or bare descriptor
    return arr


def encode_im2col_workspace(conv: Conv2d, desc: TensorDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_encode_im2col_workspace(ctypes.byref(conv), ctypes.byref(desc), ctypes.byref(n)), "hbfp_encode_im2col_workspace")
    return int(n.value)


def encode_im2col(x: torch.Tensor, conv: Conv2d, fmt: Format, contract_axis: int = 1, out: Optional[BfpTensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None) -> BfpTensor:
    """hbfp_encode_im2col on an NHWC FP32 device tensor: the lowered activation operand of a convolution
    (contract_axis 1: forward product, 0: weight gradient)."""
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and tuple(x.shape) == (conv.n, conv.h, conv.w, conv.c)
    ho, wo = conv.out_hw()
    if out is None:
        out = alloc(fmt, conv.n * ho * wo, conv.r * conv.s * conv.c, contract_axis, x.device)
    workspace = _workspace(encode_im2col_workspace(conv, out.desc), x.device, workspace)
    _check(_lib.hbfp_encode_im2col(_dev_ptr(x), ctypes.byref(conv), ctypes.byref(out.desc), _dev_ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream_ptr(stream)), "hbfp_encode_im2col")
    return out


def encode_multi_workspace(outs) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_encode_multi_workspace(len(outs), _desc_array(outs), ctypes.byref(n)), "hbfp_encode_multi_workspace")
    return int(n.value)


def encode_multi(src: torch.Tensor, outs, workspace: Optional[torch.Tensor] = None, stream=None):
    """hbfp_encode_multi: one FP32 matrix into up to three planned operand tensors (see ``alloc``)."""
    assert src.is_cuda and src.dtype == torch.float32 and src.dim() == 2 and src.stride(1) == 1
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else max(src.stride(0), cols)
    arr = _desc_array(outs)
    workspace = _workspace(encode_multi_workspace(outs), src.device, workspace)
    _check(_lib.hbfp_encode_multi(_dev_ptr(src), ld, len(outs), arr, _dev_ptr(workspace),
                                  0 if workspace is None else workspace.numel(), _stream_ptr(stream)), "hbfp_encode_multi")
    return outs



def encode_packed_workspace(outs) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_encode_packed_workspace(len(outs), _desc_array(outs), ctypes.byref(n)), "hbfp_encode_packed_workspace")
    return int(n.value)


def encode_packed(src: torch.Tensor, outs, packed, workspace: Optional[torch.Tensor] = None, stream=None):
    """hbfp_encode_packed: one FP32 matrix into planned operand tensors and their packed forms (``packed[i]`` a uint8
    device tensor of ``pack_bytes`` bytes, or None)."""
    assert src.is_cuda and src.dtype == torch.float32 and src.dim() == 2 and src.stride(1) == 1
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else max(src.stride(0), cols)
    n = len(outs)
    ptrs = (ctypes.c_void_p * n)(*[None if b is None else b.data_ptr() for b in packed])
    sizes = (ctypes.c_size_t * n)(*[0 if b is None else b.numel() for b in packed])
    workspace = _workspace(encode_packed_workspace(outs), src.device, workspace)
    _check(_lib.hbfp_encode_packed(_dev_ptr(src), ld, n, _desc_array(outs), ptrs, sizes, _dev_ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream_ptr(stream)), "hbfp_encode_packed")
    return outs


def _encode_jobs(sources):
    """sources: sequence of (src, outs, packed); returns the job array and the objects that its pointers refer to."""
    jobs, keep = (EncodeJob * len(sources))(), []
    for j, (src, outs, packed) in enumerate(sources):
        assert src.is_cuda and src.dtype == torch.float32 and src.dim() == 2 and src.stride(1) == 1
        rows, cols = src.shape
        n = len(outs)
        descs = _desc_array(outs)
        ptrs = (ctypes.c_void_p * n)(*[None if b is None else b.data_ptr() for b in packed])
        sizes = (ctypes.c_size_t * n)(*[0 if b is None else b.numel() for b in packed])
        keep += [descs, ptrs, sizes]
        jobs[j].src, jobs[j].ld, jobs[j].n = src.data_ptr(), (src.stride(0) if rows > 1 else max(src.stride(0), cols)), n
        jobs[j].outs = ctypes.cast(descs, ctypes.c_void_p)
        jobs[j].packed = ctypes.cast(ptrs, ctypes.c_void_p)
        jobs[j].packed_bytes = ctypes.cast(sizes, ctypes.c_void_p)
    return jobs, keep


def encode_packed_batch_workspace(sources) -> int:
    jobs, keep = _encode_jobs(sources)
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_encode_packed_batch_workspace(len(sources), jobs, ctypes.byref(n)), "hbfp_encode_packed_batch_workspace")
    return int(n.value)


def encode_packed_batch(sources, workspace: Optional[torch.Tensor] = None, stream=None):
    """hbfp_encode_packed_batch: sources is a sequence of (src, outs, packed), each as the arguments of encode_packed."""
    jobs, keep = _encode_jobs(sources)
    need = ctypes.c_size_t(0)
    _check(_lib.hbfp_encode_packed_batch_workspace(len(sources), jobs, ctypes.byref(need)), "hbfp_encode_packed_batch_workspace")
    workspace = _workspace(int(need.value), sources[0][0].device, workspace)
    _check(_lib.hbfp_encode_packed_batch(len(sources), jobs, _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                                         _stream_ptr(stream)), "hbfp_encode_packed_batch")
    return [s[1] for s in sources]


def probe_matrix_rate(instruction: int, words: torch.Tensor, workgroups: int, iters: int, sink: torch.Tensor,
                      clocks: torch.Tensor, stream=None) -> None:
    """hbfp_probe_matrix_rate: one launch of the register-only loop (the caller times it with events)."""
    assert words.dtype == torch.int32 and words.numel() >= 64 * 64 and sink.numel() >= workgroups * 256
    assert clocks.dtype == torch.int64 and clocks.numel() >= 2
    _check(_lib.hbfp_probe_matrix_rate(instruction, _dev_ptr(words), workgroups, iters, _dev_ptr(sink), _dev_ptr(clocks),
                                       _stream_ptr(stream)), "hbfp_probe_matrix_rate")


def gemm_conv2d_workspace(image: TensorDesc, conv: Conv2d, filters: TensorDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_gemm_conv2d_workspace(ctypes.byref(image), ctypes.byref(conv), ctypes.byref(filters), ctypes.byref(n)),
           "hbfp_gemm_conv2d_workspace")
    return int(n.value)


def gemm_conv2d(image: BfpTensor, conv: Conv2d, filters: BfpTensor, out: Optional[torch.Tensor] = None, beta: float = 0.0,
                workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """hbfp_gemm_conv2d: Y[n*ho*wo, filters] from the image encoded once as [n*h*w, c] (blocks of 32 channels) and
    the filter matrix [r*s*c, filters] (blocks of 32 down its rows)."""
    ho, wo = conv.out_hw()
    if out is None:
        out = torch.empty((conv.n * ho * wo, filters.desc.rows), dtype=torch.float32, device=image.mant.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.stride(1) == 1
    workspace = _workspace(gemm_conv2d_workspace(image.desc, conv, filters.desc), out.device, workspace)
    _check(_lib.hbfp_gemm_conv2d(ctypes.byref(image.desc), ctypes.byref(conv), ctypes.byref(filters.desc), _dev_ptr(out),
                                 out.stride(0), beta, _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                                 _stream_ptr(stream)), "hbfp_gemm_conv2d")
    return out


def gemm_conv2d_bfp_workspace(image: TensorDesc, conv: Conv2d, filters: TensorDesc, out: TensorDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_gemm_conv2d_bfp_workspace(ctypes.byref(image), ctypes.byref(conv), ctypes.byref(filters), ctypes.byref(out),
                                               ctypes.byref(n)), "hbfp_gemm_conv2d_bfp_workspace")
    return int(n.value)


def gemm_conv2d_bfp(image: BfpTensor, conv: Conv2d, filters: BfpTensor, fmt: Format, relu: bool = False, out: Optional[BfpTensor] = None,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> BfpTensor:
    """hbfp_gemm_conv2d_bfp: the convolution delivered as an encoded operand [n*ho*wo, filters] (contraction along the
    filters): the next layer's image."""
    ho, wo = conv.out_hw()
    if out is None:
        out = alloc(fmt, conv.n * ho * wo, filters.desc.rows, 1, image.mant.device)
    workspace = _workspace(gemm_conv2d_bfp_workspace(image.desc, conv, filters.desc, out.desc), image.mant.device, workspace)
    _check(_lib.hbfp_gemm_conv2d_bfp(ctypes.byref(image.desc), ctypes.byref(conv), ctypes.byref(filters.desc), ctypes.byref(out.desc),
                                     1 if relu else 0, _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                                     _stream_ptr(stream)), "hbfp_gemm_conv2d_bfp")
    return out


def gemm_conv2d_dgrad_workspace(dy: TensorDesc, conv: Conv2d, filters: TensorDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.hbfp_gemm_conv2d_dgrad_workspace(ctypes.byref(dy), ctypes.byref(conv), ctypes.byref(filters), ctypes.byref(n)),
           "hbfp_gemm_conv2d_dgrad_workspace")
    return int(n.value)


def gemm_conv2d_dgrad(dy: BfpTensor, conv: Conv2d, filters: BfpTensor, out: Optional[torch.Tensor] = None, beta: float = 0.0,
                      workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """hbfp_gemm_conv2d_dgrad: dX[n*h*w, c] of the convolution `conv` (any stride) from its output gradient encoded once
    as [n*ho*wo, filters] (blocks of 32 filters) and the mirrored filter matrix [r*s*filters, c]."""
    if out is None:
        out = torch.empty((conv.n * conv.h * conv.w, filters.desc.rows), dtype=torch.float32, device=dy.mant.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.stride(1) == 1
    workspace = _workspace(gemm_conv2d_dgrad_workspace(dy.desc, conv, filters.desc), out.device, workspace)
    _check(_lib.hbfp_gemm_conv2d_dgrad(ctypes.byref(dy.desc), ctypes.byref(conv), ctypes.byref(filters.desc), _dev_ptr(out),
                                       out.stride(0), beta, _dev_ptr(workspace), 0 if workspace is None else workspace.numel(),
                                       _stream_ptr(stream)), "hbfp_gemm_conv2d_dgrad")
    return out
