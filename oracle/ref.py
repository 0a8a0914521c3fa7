"""ctypes front end of the CPU oracle (``hbfp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
``cpu_baseline`` leg of the benchmark.  Nothing here is used by the GPU library
and nothing here uses it.

All arrays are plain numpy, host memory, in the *source* orientation of the
paper's notation: a tensor ``a`` with mantissas ``m_i`` and one exponent per
block (Eq. (1), Sec. 4), a product ``C = A B`` with ``A`` of shape [M, K] and
``B`` of shape [K, N] (Eq. (2), Sec. 4).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hbfp_oracle.c")
_LIB = os.path.join(_HERE, "libhbfp_oracle.so")

RNE = 0
STOCHASTIC = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, u64 = ctypes.c_int64, ctypes.c_int, ctypes.c_uint64
        p = ctypes.c_void_p
        lib.hbfp_ref_hash32.restype = ctypes.c_uint32
        lib.hbfp_ref_hash32.argtypes = [u64, u64]
        lib.hbfp_ref_num_threads.restype = i32
        lib.hbfp_ref_encode.argtypes = [p, i64, i64, i64, i64, i64, i32, i32, u64, p, p]
        lib.hbfp_ref_decode.argtypes = [p, p, i64, i64, i64, i64, i32, p, i64]
        lib.hbfp_ref_block_dots.argtypes = [p, p, i64, i64, i64, i64, p]
        lib.hbfp_ref_gemm.argtypes = [p, i64, p, i64, i64, i64, i64, p]
        lib.hbfp_ref_gemm_rows.argtypes = [p, i64, p, i64, i64, i64, i64, p, i64, p]
        lib.hbfp_ref_scale_accumulate.argtypes = [p, p, p, i64, i64, i64, i32, i32, p]
        lib.hbfp_ref_weight_update.argtypes = [p, p, i64, i64, i64, i64, i32, i32, u64, p, i64, ctypes.c_float,
                                               i32, i32, u64, p, p, p, p, p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_L().hbfp_ref_num_threads())


def hash32(seed: int, idx: int) -> int:
    return int(_L().hbfp_ref_hash32(ctypes.c_uint64(seed), ctypes.c_uint64(idx)))


@dataclass
class BFP:
    """A BFP tensor in source orientation: ``value = mant * 2**(exps - 125 - m)``."""

    mant: np.ndarray  # int32 [rows, cols]
    exps: np.ndarray  # uint8 [ceil(rows/br), ceil(cols/bc)]
    m: int
    br: int
    bc: int

    def unit_exponents(self) -> np.ndarray:
        """Exponent of one mantissa unit, per element, int32 [rows, cols]."""
        rows, cols = self.mant.shape
        e = self.exps.astype(np.int32) - 125 - self.m
        return np.repeat(np.repeat(e, self.br, axis=0)[:rows], self.bc, axis=1)[:, :cols]


def _blk(n: int, b: int) -> int:
    return n if (b <= 0 or b > n) else b


def encode(x: np.ndarray, br: int, bc: int, m: int, rounding: int = RNE, seed: int = 0) -> BFP:
    """FP32 [rows, cols] -> BFP with br x bc exponent blocks (0 = whole extent)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.ndim == 2
    rows, cols = x.shape
    br, bc = _blk(rows, br), _blk(cols, bc)
    nbr, nbc = -(-rows // br), -(-cols // bc)
    mant = np.empty((rows, cols), dtype=np.int32)
    exps = np.empty((nbr, nbc), dtype=np.uint8)
    rc = _L().hbfp_ref_encode(_ptr(x), rows, cols, cols, br, bc, m, rounding,
                              ctypes.c_uint64(seed), _ptr(mant), _ptr(exps))
    if rc != 0:
        raise ValueError(f"hbfp_ref_encode: {rc}")
    return BFP(mant, exps, m, br, bc)


def decode(t: BFP) -> np.ndarray:
    rows, cols = t.mant.shape
    out = np.empty((rows, cols), dtype=np.float32)
    rc = _L().hbfp_ref_decode(_ptr(np.ascontiguousarray(t.mant)), _ptr(np.ascontiguousarray(t.exps)),
                              rows, cols, t.br, t.bc, t.m, _ptr(out), cols)
    if rc != 0:
        raise ValueError(f"hbfp_ref_decode: {rc}")
    return out


def im2col(x: np.ndarray, r: int, s: int, pad_h: int, pad_w: int, stride_h: int = 1, stride_w: int = 1,
           c_block: int = 0) -> np.ndarray:
    """Activation operand of a convolution executed as a matrix product (Sec. 5.1 treats convolutions like matrix
    multiplications): x [n, h, w, c] -> [n*ho*wo, r*s*c]; row (img, oy, ox) holds the values under the filter
    window, column (fr*s + fs)*c + ch = x[img, oy*stride_h - pad_h + fr, ox*stride_w - pad_w + fs, ch], zero
    outside the image.  Written out tap by tap on a zero-padded copy.  With c_block the channels are cut into
    blocks and the columns run block by block (all taps of the first c_block channels, then the next block, ...)."""
    n, h, w, c = x.shape
    ho = (h + 2 * pad_h - r) // stride_h + 1
    wo = (w + 2 * pad_w - s) // stride_w + 1
    xp = np.zeros((n, h + 2 * pad_h, w + 2 * pad_w, c), dtype=x.dtype)
    xp[:, pad_h:pad_h + h, pad_w:pad_w + w, :] = x
    out = np.empty((n, ho, wo, r, s, c), dtype=x.dtype)
    for fr in range(r):
        for fs in range(s):
            out[:, :, :, fr, fs, :] = xp[:, fr:fr + stride_h * (ho - 1) + 1:stride_h, fs:fs + stride_w * (wo - 1) + 1:stride_w, :]
    if c_block <= 0 or c_block >= c:
        return out.reshape(n * ho * wo, r * s * c)
    return np.concatenate([out[..., c0:c0 + c_block].reshape(n * ho * wo, -1) for c0 in range(0, c, c_block)], axis=1)


def filter_matrix(w4: np.ndarray, c_block: int = 0) -> np.ndarray:
    """Filter tensor [r, s, c, f] -> the matrix [r*s*c, f] whose rows are in the column order of im2col."""
    r, s, c, f = w4.shape
    if c_block <= 0 or c_block >= c:
        return w4.reshape(r * s * c, f)
    return np.concatenate([w4[:, :, c0:c0 + c_block, :].reshape(-1, f) for c0 in range(0, c, c_block)], axis=0)


def filter_matrix_dgrad(w4: np.ndarray, c_block: int = 0) -> np.ndarray:
    """Filter of the data gradient of a stride-1 convolution (Sec. 5.1: the backward pass is executed like the
    forward pass).  With y[oy, ox, f] = sum x[oy - pad + fr, ox - pad + fs, c] w4[fr, fs, c, f], the gradient is
    dx[h, w, c] = sum dy[h + pad - fr, w + pad - fs, f] w4[fr, fs, c, f]: a convolution of dy with padding
    r - 1 - pad, whose filter is w4 mirrored in both spatial axes with its two channel axes exchanged.  Returns that
    filter as the matrix [r*s*f, c] in the column order of im2col(dy, ...)."""
    mirrored = w4[::-1, ::-1, :, :].transpose(0, 1, 3, 2)
    return filter_matrix(np.ascontiguousarray(mirrored), c_block)


def im2col_dgrad(dy: np.ndarray, h: int, w: int, r: int, s: int, pad_h: int, pad_w: int, stride_h: int = 1,
                 stride_w: int = 1) -> np.ndarray:
    """Activation operand of the data gradient of a convolution of any stride (Sec. 5.1: the backward pass is executed
    like the forward pass).  dy [n, ho, wo, f] is the gradient of y[oy, ox] = sum x[oy*stride - pad + fr, ...] w4[fr, ...];
    x has h x w positions.  dx[iy, ix] collects dy[oy, ox] * w4[fr, fs] over all oy*stride_h - pad_h + fr = iy (same in
    x), i.e. it is a stride-1 convolution of dy spread out with stride - 1 zeros between its pixels: dy[oy, ox] sits at
    position (r - 1 - pad_h + oy*stride_h, s - 1 - pad_w + ox*stride_w) of a zero canvas of (h + r - 1) x (w + s - 1), and
    row (img, iy, ix) of the result holds the canvas under the window whose corner is (iy, ix), column
    (fr' * s + fs') * f + ch: [n*h*w, r*s*f], to be multiplied by filter_matrix_dgrad."""
    n, ho, wo, f = dy.shape
    canvas = np.zeros((n, h + r - 1, w + s - 1, f), dtype=dy.dtype)
    for oy in range(ho):
        for ox in range(wo):
            cy, cx = r - 1 - pad_h + oy * stride_h, s - 1 - pad_w + ox * stride_w
            if 0 <= cy < h + r - 1 and 0 <= cx < w + s - 1:            # beyond: a window that lies wholly in the padding
                canvas[:, cy, cx, :] = dy[:, oy, ox, :]
    out = np.empty((n, h, w, r, s, f), dtype=dy.dtype)
    for fr in range(r):
        for fs in range(s):
            out[:, :, :, fr, fs, :] = canvas[:, fr:fr + h, fs:fs + w, :]
    return out.reshape(n * h * w, r * s * f)


def im2col_rows(x: np.ndarray, rows, r: int, s: int, pad_h: int, pad_w: int, stride_h: int = 1, stride_w: int = 1) -> np.ndarray:
    """The rows `rows` of im2col(x, ...) (plain window order), each written out from the definition: for checks at sizes
    where the whole lowered matrix is too large to hold."""
    n, h, w, c = x.shape
    ho = (h + 2 * pad_h - r) // stride_h + 1
    wo = (w + 2 * pad_w - s) // stride_w + 1
    out = np.zeros((len(rows), r, s, c), dtype=x.dtype)
    for i, row in enumerate(rows):
        img, rem = divmod(int(row), ho * wo)
        oy, ox = divmod(rem, wo)
        for fr in range(r):
            for fs in range(s):
                iy, ix = oy * stride_h - pad_h + fr, ox * stride_w - pad_w + fs
                if 0 <= iy < h and 0 <= ix < w:
                    out[i, fr, fs, :] = x[img, iy, ix, :]
    return out.reshape(len(rows), r * s * c)


def im2col_dgrad_rows(dy: np.ndarray, rows, h: int, w: int, r: int, s: int, pad_h: int, pad_w: int, stride_h: int = 1,
                      stride_w: int = 1) -> np.ndarray:
    """The rows `rows` of im2col_dgrad(dy, ...), each written out from the definition: entry (fr', fs') of input position
    (iy, ix) is dy[oy, ox] for the output position with oy*stride_h - pad_h + (r - 1 - fr') = iy (same in x), if there is one."""
    n, ho, wo, f = dy.shape
    out = np.zeros((len(rows), r, s, f), dtype=dy.dtype)
    for i, row in enumerate(rows):
        img, rem = divmod(int(row), h * w)
        iy, ix = divmod(rem, w)
        for fr in range(r):
            for fs in range(s):
                ny, nx = iy + pad_h - fr, ix + pad_w - fs
                if ny % stride_h == 0 and nx % stride_w == 0 and 0 <= ny // stride_h < ho and 0 <= nx // stride_w < wo:
                    out[i, r - 1 - fr, s - 1 - fs, :] = dy[img, ny // stride_h, nx // stride_w, :]
    return out.reshape(len(rows), r * s * f)


def block_dots(mA: np.ndarray, mB: np.ndarray, kb: int) -> np.ndarray:
    """Integer block partials P[i, j, b] of Eq. (2); mA [M, K], mB [K, N]."""
    mA = np.ascontiguousarray(mA, dtype=np.int32)
    mB = np.ascontiguousarray(mB, dtype=np.int32)
    M, K = mA.shape
    K2, N = mB.shape
    assert K == K2
    kb = _blk(K, kb)
    nb = -(-K // kb)
    P = np.empty((M, N, nb), dtype=np.int32)
    rc = _L().hbfp_ref_block_dots(_ptr(mA), _ptr(mB), M, N, K, kb, _ptr(P))
    if rc == -2:
        raise OverflowError("a block partial does not fit int32")
    if rc != 0:
        raise ValueError(f"hbfp_ref_block_dots: {rc}")
    return P


def gemm(A: np.ndarray, B: np.ndarray, rows=None) -> np.ndarray:
    """FP64 product of FP32 operands, by definition; optionally only some rows of A."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    if rows is None:
        C = np.empty((M, N), dtype=np.float64)
        rc = _L().hbfp_ref_gemm(_ptr(A), K, _ptr(B), N, M, N, K, _ptr(C))
    else:
        sel = np.ascontiguousarray(rows, dtype=np.int64)
        C = np.empty((sel.size, N), dtype=np.float64)
        rc = _L().hbfp_ref_gemm_rows(_ptr(A), K, _ptr(B), N, M, N, K, _ptr(sel), sel.size, _ptr(C))
    if rc != 0:
        raise ValueError(f"hbfp_ref_gemm: {rc}")
    return C


def scale_accumulate(P: np.ndarray, eA: np.ndarray, eB: np.ndarray, mA: int, mB: int) -> np.ndarray:
    """C[i,j] = sum_b P[i,j,b] * 2^(unit exponent of A block + of B block), in FP64."""
    P = np.ascontiguousarray(P, dtype=np.int32)
    M, N, nb = P.shape
    eA = np.ascontiguousarray(eA, dtype=np.uint8)
    eB = np.ascontiguousarray(eB, dtype=np.uint8)
    assert eA.shape == (M, nb) and eB.shape == (nb, N)
    C = np.empty((M, N), dtype=np.float64)
    rc = _L().hbfp_ref_scale_accumulate(_ptr(P), _ptr(eA), _ptr(eB), M, N, nb, mA, mB, _ptr(C))
    if rc != 0:
        raise ValueError(f"hbfp_ref_scale_accumulate: {rc}")
    return C


def bfp_gemm(A: np.ndarray, B: np.ndarray, fmt_a: dict, fmt_b: dict, rows=None):
    """The whole path by its definition: quantise A [M,K] and B [K,N], multiply in FP64.

    ``fmt_a`` / ``fmt_b``: dicts with keys br, bc, m and optionally rounding, seed;
    the block shapes are in each operand's own orientation.  Returns (C64, BFP(A), BFP(B)).
    """
    ta = encode(A, fmt_a["br"], fmt_a["bc"], fmt_a["m"], fmt_a.get("rounding", RNE), fmt_a.get("seed", 0))
    tb = encode(B, fmt_b["br"], fmt_b["bc"], fmt_b["m"], fmt_b.get("rounding", RNE), fmt_b.get("seed", 0))
    return gemm(decode(ta), decode(tb), rows=rows), ta, tb


def weight_update(wide: BFP, delta: np.ndarray, alpha: float, m_narrow: int, rounding_wide: int = RNE, seed_wide: int = 0,
                  rounding_narrow: int = RNE, seed_narrow: int = 0):
    """One FP32 update step on weights stored with wide mantissas (Sec. 4.2, Sec. 5.1).

    Returns (wide', narrow', w') with w' = fma(alpha, delta, value(wide)) in FP32 and both
    BFP tensors converted from w' with the block shape of ``wide``.
    """
    delta = np.ascontiguousarray(delta, dtype=np.float32)
    rows, cols = wide.mant.shape
    assert delta.shape == (rows, cols)
    wm = np.empty((rows, cols), dtype=np.int32)
    we = np.empty_like(wide.exps)
    nm = np.empty((rows, cols), dtype=np.int32)
    ne = np.empty_like(wide.exps)
    w = np.empty((rows, cols), dtype=np.float32)
    rc = _L().hbfp_ref_weight_update(_ptr(np.ascontiguousarray(wide.mant)), _ptr(np.ascontiguousarray(wide.exps)),
                                     rows, cols, wide.br, wide.bc, wide.m, rounding_wide, ctypes.c_uint64(seed_wide),
                                     _ptr(delta), cols, ctypes.c_float(alpha), m_narrow, rounding_narrow,
                                     ctypes.c_uint64(seed_narrow), _ptr(wm), _ptr(we), _ptr(nm), _ptr(ne), _ptr(w))
    if rc != 0:
        raise ValueError(f"hbfp_ref_weight_update: {rc}")
    return BFP(wm, we, wide.m, wide.br, wide.bc), BFP(nm, ne, m_narrow, wide.br, wide.bc), w

