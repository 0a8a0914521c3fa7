"""Exact-arithmetic parity of the product kernels that hbfp_gemm runs.

Eq. (2) of Sec. 4 followed by the FP accumulation of tile results: with inputs chosen so that every FP32
accumulation is exact (all running sums are integers below 2^24 times one common power of two), the FP32 result of
ANY correct evaluation order is the same number, the one the oracle's FP64 definition gives, so C must match it bit
for bit whatever kernel family computed it.  A wrong scale word, a wrong limb exponent, a stale staging buffer or a
lost k-step changes single elements and fails here, where a norm over the matrix would let it pass.
"""
import numpy as np
import pytest
import torch

from oracle import ref
from tests.util import unpack

pytestmark = pytest.mark.gpu

AUTO, INT8, SCALED, WIDE, FP16, BF16, F16P = 0, 1, 2, 3, 4, 5, 6


@pytest.fixture(scope="module")
def hb():
    from paper_1804_01526_amd import hbfp
    assert torch.cuda.is_available(), "these tests need the GPU"
    return hbfp


def _integers(rng, shape, kb, axis, top, small=None, plant_at=None):
    """Integer-valued FP32 matrix whose every block of kb along `axis` holds one entry of magnitude `top`, so that every
    block gets the same exponent byte and one mantissa unit is worth 1: the mantissas are the integers themselves.
    small: bound of the other magnitudes (default: top).  plant_at: offset of the planted entry in its block
    (default: random)."""
    small = top if small is None else small
    x = rng.integers(-small, small + 1, size=shape).astype(np.float32)
    xs = np.moveaxis(x, axis, 1)                      # view: [other, k]
    K = xs.shape[1]
    for b0 in range(0, K, kb):
        n = min(kb, K - b0)
        pos = rng.integers(0, n, size=xs.shape[0]) if plant_at is None else np.full(xs.shape[0], min(plant_at, n - 1))
        xs[np.arange(xs.shape[0]), b0 + pos] = top * rng.choice([-1.0, 1.0], size=xs.shape[0])
    return x


def _encode_pair(hb, A, B, fa, fb):
    ta = hb.encode(torch.from_numpy(A).cuda(), 1, hb.make_format(fa[2], fa[0], fa[1]))
    tb = hb.encode(torch.from_numpy(B).cuda(), 0, hb.make_format(fb[2], fb[0], fb[1]))
    oa, ob = ref.encode(A, fa[0], fa[1], fa[2]), ref.encode(B, fb[0], fb[1], fb[2])
    for t, o in ((ta, oa), (tb, ob)):
        m, e = unpack(t)
        np.testing.assert_array_equal(m, o.mant)
        np.testing.assert_array_equal(e, o.exps)
    return ta, tb, oa, ob


def _exact(hb, A, B, fa, fb, kernel, check_integers=True):
    """A [M, K], B [K, N]; fa / fb = (block rows, block cols, mantissa bits).  C must equal the oracle bit for bit."""
    print(f"[exact] A={A.shape} B={B.shape} fa={fa} fb={fb} kernel={kernel}", flush=True)
    ta, tb, oa, ob = _encode_pair(hb, A, B, fa, fb)
    C64 = ref.gemm(ref.decode(oa), ref.decode(ob))
    # the oracle's definition is exact here: it equals the scaled integer block sums of Eq. (2)
    kb = ta.desc.kblock
    if check_integers:                                # 1-D blocks: exponent arrays are [M, nblk] and [nblk, N]
        P = ref.block_dots(oa.mant, ob.mant, kb)
        np.testing.assert_array_equal(ref.scale_accumulate(P, oa.exps, ob.exps, fa[2], fb[2]), C64)
    assert np.array_equal(C64, C64.astype(np.float32).astype(np.float64)), "test input: the exact result must fit FP32"
    C = hb.gemm(ta, tb, kernel=kernel)
    torch.cuda.synchronize()
    got = C.cpu().numpy().astype(np.float64)
    bad = np.argwhere(got != C64)
    assert bad.size == 0, f"{len(bad)} elements differ, first at {bad[0]}: got {got[tuple(bad[0])]!r} want {C64[tuple(bad[0])]!r}"
    return ta, tb, C64


# ------------------------------------------------------------------ 8-bit mantissas: every product kernel
@pytest.mark.parametrize("kernel", [INT8, SCALED, BF16])
@pytest.mark.parametrize("kb,K", [(32, 1024), (24, 1000), (64, 1024), (16, 400), (8, 264)])
def test_exact_sums_8_bit_blocks(hb, kernel, kb, K):
    """Random mantissas in [-127, 127], one +-127 planted per block: equal exponent bytes, |sum| <= 1024 * 127^2 < 2^24.
    Blocks of 32 / 24 / 16 / 8 (one matrix instruction per block), 64 (two, chained): the int8 kernels' three block
    modes, the two-limb block-scaled kernel and the bf16 kernel, several 256 x 256 tiles with ragged edges."""
    rng = np.random.default_rng(1000 + kb + K + kernel)
    M, N = 300, 530
    A = _integers(rng, (M, K), kb, 1, 127)
    B = _integers(rng, (K, N), kb, 0, 127)
    _exact(hb, A, B, (1, kb, 8), (kb, 1, 8), kernel)


@pytest.mark.parametrize("kernel", [INT8, SCALED, AUTO, BF16])
@pytest.mark.parametrize("kb,K", [(128, 1024), (256, 768), (512, 1024), (0, 896)])
def test_exact_sums_8_bit_long_blocks(hb, kernel, kb, K):
    """Blocks of 128 and more, and one exponent per row / column (Sec. 4): chains of matrix instructions."""
    rng = np.random.default_rng(2000 + kb + K + kernel)
    M, N = 200, 280
    kbe = kb if kb else K
    A = _integers(rng, (M, K), kbe, 1, 127)
    B = _integers(rng, (K, N), kbe, 0, 127)
    _exact(hb, A, B, (1, kb, 8), (kb, 1, 8), kernel)


@pytest.mark.parametrize("kernel", [INT8, AUTO, WIDE])
@pytest.mark.parametrize("kb,K", [(512, 4096), (0, 4096), (384, 1536)])
def test_long_blocks_of_equal_signs_stay_exact(hb, kernel, kb, K):
    """Every mantissa +-127 with one sign per column of B: block sums of 512 * 127^2 = 8.26e6 and 4096 * 127^2 = 6.6e7,
    far beyond the 2^22 up to which an int32 sum can ride on the bit pattern of a float constant.  The result
    (127^2 * K, a 14-bit integer times a power of two) is exact in FP32."""
    if kernel == WIDE and kb != 0:
        pytest.skip("the 256 x 256-tile kernel takes one exponent per row only")
    M, N = 64, 96
    A = np.full((M, K), 127.0, dtype=np.float32)
    B = np.full((K, N), 127.0, dtype=np.float32)
    B[:, ::2] *= -1
    A[1::2] *= -1
    _exact(hb, A, B, (1, kb, 8), (kb, 1, 8), kernel)


@pytest.mark.parametrize("kernel", [INT8, SCALED, BF16])
def test_exact_sums_config4_formats(hb, kernel):
    """1 x 24 activation blocks against 24 x 24 weight tiles, ragged last block (1000 = 41 * 24 + 16)."""
    rng = np.random.default_rng(77 + kernel)
    M, K, N = 280, 1000, 300
    A = _integers(rng, (M, K), 24, 1, 127)
    B = _integers(rng, (K, N), 24, 0, 127)       # every column block holds a 127, so every 24 x 24 tile does
    _exact(hb, A, B, (1, 24, 8), (24, 24, 8), kernel, check_integers=False)


# ------------------------------------------------------------------ one block, unequal exponents
@pytest.mark.parametrize("kernel", [INT8, SCALED, BF16])
@pytest.mark.parametrize("kb", [32, 24, 64])
def test_single_block_with_unequal_exponents(hb, kernel, kb):
    """One block along k (K = kb): C[i][j] = P[i][j] * 2^(eA[i] + eB[j]) with |P| < 2^24 is exact for any exponents.
    Rows of A and columns of B are scaled by different powers of two, so every (row, column) pair of scale words is hit."""
    rng = np.random.default_rng(3000 + kb + kernel)
    M, N, K = 260, 270, kb
    A = _integers(rng, (M, K), kb, 1, 127) * np.exp2(rng.integers(-30, 31, size=(M, 1))).astype(np.float32)
    B = _integers(rng, (K, N), kb, 0, 127) * np.exp2(rng.integers(-30, 31, size=(1, N))).astype(np.float32)
    _exact(hb, A.astype(np.float32), B.astype(np.float32), (1, kb, 8), (kb, 1, 8), kernel)


@pytest.mark.parametrize("kernel", [INT8, SCALED, BF16])
def test_blocks_with_unequal_exponents_and_disjoint_support(hb, kernel):
    """Several blocks with different exponents each: row i of A is non-zero only in block i % nblk, so each output is a
    single block product and stays exact, while the kernel still walks all blocks with their own scale words."""
    rng = np.random.default_rng(3100 + kernel)
    kb, nblk = 32, 8
    M, N, K = 270, 260, kb * nblk
    A = np.zeros((M, K), dtype=np.float32)
    for i in range(M):
        b = i % nblk
        A[i, b * kb:(b + 1) * kb] = _integers(rng, (1, kb), kb, 1, 127)[0] * np.exp2(rng.integers(-20, 21))
    B = np.empty((K, N), dtype=np.float32)
    for b in range(nblk):
        B[b * kb:(b + 1) * kb] = _integers(rng, (kb, N), kb, 0, 127) * np.exp2(rng.integers(-20, 21, size=(1, N)))
    _exact(hb, A, B, (1, kb, 8), (kb, 1, 8), kernel)


# ------------------------------------------------------------------ other limb counts of the block-scaled kernel
@pytest.mark.parametrize("m", [4, 5])
def test_exact_sums_one_limb(hb, m):
    """Mantissas of at most 5 bits: one 4-bit limb, one matrix instruction per k-step (both kernel families)."""
    top = (1 << (m - 1)) - 1
    for kernel in (INT8, SCALED):
        rng = np.random.default_rng(4000 + m + kernel)
        M, N, K = 300, 300, 2048
        A = _integers(rng, (M, K), 32, 1, top)
        B = _integers(rng, (K, N), 32, 0, top)
        _exact(hb, A, B, (1, 32, m), (32, 1, m), kernel)


@pytest.mark.parametrize("ma,mb", [(8, 4), (4, 8), (9, 9)])
def test_exact_sums_mixed_limb_counts(hb, ma, mb):
    """Operands with different limb counts (2 x 1, 1 x 2) and 9-bit mantissas (two limbs, |m| up to 255)."""
    ta_, tb_ = (1 << (ma - 1)) - 1, (1 << (mb - 1)) - 1
    K = 1024 if ma * mb <= 32 else 256
    for kernel in (INT8, SCALED) + ((BF16,) if ma == mb == 9 else ()):        # 9-bit mantissas (int16 storage) are bf16 numbers too
        rng = np.random.default_rng(4100 + ma * 16 + mb + kernel)
        M, N = 260, 300
        A = _integers(rng, (M, K), 32, 1, ta_)
        B = _integers(rng, (K, N), 32, 0, tb_)
        assert K * ta_ * tb_ < 2 ** 24
        _exact(hb, A, B, (1, 32, ma), (32, 1, mb), kernel)


@pytest.mark.parametrize("kernel", [FP16, F16P])
@pytest.mark.parametrize("kb,K,m", [(32, 512, 9), (64, 1024, 9), (128, 768, 9), (256, 1024, 9), (0, 640, 9), (64, 16384, 9), (64, 256, 11),
                                    (32, 160, 12)])
def test_exact_sums_fp16_kernel(hb, kernel, kb, K, m):
    """9..12-bit mantissas as FP16 numbers on the FP16 matrix instruction: every block length the kernel takes (two
    matrix instructions per block of 32, chains for longer blocks), a contraction long enough for split-k, full-range
    9-bit mantissas (|sum| <= K * 255 * 3 ... below 2^24 by construction) and wider ones with small magnitudes around the
    planted full-width entry."""
    rng = np.random.default_rng(8000 + kb + K + m)
    M, N = (200, 280) if K < 8192 else (100, 90)
    kbe = kb if kb else K
    top = (1 << (m - 1)) - 1
    small = {9: 255 if K <= 256 else 60, 11: 30, 12: 40}[m] if K < 8192 else 25
    A = _integers(rng, (M, K), kbe, 1, top, small=small)
    B = _integers(rng, (K, N), kbe, 0, top, small=small)
    assert (np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)).max() < 2 ** 24, "test input: sums must stay exact"
    _exact(hb, A, B, (1, kb, m), (kb, 1, m), kernel)


@pytest.mark.parametrize("kernel", [INT8, SCALED, FP16, F16P])
@pytest.mark.parametrize("ma,mb", [(12, 12), (10, 12), (12, 10)])
def test_exact_sums_three_limbs(hb, kernel, ma, mb):
    """9..12-bit mantissas (three 4-bit limbs, or two int8 limbs): one full-width entry per block of 64 and small
    values elsewhere, three blocks, so that every pair of limb planes meets (planted entries coincide for some
    (row, column, block)) and the sum stays below 3 * 2047^2 + cross terms < 2^24."""
    rng = np.random.default_rng(5000 + ma * 16 + mb + kernel)
    M, N, K, kb = 270, 300, 192, 64
    ta_, tb_ = (1 << (ma - 1)) - 1, (1 << (mb - 1)) - 1
    A = _integers(rng, (M, K), kb, 1, ta_, small=3)
    B = _integers(rng, (K, N), kb, 0, tb_, small=3)
    # make sure full-width x full-width products occur: same planted position in some rows and columns
    A[:40] = _integers(rng, (40, K), kb, 1, ta_, small=3, plant_at=5)
    B[:, :40] = _integers(rng, (K, 40), kb, 0, tb_, small=3, plant_at=5)
    assert 3 * ta_ * tb_ + 2 * 3 * 3 * max(ta_, tb_) + 9 * K < 2 ** 24
    _exact(hb, A, B, (1, kb, ma), (kb, 1, mb), kernel)


# ------------------------------------------------------------------ the product delivered as an encoded operand
@pytest.mark.parametrize("kernel", [SCALED, INT8, BF16])
@pytest.mark.parametrize("out_kb,out_m,relu", [(32, 8, False), (64, 8, True), (32, 12, True), (24, 8, False)])
def test_encoded_output_of_an_exact_product(hb, kernel, out_kb, out_m, relu):
    """hbfp_gemm_bfp on a product whose FP32 value is exact: the encoded output must equal the ORACLE's conversion of
    the ORACLE's product (nothing of the library's own feeds the expected value).  Blocks of 32 / 64 take the fused
    epilogue of the block-scaled kernel (operands of the matrix instruction exchanged), 24 the workspace route."""
    rng = np.random.default_rng(6000 + out_kb + out_m + kernel)
    M, N, K = 300, 330, 512
    A = _integers(rng, (M, K), 32, 1, 127)
    B = _integers(rng, (K, N), 32, 0, 127)
    ta, tb, oa, ob = _encode_pair(hb, A, B, (1, 32, 8), (32, 1, 8))
    C64 = ref.gemm(ref.decode(oa), ref.decode(ob))
    C32 = C64.astype(np.float32)
    assert np.array_equal(C32.astype(np.float64), C64)
    if relu:
        C32 = np.maximum(C32, 0.0)
    want = ref.encode(C32, 1, out_kb, out_m)
    got = hb.gemm_bfp(ta, tb, hb.make_format(out_m, 1, out_kb), 1, relu=relu, kernel=kernel)
    torch.cuda.synchronize()
    m, e = unpack(got)
    np.testing.assert_array_equal(e, want.exps)
    np.testing.assert_array_equal(m, want.mant)


# ------------------------------------------------------------------ dense packing of blocks shorter than 32
def _stepped(rng, shape, kb, axis, steps, small=15):
    """Integer mantissas with one +-127 per block as in _integers, block b of every operand row scaled by 2^steps[row, b]."""
    x = _integers(rng, shape, kb, axis, 127, small=small)
    xs = np.moveaxis(x, axis, 1)
    K = xs.shape[1]
    for b, b0 in enumerate(range(0, K, kb)):
        xs[:, b0:b0 + kb] *= np.exp2(steps[:, b])[:, None].astype(np.float32)
    return x


@pytest.mark.parametrize("kernel", [SCALED, INT8])
@pytest.mark.parametrize("kb", [24, 16, 8])
@pytest.mark.parametrize("which", ["a", "b", "both"])
def test_dense_packing_neighbouring_blocks_up_to_three_binades_apart(hb, kernel, kb, which):
    """Blocks shorter than 32 are packed without their padding for the block-scaled kernel: a group of 32 consecutive
    elements spans two to four blocks, takes the smallest of their exponents and holds the other blocks' magnitudes
    shifted left by up to 3 bits (one in the limbs, two in the codes' own exponent bits).  Exponents of neighbouring
    blocks differ by 0 to 3 here; every sum stays below 2^24."""
    rng = np.random.default_rng(7000 + kb + kernel + len(which))
    M, N, K = 270, 280, {24: 480, 16: 400, 8: 264}[kb]
    nblk = -(-K // kb)
    sa = rng.integers(0, 4, size=(M, nblk)) if which in ("a", "both") else np.zeros((M, nblk), dtype=np.int64)
    sb = rng.integers(0, 4, size=(N, nblk)) if which in ("b", "both") else np.zeros((N, nblk), dtype=np.int64)
    small = 20 if which == "both" else 90
    A = _stepped(rng, (M, K), kb, 1, sa, small)
    B = _stepped(rng, (K, N), kb, 0, sb, small)
    assert (np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)).max() < 2 ** 24, "test input: sums must stay exact"
    _exact(hb, A, B, (1, kb, 8), (kb, 1, 8), kernel)


@pytest.mark.parametrize("kb", [24, 16])
def test_dense_packing_falls_back_when_blocks_are_far_apart(hb, kb):
    """A jump of four and more binades between neighbouring blocks cannot be written into one group of 32: the
    call must still deliver the exact product (the int8 kernels behind the block-scaled kernel compute it)."""
    rng = np.random.default_rng(7100 + kb)
    M, N, K = 260, 300, 240
    nblk = -(-K // kb)
    sa = np.zeros((M, nblk), dtype=np.int64)
    sa[5, 3] = 4                                   # a single far block in one row is enough
    sa[200:, ::2] = 6
    A = _stepped(rng, (M, K), kb, 1, sa, small=3)
    B = _integers(rng, (K, N), kb, 0, 127, small=3)
    _exact(hb, A, B, (1, kb, 8), (kb, 1, 8), SCALED)
    # all-zero blocks between non-zero ones take any exponent: no fallback needed, still exact
    A2 = _integers(rng, (M, K), kb, 1, 127)
    A2[:, kb:2 * kb] = 0.0
    A2[7, :] = 0.0
    _exact(hb, A2, B, (1, kb, 8), (kb, 1, 8), SCALED)
