"""hbfp_gemm_conv2d: the convolution whose activation operand is gathered from the image converted once (Sec. 5.1:
convolutions are executed like matrix products), against the oracle - which lowers the image explicitly - and against
the library's own product on the lowered operand of hbfp_encode_im2col (bit for bit: a block of 32 channels of a pixel
is the same block in the image and in every window that contains the pixel).  hbfp_gemm_conv2d_dgrad: the data gradient
of a convolution of any stride, gathered from the output gradient converted once."""
import numpy as np
import pytest
import torch

from oracle import ref
from tests.util import random_cases, rel_fro

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def hb():
    from paper_1804_01526_amd import hbfp
    assert torch.cuda.is_available(), "these tests need the GPU"
    return hbfp


def _conv_case(hb, n, h, w, c, f, r, s, pad_h, pad_w, sh, sw, seed, beta=0.0, against_lowered=True):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((n, h, w, c)) * np.exp2(rng.integers(-3, 4, size=(n, h, w, 1)))).astype(np.float32)
    wm = (rng.standard_normal((r * s * c, f)) * 0.1).astype(np.float32)
    conv = hb.Conv2d(n, h, w, c, r, s, pad_h, pad_w, sh, sw, 0, 0)
    ho, wo = conv.out_hw()
    print(f"[conv] n={n} h={h} w={w} c={c} f={f} r={r} s={s} pad=({pad_h},{pad_w}) stride=({sh},{sw}) -> {n * ho * wo} x {f}", flush=True)
    img = hb.encode(torch.from_numpy(x.reshape(n * h * w, c)).cuda(), 1, hb.make_format(8, 1, 32))
    flt = hb.encode(torch.from_numpy(wm).cuda(), 0, hb.make_format(8, 32, 1))
    y0 = None
    if beta:
        y0 = rng.standard_normal((n * ho * wo, f)).astype(np.float32)
        y = hb.gemm_conv2d(img, conv, flt, out=torch.from_numpy(y0).cuda(), beta=1.0)
    else:
        y = hb.gemm_conv2d(img, conv, flt)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    # the oracle: convert the image (blocks of 32 channels), lower the decoded values tap by tap, multiply in FP64
    xq = ref.decode(ref.encode(x.reshape(n * h * w, c), 1, 32, 8)).reshape(n, h, w, c)
    low = ref.im2col(xq, r, s, pad_h, pad_w, sh, sw)
    # converting the lowered matrix instead gives the same operand (pinned here on the CPU side of the test)
    np.testing.assert_array_equal(ref.decode(ref.encode(ref.im2col(x, r, s, pad_h, pad_w, sh, sw), 1, 32, 8)), low)
    want = ref.gemm(low, ref.decode(ref.encode(wm, 32, 1, 8)))
    if y0 is not None:
        want = want + y0.astype(np.float64)
    err = rel_fro(y, want)
    print(f"        rel fro err = {err:.3e}", flush=True)
    assert err <= TOL
    if against_lowered and not beta:
        ta = hb.encode_im2col(torch.from_numpy(x).cuda(), conv, hb.make_format(8, 1, 32))
        yl = hb.gemm(ta, flt, kernel=hb.KERNEL_INT8)
        torch.cuda.synchronize()
        assert np.array_equal(y, yl.cpu().numpy()), "differs from the product on the lowered operand"


@pytest.mark.parametrize("geom", [
    # n, h, w, c, f, r, s, pad_h, pad_w, stride_h, stride_w
    (2, 12, 13, 64, 40, 3, 3, 1, 1, 1, 1),
    (3, 9, 9, 128, 130, 3, 3, 1, 1, 1, 1),
    (2, 10, 11, 64, 24, 1, 1, 0, 0, 1, 1),          # a 1 x 1 convolution: a plain product, k = 64 stored as 128
    (2, 14, 9, 64, 50, 5, 3, 2, 1, 1, 1),
    (2, 15, 16, 128, 64, 3, 3, 1, 1, 2, 2),          # strided
    (1, 8, 8, 192, 33, 3, 3, 0, 0, 1, 1),            # no padding, three 64-channel stages per tap (27 stages: odd)
    (2, 7, 7, 64, 20, 3, 3, 2, 2, 1, 3),             # padding wider than the usual, mixed strides
    (5, 6, 6, 64, 16, 2, 2, 0, 1, 2, 1),
])
def test_conv_geometries(hb, geom):
    _conv_case(hb, *geom, seed=sum(geom))


def test_conv_accumulates_and_splits_k(hb):
    _conv_case(hb, 2, 12, 13, 64, 40, 3, 3, 1, 1, 1, 1, seed=5, beta=1.0)
    _conv_case(hb, 1, 6, 6, 1024, 100, 3, 3, 1, 1, 1, 1, seed=6)            # few tiles, k = 9216: split along k
    _conv_case(hb, 1, 6, 6, 1024, 100, 3, 3, 1, 1, 1, 1, seed=7, beta=1.0)


def test_conv_random_geometries(hb):
    for seed in random_cases(12):
        rng = np.random.default_rng(9000 + seed)
        r, s = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        h, w = int(rng.integers(r, 14)), int(rng.integers(s, 14))
        geom = (int(rng.integers(1, 4)), h, w, 64 * int(rng.integers(1, 4)), int(rng.integers(1, 150)), r, s,
                int(rng.integers(0, r)), int(rng.integers(0, s)), int(rng.integers(1, 3)), int(rng.integers(1, 3)))
        _conv_case(hb, *geom, seed=seed)


def test_conv_data_gradient_of_a_stride_one_convolution(hb):
    """dX of y = conv(x, w) with padding 1: the same call on dY with padding r - 1 - pad = 1 and the mirrored filter with
    its channel axes exchanged, against the adjoint of the convolution sum taken in FP64 from the decoded operands."""
    rng = np.random.default_rng(44)
    n, h, w, c, f = 2, 9, 10, 64, 128
    w4 = (rng.standard_normal((3, 3, c, f)) * 0.1).astype(np.float32)
    dy = (rng.standard_normal((n, h, w, f)) * 1e-2).astype(np.float32)
    wd = ref.filter_matrix_dgrad(w4)                                       # [3*3*f, c]
    conv = hb.Conv2d(n, h, w, f, 3, 3, 1, 1, 1, 1, 0, 0)
    img = hb.encode(torch.from_numpy(dy.reshape(n * h * w, f)).cuda(), 1, hb.make_format(8, 1, 32))
    flt = hb.encode(torch.from_numpy(np.ascontiguousarray(wd)).cuda(), 0, hb.make_format(8, 32, 1))
    dx = hb.gemm_conv2d(img, conv, flt)
    torch.cuda.synchronize()
    dyq = ref.decode(ref.encode(dy.reshape(n * h * w, f), 1, 32, 8)).reshape(n, h, w, f).astype(np.float64)
    wq = ref.decode(ref.encode(np.ascontiguousarray(wd), 32, 1, 8)).astype(np.float64).reshape(3, 3, f, c)   # mirrored, [fr][fs][f][c]
    # adjoint, written out: dx[img, y, x, ch] = sum_{fr, fs, f} dy[img, y + 1 - fr, x + 1 - fs, f] * w4[fr, fs, ch, f]
    # where wq[2 - fr, 2 - fs, f, ch] is the quantised w4[fr, fs, ch, f]
    want = np.zeros((n, h, w, c))
    dyp = np.zeros((n, h + 2, w + 2, f))
    dyp[:, 1:-1, 1:-1] = dyq
    for fr in range(3):
        for fs in range(3):
            want += dyp[:, 2 - fr:2 - fr + h, 2 - fs:2 - fs + w, :] @ wq[2 - fr, 2 - fs]
    assert rel_fro(dx.cpu().numpy(), want.reshape(n * h * w, c)) <= TOL


def _slot_case(hb, n, h, w, c, f, r, s, pad_h, pad_w, sh, sw, kb, by_block, per_image, tiles, seed, beta=0.0):
    """The general gather: channels in blocks of kb (stored padded to 32), window entries tap by tap or channel block by
    channel block (by_block), the image with one exponent per pixel and block or one per training input (per_image), the
    filter with one exponent per column and block or in tiles (tiles: kb x kb tap by tap, the whole window x kb channels
    x 24 filters by block - the tiling of the two outer filter dimensions of Sec. 5.1)."""
    rng = np.random.default_rng(seed)
    x = (np.maximum(rng.standard_normal((n, h, w, c)), -0.5) * np.exp2(rng.integers(-3, 4, size=(n, 1, 1, 1)))).astype(np.float32)
    w4 = (rng.standard_normal((r, s, c, f)) * np.exp2(rng.integers(-4, 5, size=(1, 1, c, 1))) * 0.1).astype(np.float32)
    cb = kb if by_block else 0
    wmat = np.ascontiguousarray(ref.filter_matrix(w4, cb))
    conv = hb.Conv2d(n, h, w, c, r, s, pad_h, pad_w, sh, sw, cb, 0)
    ho, wo = conv.out_hw()
    print(f"[slots] n={n} h={h} w={w} c={c} f={f} r={r} s={s} pad=({pad_h},{pad_w}) stride=({sh},{sw}) blocks of {kb} "
          f"{'by block' if by_block else 'by tap'} {'per image' if per_image else 'per pixel'} {'tiles' if tiles else 'columns'}", flush=True)
    x2 = x.reshape(n * h * w, c)
    if per_image:
        img = hb.encode(torch.from_numpy(x2).cuda(), 1, hb.make_format(8, h * w, 0, k_slot=kb))
        xq = ref.decode(ref.encode(x.reshape(n, -1), 1, 0, 8)).reshape(n, h, w, c)
        low_fmt = hb.make_format(8, ho * wo, 0, k_slot=kb)
    else:
        img = hb.encode(torch.from_numpy(x2).cuda(), 1, hb.make_format(8, 1, kb))
        xq = ref.decode(ref.encode(x2, 1, kb, 8)).reshape(n, h, w, c)
        low_fmt = hb.make_format(8, 1, kb)
    if tiles and by_block:
        flt = hb.encode(torch.from_numpy(wmat).cuda(), 0, hb.make_format(8, r * s * kb, 24, k_slot=kb))
        wq = ref.decode(ref.encode(wmat, r * s * kb, 24, 8))
    elif tiles:
        flt = hb.encode(torch.from_numpy(wmat).cuda(), 0, hb.make_format(8, kb, kb))
        wq = ref.decode(ref.encode(wmat, kb, kb, 8))
    else:
        flt = hb.encode(torch.from_numpy(wmat).cuda(), 0, hb.make_format(8, kb, 1))
        wq = ref.decode(ref.encode(wmat, kb, 1, 8))
    y0 = None
    if beta:
        y0 = rng.standard_normal((n * ho * wo, f)).astype(np.float32)
        y = hb.gemm_conv2d(img, conv, flt, out=torch.from_numpy(y0).cuda(), beta=1.0)
    else:
        y = hb.gemm_conv2d(img, conv, flt)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    want = ref.gemm(ref.im2col(xq, r, s, pad_h, pad_w, sh, sw, cb), wq)
    if y0 is not None:
        want = want + y0.astype(np.float64)
    err = rel_fro(y, want)
    print(f"        rel fro err = {err:.3e}", flush=True)
    assert np.linalg.norm(want) > 0 and err <= TOL
    if not beta and not (per_image and ho * wo == 1):     # hbfp_encode_im2col has no one-exponent-per-row form with k_slot
        ta = hb.encode_im2col(torch.from_numpy(x).cuda(), conv, low_fmt)
        yl = hb.gemm(ta, flt, kernel=hb.KERNEL_INT8)
        torch.cuda.synchronize()
        if by_block and per_image and tiles and r * s > 1:
            # both operands repeat their exponents over the taps of a channel block: the gather scales such a run once,
            # the product on the lowered operand block by block - the same sum with fewer roundings
            assert rel_fro(y, yl.cpu().numpy()) <= 2e-6
        else:
            assert np.array_equal(y, yl.cpu().numpy()), "differs from the product on the lowered operand"


@pytest.mark.parametrize("geom", [
    # n, h, w, c, f, r, s, pad_h, pad_w, stride_h, stride_w, block, by block, per image, filter tiles
    (3, 9, 9, 48, 50, 3, 3, 1, 1, 1, 1, 24, True, True, True),          # the format of Sec. 5.1 in full
    (2, 10, 8, 72, 30, 3, 3, 1, 1, 1, 1, 24, True, True, True),         # 27 slots: an odd number, the last stage half empty
    (2, 10, 8, 72, 30, 3, 3, 1, 1, 2, 2, 24, True, False, False),
    (2, 9, 11, 48, 70, 3, 3, 1, 1, 1, 1, 24, False, True, True),        # tap by tap, 24 x 24 filter tiles
    (2, 9, 11, 96, 40, 3, 3, 1, 1, 1, 1, 32, False, False, False),      # blocks of 32 but 96 channels: three slots per tap
    (2, 8, 8, 32, 20, 5, 3, 2, 1, 1, 1, 32, False, False, False),       # one slot per tap
    (2, 8, 8, 32, 20, 3, 3, 1, 1, 1, 1, 16, True, False, False),        # blocks of 16
    (3, 7, 9, 24, 24, 1, 1, 0, 0, 1, 1, 8, False, False, False),        # blocks of 8, a 1 x 1 convolution
    (2, 12, 12, 24, 40, 2, 2, 0, 0, 2, 2, 24, True, True, True),        # a single channel block
    (1, 6, 6, 960, 100, 3, 3, 1, 1, 1, 1, 24, True, True, True),        # few tiles, 360 slots: split along k
    (1, 2, 1, 8, 128, 1, 1, 0, 0, 1, 1, 8, True, True, False),          # two pixels, one slot
    (2, 9, 9, 64, 40, 3, 3, 1, 1, 1, 1, 32, True, True, True),          # runs of 9 blocks of 32: scaled after 8 and after 1
    (2, 8, 10, 48, 30, 5, 5, 2, 2, 1, 1, 24, True, True, True),         # runs of 25
    (2, 11, 7, 16, 30, 2, 1, 0, 0, 1, 1, 8, True, True, True),          # runs of 2 blocks of 8
])
def test_conv_general_gather(hb, geom):
    _slot_case(hb, *geom, seed=sum(int(g) for g in geom))


def test_conv_general_gather_accumulates(hb):
    _slot_case(hb, 3, 9, 9, 48, 50, 3, 3, 1, 1, 1, 1, 24, True, True, True, seed=3, beta=1.0)
    _slot_case(hb, 1, 6, 6, 960, 100, 3, 3, 1, 1, 1, 1, 24, True, True, True, seed=4, beta=1.0)


def test_conv_general_gather_random(hb):
    for seed in random_cases(12):
        rng = np.random.default_rng(9700 + seed)
        r, s = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        h, w = int(rng.integers(r, 13)), int(rng.integers(s, 13))
        kb = int(rng.choice([8, 16, 24, 32]))
        geom = (int(rng.integers(1, 4)), h, w, kb * int(rng.integers(1, 6)), int(rng.integers(1, 150)), r, s,
                int(rng.integers(0, r)), int(rng.integers(0, s)), int(rng.integers(1, 3)), int(rng.integers(1, 3)),
                kb, bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2)))
        _slot_case(hb, *geom, seed=seed)


def _conv_bfp_case(hb, n, h, w, c, f, r, s, pad, st, kb, by_block, per_image, tiles, out_fmt, relu, seed):
    """hbfp_gemm_conv2d_bfp against the oracle's conversion of the library's own FP32 convolution (bit for bit: the same
    product, converted in the kernel or behind it), whose parity with the oracle the tests above establish."""
    from tests.util import unpack
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((n, h, w, c)) * np.exp2(rng.integers(-3, 4, size=(n, 1, 1, 1)))).astype(np.float32)
    w4 = (rng.standard_normal((r, s, c, f)) * 0.1).astype(np.float32)
    cb = kb if by_block else 0
    wmat = np.ascontiguousarray(ref.filter_matrix(w4, cb))
    conv = hb.Conv2d(n, h, w, c, r, s, pad, pad, st, st, cb, 0)
    ho, wo = conv.out_hw()
    f_img = hb.make_format(8, h * w, 0, k_slot=kb) if per_image else hb.make_format(8, 1, kb)
    f_flt = (hb.make_format(8, r * s * kb, 24, k_slot=kb) if by_block else hb.make_format(8, kb, kb)) if tiles else hb.make_format(8, kb, 1)
    img = hb.encode(torch.from_numpy(x.reshape(n * h * w, c)).cuda(), 1, f_img)
    flt = hb.encode(torch.from_numpy(wmat).cuda(), 0, f_flt)
    print(f"[conv bfp] n={n} h={h} w={w} c={c} f={f} r={r} s={s} pad={pad} stride={st} blocks of {kb} by_block={by_block} "
          f"per_image={per_image} tiles={tiles} out={out_fmt} relu={relu}", flush=True)
    m, br, bc, rounding, sd = out_fmt
    out = hb.gemm_conv2d_bfp(img, conv, flt, hb.make_format(m, br, bc, rounding, sd), relu=relu)
    y = hb.gemm_conv2d(img, conv, flt)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    if relu:
        y = np.maximum(y, 0.0)
    want = ref.encode(y, br, bc, m, rounding, sd)
    mant, exps = unpack(out)
    np.testing.assert_array_equal(exps, want.exps)
    np.testing.assert_array_equal(mant, want.mant)
    assert np.abs(mant).max() > 0


@pytest.mark.parametrize("case", [
    # n, h, w, c, f, r, s, pad, stride, block, by block, per image, tiles, (m, block rows, block cols, rounding, seed), relu
    (2, 12, 13, 64, 40, 3, 3, 1, 1, 32, False, False, False, (8, 1, 32, 0, 0), True),       # 64 channels per stage; 40 filters: a ragged block
    (3, 9, 9, 128, 130, 3, 3, 1, 1, 32, False, False, False, (8, 1, 32, 1, 77), False),      # stochastic rounding, two column tiles
    (2, 15, 16, 128, 64, 3, 3, 1, 2, 32, False, False, False, (6, 1, 32, 0, 0), True),       # strided, 6-bit output
    (3, 9, 9, 48, 50, 3, 3, 1, 1, 24, True, True, True, (8, 1, 32, 0, 0), True),             # Sec. 5.1's pairing, runs scaled once
    (2, 10, 8, 72, 96, 3, 3, 1, 1, 24, False, False, False, (8, 1, 32, 1, 5), True),         # slot by slot
    (2, 12, 13, 64, 40, 3, 3, 1, 1, 32, False, False, False, (8, 1, 24, 0, 0), True),        # blocks of 24: converted behind the product
    (2, 12, 13, 64, 40, 3, 3, 1, 1, 32, False, False, False, (12, 1, 32, 0, 0), False),      # 12 bits: behind the product
    (1, 6, 6, 1024, 100, 3, 3, 1, 1, 32, False, False, False, (8, 1, 32, 0, 0), True),       # split along k: behind the product
    (2, 12, 12, 24, 40, 2, 2, 0, 2, 24, True, True, True, (8, 144 // 4, 0, 0, 0), False),    # one exponent per training input out: behind
])
def test_conv_delivered_as_an_encoded_operand(hb, case):
    _conv_bfp_case(hb, *case, seed=sum(int(v) for v in case[:9]))


def test_conv_delivered_as_an_encoded_operand_random(hb):
    for seed in random_cases(10):
        rng = np.random.default_rng(9800 + seed)
        r, s = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        h, w = int(rng.integers(max(r, s), 14)), int(rng.integers(max(r, s), 14))
        kb = int(rng.choice([8, 16, 24, 32]))
        by_block = bool(rng.integers(0, 2))
        per_image = bool(rng.integers(0, 2))
        _conv_bfp_case(hb, int(rng.integers(1, 4)), h, w, kb * int(rng.integers(1, 6)), int(rng.integers(1, 200)), r, s,
                       int(rng.integers(0, min(r, s))), int(rng.integers(1, 3)), kb, by_block, per_image, by_block and per_image,
                       (int(rng.integers(4, 9)), 1, 32, int(rng.integers(0, 2)), seed), bool(rng.integers(0, 2)), seed)


def test_conv_data_gradient_of_a_stride_one_convolution_in_the_format_of_the_experiments(hb):
    """Stride 1: the data gradient is hbfp_gemm_conv2d itself on dY (padding r - 1 - pad) in any format the gather takes;
    here dY with one exponent per training input in blocks of 24 filters, the mirrored filter in tiles over the whole
    window, 24 filters and 24 channels, against the oracle's lowered dY times its decoded filter."""
    rng = np.random.default_rng(52)
    n, h, w, c, f, r, s, pad = 3, 9, 10, 50, 72, 3, 3, 1
    dy = (rng.standard_normal((n, h, w, f)) * 1e-2 * np.exp2(rng.integers(-3, 4, size=(n, 1, 1, 1)))).astype(np.float32)
    w4 = (rng.standard_normal((r, s, c, f)) * np.exp2(rng.integers(-3, 4, size=(1, 1, 1, f))) * 0.1).astype(np.float32)
    wd = np.ascontiguousarray(ref.filter_matrix_dgrad(w4, 24))                                  # [(f block, tap, f in block), c]
    conv = hb.Conv2d(n, h, w, f, r, s, r - 1 - pad, s - 1 - pad, 1, 1, 24, 0)
    img = hb.encode(torch.from_numpy(dy.reshape(n * h * w, f)).cuda(), 1, hb.make_format(8, h * w, 0, k_slot=24))
    flt = hb.encode(torch.from_numpy(wd).cuda(), 0, hb.make_format(8, r * s * 24, 24, k_slot=24))
    dx = hb.gemm_conv2d(img, conv, flt)
    torch.cuda.synchronize()
    dyq = ref.decode(ref.encode(dy.reshape(n, -1), 1, 0, 8)).reshape(n, h, w, f)
    low = ref.im2col_dgrad(dyq, h, w, r, s, pad, pad)                                             # columns (tap, f)
    low = low.reshape(n * h * w, r * s, f // 24, 24).transpose(0, 2, 1, 3).reshape(n * h * w, -1)  # -> (f block, tap, f in block)
    want = ref.gemm(low, ref.decode(ref.encode(wd, r * s * 24, 24, 8)))
    assert np.linalg.norm(want) > 0 and rel_fro(dx.cpu().numpy(), want) <= TOL


def _dgrad_case(hb, n, h, w, c, f, r, s, pad_h, pad_w, sh, sw, seed, beta=0.0, kb=32, by_block=False, per_image=False, tiles=False):
    """hbfp_gemm_conv2d_dgrad against the oracle (dY converted, spread out and lowered explicitly, FP64 product with the
    converted mirrored filter) and, bit for bit, against hbfp_gemm_conv2d on a dY whose zeros are really stored.
    kb / by_block / per_image / tiles: the formats of _slot_case, with the filters of dY in the place of the channels."""
    rng = np.random.default_rng(seed)
    ho, wo = (h + 2 * pad_h - r) // sh + 1, (w + 2 * pad_w - s) // sw + 1
    print(f"[dgrad] n={n} h={h} w={w} c={c} f={f} r={r} s={s} pad=({pad_h},{pad_w}) stride=({sh},{sw}) dy {ho}x{wo} blocks of {kb} "
          f"{'by block' if by_block else 'by tap'} {'per image' if per_image else 'per pixel'} {'tiles' if tiles else 'columns'}", flush=True)
    dy = (rng.standard_normal((n, ho, wo, f)) * 1e-2 * np.exp2(rng.integers(-3, 4, size=(n, 1 if per_image else ho, 1 if per_image else wo, 1)))).astype(np.float32)
    w4 = (rng.standard_normal((r, s, c, f)) * 0.1).astype(np.float32)
    cb = kb if by_block else 0
    wd = np.ascontiguousarray(ref.filter_matrix_dgrad(w4, cb))             # [r*s*f, c]
    conv = hb.Conv2d(n, h, w, c, r, s, pad_h, pad_w, sh, sw, cb, 0)
    assert conv.out_hw() == (ho, wo)
    f_img = (lambda rows: hb.make_format(8, rows, 0, k_slot=kb)) if per_image else (lambda rows: hb.make_format(8, 1, kb))
    f_flt = (hb.make_format(8, r * s * kb, 24, k_slot=kb) if by_block else hb.make_format(8, kb, kb)) if tiles else hb.make_format(8, kb, 1)
    o_flt = ((r * s * kb, 24) if by_block else (kb, kb)) if tiles else (kb, 1)
    img = hb.encode(torch.from_numpy(dy.reshape(n * ho * wo, f)).cuda(), 1, f_img(ho * wo))
    flt = hb.encode(torch.from_numpy(wd).cuda(), 0, f_flt)
    x0 = None
    if beta:
        x0 = rng.standard_normal((n * h * w, c)).astype(np.float32)
        dx = hb.gemm_conv2d_dgrad(img, conv, flt, out=torch.from_numpy(x0).cuda(), beta=1.0)
    else:
        dx = hb.gemm_conv2d_dgrad(img, conv, flt)
    torch.cuda.synchronize()
    dx = dx.cpu().numpy()
    dyq = (ref.decode(ref.encode(dy.reshape(n, -1), 1, 0, 8)) if per_image else ref.decode(ref.encode(dy.reshape(n * ho * wo, f), 1, kb, 8))).reshape(n, ho, wo, f)
    low = ref.im2col_dgrad(dyq, h, w, r, s, pad_h, pad_w, sh, sw)          # columns (tap, filter)
    if by_block:                                                           # -> (filter block, tap, filter in block)
        low = low.reshape(n * h * w, r * s, f // kb, kb).transpose(0, 2, 1, 3).reshape(n * h * w, -1)
    want = ref.gemm(low, ref.decode(ref.encode(wd, o_flt[0], o_flt[1], 8)))
    if x0 is not None:
        want = want + x0.astype(np.float64)
    err = rel_fro(dx, want)
    print(f"        rel fro err = {err:.3e}", flush=True)
    assert err <= TOL
    ph, pw = r - 1 - pad_h, s - 1 - pad_w
    if ph >= 0 and pw >= 0 and not beta:
        hc, wc = h + r - 1 - 2 * ph, w + s - 1 - 2 * pw                 # the spread-out dY, with the rows no window reaches
        spread = np.zeros((n, hc, wc, f), dtype=np.float32)
        spread[:, 0:(ho - 1) * sh + 1:sh, 0:(wo - 1) * sw + 1:sw, :] = dy
        simg = hb.encode(torch.from_numpy(spread.reshape(n * hc * wc, f)).cuda(), 1, f_img(hc * wc))
        sconv = hb.Conv2d(n, hc, wc, f, r, s, ph, pw, 1, 1, cb, 0)
        assert sconv.out_hw() == (h, w)
        ds = hb.gemm_conv2d(simg, sconv, flt)
        torch.cuda.synchronize()
        assert np.array_equal(dx, ds.cpu().numpy()), "differs from the convolution of the stored spread-out gradient"


@pytest.mark.parametrize("geom", [
    # n, h, w, c, f, r, s, pad_h, pad_w, stride_h, stride_w   (of the forward convolution)
    (2, 12, 12, 40, 64, 3, 3, 1, 1, 2, 2),           # the last row and column of x are reached by part of a window only
    (2, 13, 11, 128, 128, 3, 3, 1, 1, 2, 2),
    (3, 9, 10, 64, 64, 3, 3, 1, 1, 1, 1),            # stride 1: the plain gather
    (2, 14, 14, 130, 64, 1, 1, 0, 0, 2, 2),          # a strided 1 x 1 convolution: three quarters of dx are zero
    (1, 17, 15, 24, 192, 5, 3, 2, 1, 3, 2),
    (2, 10, 9, 64, 64, 2, 2, 0, 0, 2, 2),            # windows that tile the image
    (2, 9, 9, 33, 64, 3, 3, 0, 0, 4, 4),             # stride beyond the window: rows of x that no window touches
    (2, 6, 7, 20, 64, 2, 2, 3, 2, 2, 2),             # padding wider than the window
])
def test_conv_data_gradient_geometries(hb, geom):
    _dgrad_case(hb, *geom, seed=sum(geom) + 1)


@pytest.mark.parametrize("geom", [
    # n, h, w, c, f, r, s, pad_h, pad_w, stride_h, stride_w, block, by block, per image, filter tiles
    (2, 12, 12, 40, 48, 3, 3, 1, 1, 2, 2, 24, True, True, True),       # the format of Sec. 5.1, strided
    (2, 11, 9, 30, 72, 3, 3, 1, 1, 2, 1, 24, False, True, True),
    (2, 10, 10, 50, 96, 3, 3, 1, 1, 2, 2, 32, False, False, False),    # 96 filters in blocks of 32: three slots per tap
    (2, 9, 9, 20, 32, 2, 2, 0, 0, 3, 3, 16, True, False, False),
    (3, 8, 8, 24, 48, 3, 3, 1, 1, 1, 1, 24, True, True, True),         # stride 1 in that format
    (1, 7, 7, 100, 960, 3, 3, 1, 1, 2, 2, 24, True, True, True),       # few tiles, 360 slots: split along k
])
def test_conv_data_gradient_general_formats(hb, geom):
    n, h, w, c, f, r, s, ph, pw, sh, sw, kb, by_block, per_image, tiles = geom
    _dgrad_case(hb, n, h, w, c, f, r, s, ph, pw, sh, sw, seed=sum(int(g) for g in geom), kb=kb, by_block=by_block, per_image=per_image, tiles=tiles)


def test_conv_data_gradient_general_formats_random(hb):
    for seed in random_cases(12):
        rng = np.random.default_rng(9900 + seed)
        r, s = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        h, w = int(rng.integers(r, 14)), int(rng.integers(s, 14))
        kb = int(rng.choice([8, 16, 24, 32]))
        _dgrad_case(hb, int(rng.integers(1, 4)), h, w, int(rng.integers(1, 150)), kb * int(rng.integers(1, 6)), r, s,
                    int(rng.integers(0, r + 1)), int(rng.integers(0, s + 1)), int(rng.integers(1, 4)), int(rng.integers(1, 4)), seed=seed,
                    kb=kb, by_block=bool(rng.integers(0, 2)), per_image=bool(rng.integers(0, 2)), tiles=bool(rng.integers(0, 2)))


def test_conv_data_gradient_accumulates_and_splits_k(hb):
    _dgrad_case(hb, 2, 12, 12, 40, 64, 3, 3, 1, 1, 2, 2, seed=15, beta=1.0)
    _dgrad_case(hb, 1, 8, 8, 100, 1024, 3, 3, 1, 1, 2, 2, seed=16)         # few tiles, k = 9216: split along k
    _dgrad_case(hb, 1, 8, 8, 100, 1024, 3, 3, 1, 1, 2, 2, seed=17, beta=1.0)


def test_conv_data_gradient_random_geometries(hb):
    for seed in random_cases(12):
        rng = np.random.default_rng(9500 + seed)
        r, s = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        h, w = int(rng.integers(r, 16)), int(rng.integers(s, 16))
        geom = (int(rng.integers(1, 4)), h, w, int(rng.integers(1, 150)), 64 * int(rng.integers(1, 4)), r, s,
                int(rng.integers(0, r + 1)), int(rng.integers(0, s + 1)), int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        _dgrad_case(hb, *geom, seed=seed)


def test_conv_data_gradient_under_graph_replay(hb):
    """Conversion of dY + hbfp_gemm_conv2d_dgrad (phase by phase) captured in a HIP graph and replayed on new gradients in
    the same buffers, with eager work in between; every replay against the eager result (bit for bit) and the oracle."""
    n, h, w, c, f, r, s, pad, st = 2, 11, 12, 48, 64, 3, 3, 1, 2
    conv = hb.Conv2d(n, h, w, c, r, s, pad, pad, st, st, 0, 0)
    ho, wo = conv.out_hw()
    rng = np.random.default_rng(71)
    w4 = (rng.standard_normal((r, s, c, f)) * 0.1).astype(np.float32)
    wd = np.ascontiguousarray(ref.filter_matrix_dgrad(w4))
    flt = hb.encode(torch.from_numpy(wd).cuda(), 0, hb.make_format(8, 32, 1))
    fmt = hb.make_format(8, 1, 32)
    dy = torch.zeros((n * ho * wo, f), device="cuda")
    td = hb.encode(dy, 1, fmt)
    dx = torch.empty((n * h * w, c), device="cuda")
    ws = torch.empty(hb.gemm_conv2d_dgrad_workspace(td.desc, conv, flt.desc), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        hb.encode(dy, 1, fmt, out=td, stream=stream)
        hb.gemm_conv2d_dgrad(td, conv, flt, out=dx, workspace=ws, stream=stream)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            hb.encode(dy, 1, fmt, out=td, stream=stream)
            hb.gemm_conv2d_dgrad(td, conv, flt, out=dx, workspace=ws, stream=stream)
    for i, scale in enumerate([1e-2, 3.0, 2.0 ** -100, 1e-3]):
        g = (rng.standard_normal((n, ho, wo, f)) * scale).astype(np.float32)
        dy.copy_(torch.from_numpy(g.reshape(n * ho * wo, f)).cuda())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = dx.cpu().numpy().copy()
        eager = hb.gemm_conv2d_dgrad(hb.encode(dy, 1, fmt), conv, flt)
        torch.cuda.synchronize()
        print(f"[case] dgrad graph replay {i} scale={scale}", flush=True)
        assert np.array_equal(got, eager.cpu().numpy())
        gq = ref.decode(ref.encode(g.reshape(n * ho * wo, f), 1, 32, 8)).reshape(n, ho, wo, f)
        want = ref.gemm(ref.im2col_dgrad(gq, h, w, r, s, pad, pad, st, st), ref.decode(ref.encode(wd, 32, 1, 8)))
        assert np.linalg.norm(want) > 0 and rel_fro(got, want) <= TOL


def test_conv_data_gradient_rejects_what_it_does_not_cover(hb):
    import ctypes
    conv = hb.Conv2d(2, 8, 8, 48, 3, 3, 1, 1, 2, 2, 0, 0)                  # dy 4 x 4
    dy = hb.encode(torch.zeros((2 * 4 * 4, 64), device="cuda"), 1, hb.make_format(8, 1, 32))
    flt = hb.encode(torch.zeros((9 * 64, 48), device="cuda"), 0, hb.make_format(8, 32, 1))
    dx = torch.empty((128, 48), device="cuda")
    ws = torch.empty(hb.gemm_conv2d_dgrad_workspace(dy.desc, conv, flt.desc), dtype=torch.uint8, device="cuda")
    call = lambda d, c, f_, ldx=48, beta=0.0, w=ws: hb._lib.hbfp_gemm_conv2d_dgrad(
        ctypes.byref(d.desc), ctypes.byref(c), ctypes.byref(f_.desc), dx.data_ptr(), ldx, beta, w.data_ptr(), w.numel(), None)
    assert call(dy, conv, flt) == hb.OK
    assert call(dy, conv, flt, ldx=40) == hb.ERR_ARG
    assert call(dy, conv, flt, beta=2.0) == hb.ERR_ARG
    assert call(dy, hb.Conv2d(2, 8, 8, 48, 3, 3, 1, 1, 1, 1, 0, 0), flt) == hb.ERR_LAYOUT              # dy of another stride
    assert call(dy, hb.Conv2d(2, 8, 8, 40, 3, 3, 1, 1, 2, 2, 0, 0), flt) == hb.ERR_LAYOUT              # filter of other channels
    assert call(dy, hb.Conv2d(2, 8, 8, 48, 3, 3, 1, 1, 2, 2, 16, 0), flt) == hb.ERR_FORMAT             # channel-block order
    dy24 = hb.encode(torch.zeros((2 * 4 * 4, 64), device="cuda"), 1, hb.make_format(8, 1, 16))
    assert call(dy24, conv, flt) == hb.ERR_FORMAT                                                      # blocks of 16 filters
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    assert call(dy, conv, flt, w=small) == hb.ERR_WORKSPACE
    torch.cuda.synchronize()


def test_conv_rejects_what_it_does_not_cover(hb):
    import ctypes
    x = torch.zeros((2 * 8 * 8, 64), device="cuda")
    img = hb.encode(x, 1, hb.make_format(8, 1, 32))
    flt = hb.encode(torch.zeros((9 * 64, 16), device="cuda"), 0, hb.make_format(8, 32, 1))
    conv = hb.Conv2d(2, 8, 8, 64, 3, 3, 1, 1, 1, 1, 0, 0)
    y = torch.empty((128, 16), device="cuda")
    ws = torch.empty(hb.gemm_conv2d_workspace(img.desc, conv, flt.desc), dtype=torch.uint8, device="cuda")
    call = lambda i, c, f_, ldy=16, beta=0.0, w=ws: hb._lib.hbfp_gemm_conv2d(
        ctypes.byref(i.desc), ctypes.byref(c), ctypes.byref(f_.desc), y.data_ptr(), ldy, beta, w.data_ptr(), w.numel(), None)
    assert call(img, conv, flt) == hb.OK
    assert call(img, conv, flt, ldy=8) == hb.ERR_ARG
    assert call(img, conv, flt, beta=0.5) == hb.ERR_ARG
    assert call(img, hb.Conv2d(2, 8, 8, 64, 3, 3, 1, 1, 1, 1, 16, 0), flt) == hb.ERR_FORMAT            # channel blocks that are not the stored blocks
    assert call(img, hb.Conv2d(2, 8, 9, 64, 3, 3, 1, 1, 1, 1, 0, 0), flt) == hb.ERR_LAYOUT             # not this image
    img24 = hb.encode(x, 1, hb.make_format(8, 1, 24))
    assert call(img24, conv, flt) == hb.ERR_FORMAT                                                       # blocks of 24: 64 channels are no multiple, and the filter has 32
    img16 = hb.encode(x, 1, hb.make_format(8, 1, 16))
    assert call(img16, conv, flt) == hb.ERR_FORMAT                                                       # blocks of 16 against a filter in blocks of 32
    flt5 = hb.encode(torch.zeros((25 * 64, 16), device="cuda"), 0, hb.make_format(8, 32, 1))
    assert call(img, conv, flt5) == hb.ERR_LAYOUT
    assert hb._lib.hbfp_gemm_conv2d(ctypes.byref(img.desc), ctypes.byref(conv), ctypes.byref(flt.desc), y.data_ptr(), 16, 0.0,
                                    None, 0, None) == hb.ERR_WORKSPACE
    torch.cuda.synchronize()
