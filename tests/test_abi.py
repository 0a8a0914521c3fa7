"""CPU-only checks of the C ABI: the library loads, exports what include/hbfp.h declares,
plans the documented geometry and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

from paper_1804_01526_amd import hbfp  # noqa: E402


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hbfp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hbfp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"hbfp_plan", "hbfp_encode", "hbfp_decode", "hbfp_gemm", "hbfp_gemm_partials", "hbfp_gemm_f32"} <= set(names)
    lib = ctypes.CDLL(hbfp.library_path())
    for n in names:
        assert hasattr(lib, n), n
    assert hbfp.version() >= 100
    assert hbfp.status_string(0) == "ok" and "workspace" in hbfp.status_string(hbfp.ERR_WORKSPACE)


def test_sizes_is_the_plan_in_three_numbers():
    for rows, cols, axis, br, bc, m in ((4096, 4096, 1, 1, 24, 8), (8192, 8192, 0, 64, 1, 12), (100, 1000, 1, 1, 0, 8), (77, 130, 0, 24, 24, 16)):
        fmt = hbfp.make_format(m, br, bc)
        d = hbfp.plan(fmt, rows, cols, axis)
        assert hbfp.sizes(fmt, rows, cols, axis) == (d.mant_bytes, d.exp_bytes, d.kpad)
    fmt = hbfp.make_format(8, 1, 32)
    assert hbfp._lib.hbfp_sizes(ctypes.byref(fmt), 0, 5, 1, None, None, None) == hbfp.ERR_ARG
    assert hbfp._lib.hbfp_sizes(ctypes.byref(fmt), 5, 5, 1, None, None, None) == hbfp.OK
    bad = hbfp.make_format(17, 1, 32)
    assert hbfp._lib.hbfp_sizes(ctypes.byref(bad), 5, 5, 1, None, None, None) == hbfp.ERR_FORMAT


def test_struct_sizes_match_the_header():
    assert ctypes.sizeof(hbfp.Format) == 40
    assert ctypes.sizeof(hbfp.TensorDesc) == 144


@pytest.mark.parametrize("rows,cols,axis,br,bc,m,want", [
    # rows cols axis br bc m   -> (R, K, kblock, kbp, nblk, kpad, exp_ld, rblock, mant_bytes)
    (256, 256, 1, 1, 32, 8, (256, 256, 32, 32, 8, 256, 8, 1, 256 * 256)),
    (256, 256, 0, 32, 1, 8, (256, 256, 32, 32, 8, 256, 8, 1, 256 * 256)),
    (4096, 4096, 1, 1, 24, 8, (4096, 4096, 24, 32, 171, 5504, 172, 1, 4096 * 5504)),
    (4096, 4096, 0, 24, 24, 8, (4096, 4096, 24, 32, 171, 5504, 172, 24, 4096 * 5504)),
    (8192, 8192, 1, 1, 64, 12, (8192, 8192, 64, 64, 128, 8192, 128, 1, 8192 * 8192 * 2)),
    (100, 1000, 1, 1, 0, 8, (100, 1000, 1000, 1024, 1, 1024, 4, 1, 100 * 1024)),
    (100, 1000, 0, 0, 0, 16, (1000, 100, 100, 128, 1, 128, 4, 1000, 1000 * 128 * 2)),
    (1, 1 << 26, 1, 1, 32, 8, (1, 1 << 26, 32, 32, 1 << 21, 1 << 26, 1 << 21, 1, 1 << 26)),
])
def test_plan_geometry(rows, cols, axis, br, bc, m, want):
    d = hbfp.plan(hbfp.make_format(m, br, bc), rows, cols, axis)
    got = (d.rows, d.kdim, d.kblock, d.kblock_pad, d.nblk, d.kpad, d.exp_ld, d.rblock, d.mant_bytes)
    assert got == want
    assert d.exp_bytes == d.rows * d.exp_ld and d.mant is None and d.exps is None


@pytest.mark.parametrize("rows,cols,axis,br,bc,slot,want", [
    # exponent blocks longer than the stored blocks -> (kblock, kbp, nblk, kshare, kpad, exp_ld, rblock)
    (64, 4096, 1, 1, 0, 24, (24, 32, 171, 171, 5504, 172, 1)),          # one exponent per row, stored like 24-wide tiles
    (4096, 64, 0, 0, 1, 24, (24, 32, 171, 171, 5504, 172, 1)),
    (64, 4096, 1, 1, 96, 24, (24, 32, 171, 4, 5504, 172, 1)),
    (128, 4096, 1, 64, 64, 32, (32, 32, 128, 2, 4096, 128, 64)),
    (64, 4096, 1, 1, 24, 24, (24, 32, 171, 1, 5504, 172, 1)),           # slot = block: nothing changes
    (64, 4096, 1, 1, 24, 32, (24, 32, 171, 1, 5504, 172, 1)),           # slot longer than the block: ignored
    (64, 100, 1, 1, 0, 128, (100, 128, 1, 1, 128, 4, 1)),
])
def test_plan_geometry_with_k_slot(rows, cols, axis, br, bc, slot, want):
    d = hbfp.plan(hbfp.make_format(8, br, bc, k_slot=slot), rows, cols, axis)
    assert (d.kblock, d.kblock_pad, d.nblk, d.kshare, d.kpad, d.exp_ld, d.rblock) == want
    n = hbfp.encode_workspace(d)
    assert (n > 0) == (d.kshare > 1 or d.kblock > 128)


def test_k_slot_must_divide_the_exponent_block():
    with pytest.raises(hbfp.HbfpError) as e:
        hbfp.plan(hbfp.make_format(8, 1, 100, k_slot=24), 64, 4096, 1)
    assert e.value.status == hbfp.ERR_FORMAT
    with pytest.raises(hbfp.HbfpError) as e:
        hbfp.plan(hbfp.make_format(8, 1, 0, k_slot=-1), 64, 4096, 1)
    assert e.value.status == hbfp.ERR_FORMAT


def _status(fn, *a):
    try:
        fn(*a)
    except hbfp.HbfpError as e:
        return e.status
    return 0


def test_plan_rejects_bad_arguments():
    ok = hbfp.make_format(8, 1, 32)
    assert _status(hbfp.plan, ok, 0, 10, 1) == hbfp.ERR_ARG
    assert _status(hbfp.plan, ok, 10, -1, 1) == hbfp.ERR_ARG
    assert _status(hbfp.plan, ok, 10, 10, 2) == hbfp.ERR_ARG
    assert _status(hbfp.plan, hbfp.make_format(1, 1, 32), 10, 10, 1) == hbfp.ERR_FORMAT
    assert _status(hbfp.plan, hbfp.make_format(17, 1, 32), 10, 10, 1) == hbfp.ERR_FORMAT
    assert _status(hbfp.plan, hbfp.make_format(8, -1, 32), 10, 10, 1) == hbfp.ERR_FORMAT
    assert _status(hbfp.plan, hbfp.make_format(8, 1, 32, rounding=2), 10, 10, 1) == hbfp.ERR_FORMAT


def test_encode_im2col_workspace_sizes():
    """One exponent per training input needs 4 bytes per image at any image size (also where hbfp_encode converts the
    same plan in one pass); blocks inside a pixel need nothing; a plan of another shape is refused."""
    import ctypes
    conv = hbfp.Conv2d(3, 2, 1, 8, 1, 1, 0, 0, 1, 1, 8, 0)                    # three images of 2 x 1 pixels
    per_input = hbfp.plan(hbfp.make_format(8, 2, 0, k_slot=8), 6, 8, 1)
    assert hbfp.encode_workspace(per_input) == 0
    assert hbfp.encode_im2col_workspace(conv, per_input) == 256
    assert hbfp.encode_im2col_workspace(conv, hbfp.plan(hbfp.make_format(8, 1, 8), 6, 8, 1)) == 0
    big = hbfp.Conv2d(100, 28, 28, 24, 3, 3, 1, 1, 1, 1, 0, 0)
    assert hbfp.encode_im2col_workspace(big, hbfp.plan(hbfp.make_format(8, 784, 0, k_slot=24), 78400, 216, 1)) == 512
    n = ctypes.c_size_t(0)
    other = hbfp.plan(hbfp.make_format(8, 1, 8), 7, 8, 1)
    assert hbfp._lib.hbfp_encode_im2col_workspace(ctypes.byref(conv), ctypes.byref(other), ctypes.byref(n)) == hbfp.ERR_LAYOUT
    assert hbfp._lib.hbfp_encode_im2col_workspace(ctypes.byref(conv), ctypes.byref(per_input), None) == hbfp.ERR_ARG


def test_encode_workspace_sizes():
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 1, 32), 64, 256, 1)) == 0
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 32, 1), 256, 64, 0)) == 0
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 1, 128), 64, 256, 1)) == 0
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 128, 1), 256, 64, 0)) > 0
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 24, 24), 100, 100, 0)) == 0
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 24, 24), 100, 100, 1)) == 0
    n = hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 96, 96), 500, 500, 0))
    assert n >= 6 * 6 * 4 and n % 256 == 0
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 32, 100), 100, 100, 1)) == 0
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 0, 0), 100, 100, 1)) == 256
    assert hbfp.encode_workspace(hbfp.plan(hbfp.make_format(8, 0, 0), 2000, 2000, 1)) == 256


def _raw():
    return ctypes.CDLL(hbfp.library_path())


def test_entry_points_validate_before_launching():
    """Every call below must come back with an argument error; none may reach a launch
    (this box has no GPU: a launch would report HBFP_ERR_LAUNCH instead)."""
    lib = hbfp._lib
    fmt = hbfp.make_format(8, 1, 32)
    d = hbfp.plan(fmt, 64, 256, 1)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced on the host
    byref = ctypes.byref
    # null pointers
    assert lib.hbfp_encode(None, 64, 256, 256, 1, byref(fmt), byref(d), None, 0, None) == hbfp.ERR_ARG
    assert lib.hbfp_encode(fake, 64, 256, 256, 1, byref(fmt), byref(d), None, 0, None) == hbfp.ERR_ARG  # mant/exps null
    d.mant, d.exps = 0x10000, 0x20000
    assert lib.hbfp_encode(fake, 64, 256, 100, 1, byref(fmt), byref(d), None, 0, None) == hbfp.ERR_ARG   # ld < cols
    # descriptor planned for another shape
    assert lib.hbfp_encode(fake, 64, 128, 128, 1, byref(fmt), byref(d), None, 0, None) == hbfp.ERR_LAYOUT
    assert lib.hbfp_encode(fake, 64, 256, 256, 0, byref(fmt), byref(d), None, 0, None) == hbfp.ERR_LAYOUT
    bad = hbfp.make_format(8, 1, 32, rounding=7)
    assert lib.hbfp_encode(fake, 64, 256, 256, 1, byref(bad), byref(d), None, 0, None) == hbfp.ERR_FORMAT
    # misaligned buffers
    d.mant = 0x10001
    assert lib.hbfp_encode(fake, 64, 256, 256, 1, byref(fmt), byref(d), None, 0, None) == hbfp.ERR_ARG
    d.mant = 0x10000
    # tile path without workspace
    f2 = hbfp.make_format(8, 96, 96)
    d2 = hbfp.plan(f2, 100, 100, 0)
    d2.mant, d2.exps = 0x10000, 0x20000
    assert lib.hbfp_encode(fake, 100, 100, 100, 0, byref(f2), byref(d2), None, 0, None) == hbfp.ERR_WORKSPACE
    assert lib.hbfp_encode(fake, 100, 100, 100, 0, byref(f2), byref(d2), fake, 16, None) == hbfp.ERR_WORKSPACE
    # decode
    assert lib.hbfp_decode(byref(d), None, 256, None) == hbfp.ERR_ARG
    assert lib.hbfp_decode(byref(d), fake, 100, None) == hbfp.ERR_ARG
    broken = hbfp.plan(fmt, 64, 256, 1)
    broken.mant, broken.exps, broken.kpad = 0x10000, 0x20000, 300
    assert lib.hbfp_decode(byref(broken), fake, 256, None) == hbfp.ERR_LAYOUT


def test_gemm_validation():
    lib = hbfp._lib
    byref = ctypes.byref
    fake = ctypes.c_void_p(0x1000)

    def desc(m, rows, cols, axis, br, bc):
        d = hbfp.plan(hbfp.make_format(m, br, bc), rows, cols, axis)
        d.mant, d.exps = 0x10000, 0x20000
        return d

    a = desc(8, 128, 256, 1, 1, 32)
    b = desc(8, 256, 64, 0, 32, 1)
    assert lib.hbfp_gemm(byref(a), byref(b), None, 64, 0.0, None, 0, None) == hbfp.ERR_ARG
    assert lib.hbfp_gemm(byref(a), byref(b), fake, 32, 0.0, None, 0, None) == hbfp.ERR_ARG       # ldc < N
    assert lib.hbfp_gemm(byref(a), byref(b), fake, 64, 0.5, None, 0, None) == hbfp.ERR_ARG       # beta not 0/1
    b_k = desc(8, 128, 64, 0, 32, 1)                                                               # other K
    assert lib.hbfp_gemm(byref(a), byref(b_k), fake, 64, 0.0, None, 0, None) == hbfp.ERR_LAYOUT
    b_blk = desc(8, 256, 64, 0, 64, 1)                                                             # other block length
    assert lib.hbfp_gemm(byref(a), byref(b_blk), fake, 64, 0.0, None, 0, None) == hbfp.ERR_LAYOUT
    b12 = desc(12, 256, 64, 0, 32, 1)                                                              # mixed mantissa classes
    assert lib.hbfp_gemm(byref(a), byref(b12), fake, 64, 0.0, None, 0, None) == hbfp.ERR_FORMAT
    a16, b16 = desc(16, 128, 256, 1, 1, 32), desc(16, 256, 64, 0, 32, 1)                           # too wide for the product
    assert lib.hbfp_gemm(byref(a16), byref(b16), fake, 64, 0.0, fake, 1 << 20, None) == hbfp.ERR_FORMAT
    # accumulator bound: 12-bit mantissas allow blocks of at most 512
    big_a, big_b = desc(12, 8, 1024, 1, 1, 1024), desc(12, 1024, 8, 0, 1024, 1)
    assert lib.hbfp_gemm(byref(big_a), byref(big_b), fake, 8, 0.0, fake, 1 << 20, None) == hbfp.ERR_RANGE
    # 8-bit mantissas: 133144 fits, 133145 does not (133145 * 127^2 >= 2^31)
    fits_a, fits_b = desc(8, 8, 133144, 1, 1, 0), desc(8, 133144, 8, 0, 0, 1)
    assert lib.hbfp_gemm(byref(fits_a), byref(fits_b), None, 8, 0.0, None, 0, None) == hbfp.ERR_ARG  # passes the range test
    over_a, over_b = desc(8, 8, 133145, 1, 1, 0), desc(8, 133145, 8, 0, 0, 1)
    assert lib.hbfp_gemm(byref(over_a), byref(over_b), fake, 8, 0.0, None, 0, None) == hbfp.ERR_RANGE
    assert lib.hbfp_gemm_partials(byref(a), byref(b), None, None, 0, None) == hbfp.ERR_ARG
    # a window of the block sums must lie inside the product (a: 128 operand rows, b: 64)
    big = 1 << 22
    for row0, rows, col0, cols in ((0, 0, 0, 8), (-1, 8, 0, 8), (121, 8, 0, 8), (0, 129, 0, 8), (0, 8, 57, 8), (0, 8, 0, 65), (0, 8, -2, 4)):
        assert lib.hbfp_gemm_partials_window(byref(a), byref(b), row0, rows, col0, cols, fake, fake, big, None) == hbfp.ERR_ARG
    assert lib.hbfp_gemm_partials_window(byref(a), byref(b), 0, 8, 0, 8, None, fake, big, None) == hbfp.ERR_ARG
    assert lib.hbfp_gemm_partials_window(byref(a), byref(b), 120, 8, 56, 8, fake, None, 0, None) == hbfp.ERR_WORKSPACE


def test_gemm_select_validation():
    """Kernel choice: unknown kernel rejected; the block-scaled kernel needs room for its limb planes; the automatic
    choice takes it only for large products in the formats where it is the faster one."""
    lib = hbfp._lib
    byref = ctypes.byref
    fake = ctypes.c_void_p(0x1000)

    def desc(m, rows, cols, axis, br, bc):
        d = hbfp.plan(hbfp.make_format(m, br, bc), rows, cols, axis)
        d.mant, d.exps = 0x10000, 0x20000
        return d

    a, b = desc(8, 128, 256, 1, 1, 32), desc(8, 256, 64, 0, 32, 1)
    assert lib.hbfp_gemm_select(byref(a), byref(b), fake, 64, 0.0, 7, fake, 1 << 20, None) == hbfp.ERR_ARG
    # the bf16 kernel is for 6..9-bit mantissas on both sides; its workspace holds the bf16 planes of both operands
    # (whole panels of 256 rows, 2 bytes per stored element, a 256-byte header each)
    for m in (4, 5, 10, 12):
        am, bm = desc(m, 128, 256, 1, 1, 32), desc(m, 256, 64, 0, 32, 1)
        assert lib.hbfp_gemm_select(byref(am), byref(bm), fake, 64, 0.0, hbfp.KERNEL_BF16, fake, 1 << 24, None) == hbfp.ERR_FORMAT
    a4 = desc(4, 128, 256, 1, 1, 32)
    assert lib.hbfp_gemm_select(byref(a4), byref(b), fake, 64, 0.0, hbfp.KERNEL_BF16, fake, 1 << 24, None) == hbfp.ERR_FORMAT
    for m in (6, 8, 9):
        am, bm = desc(m, 128, 256, 1, 1, 32), desc(m, 256, 64, 0, 32, 1)
        n_bf = hbfp.gemm_select_workspace(am, bm, hbfp.KERNEL_BF16)
        assert n_bf == 2 * (256 + 256 * 256 * 2) == hbfp.pack_bytes(am) + hbfp.pack_bytes(bm)
        assert lib.hbfp_gemm_select(byref(am), byref(bm), fake, 64, 0.0, hbfp.KERNEL_BF16, fake, n_bf - 256, None) == hbfp.ERR_WORKSPACE
    # the FP16 kernel is for 9..12-bit mantissas in blocks stored as 32, 64 or a multiple of 128 elements
    assert lib.hbfp_gemm_select(byref(a), byref(b), fake, 64, 0.0, hbfp.KERNEL_FP16, fake, 1 << 24, None) == hbfp.ERR_FORMAT
    a12, b12 = desc(12, 128, 256, 1, 1, 32), desc(8, 256, 64, 0, 32, 1)          # both operands have to be wide
    assert lib.hbfp_gemm_select(byref(a12), byref(b12), fake, 64, 0.0, hbfp.KERNEL_FP16, fake, 1 << 24, None) == hbfp.ERR_FORMAT
    # the 256 x 256-tile int8 kernel is for one exponent per operand row: these operands have 8 blocks of 32
    assert lib.hbfp_gemm_select(byref(a), byref(b), fake, 64, 0.0, hbfp.KERNEL_INT8_WIDE, fake, 1 << 20, None) == hbfp.ERR_FORMAT
    a1, b1 = desc(8, 128, 256, 1, 1, 0), desc(8, 256, 64, 0, 0, 1)
    assert hbfp.gemm_select_workspace(a1, b1, hbfp.KERNEL_INT8_WIDE) == hbfp.gemm_select_workspace(a1, b1, hbfp.KERNEL_INT8)
    a12, b12 = desc(12, 128, 256, 1, 1, 0), desc(12, 256, 64, 0, 0, 1)
    assert lib.hbfp_gemm_select(byref(a12), byref(b12), fake, 64, 0.0, hbfp.KERNEL_INT8_WIDE, fake, 1 << 24, None) == hbfp.ERR_FORMAT
    assert lib.hbfp_gemm_select(byref(a), byref(b), fake, 64, 0.0, -1, fake, 1 << 20, None) == hbfp.ERR_ARG
    assert _status(hbfp.gemm_select_workspace, a, b, 7) == hbfp.ERR_ARG
    n_int8 = hbfp.gemm_select_workspace(a, b, hbfp.KERNEL_INT8)
    n_scaled = hbfp.gemm_select_workspace(a, b, hbfp.KERNEL_SCALED)
    assert hbfp.gemm_select_workspace(a, b, hbfp.KERNEL_AUTO) == n_int8 == hbfp.gemm_workspace(a, b)   # small: int8
    # one 256-row panel per operand, 4 k-steps of 64, two limbs: 8 row tiles x (2 x 1536 + 256) bytes per k-step
    assert n_scaled >= n_int8 + 2 * 4 * 8 * 3328
    assert lib.hbfp_gemm_select(byref(a), byref(b), fake, 64, 0.0, hbfp.KERNEL_SCALED, fake, n_int8, None) == hbfp.ERR_WORKSPACE
    # automatic choice on a 4096^3 product: 6..9-bit mantissas in blocks of 24 (padded to 32) and of 32 -> bf16; blocks of
    # 64 -> int8; 4-bit mantissas -> block-scaled; a 2048^3 product (64 tiles of 256 x 256) -> int8; 12-bit mantissas on
    # both sides -> the FP16 instruction, 12-bit against 8-bit -> block-scaled
    def auto_is(m, blk, kernel):
        x, w = desc(m, 4096, 4096, 1, 1, blk), desc(m, 4096, 4096, 0, blk, 1)
        n = hbfp.gemm_workspace(x, w)
        return n == hbfp.gemm_select_workspace(x, w, kernel) and (kernel == hbfp.KERNEL_INT8 or n != hbfp.gemm_select_workspace(x, w, hbfp.KERNEL_INT8))
    def auto_is_scaled(m, blk):
        return auto_is(m, blk, hbfp.KERNEL_SCALED)
    assert auto_is(8, 32, hbfp.KERNEL_BF16) and auto_is(8, 24, hbfp.KERNEL_BF16) and auto_is(6, 16, hbfp.KERNEL_BF16)
    assert auto_is(9, 32, hbfp.KERNEL_BF16) and auto_is(8, 64, hbfp.KERNEL_INT8)
    x, w = desc(8, 2048, 2048, 1, 1, 32), desc(8, 2048, 2048, 0, 32, 1)
    assert hbfp.gemm_workspace(x, w) == hbfp.gemm_select_workspace(x, w, hbfp.KERNEL_INT8)
    assert auto_is_scaled(4, 64) and auto_is_scaled(5, 24)
    # 12-bit mantissas on both sides: FP16 planes on the 256 x 256-tile kernel where those tiles pay (header, a scale
    # word per row and 2 bytes per stored element for each operand), the FP16 instruction on 128 x 128 tiles elsewhere
    x, w = desc(12, 4096, 4096, 1, 1, 64), desc(12, 4096, 4096, 0, 64, 1)
    planes = hbfp.gemm_select_workspace(x, w, hbfp.KERNEL_FP16_PLANES)
    assert hbfp.gemm_workspace(x, w) == planes == 2 * (256 + 4096 * 4 + 4096 * 4096 * 2)
    assert planes != hbfp.gemm_select_workspace(x, w, hbfp.KERNEL_FP16)
    x, w = desc(12, 1024, 4096, 1, 1, 64), desc(12, 4096, 1024, 0, 64, 1)
    assert hbfp.gemm_workspace(x, w) == hbfp.gemm_select_workspace(x, w, hbfp.KERNEL_FP16)
    for m in (4, 8):
        am, bm = desc(m, 128, 256, 1, 1, 32), desc(m, 256, 64, 0, 32, 1)
        assert lib.hbfp_gemm_select(byref(am), byref(bm), fake, 64, 0.0, hbfp.KERNEL_FP16_PLANES, fake, 1 << 24, None) == hbfp.ERR_FORMAT
    x, w = desc(12, 4096, 4096, 1, 1, 64), desc(12, 4096, 4096, 0, 64, 1)
    w = desc(8, 4096, 4096, 0, 64, 1)
    assert hbfp.gemm_workspace(x, w) == hbfp.gemm_select_workspace(x, w, hbfp.KERNEL_SCALED)
    # narrow output: tiles of 256 x 256 would be half empty
    x, w = desc(8, 100352, 1152, 1, 1, 32), desc(8, 1152, 128, 0, 32, 1)
    assert hbfp.gemm_workspace(x, w) == hbfp.gemm_select_workspace(x, w, hbfp.KERNEL_INT8)


def test_gemm_batch_validation():
    """hbfp_gemm_batch: argument checks happen before any launch; products that fill the chip only together are
    grouped by the automatic choice (seen through the workspace, which then holds the packed operands)."""
    lib = hbfp._lib
    fake = ctypes.c_void_p(0x1000)

    def desc(m, rows, cols, axis, br, bc):
        d = hbfp.plan(hbfp.make_format(m, br, bc), rows, cols, axis)
        d.mant, d.exps = 0x10000, 0x20000
        return d

    def pair(m, M, N, K, blk):
        return desc(m, M, K, 1, 1, blk), desc(m, K, N, 0, blk, 1)

    def call(pairs, kernel=0, ws_bytes=1 << 30, n=None, ldc=None):
        n = len(pairs) if n is None else n
        a, b = hbfp._desc_array([p[0] for p in pairs]), hbfp._desc_array([p[1] for p in pairs])
        c = (ctypes.c_void_p * len(pairs))(*[0x3000] * len(pairs))
        ld = (ctypes.c_int64 * len(pairs))(*(ldc or [p[1].rows for p in pairs]))
        return lib.hbfp_gemm_batch(n, a, b, c, ld, 0.0, kernel, fake, ws_bytes, None)

    small = pair(8, 128, 64, 256, 32)
    assert call([small] * 5) == hbfp.ERR_ARG and call([small], n=0) == hbfp.ERR_ARG
    assert call([small, small], kernel=9) == hbfp.ERR_ARG
    assert call([small, small], ldc=[64, 63]) == hbfp.ERR_ARG
    assert call([small, (small[0], desc(8, 256, 64, 0, 64, 1))]) != hbfp.OK            # blocks disagree
    need = hbfp.gemm_batch_workspace([small, small], hbfp.KERNEL_SCALED)
    assert need == 2 * hbfp.gemm_select_workspace(small[0], small[1], hbfp.KERNEL_SCALED)
    assert call([small, small], kernel=hbfp.KERNEL_SCALED, ws_bytes=need - 256) == hbfp.ERR_WORKSPACE
    assert hbfp.gemm_batch_workspace([small, small]) == 2 * hbfp.gemm_workspace(small[0], small[1])
    # four products of 64 tiles each: alone each takes the int8 kernels, together the bf16 kernel (8-bit mantissas) or
    # the block-scaled kernel (4-bit mantissas)
    q = pair(8, 2048, 2048, 2048, 32)
    alone, scaled = hbfp.gemm_workspace(q[0], q[1]), hbfp.gemm_select_workspace(q[0], q[1], hbfp.KERNEL_SCALED)
    bf = hbfp.gemm_select_workspace(q[0], q[1], hbfp.KERNEL_BF16)
    assert alone < scaled and bf != scaled and bf != alone
    assert hbfp.gemm_batch_workspace([q] * 4) == 4 * bf == hbfp.gemm_batch_workspace([q] * 4, hbfp.KERNEL_BF16)
    assert hbfp.gemm_batch_workspace([q] * 4, hbfp.KERNEL_SCALED) == 4 * scaled
    q4 = pair(4, 2048, 2048, 2048, 32)
    assert hbfp.gemm_batch_workspace([q4] * 4) == 4 * hbfp.gemm_select_workspace(q4[0], q4[1], hbfp.KERNEL_SCALED)
    assert hbfp.gemm_batch_workspace([q] * 2) == 2 * alone                         # 128 tiles: not together either
    assert hbfp.gemm_batch_workspace([q] * 4, hbfp.KERNEL_INT8) == 4 * alone
    q64 = pair(8, 2048, 2048, 2048, 64)                                            # blocks of 64: the int8 kernels are ahead
    assert hbfp.gemm_batch_workspace([q64] * 4) == 4 * hbfp.gemm_workspace(q64[0], q64[1])
    q12 = pair(12, 2048, 2048, 2048, 64)                                           # limb counts differ: one after the other
    assert hbfp.gemm_batch_workspace([q, q, q12, q12]) == 2 * alone + 2 * hbfp.gemm_workspace(q12[0], q12[1])


def test_gemm_packed_batch_validation():
    """hbfp_gemm_packed_batch: every check happens before the launch."""
    lib = hbfp._lib
    fake = ctypes.c_void_p(0x1000)

    def desc(m, rows, cols, axis, br, bc):
        d = hbfp.plan(hbfp.make_format(m, br, bc), rows, cols, axis)
        d.mant, d.exps = 0x10000, 0x20000
        return d

    def call(pairs, n=None, packed=0x4000, c=0x3000, ldc=None, beta=0.0, ws=fake, ws_bytes=1 << 30):
        k = len(pairs)
        n = k if n is None else n
        a, b = hbfp._desc_array([p[0] for p in pairs]), hbfp._desc_array([p[1] for p in pairs])
        pa, pb = (ctypes.c_void_p * k)(*[packed] * k), (ctypes.c_void_p * k)(*[0x8000] * k)
        cs = (ctypes.c_void_p * k)(*[c] * k)
        ld = (ctypes.c_int64 * k)(*(ldc or [p[1].rows for p in pairs]))
        return lib.hbfp_gemm_packed_batch(n, a, pa, b, pb, cs, ld, beta, ws, ws_bytes, None)

    p8 = (desc(8, 128, 256, 1, 1, 24), desc(8, 256, 64, 0, 24, 1))
    p4 = (desc(4, 128, 256, 1, 1, 24), desc(4, 256, 64, 0, 24, 1))
    assert call([p8] * 5) == hbfp.ERR_ARG and call([p8], n=0) == hbfp.ERR_ARG
    assert call([p8, p8], packed=0x4010) == hbfp.ERR_ARG and call([p8, p8], packed=0) == hbfp.ERR_ARG
    assert call([p8, p8], c=0x3001) == hbfp.ERR_ARG and call([p8, p8], ldc=[64, 63]) == hbfp.ERR_ARG
    assert call([p8, p8], beta=0.5) == hbfp.ERR_ARG
    assert call([p8, p4]) == hbfp.ERR_FORMAT
    assert call([p8, (p8[0], desc(8, 256, 64, 0, 32, 1))]) != hbfp.OK            # blocks disagree
    need = hbfp.gemm_packed_batch_workspace([p8, p8])
    assert need == 2 * ((hbfp.gemm_packed_workspace(*p8) + 255) // 256 * 256)
    if need:
        assert call([p8, p8], ws_bytes=need - 256) == hbfp.ERR_WORKSPACE
        assert call([p8, p8], ws=None) == hbfp.ERR_WORKSPACE


def test_encode_packed_batch_validation():
    """hbfp_encode_packed_batch: the checks of hbfp_encode_packed for every job, all before the first launch."""
    lib = hbfp._lib

    def desc(m, rows, cols, axis, br, bc):
        d = hbfp.plan(hbfp.make_format(m, br, bc), rows, cols, axis)
        d.mant, d.exps = 0x10000, 0x20000
        return d

    def job(outs, src=0x100000, ld=None, packed=0x4000, size=1 << 40):
        n = len(outs)
        descs = hbfp._desc_array(outs)
        ptrs, sizes = (ctypes.c_void_p * n)(*[packed] * n), (ctypes.c_size_t * n)(*[size] * n)
        j = hbfp.EncodeJob(src, outs[0].src_cols if ld is None else ld, n, 0, ctypes.cast(descs, ctypes.c_void_p),
                           ctypes.cast(ptrs, ctypes.c_void_p), ctypes.cast(sizes, ctypes.c_void_p))
        return j, (descs, ptrs, sizes)

    def call(jobs, n=None):
        arr = (hbfp.EncodeJob * len(jobs))(*[j[0] for j in jobs])
        return lib.hbfp_encode_packed_batch(len(jobs) if n is None else n, arr, None, 0, None)

    x = [desc(8, 96, 240, 1, 1, 24), desc(8, 96, 240, 0, 24, 1)]
    w = [desc(8, 240, 48, 0, 24, 24)]
    good = job(x)
    assert call([good] * 5) == hbfp.ERR_ARG and call([good], n=0) == hbfp.ERR_ARG
    assert lib.hbfp_encode_packed_batch(1, None, None, 0, None) == hbfp.ERR_ARG
    assert call([good, job(w, src=0)]) == hbfp.ERR_ARG and call([good, job(w, src=0x100002)]) == hbfp.ERR_ARG
    assert call([good, job(w, ld=47)]) == hbfp.ERR_ARG
    odd = job(w)
    odd[0].reserved = 1
    assert call([good, odd]) == hbfp.ERR_ARG
    assert call([good, job(w, packed=0x4010)]) == hbfp.ERR_ARG
    assert call([good, job(w, size=1024)]) == hbfp.ERR_WORKSPACE
    assert call([good, job([desc(16, 240, 48, 0, 24, 24)])]) == hbfp.ERR_FORMAT          # too wide for the packed form
    assert call([good, job([x[0], w[0]])]) == hbfp.ERR_LAYOUT                             # outputs of different source shapes
    # a job whose conversion needs scratch (one exponent per matrix) makes the batch need it
    whole = [desc(8, 96, 240, 1, 96, 240)]
    scratch_job = job(whole)                                                              # holds the arrays the job points to
    arr = (hbfp.EncodeJob * 2)(good[0], scratch_job[0])
    need = ctypes.c_size_t(0)
    assert lib.hbfp_encode_packed_batch_workspace(2, arr, ctypes.byref(need)) == hbfp.OK
    assert need.value == hbfp.encode_packed_workspace(whole) and need.value > 0
    assert call([good, scratch_job]) == hbfp.ERR_WORKSPACE


def test_gemm_bfp_validation():
    """hbfp_gemm_bfp: the output plan must be that of an A->rows x B->rows matrix; the workspace always holds the FP32
    product (for the int8 kernels that stand by, or as the route to the conversion kernels) plus the product's own
    and, for two-pass output formats, the conversion's."""
    lib = hbfp._lib
    byref = ctypes.byref
    fake = ctypes.c_void_p(0x1000)

    def desc(m, rows, cols, axis, br, bc):
        d = hbfp.plan(hbfp.make_format(m, br, bc), rows, cols, axis)
        d.mant, d.exps = 0x10000, 0x20000
        return d

    a, b = desc(8, 128, 256, 1, 1, 32), desc(8, 256, 64, 0, 32, 1)
    out = desc(8, 128, 64, 1, 1, 32)
    c_bytes = 128 * 64 * 4
    for kernel in (hbfp.KERNEL_AUTO, hbfp.KERNEL_INT8, hbfp.KERNEL_SCALED):
        assert hbfp.gemm_bfp_workspace(a, b, out, kernel) == c_bytes + -(-hbfp.gemm_select_workspace(a, b, kernel) // 256) * 256
    row_exp = desc(8, 128, 64, 1, 1, 0)                                   # one exponent per row: two-pass conversion
    assert hbfp.gemm_bfp_workspace(a, b, row_exp, hbfp.KERNEL_SCALED) == \
        hbfp.gemm_bfp_workspace(a, b, out, hbfp.KERNEL_SCALED) + -(-hbfp.encode_workspace(row_exp) // 256) * 256
    assert _status(hbfp.gemm_bfp_workspace, a, b, desc(8, 128, 65, 1, 1, 32), 0) == hbfp.ERR_LAYOUT
    assert _status(hbfp.gemm_bfp_workspace, a, b, desc(8, 64, 128, 1, 1, 32), 0) == hbfp.ERR_LAYOUT
    assert _status(hbfp.gemm_bfp_workspace, a, b, out, 7) == hbfp.ERR_ARG
    need = hbfp.gemm_bfp_workspace(a, b, out, hbfp.KERNEL_SCALED)
    call = lib.hbfp_gemm_bfp
    assert call(byref(a), byref(b), byref(out), 0, hbfp.KERNEL_SCALED, fake, need - 1, None) == hbfp.ERR_WORKSPACE
    assert call(byref(a), byref(b), byref(out), 0, hbfp.KERNEL_SCALED, None, need, None) == hbfp.ERR_WORKSPACE
    assert call(byref(a), byref(b), byref(out), 2, hbfp.KERNEL_SCALED, fake, need, None) == hbfp.ERR_ARG
    assert call(byref(a), None, byref(out), 0, 0, fake, need, None) == hbfp.ERR_ARG
    no_ptr = hbfp.plan(hbfp.make_format(8, 1, 32), 128, 64, 1)
    assert call(byref(a), byref(b), byref(no_ptr), 0, 0, fake, need, None) == hbfp.ERR_ARG


def test_gemm_f32_validation():
    lib = hbfp._lib
    byref = ctypes.byref
    fake = ctypes.c_void_p(0x1000)
    fa, fb = hbfp.make_format(8, 1, 32), hbfp.make_format(8, 32, 1)
    n = hbfp.gemm_f32_workspace(0, 0, 128, 64, 256, fa, fb)
    assert n >= 128 * 256 + 64 * 256 and n % 256 == 0
    assert lib.hbfp_gemm_f32(0, 0, 128, 64, 256, fake, 256, fake, 64, fake, 64, byref(fa), byref(fb), None, 0, None) \
        == hbfp.ERR_WORKSPACE
    assert lib.hbfp_gemm_f32(0, 0, 128, 64, 256, fake, 100, fake, 64, fake, 64, byref(fa), byref(fb), fake, n, None) \
        == hbfp.ERR_ARG
    assert lib.hbfp_gemm_f32(2, 0, 128, 64, 256, fake, 256, fake, 64, fake, 64, byref(fa), byref(fb), fake, n, None) \
        == hbfp.ERR_ARG
    fb_bad = hbfp.make_format(8, 64, 1)                   # A cuts k in 32s, B in 64s
    assert _status(hbfp.gemm_f32_workspace, 0, 0, 128, 64, 256, fa, fb_bad) == hbfp.ERR_LAYOUT
    # weight-gradient shape: both operands are blocked down their rows
    fx, fdy = hbfp.make_format(8, 32, 1), hbfp.make_format(8, 32, 1)
    assert hbfp.gemm_f32_workspace(1, 0, 128, 64, 4096, fx, fdy) > 0


def test_weight_update_validation():
    lib = hbfp._lib
    byref = ctypes.byref
    fake = ctypes.c_void_p(0x1000)

    def planned(rows, cols, axis, m, br=24, bc=24):
        d = hbfp.plan(hbfp.make_format(m, br, bc), rows, cols, axis)
        d.mant, d.exps = 0x10000, 0x20000
        return d

    wide, n0, n1 = planned(100, 200, 1, 16), planned(100, 200, 0, 8), planned(100, 200, 1, 8)
    n = ctypes.c_size_t(0)
    assert lib.hbfp_weight_update_workspace(byref(wide), byref(n0), byref(n1), byref(n)) == hbfp.OK
    assert n.value >= 100 * 200 * 4 and n.value % 256 == 0
    assert lib.hbfp_weight_update_workspace(byref(wide), None, None, byref(n)) == hbfp.OK
    assert lib.hbfp_weight_update_workspace(None, None, None, byref(n)) == hbfp.ERR_ARG
    other = planned(100, 201, 1, 8)
    assert lib.hbfp_weight_update_workspace(byref(wide), byref(other), None, byref(n)) == hbfp.ERR_LAYOUT
    ws = 1 << 20
    assert lib.hbfp_weight_update(byref(wide), None, 200, 1.0, None, None, fake, ws, None) == hbfp.ERR_ARG
    assert lib.hbfp_weight_update(byref(wide), fake, 199, 1.0, None, None, fake, ws, None) == hbfp.ERR_ARG
    assert lib.hbfp_weight_update(byref(wide), fake, 200, 1.0, byref(n0), byref(n1), None, 0, None) == hbfp.ERR_WORKSPACE
    assert lib.hbfp_weight_update(byref(wide), fake, 200, 1.0, byref(n0), byref(n1), fake, 1024, None) == hbfp.ERR_WORKSPACE
    nobuf = hbfp.plan(hbfp.make_format(8, 24, 24), 100, 200, 0)
    assert lib.hbfp_weight_update(byref(wide), fake, 200, 1.0, byref(nobuf), None, fake, ws, None) != hbfp.OK


def test_encode_multi_validation():
    lib = hbfp._lib
    T = ctypes.POINTER(hbfp.TensorDesc)
    fake = ctypes.c_void_p(0x1000)

    def planned(rows, cols, axis, br, bc):
        d = hbfp.plan(hbfp.make_format(8, br, bc), rows, cols, axis)
        d.mant, d.exps = 0x10000, 0x20000
        return d

    a, b, c = planned(96, 200, 1, 1, 24), planned(96, 200, 0, 24, 1), planned(96, 204, 0, 24, 1)
    n = ctypes.c_size_t(7)
    arr = (T * 2)(ctypes.pointer(a), ctypes.pointer(b))
    assert lib.hbfp_encode_multi_workspace(2, arr, ctypes.byref(n)) == hbfp.OK and n.value == 0
    assert lib.hbfp_encode_multi_workspace(0, arr, ctypes.byref(n)) == hbfp.ERR_ARG
    assert lib.hbfp_encode_multi_workspace(4, arr, ctypes.byref(n)) == hbfp.ERR_ARG
    bad = (T * 2)(ctypes.pointer(a), ctypes.pointer(c))
    assert lib.hbfp_encode_multi_workspace(2, bad, ctypes.byref(n)) == hbfp.ERR_LAYOUT
    assert lib.hbfp_encode_multi(None, 200, 2, arr, None, 0, None) == hbfp.ERR_ARG
    assert lib.hbfp_encode_multi(fake, 100, 2, arr, None, 0, None) == hbfp.ERR_ARG       # ld < src_cols
    big = planned(96, 200, 1, 96, 200)                                                    # one block for the matrix: needs scratch
    arr2 = (T * 2)(ctypes.pointer(a), ctypes.pointer(big))
    assert lib.hbfp_encode_multi_workspace(2, arr2, ctypes.byref(n)) == hbfp.OK and n.value > 0
    assert lib.hbfp_encode_multi(fake, 200, 2, arr2, None, 0, None) == hbfp.ERR_WORKSPACE
