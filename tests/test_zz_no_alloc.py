"""hbfp_encode_static (the conversion whose scratch is a fixed device array inside the library) against hbfp_encode
with a caller-supplied workspace and against the oracle, through the C ABI: bit for bit, two calls in a row on the
same stream, the second with a smaller input (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import ref
from tests.util import unpack

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_1804_01526_amd import hbfp
    assert torch.cuda.is_available(), "these tests need the GPU"
    return hbfp


def _rand(shape, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * np.exp2(rng.integers(-6, 7, size=shape))).astype(np.float32)


# (block rows, block cols, mantissa bits, rounding, seed, contraction axis): formats whose conversion takes two passes
FORMATS = [
    (0, 0, 8, 0, 0, 1),          # one exponent for the whole matrix
    (64, 64, 8, 0, 0, 1),        # 64 x 64 tiles, k along the rows
    (256, 1, 12, 1, 99, 0),      # blocks of 256 down the rows, stochastic rounding
    (0, 1, 8, 0, 0, 0),          # one exponent per column
]


def _both(hb, x, fmt_t):
    br, bc, m, rounding, seed, axis = fmt_t
    fmt = hb.make_format(m, br, bc, rounding, seed)
    src = torch.from_numpy(x).cuda()
    want = hb.encode(src, axis, fmt)                               # workspace allocated by the binding
    assert hb.encode_workspace(want.desc) > 0, "test input: this format must need the table"
    got = hb.alloc(fmt, x.shape[0], x.shape[1], axis)
    got.mant.fill_(77)
    got.exps.fill_(77)
    before = torch.cuda.memory_allocated()
    hb.encode_static(src, axis, fmt, got)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert torch.equal(got.mant, want.mant) and torch.equal(got.exps, want.exps)
    o = ref.encode(x, br, bc, m, rounding, seed)
    mant, exps = unpack(got)
    np.testing.assert_array_equal(mant, o.mant)
    np.testing.assert_array_equal(exps, o.exps)


@pytest.mark.parametrize("fmt_t", FORMATS)
def test_static_scratch_two_calls_in_a_row(hb, fmt_t):
    print(f"[static] format={fmt_t}", flush=True)
    _both(hb, _rand((700, 900), 1), fmt_t)
    _both(hb, _rand((130, 260) if fmt_t[0] != 256 else (520, 70), 2) * 1e-3, fmt_t)    # smaller input, smaller values


def test_static_scratch_without_a_table_and_over_the_limit(hb):
    # a format that needs no table does not touch the array
    x = _rand((100, 320), 3)
    fmt = hb.make_format(8, 1, 32)
    src = torch.from_numpy(x).cuda()
    got = hb.encode_static(src, 1, fmt, hb.alloc(fmt, 100, 320, 1))
    want = hb.encode(src, 1, fmt)
    torch.cuda.synchronize()
    assert torch.equal(got.mant, want.mant) and torch.equal(got.exps, want.exps)
    # more exponent blocks than the array holds: rejected on the host, nothing launched
    assert hb.encode_static_limit() == 1 << 20
    rows = (1 << 18) + 64
    fmt = hb.make_format(8, 1, 0, k_slot=32)                       # one exponent per row, stored in blocks of 32
    d = hb.plan(fmt, rows, 64, 1)
    assert hb.encode_workspace(d) > hb.encode_static_limit()
    d.mant, d.exps = 0x10000, 0x20000
    rc = hb._lib.hbfp_encode_static(ctypes.c_void_p(0x1000), rows, 64, 64, 1, ctypes.byref(fmt), ctypes.byref(d), None)
    assert rc == hb.ERR_WORKSPACE
