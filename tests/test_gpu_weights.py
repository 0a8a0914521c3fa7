"""GPU parity of the wide-weight update step (Sec. 4.2 "Wide weight storage", Sec. 5.1) against
the CPU oracle, through the C ABI: the wide copy and both narrow copies must match bit for bit
(which pins the FP32 result they are conversions of)."""
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


def _case(hb, rows, cols, br, bc, m_wide, m_narrow, alpha, seed, rounding=0, steps=1, wide_axis=1, slot=0):
    print(f"[case] {rows}x{cols} tiles {br}x{bc} m {m_wide}->{m_narrow} alpha={alpha} rounding={rounding} "
          f"steps={steps} wide_axis={wide_axis}", flush=True)
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((rows, cols)) * 0.05).astype(np.float32)
    f_wide = hb.make_format(m_wide, br, bc, rounding, 77, k_slot=slot)
    f_nar = hb.make_format(m_narrow, br, bc, rounding, 78, k_slot=slot)
    wide = hb.encode(torch.from_numpy(W).cuda(), wide_axis, f_wide)
    na = hb.alloc(f_nar, rows, cols, 0)     # operand of the forward product: contraction down the rows
    nb = hb.alloc(f_nar, rows, cols, 1)     # operand of the data gradient: contraction along the rows
    o_wide = ref.encode(W, br, bc, m_wide, rounding, 77)
    for step in range(steps):
        G = (rng.standard_normal((rows, cols)) * np.exp2(rng.integers(-8, 2, size=(rows, cols)))).astype(np.float32)
        ws = hb.weight_update(wide, torch.from_numpy(G).cuda(), alpha, na, nb)
        torch.cuda.synchronize()
        o_wide, o_nar, w = ref.weight_update(o_wide, G, alpha, m_narrow, rounding, 77, rounding, 78)
        for t, o in ((wide, o_wide), (na, o_nar), (nb, o_nar)):
            m, e = unpack(t)
            np.testing.assert_array_equal(m, o.mant)
            np.testing.assert_array_equal(e, o.exps)


@pytest.mark.parametrize("rows,cols,br,bc,mn", [
    (96, 160, 24, 24, 8), (100, 130, 24, 24, 8), (64, 64, 1, 32, 8), (70, 200, 16, 5, 12), (33, 47, 0, 0, 8), (257, 129, 64, 64, 12),
])
def test_weight_update_matches_oracle(hb, rows, cols, br, bc, mn):
    _case(hb, rows, cols, br, bc, 16, mn, -0.01, rows + cols)


def test_weight_update_several_steps_and_stochastic_rounding(hb):
    _case(hb, 120, 168, 24, 24, 16, 8, -0.05, 3, steps=4)
    _case(hb, 120, 168, 24, 24, 16, 8, -0.05, 4, rounding=1, steps=3)
    _case(hb, 90, 100, 24, 24, 16, 8, 0.02, 5, wide_axis=0, steps=2)
    _case(hb, 90, 100, 24, 24, 12, 8, 0.02, 6)


def test_weight_update_of_a_filter_matrix_with_tiles_over_the_outer_filter_dimensions(hb):
    """The filter matrix of a 3 x 3 convolution (56 channels in blocks of 24, 50 filters) in tiles of (9 * 24) x 24,
    stored in blocks of 24 (k_slot): wide storage along k, narrow copies in both orientations."""
    _case(hb, 504, 50, 216, 24, 16, 8, -0.02, 11, wide_axis=0, slot=24, steps=2)
    _case(hb, 504, 50, 216, 24, 16, 8, -0.02, 12, rounding=1, wide_axis=0, slot=24)
    _case(hb, 300, 90, 1, 0, 16, 8, 0.01, 13, slot=24)                     # one exponent per row, stored in blocks of 24


def test_weight_update_zero_step_is_identity(hb):
    rng = np.random.default_rng(9)
    W = (rng.standard_normal((96, 96)) * 0.1).astype(np.float32)
    f = hb.make_format(16, 24, 24)
    wide = hb.encode(torch.from_numpy(W).cuda(), 1, f)
    before = (wide.mant.clone(), wide.exps.clone())
    hb.weight_update(wide, torch.ones((96, 96), device="cuda"), 0.0)
    torch.cuda.synchronize()
    assert torch.equal(wide.mant, before[0]) and torch.equal(wide.exps, before[1])


def test_weight_update_config4_weights_full_size(hb):
    """4096 x 4096 weights in 24 x 24 tiles (config 4), 16-bit storage, 8-bit views for the forward and data-gradient products."""
    import synth
    _, W, _ = synth.c4_linear()
    rng = np.random.default_rng(12)
    G = rng.standard_normal(W.shape).astype(np.float32)
    f_wide, f_nar = hb.make_format(16, 24, 24), hb.make_format(8, 24, 24)
    wide = hb.encode(torch.from_numpy(W).cuda(), 1, f_wide)
    na, nb = hb.alloc(f_nar, 4096, 4096, 0), hb.alloc(f_nar, 4096, 4096, 1)
    hb.weight_update(wide, torch.from_numpy(G).cuda(), -1e-3, na, nb)
    torch.cuda.synchronize()
    o_wide, o_nar, _ = ref.weight_update(ref.encode(W, 24, 24, 16), G, -1e-3, 8)
    for t, o in ((wide, o_wide), (na, o_nar), (nb, o_nar)):
        m, e = unpack(t)
        np.testing.assert_array_equal(m, o.mant)
        np.testing.assert_array_equal(e, o.exps)
