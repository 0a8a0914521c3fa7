"""Pins for the CPU oracle: it is checked against things other than itself.

Hand-worked examples (tests/golden), closed forms, invariants, special cases that
reduce to library routines (numpy/torch casts, np.rint, integer matmul) and brute
force on tiny inputs.  None of these needs a GPU.
"""
import os

import numpy as np
import pytest
import torch

from oracle import ref


def _read_rows(path):
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [p.strip() for p in line.split(";")]


# ---------------------------------------------------------------- hand-worked examples
def test_golden_rne_examples(golden_dir):
    n = 0
    for m, vals, e, mant in _read_rows(os.path.join(golden_dir, "encode_rne_examples.txt")):
        m, e = int(m), int(e)
        x = np.array([[float(v) for v in vals.split()]], dtype=np.float32)
        want = np.array([int(v) for v in mant.split()], dtype=np.int32)
        t = ref.encode(x, 1, 0, m)
        assert t.exps.shape == (1, 1)
        assert int(t.exps[0, 0]) - 125 - m == e, (vals, t.exps)
        np.testing.assert_array_equal(t.mant[0], want, err_msg=vals)
        np.testing.assert_array_equal(ref.decode(t)[0], want.astype(np.float64) * 2.0 ** e)
        n += 1
    assert n >= 8


def test_golden_dot_examples(golden_dir):
    for a, b, ea, eb, idot, val in _read_rows(os.path.join(golden_dir, "dot_examples.txt")):
        a = np.array([[float(v) for v in a.split()]], dtype=np.float32)          # [1, K]
        b = np.array([[float(v)] for v in b.split()], dtype=np.float32)          # [K, 1]
        ta, tb = ref.encode(a, 1, 0, 8), ref.encode(b, 0, 1, 8)
        assert int(ta.exps[0, 0]) - 133 == int(ea) and int(tb.exps[0, 0]) - 133 == int(eb)
        P = ref.block_dots(ta.mant, tb.mant, 0)
        assert P.shape == (1, 1, 1) and int(P[0, 0, 0]) == int(idot)
        C = ref.gemm(ref.decode(ta), ref.decode(tb))
        assert C[0, 0] == float(val)
        C2 = ref.scale_accumulate(P, ta.exps, tb.exps, 8, 8)
        assert C2[0, 0] == float(val)


# ---------------------------------------------------------------- an independent formulation
def _encode_rne_float64(x, br, bc, m):
    """Same quantiser written with frexp / rint in FP64 instead of integer bit
    operations (x / unit is exact in FP64, np.rint rounds half to even)."""
    rows, cols = x.shape
    br = rows if br <= 0 or br > rows else br
    bc = cols if bc <= 0 or bc > cols else bc
    mant = np.zeros((rows, cols), dtype=np.int64)
    unit_exp = np.zeros((-(-rows // br), -(-cols // bc)), dtype=np.int64)
    for i, r0 in enumerate(range(0, rows, br)):
        for j, c0 in enumerate(range(0, cols, bc)):
            blk = x[r0:r0 + br, c0:c0 + bc].astype(np.float64)
            amax = np.abs(blk).max()
            _, ex = np.frexp(amax)                       # amax = f * 2^ex, f in [0.5, 1)
            emax = max(int(ex) - 1, -126)                # exponent of the leading bit (subnormals pinned)
            e = emax - (m - 2)
            q = np.rint(blk / 2.0 ** e)
            if np.abs(q).max() >= 2 ** (m - 1):
                e += 1
                q = np.rint(blk / 2.0 ** e)
            mant[r0:r0 + br, c0:c0 + bc] = q.astype(np.int64)
            unit_exp[i, j] = e
    return mant, unit_exp


@pytest.mark.parametrize("m", [2, 4, 8, 9, 12, 16])
@pytest.mark.parametrize("shape,br,bc", [((7, 96), 1, 32), ((50, 70), 24, 24), ((64, 5), 32, 1),
                                         ((3, 100), 1, 0), ((33, 33), 0, 0), ((1, 1000), 1, 64)])
def test_rne_matches_float64_formulation(m, shape, br, bc):
    rng = np.random.default_rng(m * 1000 + shape[0])
    x = (rng.standard_normal(shape) * np.exp2(rng.integers(-30, 30, size=shape))).astype(np.float32)
    x[rng.random(shape) < 0.05] = 0.0
    t = ref.encode(x, br, bc, m)
    mant, ue = _encode_rne_float64(x, br, bc, m)
    np.testing.assert_array_equal(t.mant, mant)
    np.testing.assert_array_equal(t.exps.astype(np.int64) - 125 - m, ue)


def test_rne_near_power_of_two_maxima_and_ties():
    # maxima just below a power of two force the exponent raise; exact ties test half-to-even
    for m in (4, 8, 12, 16):
        top = np.float32(2.0)
        vals = [np.nextafter(top, np.float32(0)), top * (1 - 2.0 ** -(m - 1)), top * (1 - 2.0 ** -m),
                top * (1 - 2.0 ** -(m + 1)), 1.0, 2.0 ** -(m - 2) * 0.5, 2.0 ** -(m - 2) * 1.5, 2.0 ** -(m - 2) * 2.5]
        for v in vals[:4]:
            x = np.array([[v] + vals[4:]], dtype=np.float32)
            t = ref.encode(x, 1, 0, m)
            mant, ue = _encode_rne_float64(x, 1, 0, m)
            np.testing.assert_array_equal(t.mant, mant)
            assert int(t.exps[0, 0]) - 125 - m == int(ue[0, 0])
            assert np.abs(t.mant).max() <= 2 ** (m - 1) - 1


# ---------------------------------------------------------------- invariants
def _lsb(t):
    return np.exp2(t.unit_exponents().astype(np.float64))


@pytest.mark.parametrize("m", [4, 8, 12, 16])
@pytest.mark.parametrize("rounding", [ref.RNE, ref.STOCHASTIC])
def test_power_of_two_blocks_are_exact(m, rounding):
    rng = np.random.default_rng(7 + m)
    rows, cols, B = 16, 128, 32
    kmax = rng.integers(-100, 100, size=(rows, cols // B, 1))
    k = kmax - rng.integers(0, m - 1, size=(rows, cols // B, B))      # within the m-1 magnitude bits
    k[:, :, 0] = kmax[:, :, 0]
    sign = rng.choice([-1.0, 1.0], size=k.shape)
    x = (sign * np.exp2(k.astype(np.float64))).reshape(rows, cols).astype(np.float32)
    t = ref.encode(x, 1, B, m, rounding, seed=99)
    np.testing.assert_array_equal(ref.decode(t), x)
    # the block maximum sits on the top magnitude bit
    assert (np.abs(t.mant).reshape(rows, cols // B, B).max(axis=2) == 2 ** (m - 2)).all()


@pytest.mark.parametrize("m", [4, 8, 12, 16])
def test_rne_error_at_most_half_unit_and_normalised(m):
    x = (np.random.default_rng(m).standard_normal((64, 256)) * 3).astype(np.float32)
    t = ref.encode(x, 1, 32, m)
    err = np.abs(ref.decode(t).astype(np.float64) - x.astype(np.float64))
    assert (err <= 0.5 * _lsb(t)).all()
    top = np.abs(t.mant).reshape(64, 8, 32).max(axis=2)
    assert (top >= 2 ** (m - 2)).all() and (top <= 2 ** (m - 1) - 1).all()


@pytest.mark.parametrize("m", [4, 8, 12])
def test_sr_error_below_one_unit_unbiased_and_floor_or_ceil(m):
    rng = np.random.default_rng(100 + m)
    x = (rng.standard_normal((256, 1024)) * np.exp2(rng.integers(-3, 3, size=(256, 1024)))).astype(np.float32)
    t = ref.encode(x, 1, 32, m, ref.STOCHASTIC, seed=1234)
    lsb = _lsb(t)
    exact = x.astype(np.float64) / lsb
    q = t.mant.astype(np.float64)
    mag, qm = np.abs(exact), np.abs(q)
    assert ((qm == np.floor(mag)) | (qm == np.ceil(mag))).all()          # only the two neighbours
    assert (np.abs(q - exact) < 1.0).all()
    assert (np.sign(q) * np.sign(exact) >= 0).all()
    d = (q - exact).ravel()                                              # error in units
    n = d.size
    assert abs(d.mean()) < 4.0 * d.std() / np.sqrt(n)                    # unbiased
    assert np.abs(t.mant).max() <= 2 ** (m - 1) - 1


def test_sr_round_up_frequency_equals_fraction():
    # a block [64.0, f, f, ...] with m=8 has unit 1, so element f in (0,1) must round up with probability f
    for f in (0.125, 0.3, 0.5, 0.9):
        n = 1 << 16
        x = np.full((n // 32, 32), f, dtype=np.float32)
        x[:, 0] = 64.0
        t = ref.encode(x, 1, 32, 8, ref.STOCHASTIC, seed=42)
        assert (t.exps == 133).all()
        ups = t.mant[:, 1:].ravel()
        assert set(np.unique(ups)) <= {0, 1}
        p = ups.mean()
        fx = float(np.float32(f))
        assert abs(p - fx) < 4.0 * np.sqrt(fx * (1 - fx) / ups.size)


def test_sr_depends_on_seed_and_logical_index_only():
    x = np.random.default_rng(5).standard_normal((32, 64)).astype(np.float32)
    a = ref.encode(x, 1, 32, 8, ref.STOCHASTIC, seed=1)
    b = ref.encode(x, 1, 32, 8, ref.STOCHASTIC, seed=1)
    c = ref.encode(x, 1, 32, 8, ref.STOCHASTIC, seed=2)
    np.testing.assert_array_equal(a.mant, b.mant)
    assert (a.mant != c.mant).mean() > 0.2
    np.testing.assert_array_equal(a.exps, c.exps)
    # block shape does not change the random draw of an element: with a common exponent the mantissas agree
    y = np.ones((4, 64), dtype=np.float32) * 0.3
    y[:, ::8] = 1.0
    d = ref.encode(y, 1, 8, 8, ref.STOCHASTIC, seed=3)
    e = ref.encode(y, 4, 64, 8, ref.STOCHASTIC, seed=3)
    np.testing.assert_array_equal(d.mant, e.mant)


def test_hash_statistics():
    idx = np.arange(1 << 16, dtype=np.uint64)
    h = np.array([ref.hash32(77, int(i)) for i in idx], dtype=np.uint64)
    top = (h >> np.uint64(24)).astype(np.int64)
    counts = np.bincount(top, minlength=256)
    expected = idx.size / 256.0
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert chi2 < 255 + 5 * np.sqrt(2 * 255)                              # uniform top byte
    low = (h & np.uint64(0xFF)).astype(np.int64)
    chi2l = ((np.bincount(low, minlength=256) - expected) ** 2 / expected).sum()
    assert chi2l < 255 + 5 * np.sqrt(2 * 255)
    h2 = np.array([ref.hash32(78, int(i)) for i in idx[:4096]], dtype=np.uint64)
    diff = np.array([bin(int(a ^ b)).count("1") for a, b in zip(h[:4096], h2)])
    assert abs(diff.mean() - 16.0) < 0.5                                  # other seed: half the bits flip
    hs = np.array([ref.hash32(77, int(i) + (1 << 32)) for i in idx[:4096]], dtype=np.uint64)
    assert (hs != h[:4096]).mean() > 0.99                                  # the high index word matters
    # serial correlation of consecutive outputs
    u = h.astype(np.float64) / 2 ** 32
    r = np.corrcoef(u[:-1], u[1:])[0, 1]
    assert abs(r) < 4.0 / np.sqrt(u.size)


@pytest.mark.parametrize("m", [8, 12])
def test_equivariances(m):
    rng = np.random.default_rng(31 + m)
    x = rng.standard_normal((16, 96)).astype(np.float32)
    t = ref.encode(x, 1, 24, m)
    for k in (-40, -3, 5, 60):
        tk = ref.encode((x.astype(np.float64) * 2.0 ** k).astype(np.float32), 1, 24, m)
        np.testing.assert_array_equal(tk.mant, t.mant)
        np.testing.assert_array_equal(tk.exps.astype(int), t.exps.astype(int) + k)
    tn = ref.encode(-x, 1, 24, m)
    np.testing.assert_array_equal(tn.mant, -t.mant)
    np.testing.assert_array_equal(tn.exps, t.exps)
    ts = ref.encode(x, 1, 24, m, ref.STOCHASTIC, seed=8)
    tsn = ref.encode(-x, 1, 24, m, ref.STOCHASTIC, seed=8)
    np.testing.assert_array_equal(tsn.mant, -ts.mant)
    # idempotence: a decoded BFP tensor encodes to itself
    t2 = ref.encode(ref.decode(t), 1, 24, m)
    np.testing.assert_array_equal(t2.mant, t.mant)
    np.testing.assert_array_equal(t2.exps, t.exps)


def test_block_of_one_is_a_float_cast():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal(20000) * np.exp2(rng.integers(-13, 15, size=20000))).astype(np.float32)
    x = x[(np.abs(x) >= 2.0 ** -14) & (np.abs(x) < 65000.0)].reshape(1, -1)
    # 12-bit mantissa incl. sign = 11 significant bits = IEEE half precision
    got = ref.decode(ref.encode(x, 1, 1, 12))
    np.testing.assert_array_equal(got, x.astype(np.float16).astype(np.float32))
    # 9 bits incl. sign = 8 significant bits = bfloat16
    y = (rng.standard_normal(20000) * np.exp2(rng.integers(-100, 100, size=20000))).astype(np.float32).reshape(1, -1)
    got = ref.decode(ref.encode(y, 1, 1, 9))
    want = torch.from_numpy(y).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("m,kb", [(6, 24), (8, 24), (8, 32), (9, 64)])
def test_decoded_values_of_narrow_mantissas_are_bfloat16_numbers(m, kb):
    """What the bf16 product route rests on: a mantissa of at most 9 bits times its block's power of two (Eq. (1)) is a
    bfloat16 number for every exponent byte up to 253, subnormal blocks included; the library cast is the check."""
    rng = np.random.default_rng(40 + m)
    x = (rng.standard_normal((64, 960)) * np.exp2(rng.integers(-126, 126, size=(64, 1)))).astype(np.float32)
    x[:4] = (rng.standard_normal((4, 960)) * 2.0 ** -132).astype(np.float32)   # FP32 subnormals: exponent byte 1
    x[4:8, ::7] = 0.0
    t = ref.encode(x, 1, kb, m)
    assert int(t.exps.max()) <= 253 and int(t.exps.min()) == 1
    d = ref.decode(t)
    assert np.isfinite(d).all()
    np.testing.assert_array_equal(torch.from_numpy(d).to(torch.bfloat16).to(torch.float32).numpy(), d)


@pytest.mark.parametrize("m", [10, 11, 12])
def test_wide_mantissas_relative_to_the_row_maximum_are_half_precision_numbers(m):
    """What the FP16-planes route rests on: mant * 2^(E - Eref + 4), Eref the largest exponent byte of the operand row, is an
    IEEE half-precision number (subnormals included) whenever the block lies at most 28 binades below the row's largest,
    its magnitude stays below 2^15, and decode = that number times 2^(Eref - 4 - 125 - m) exactly."""
    rng = np.random.default_rng(50 + m)
    kb, nb = 64, 16
    x = rng.standard_normal((48, kb * nb)).astype(np.float32)
    for b in range(nb):                                                       # blocks of a row 0..28 binades apart
        x[:, b * kb:(b + 1) * kb] *= np.float32(2.0 ** -(28 * b // (nb - 1)))
    x *= np.exp2(rng.integers(-60, 60, size=(48, 1))).astype(np.float32)
    t = ref.encode(x, 1, kb, m)
    e = t.exps.astype(np.int64)                                               # [rows, blocks]
    eref = e.max(axis=1, keepdims=True)
    assert int((eref - e).max()) >= 27
    shift = np.repeat(e - eref + 4, kb, axis=1)
    rel = np.ldexp(t.mant.astype(np.float64), shift)
    ok = np.repeat(eref - e <= 28, kb, axis=1)
    assert np.abs(rel).max() < 2.0 ** 15
    half = rel.astype(np.float16).astype(np.float64)
    np.testing.assert_array_equal(half[ok], rel[ok])
    np.testing.assert_array_equal(np.ldexp(rel, np.broadcast_to(eref - 4 - 125 - m, rel.shape)).astype(np.float32), ref.decode(t))
    # one binade further and the last bit of an odd mantissa is lost
    assert np.float64(np.float16(np.ldexp(1.0, -25))) == 0.0


def test_zero_subnormal_and_signed_zero():
    x = np.zeros((2, 32), dtype=np.float32)
    x[1, 3] = -0.0
    t = ref.encode(x, 1, 32, 8)
    assert (t.mant == 0).all() and (t.exps == 1).all()
    tiny = np.float32(2.0 ** -149)
    for m in (8, 16):
        unit = 2.0 ** (1 - 125 - m)                                       # smallest unit a block can have
        k = np.arange(-20, 21, dtype=np.float64)
        y = (k * unit).astype(np.float32).reshape(1, -1)                   # subnormal-range multiples of the unit
        assert np.abs(y).max() < 2.0 ** -126
        t = ref.encode(y, 1, 0, m)
        assert int(t.exps[0, 0]) == 1
        np.testing.assert_array_equal(t.mant[0], k.astype(np.int32))
        np.testing.assert_array_equal(ref.decode(t), y)
    z = np.array([[tiny, -tiny, 0.0, 3 * tiny]], dtype=np.float32)
    t = ref.encode(z, 1, 0, 16)
    np.testing.assert_array_equal(t.mant[0], [0, 0, 0, 0])               # far below one unit (2^-140)


def test_two_d_tiles_and_ragged_edges_share_one_exponent():
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((50, 70)) * np.exp2(rng.integers(-8, 8, size=(50, 70)))).astype(np.float32)
    t = ref.encode(x, 24, 24, 8)
    assert t.exps.shape == (3, 3)
    for i in range(3):
        for j in range(3):
            blk = x[24 * i:24 * i + 24, 24 * j:24 * j + 24]
            amax = np.abs(blk).max()
            _, ex = np.frexp(amax)
            eb = int(ex) - 1 + 127
            assert int(t.exps[i, j]) in (eb, eb + 1)
            sub = ref.encode(np.ascontiguousarray(blk), 0, 0, 8)
            np.testing.assert_array_equal(sub.mant, t.mant[24 * i:24 * i + 24, 24 * j:24 * j + 24])
            assert int(sub.exps[0, 0]) == int(t.exps[i, j])


# ---------------------------------------------------------------- integer dot products
def test_block_dots_brute_force():
    rng = np.random.default_rng(3)
    M, N, K, kb = 4, 5, 70, 32
    mA = rng.integers(-127, 128, size=(M, K)).astype(np.int32)
    mB = rng.integers(-127, 128, size=(K, N)).astype(np.int32)
    P = ref.block_dots(mA, mB, kb)
    assert P.shape == (M, N, 3)
    for i in range(M):
        for j in range(N):
            for b in range(3):
                s = 0
                for k in range(b * kb, min(K, (b + 1) * kb)):
                    s += int(mA[i, k]) * int(mB[k, j])
                assert int(P[i, j, b]) == s
    # extreme block: every mantissa +-127, 32 per block -> 32 * 127^2 = 516128
    a = np.full((2, 64), 127, dtype=np.int32)
    b = np.full((64, 2), -127, dtype=np.int32)
    P = ref.block_dots(a, b, 32)
    assert (P == -516128).all()
    # library routine: integer matmul over the whole K
    P = ref.block_dots(mA, mB, 0)
    np.testing.assert_array_equal(P[:, :, 0], mA.astype(np.int64) @ mB.astype(np.int64))


def test_block_dots_reports_accumulator_overflow():
    a = np.full((1, 40000), 2047, dtype=np.int32)
    b = np.full((40000, 1), 2047, dtype=np.int32)
    with pytest.raises(OverflowError):
        ref.block_dots(a, b, 0)
    assert ref.block_dots(a, b, 512).max() == 512 * 2047 * 2047           # 12-bit mantissas, blocks of 512 fit


def test_limb_identity_for_12_bit_mantissas_exhaustive():
    # every 12-bit pair: v = 64 h + l with h in [-32, 31], l in [0, 63]; the four limb
    # products recombine to the exact product (the identity a limb-split GEMM relies on)
    v = np.arange(-2047, 2048, dtype=np.int64)
    h, l = v >> 6, v & 63
    assert h.min() >= -32 and h.max() <= 31 and l.min() >= 0 and l.max() <= 63
    prod = np.multiply.outer(v, v)
    rec = (np.multiply.outer(h, h) << 12) + ((np.multiply.outer(h, l) + np.multiply.outer(l, h)) << 6) \
        + np.multiply.outer(l, l)
    np.testing.assert_array_equal(prod, rec)


def test_four_bit_limb_identity_and_scale_bytes_exhaustive():
    """The identity a product on 4-bit sign-magnitude limbs relies on (host-side check of the arithmetic, no GPU):
    |v| = sum_i n_i 16^i with n_i in 0..15; limb i of a block with stored exponent byte E and m-bit mantissas is the
    narrow float +-n_i / 8 times 2^(byte_i - 127) with byte_i = E + 5 + 4 i - m; summed over the limbs that is
    Eq. (1), v * 2^(E - 125 - m), and the products of all limb pairs sum to the product of two decoded values."""
    for m, limbs in ((4, 1), (5, 1), (8, 2), (9, 2), (12, 3)):
        q = (1 << (m - 1)) - 1
        v = np.arange(-q, q + 1, dtype=np.int64)
        a = np.abs(v)
        n = [(a >> (4 * i)) & 15 for i in range(limbs)]
        assert sum(ni << (4 * i) for i, ni in enumerate(n)).tolist() == a.tolist()      # nothing left above the top limb
        for E in (m - 5, 97, 140, 250 - 4 * (limbs - 1)):                               # both ends of the byte range
            byte = [E + 5 + 4 * i - m for i in range(limbs)]
            assert min(byte) >= 0 and max(byte) <= 254
            val = sum(np.sign(v) * (ni / 8.0) * np.exp2(float(b - 127)) for ni, b in zip(n, byte))
            np.testing.assert_array_equal(val, v * np.exp2(float(E - 125 - m)))
    # all limb pairs of two 8-bit mantissas with their own exponents: exact in FP64, equal to the decoded product
    v = np.arange(-127, 128, dtype=np.int64)
    a = np.abs(v)
    lo, hi = a & 15, a >> 4
    Ea, Eb = 131, 118
    limb = lambda e: [np.sign(v) * (lo / 8.0) * np.exp2(e - 3.0 - 127.0), np.sign(v) * (hi / 8.0) * np.exp2(e + 1.0 - 127.0)]
    total = sum(np.multiply.outer(x, y) for x in limb(Ea) for y in limb(Eb))
    want = np.multiply.outer(v * np.exp2(Ea - 133.0), v * np.exp2(Eb - 133.0))
    np.testing.assert_array_equal(total, want)


# ---------------------------------------------------------------- GEMM
@pytest.mark.parametrize("h,w,c,r,s,pad_h,pad_w,sh,sw,cb", [(5, 6, 3, 3, 3, 1, 1, 1, 1, 0), (7, 5, 2, 3, 2, 0, 1, 2, 1, 0), (4, 4, 4, 1, 1, 0, 0, 1, 1, 0),
                                                            (6, 7, 2, 5, 3, 2, 1, 2, 3, 0), (5, 6, 7, 3, 3, 1, 1, 1, 1, 3), (6, 5, 8, 2, 3, 1, 0, 1, 2, 4)])
def test_im2col_times_filter_matrix_is_the_convolution_sum(h, w, c, r, s, pad_h, pad_w, sh, sw, cb):
    """The lowered operand against the textbook definition: y[img, oy, ox, f] = sum over (fr, fs, ch) of
    x[img, oy*sh - pad_h + fr, ox*sw - pad_w + fs, ch] * wgt[fr, fs, ch, f], by brute-force loops."""
    rng = np.random.default_rng(h * 100 + w)
    n, f = 2, 3
    x = rng.integers(-4, 5, size=(n, h, w, c)).astype(np.float64)
    wgt = rng.integers(-3, 4, size=(r, s, c, f)).astype(np.float64)
    ho, wo = (h + 2 * pad_h - r) // sh + 1, (w + 2 * pad_w - s) // sw + 1
    want = np.zeros((n, ho, wo, f))
    for img in range(n):
        for oy in range(ho):
            for ox in range(wo):
                for fr in range(r):
                    for fs in range(s):
                        iy, ix = oy * sh - pad_h + fr, ox * sw - pad_w + fs
                        if 0 <= iy < h and 0 <= ix < w:
                            for ch in range(c):
                                want[img, oy, ox, :] += x[img, iy, ix, ch] * wgt[fr, fs, ch, :]
    got = ref.im2col(x, r, s, pad_h, pad_w, sh, sw, cb) @ ref.filter_matrix(wgt, cb)     # cb: channel-block order of the columns
    np.testing.assert_array_equal(got.reshape(n, ho, wo, f), want)


@pytest.mark.parametrize("h,w,c,f,r,s,pad_h,pad_w,cb", [(5, 6, 3, 4, 3, 3, 1, 1, 0), (6, 5, 2, 3, 3, 2, 0, 1, 0), (4, 7, 4, 8, 5, 3, 2, 1, 4),
                                                        (5, 5, 3, 2, 1, 1, 0, 0, 0), (6, 6, 2, 6, 3, 3, 2, 2, 3)])
def test_data_gradient_of_a_convolution_as_a_forward_product(h, w, c, f, r, s, pad_h, pad_w, cb):
    """Stride 1: the gradient with respect to the input, written out from its definition as the adjoint of the
    convolution sum (every product x * wgt that feeds y[oy, ox, f] sends dy[oy, ox, f] * wgt back to that x), equals
    the lowered dy with padding r - 1 - pad times the mirrored, channel-exchanged filter; and <y, dy> = <x, dx>."""
    rng = np.random.default_rng(h * 10 + w + r)
    n = 2
    ho, wo = h + 2 * pad_h - r + 1, w + 2 * pad_w - s + 1
    x = rng.integers(-4, 5, size=(n, h, w, c)).astype(np.float64)
    wgt = rng.integers(-3, 4, size=(r, s, c, f)).astype(np.float64)
    dy = rng.integers(-5, 6, size=(n, ho, wo, f)).astype(np.float64)
    want = np.zeros((n, h, w, c))
    for img in range(n):
        for oy in range(ho):
            for ox in range(wo):
                for fr in range(r):
                    for fs in range(s):
                        iy, ix = oy - pad_h + fr, ox - pad_w + fs
                        if 0 <= iy < h and 0 <= ix < w:
                            want[img, iy, ix, :] += wgt[fr, fs, :, :] @ dy[img, oy, ox, :]
    got = ref.im2col(dy, r, s, r - 1 - pad_h, s - 1 - pad_w, 1, 1, cb) @ ref.filter_matrix_dgrad(wgt, cb)
    assert got.shape == (n * h * w, c)
    np.testing.assert_array_equal(got.reshape(n, h, w, c), want)
    y = (ref.im2col(x, r, s, pad_h, pad_w) @ ref.filter_matrix(wgt)).reshape(n, ho, wo, f)
    assert np.sum(y * dy) == np.sum(x * want)


@pytest.mark.parametrize("h,w,c,f,r,s,pad_h,pad_w,sh,sw", [(7, 8, 3, 4, 3, 3, 1, 1, 2, 2), (8, 8, 2, 3, 3, 3, 1, 1, 2, 2), (9, 7, 2, 3, 3, 2, 0, 1, 3, 2),
                                                           (6, 9, 3, 2, 1, 1, 0, 0, 2, 3), (10, 10, 2, 2, 5, 5, 2, 2, 4, 1), (5, 6, 2, 3, 2, 2, 3, 2, 2, 2),
                                                           (6, 6, 3, 2, 3, 3, 1, 1, 1, 1)])
def test_data_gradient_of_a_strided_convolution_as_a_forward_product(h, w, c, f, r, s, pad_h, pad_w, sh, sw):
    """Any stride: the adjoint of the convolution sum, written out from its definition, equals the lowered, spread-out dy
    times the mirrored, channel-exchanged filter, at every position of x (also those that only some windows reach, and
    with padding wider than the window); and <y, dy> = <x, dx>."""
    rng = np.random.default_rng(h * 100 + w * 10 + r + sh)
    n = 2
    ho, wo = (h + 2 * pad_h - r) // sh + 1, (w + 2 * pad_w - s) // sw + 1
    x = rng.integers(-4, 5, size=(n, h, w, c)).astype(np.float64)
    wgt = rng.integers(-3, 4, size=(r, s, c, f)).astype(np.float64)
    dy = rng.integers(-5, 6, size=(n, ho, wo, f)).astype(np.float64)
    want = np.zeros((n, h, w, c))
    for img in range(n):
        for oy in range(ho):
            for ox in range(wo):
                for fr in range(r):
                    for fs in range(s):
                        iy, ix = oy * sh - pad_h + fr, ox * sw - pad_w + fs
                        if 0 <= iy < h and 0 <= ix < w:
                            want[img, iy, ix, :] += wgt[fr, fs, :, :] @ dy[img, oy, ox, :]
    got = ref.im2col_dgrad(dy, h, w, r, s, pad_h, pad_w, sh, sw) @ ref.filter_matrix_dgrad(wgt)
    assert got.shape == (n * h * w, c)
    np.testing.assert_array_equal(got.reshape(n, h, w, c), want)
    y = (ref.im2col(x, r, s, pad_h, pad_w, sh, sw) @ ref.filter_matrix(wgt)).reshape(n, ho, wo, f)
    assert np.sum(y * dy) == np.sum(x * want)
    if sh == 1 and sw == 1 and pad_h < r and pad_w < s:
        np.testing.assert_array_equal(ref.im2col_dgrad(dy, h, w, r, s, pad_h, pad_w), ref.im2col(dy, r, s, r - 1 - pad_h, s - 1 - pad_w))


def test_sampled_rows_of_the_lowered_operands_equal_the_whole_matrices():
    """im2col_rows / im2col_dgrad_rows (used where the lowered matrix is too large) against im2col / im2col_dgrad, which the
    tests above pin to the convolution sum and its adjoint."""
    rng = np.random.default_rng(77)
    for (h, w, c, f, r, s, ph, pw, sh, sw) in [(7, 8, 3, 4, 3, 3, 1, 1, 2, 2), (9, 7, 2, 3, 3, 2, 0, 1, 3, 2), (6, 6, 3, 2, 3, 3, 1, 1, 1, 1),
                                               (5, 6, 2, 3, 2, 2, 3, 2, 2, 2)]:
        n = 2
        ho, wo = (h + 2 * ph - r) // sh + 1, (w + 2 * pw - s) // sw + 1
        x = rng.standard_normal((n, h, w, c))
        dy = rng.standard_normal((n, ho, wo, f))
        rows = np.arange(n * ho * wo)
        np.testing.assert_array_equal(ref.im2col_rows(x, rows, r, s, ph, pw, sh, sw), ref.im2col(x, r, s, ph, pw, sh, sw))
        rows = rng.permutation(n * h * w)
        np.testing.assert_array_equal(ref.im2col_dgrad_rows(dy, rows, h, w, r, s, ph, pw, sh, sw), ref.im2col_dgrad(dy, h, w, r, s, ph, pw, sh, sw)[rows])


def test_filter_matrix_tiles_in_channel_block_order_are_the_outer_dimension_tiles():
    """Sec. 5.1 tiles the two outer dimensions of a convolution's filter.  With the window entries in channel-block order
    a tile of (r*s*cb) x fb of the filter matrix holds exactly one (channel block, filter block) pair with the whole
    window: its exponent must be that of the largest magnitude over w4[:, :, channel block, filter block], and every
    element's decoded value must lie within half a unit of that exponent."""
    rng = np.random.default_rng(15)
    r, s, c, f, cb, fb, m = 3, 3, 56, 50, 24, 24, 8
    w4 = (rng.standard_normal((r, s, c, f)) * np.exp2(rng.integers(-5, 6, size=(1, 1, c, 1)))).astype(np.float32)
    wmat = ref.filter_matrix(w4, cb)
    enc = ref.encode(wmat, r * s * cb, fb, m)
    dec = ref.decode(enc)
    row0 = 0
    for ci, c0 in enumerate(range(0, c, cb)):
        cw = min(cb, c - c0)
        for fi, f0 in enumerate(range(0, f, fb)):
            block = w4[:, :, c0:c0 + cw, f0:f0 + fb]
            top = np.abs(block).max()
            e_ieee = int(np.frexp(top)[1]) + 126                                  # biased exponent of the maximum
            assert enc.exps[ci, fi] in (e_ieee, e_ieee + 1)                         # + 1 only when the maximum rounds up
            unit = 2.0 ** (int(enc.exps[ci, fi]) - 125 - m)
            got = dec[row0:row0 + r * s * cw, f0:f0 + fb].reshape(r, s, cw, -1)     # rows of the tile: (fr, fs, ci)
            assert np.abs(got.astype(np.float64) - block.astype(np.float64)).max() <= unit / 2
        row0 += r * s * cw


def test_gemm_is_the_fp64_product():
    rng = np.random.default_rng(17)
    A = rng.standard_normal((37, 129)).astype(np.float32)
    B = rng.standard_normal((129, 41)).astype(np.float32)
    C = ref.gemm(A, B)
    want = A.astype(np.float64) @ B.astype(np.float64)
    np.testing.assert_allclose(C, want, rtol=0, atol=1e-12 * np.abs(want).max() * 129)
    sel = np.array([5, 0, 36, 5])
    np.testing.assert_array_equal(ref.gemm(A, B, rows=sel), C[sel])
    # a transposed operand must not pass
    Bt = rng.standard_normal((129, 129)).astype(np.float32)
    A2 = rng.standard_normal((129, 129)).astype(np.float32)
    assert np.abs(ref.gemm(A2, Bt) - A2.astype(np.float64) @ Bt.T.astype(np.float64)).max() > 1.0


def test_gemm_power_of_two_inputs_is_exact_fp32_gemm():
    rng = np.random.default_rng(23)
    M, K, N = 16, 64, 24
    A = (rng.choice([-1.0, 1.0], size=(M, K)) * np.exp2(rng.integers(-3, 3, size=(M, K)))).astype(np.float32)
    B = (rng.choice([-1.0, 1.0], size=(K, N)) * np.exp2(rng.integers(-3, 3, size=(K, N)))).astype(np.float32)
    C, ta, tb = ref.bfp_gemm(A, B, dict(br=1, bc=32, m=8), dict(br=32, bc=1, m=8))
    np.testing.assert_array_equal(ref.decode(ta), A)
    np.testing.assert_array_equal(C, A.astype(np.float64) @ B.astype(np.float64))   # small integers * 2^-6: exact


def test_gemm_whole_k_blocks_is_scaled_integer_gemm():
    # Sec. 4: one exponent per row of A and per column of B suffices
    rng = np.random.default_rng(29)
    M, K, N = 9, 200, 7
    A = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-10, 10, size=(M, 1)))).astype(np.float32)
    B = (rng.standard_normal((K, N)) * np.exp2(rng.integers(-10, 10, size=(1, N)))).astype(np.float32)
    C, ta, tb = ref.bfp_gemm(A, B, dict(br=1, bc=0, m=8), dict(br=0, bc=1, m=8))
    assert ta.exps.shape == (M, 1) and tb.exps.shape == (1, N)
    I = ta.mant.astype(np.int64) @ tb.mant.astype(np.int64)
    e = (ta.exps.astype(np.int64) - 133) + (tb.exps.astype(np.int64) - 133)
    np.testing.assert_array_equal(C, I.astype(np.float64) * np.exp2(e.astype(np.float64)))


@pytest.mark.parametrize("m,kb", [(8, 32), (8, 24), (12, 64)])
def test_block_partials_scaled_and_summed_equal_the_definition(m, kb):
    rng = np.random.default_rng(m + kb)
    M, K, N = 12, 200, 10
    A = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-6, 6, size=(M, K)))).astype(np.float32)
    B = (rng.standard_normal((K, N)) * np.exp2(rng.integers(-6, 6, size=(K, N)))).astype(np.float32)
    C, ta, tb = ref.bfp_gemm(A, B, dict(br=1, bc=kb, m=m), dict(br=kb, bc=1, m=m))
    P = ref.block_dots(ta.mant, tb.mant, kb)
    C2 = ref.scale_accumulate(P, ta.exps, tb.exps, m, m)
    np.testing.assert_allclose(C2, C, rtol=1e-13, atol=1e-13 * np.abs(C).max())
    # and the quantised product is close to the FP32 one, as the format promises (8+ bit mantissas)
    exact = A.astype(np.float64) @ B.astype(np.float64)
    rel = np.linalg.norm(C - exact) / np.linalg.norm(exact)
    assert rel < 2.0 ** -(m - 3)


# ---------------------------------------------------------------- wide weight storage (Sec. 4.2, Sec. 5.1)
def _bfp_block(mant, unit_exp, m):
    mant = np.array([mant], dtype=np.int32)
    return ref.BFP(mant, np.array([[unit_exp + 125 + m]], dtype=np.uint8), m, 1, mant.shape[1])


def test_golden_weight_update_examples(golden_dir):
    n = 0
    for row in _read_rows(os.path.join(golden_dir, "weight_update_examples.txt")):
        mw, mn, wm, ew, delta, alpha, ew2, wm2, en2, nm2 = row
        mw, mn, ew, ew2, en2 = int(mw), int(mn), int(ew), int(ew2), int(en2)
        wide = _bfp_block([int(v) for v in wm.split()], ew, mw)
        d = np.array([[float(v) for v in delta.split()]], dtype=np.float32)
        w2, n2, _ = ref.weight_update(wide, d, float(alpha), mn)
        assert int(w2.exps[0, 0]) - 125 - mw == ew2 and int(n2.exps[0, 0]) - 125 - mn == en2, row
        np.testing.assert_array_equal(w2.mant[0], [int(v) for v in wm2.split()], err_msg=str(row))
        np.testing.assert_array_equal(n2.mant[0], [int(v) for v in nm2.split()], err_msg=str(row))
        n += 1
    assert n >= 5


def _round_to_f32(x):
    """Exact rational -> nearest FP32 (ties to even), by integer arithmetic."""
    from fractions import Fraction
    if x == 0:
        return np.float32(0.0)
    sign, ax = (-1 if x < 0 else 1), abs(x)
    e = ax.numerator.bit_length() - ax.denominator.bit_length()
    if Fraction(2) ** e > ax:
        e -= 1
    e = max(e, -126)
    q = ax / Fraction(2) ** (e - 23)
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (fl & 1)):
        fl += 1
    return np.float32(sign * float(fl) * 2.0 ** (e - 23))


def test_weight_update_step_is_one_fp32_rounding_of_the_exact_sum():
    """w' must equal alpha*delta + w computed exactly (rationals) and rounded once to FP32."""
    from fractions import Fraction
    rng = np.random.default_rng(31)
    x = (rng.standard_normal((6, 40)) * np.exp2(rng.integers(-6, 7, size=(6, 40)))).astype(np.float32)
    wide = ref.encode(x, 3, 8, 16)
    delta = (rng.standard_normal((6, 40)) * np.exp2(rng.integers(-12, 3, size=(6, 40)))).astype(np.float32)
    alpha = np.float32(-0.0123)
    _, _, w = ref.weight_update(wide, delta, float(alpha), 8)
    unit = wide.unit_exponents()
    for r in range(6):
        for c in range(40):
            exact = Fraction(float(alpha)) * Fraction(float(delta[r, c])) + Fraction(int(wide.mant[r, c])) * Fraction(2) ** int(unit[r, c])
            assert w[r, c] == _round_to_f32(exact), (r, c)


@pytest.mark.parametrize("br,bc,mn", [(1, 32, 8), (24, 24, 8), (16, 5, 12), (0, 0, 8)])
def test_weight_update_properties(br, bc, mn):
    rng = np.random.default_rng(5 + br + bc)
    x = (rng.standard_normal((70, 100)) * 0.02).astype(np.float32)
    wide = ref.encode(x, br, bc, 16)
    # a zero step changes nothing: a BFP tensor is a fixed point of its own conversion
    w0, n0, w = ref.weight_update(wide, np.ones_like(x), 0.0, mn)
    np.testing.assert_array_equal(w0.mant, wide.mant)
    np.testing.assert_array_equal(w0.exps, wide.exps)
    np.testing.assert_array_equal(w, wide.mant.astype(np.float64) * np.exp2(wide.unit_exponents().astype(np.float64)))
    # a real step: both copies are within half a unit of the FP32 result, and where they share the
    # exponent the narrow mantissas are the wide ones rounded to the top mn bits
    delta = rng.standard_normal(x.shape).astype(np.float32)
    w1, n1, w = ref.weight_update(wide, delta, -0.001, mn)
    for t in (w1, n1):
        u = np.exp2(t.unit_exponents().astype(np.float64))
        assert np.all(np.abs(t.mant * u - w.astype(np.float64)) <= 0.5 * u)
        assert np.abs(t.mant).max() <= 2 ** (t.m - 1) - 1
    same = np.repeat(np.repeat(w1.exps == n1.exps, w1.br, axis=0)[:70], w1.bc, axis=1)[:, :100]
    assert same.mean() > 0.9
    assert np.all(np.abs(n1.mant.astype(np.int64) * 2 ** (16 - mn) - w1.mant)[same] <= 2 ** (15 - mn))

