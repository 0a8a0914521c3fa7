"""Configs 3, 4 and 5 at full size, in the launch configuration the benchmark times, against the oracle on at least
64 operand rows per product: half of them the first and last rows of 256-row panels (and of the ragged last tile),
half drawn at random.  Three checks per product:
  * the encoded operands equal the oracle's bit for bit (all of them, not a sample);
  * C on the sampled rows is within 1e-5 relative Frobenius error of the FP64 oracle AND within an element-wise
    bound: |C - C64| <= n_acc * 2^-24 * sum_b |term_b|, term_b the scaled integer sum of block b (Eq. (2)) taken
    from the oracle's block sums, n_acc the number of FP32 accumulations an output receives (one per block on
    the int8 kernels; limb pairs x groups of 32 on the block-scaled kernel, where every limb product of a group is
    accumulated by an instruction of its own).  On the bf16 kernel and on FP16 planes the sums inside a block are FP32 sums
    too, so there the bound is taken against the sum of |a_k b_k| over all k, with two roundings allowed per matrix instruction
    (16 products);
  * the integer block sums of four random 32 x 32 windows of the product (hbfp_gemm_partials_window) equal the
    oracle's bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ref
from tests.util import rel_fro, unpack

pytestmark = pytest.mark.gpu
TOL = 1e-5
AUTO, INT8, SCALED = 0, 1, 2


@pytest.fixture(scope="module")
def hb():
    from paper_1804_01526_amd import hbfp
    assert torch.cuda.is_available(), "these tests need the GPU"
    return hbfp


def _rows_with_edges(M, rng, n=64, panel=256):
    edges = set()
    for p0 in range(0, M, panel):
        edges.update((p0, min(p0 + panel, M) - 1))
    edges.update((M - 1, (M - 1) // 32 * 32, max(M - 2, 0)))          # the ragged last tile
    edges = sorted(edges)
    if len(edges) > n // 2:
        keep = rng.choice(len(edges), size=n // 2 - 2, replace=False)
        edges = sorted(set([edges[i] for i in keep] + [0, M - 1]))
    rest = rng.choice(M, size=min(M, n), replace=False)
    rows = list(edges)
    for r in rest:
        if len(rows) >= min(M, n):
            break
        if int(r) not in edges:
            rows.append(int(r))
    return np.array(sorted(rows), dtype=np.int64)


def _expand(exps, rows, block, axis):
    """[blocks] -> one entry per element along `axis` (exponents of 2-D tiles repeat over the tile)."""
    return np.repeat(exps, block, axis=axis).take(np.arange(rows), axis=axis) if block > 1 else exps


def _check_product(hb, name, ta, tb, oa, ob, fa, fb, C, rows, kernel_is_scaled, rng, windows=True, src_a=None, src_b=None):
    """ta/tb: GPU operands of A [M, K] and B [K, N]; oa/ob the oracle's in that orientation; fa/fb = (block rows, block
    cols, m).  src_a/src_b: the oracle's tensors in the orientation of the matrix the GPU operand was converted from,
    where that is the transpose of A or B."""
    M, K = oa.mant.shape
    N = ob.mant.shape[1]
    for t, o in ((ta, src_a or oa), (tb, src_b or ob)):
        m, e = unpack(t)
        np.testing.assert_array_equal(m, o.mant)
        np.testing.assert_array_equal(e, o.exps)
    kb = ta.desc.kblock
    nblk = ta.desc.nblk
    got = C[rows].cpu().numpy().astype(np.float64)
    A_dec, B_dec = ref.decode(oa), ref.decode(ob)
    C64 = ref.gemm(A_dec, B_dec, rows=rows)
    err = rel_fro(got, C64)
    # element-wise: sum over blocks of |scaled block sum|, from the oracle's integer block sums of the sampled rows
    P = ref.block_dots(oa.mant[rows], ob.mant, kb)
    ea = _expand(oa.exps, M, fa[0] if fa[0] else M, 0)[rows]
    eb = _expand(ob.exps, N, fb[1] if fb[1] else N, 1)
    np.testing.assert_allclose(ref.scale_accumulate(P, ea, eb, fa[2], fb[2]), C64, rtol=1e-11, atol=0)   # the oracle agrees with itself both ways (FP64 summation order apart)
    terms = ref.scale_accumulate(np.abs(P), ea, eb, fa[2], fb[2])
    limbs = lambda m: 1 if m <= 5 else 2 if m <= 9 else 3
    if kernel_is_scaled == "bf16":
        terms = np.abs(A_dec[rows]) @ np.abs(B_dec)
        n_acc = 2 * -(-K // 16)
    elif kernel_is_scaled == "fp16":     # every FP16 matrix instruction (16 products) may round once, then one per block
        n_acc = nblk + -(-ta.desc.kpad // 16)
    else:
        n_acc = max(nblk, limbs(fa[2]) * limbs(fb[2]) * 2 * (-(-K // 64))) if kernel_is_scaled else nblk
    excess = np.abs(got - C64) - n_acc * 2.0 ** -24 * terms
    worst = float((np.abs(got - C64) / np.maximum(terms, 1e-300)).max())
    print(f"[{name}] rows={len(rows)} rel fro {err:.2e}  worst |C-C64| / sum|term| = {worst:.2e} (bound {n_acc * 2.0 ** -24:.2e})", flush=True)
    assert err <= TOL
    assert (excess <= 0).all(), f"{int((excess > 0).sum())} elements outside the element-wise bound"
    if windows:
        for _ in range(4):
            r0, c0 = int(rng.integers(0, max(M - 32, 0) + 1)), int(rng.integers(0, max(N - 32, 0) + 1))
            nr, nc = min(32, M), min(32, N)
            Pw = hb.gemm_partials_window(ta, tb, r0, nr, c0, nc)
            torch.cuda.synchronize()
            want = ref.block_dots(oa.mant[r0:r0 + nr], ob.mant[:, c0:c0 + nc], kb)
            np.testing.assert_array_equal(Pw.cpu().numpy(), want)


def test_config4_step_as_the_benchmark_runs_it(hb):
    """The three products of config 4 from operands converted and packed by hbfp_encode_packed_batch (input and
    weights) and hbfp_encode_packed (gradient) and multiplied by hbfp_gemm_packed (forward) and hbfp_gemm_packed_batch (both backward products in one launch);
    then the forward product once more on the int8 kernels."""
    import synth
    X, W, dY = synth.c4_linear()
    rng = np.random.default_rng(5)
    act_r, act_c, tile = (1, 24, 8), (24, 1, 8), (24, 24, 8)
    enc, jobs = {}, {}
    for name, src, specs in (("x", X, [(act_r, 1), (act_c, 0)]), ("w", W, [(tile, 0), (tile, 1)]), ("dy", dY, [(act_r, 1), (act_c, 0)])):
        g = torch.from_numpy(src).cuda()
        outs = [hb.alloc(hb.make_format(f[2], f[0], f[1]), 4096, 4096, ax) for f, ax in specs]
        packs = [torch.empty(hb.pack_bytes(o.desc), dtype=torch.uint8, device="cuda") for o in outs]
        jobs[name] = (g, outs, packs)
        enc[name] = list(zip(outs, packs))
    # as in the benchmark's step: input and weights in one launch, the gradient on its own
    hb.encode_packed_batch([jobs["x"], jobs["w"]])
    hb.encode_packed(*jobs["dy"])
    torch.cuda.synchronize()
    del jobs
    for _, (o, pk) in ((k, v) for k, vs in enc.items() for v in vs):
        w = pk[:8].view(torch.int32).cpu().numpy()
        assert w[0] != w[1], "config 4's operands are expected to pack densely (no fallback)"
    oX_r, oX_c = ref.encode(X, 1, 24, 8), ref.encode(X, 24, 1, 8)
    oW = ref.encode(W, 24, 24, 8)
    oD_r, oD_c = ref.encode(dY, 1, 24, 8), ref.encode(dY, 24, 1, 8)
    T = lambda o: ref.BFP(np.ascontiguousarray(o.mant.T), np.ascontiguousarray(o.exps.T), o.m, o.bc, o.br)
    (x_f, px_f), (x_w, px_w) = enc["x"]
    (w_f, pw_f), (w_d, pw_d) = enc["w"]
    (d_d, pd_d), (d_w, pd_w) = enc["dy"]
    rows = _rows_with_edges(4096, rng)
    cases = (("c4 fwd", x_f, px_f, w_f, pw_f, oX_r, oW, act_r, tile, None, None),
             ("c4 dgrad", d_d, pd_d, w_d, pw_d, oD_r, T(oW), act_r, tile, None, oW),
             ("c4 wgrad", x_w, px_w, d_w, pd_w, T(oX_c), oD_c, act_r, act_c, oX_c, None))
    # as in the benchmark's step: the forward product alone, both backward products in one launch
    outs = [hb.gemm_packed(x_f, px_f, w_f, pw_f)]
    outs += hb.gemm_packed_batch([(d_d, pd_d, w_d, pw_d), (x_w, px_w, d_w, pd_w)],
                                 [torch.full((4096, 4096), float("nan"), device="cuda") for _ in range(2)])
    torch.cuda.synchronize()
    for (name, a, pa, b, pb, oa, ob, fa, fb, sa, sb), C in zip(cases, outs):
        _check_product(hb, name, a, b, oa, ob, fa, fb, C, rows, "bf16", rng, src_a=sa, src_b=sb)
    one = hb.gemm_packed(d_d, pd_d, w_d, pw_d)
    torch.cuda.synchronize()
    assert torch.equal(one, outs[1])                       # the shared launch changes no bit
    del outs, one
    C = hb.gemm(x_f, w_f, kernel=INT8)
    torch.cuda.synchronize()
    _check_product(hb, "c4 fwd int8", x_f, w_f, oX_r, oW, act_r, tile, C, rows, False, rng, windows=False)


def test_config3_conv_shapes(hb):
    """Config 3 (a 3 x 3 convolution on 128 x 28 x 28 outputs lowered to a product): forward, data gradient, weight
    gradient with blocks of 32, the library's choice of kernel."""
    import synth
    X, W, dY = synth.c3_conv_as_gemm()
    rng = np.random.default_rng(3)
    f_row, f_col = (1, 32, 8), (32, 1, 8)
    for name, A, B in (("c3 fwd", X, W), ("c3 dgrad", dY, np.ascontiguousarray(W.T)), ("c3 wgrad", np.ascontiguousarray(X.T), dY)):
        ta = hb.encode(torch.from_numpy(A).cuda(), 1, hb.make_format(8, 1, 32))
        tb = hb.encode(torch.from_numpy(B).cuda(), 0, hb.make_format(8, 32, 1))
        C = hb.gemm(ta, tb)
        torch.cuda.synchronize()
        oa, ob = ref.encode(A, 1, 32, 8), ref.encode(B, 32, 1, 8)
        scaled = hb.gemm_workspace(ta.desc, tb.desc) > hb.gemm_select_workspace(ta.desc, tb.desc, INT8)
        _check_product(hb, name, ta, tb, oa, ob, f_row, f_col, C, _rows_with_edges(A.shape[0], rng), scaled, rng)
        del ta, tb, C, oa, ob


def _check_gathered(name, got, low, flt_dec, nblk):
    """Sampled rows of a convolution product against the FP64 product of the oracle's lowered rows and decoded filter:
    relative Frobenius error, and element-wise |C - C64| <= blocks * 2^-24 * sum_k |a_k b_k| (one FP32 accumulation per
    block of 32; a block's integer sum is no larger than the sum of its products' magnitudes)."""
    C64 = ref.gemm(low, flt_dec)
    err = rel_fro(got, C64)
    terms = np.abs(low).astype(np.float64) @ np.abs(flt_dec).astype(np.float64)
    worst = float((np.abs(got - C64) / np.maximum(terms, 1e-300)).max())
    print(f"[{name}] rows={len(low)} rel fro {err:.2e}  worst |C-C64| / sum|a b| = {worst:.2e} (bound {nblk * 2.0 ** -24:.2e})", flush=True)
    assert np.linalg.norm(C64) > 0
    assert err <= TOL
    assert (np.abs(got - C64) <= nblk * 2.0 ** -24 * terms).all()


def test_config3_convolution_gathered_by_the_product(hb):
    """Config 3 as the convolution it is (hbfp_gemm_conv2d, as the benchmark runs it): the image converted once, bit for bit
    against the oracle; the product on 64 output positions (panel edges and random) against the oracle's explicitly
    lowered rows.  Then the data gradient of the strided convolution that would produce config 3's activations
    (128 x 56 x 56 x 64 -> 3 x 3, stride 2 -> 128 x 28 x 28 x 128; hbfp_gemm_conv2d_dgrad, phase by phase), the same way."""
    import synth
    X, W, dY = synth.c3_conv_as_gemm()
    rng = np.random.default_rng(33)
    n, h, w, c, f = 128, 28, 28, 128, 128
    img = np.maximum(synth.normal((n, h, w, c), 3, 7), 0.0)                      # activations after a ReLU, as config 3's X
    conv = hb.Conv2d(n, h, w, c, 3, 3, 1, 1, 1, 1, 0, 0)
    ti = hb.encode(torch.from_numpy(img.reshape(n * h * w, c)).cuda(), 1, hb.make_format(8, 1, 32))
    tf = hb.encode(torch.from_numpy(W).cuda(), 0, hb.make_format(8, 32, 1))
    y = hb.gemm_conv2d(ti, conv, tf)
    torch.cuda.synchronize()
    oi, of = ref.encode(img.reshape(n * h * w, c), 1, 32, 8), ref.encode(W, 32, 1, 8)
    for t, o in ((ti, oi), (tf, of)):
        m, e = unpack(t)
        np.testing.assert_array_equal(m, o.mant)
        np.testing.assert_array_equal(e, o.exps)
    rows = _rows_with_edges(n * h * w, rng)
    low = ref.im2col_rows(ref.decode(oi).reshape(n, h, w, c), rows, 3, 3, 1, 1)
    _check_gathered("c3 conv2d fwd", y[rows].cpu().numpy().astype(np.float64), low, ref.decode(of), 36)
    del ti, y, oi, low

    hx, wx, cx = 56, 56, 64
    w4 = np.ascontiguousarray(W.reshape(3, 3, 128, 128)[:, :, :cx, :])          # [r, s, c, f] of the strided convolution
    wd = np.ascontiguousarray(ref.filter_matrix_dgrad(w4))                         # [9 * 128, 64]
    sconv = hb.Conv2d(n, hx, wx, cx, 3, 3, 1, 1, 2, 2, 0, 0)
    assert sconv.out_hw() == (h, w)
    td = hb.encode(torch.from_numpy(dY).cuda(), 1, hb.make_format(8, 1, 32))
    tw = hb.encode(torch.from_numpy(wd).cuda(), 0, hb.make_format(8, 32, 1))
    dx = hb.gemm_conv2d_dgrad(td, sconv, tw)
    torch.cuda.synchronize()
    od, ow = ref.encode(dY, 1, 32, 8), ref.encode(wd, 32, 1, 8)
    for t, o in ((td, od), (tw, ow)):
        m, e = unpack(t)
        np.testing.assert_array_equal(m, o.mant)
        np.testing.assert_array_equal(e, o.exps)
    rows = _rows_with_edges(n * hx * wx, rng)
    low = ref.im2col_dgrad_rows(ref.decode(od).reshape(n, h, w, f), rows, hx, wx, 3, 3, 1, 1, 2, 2)
    _check_gathered("strided dgrad into 128x56x56x64", dx[rows].cpu().numpy().astype(np.float64), low, ref.decode(ow), 36)


def test_config5_wide_range_bfp12(hb):
    """Config 5: 8192^3, 12-bit mantissas, blocks of 64, stochastic rounding, rows spanning 2^+-20: the library's choice
    (FP16 planes relative to the rows' largest exponents on the 256 x 256-tile kernel), then the FP16 matrix instruction
    with per-block scaling, then the block-scaled kernel with three limbs per mantissa, then the int8 limb kernels."""
    import synth
    A, B = synth.c5_wide_range()
    rng = np.random.default_rng(6)
    ta = hb.encode(torch.from_numpy(A).cuda(), 1, hb.make_format(12, 1, 64, 1, 51))
    tb = hb.encode(torch.from_numpy(B).cuda(), 0, hb.make_format(12, 64, 1, 1, 52))
    oa, ob = ref.encode(A, 1, 64, 12, 1, 51), ref.encode(B, 64, 1, 12, 1, 52)
    rows = _rows_with_edges(8192, rng)
    C = hb.gemm(ta, tb)
    torch.cuda.synchronize()
    assert hb.gemm_workspace(ta.desc, tb.desc) == hb.gemm_select_workspace(ta.desc, tb.desc, hb.KERNEL_FP16_PLANES)
    _check_product(hb, "c5 fp16 planes", ta, tb, oa, ob, (1, 64, 12), (64, 1, 12), C, rows, "bf16", rng)
    C.zero_()
    C = hb.gemm(ta, tb, out=C, kernel=hb.KERNEL_FP16)
    torch.cuda.synchronize()
    _check_product(hb, "c5 fp16", ta, tb, oa, ob, (1, 64, 12), (64, 1, 12), C, rows, "fp16", rng, windows=False)
    C.zero_()
    C = hb.gemm(ta, tb, out=C, kernel=hb.KERNEL_SCALED)
    torch.cuda.synchronize()
    _check_product(hb, "c5 scaled", ta, tb, oa, ob, (1, 64, 12), (64, 1, 12), C, rows, True, rng, windows=False)
    C.zero_()
    C = hb.gemm(ta, tb, out=C, kernel=INT8)
    torch.cuda.synchronize()
    # the int8 limb kernels convert block sums of up to 2.7e8 to FP32 (one rounding each) before scaling them
    _check_product(hb, "c5 int8 limbs", ta, tb, oa, ob, (1, 64, 12), (64, 1, 12), C, rows, False, rng, windows=False)
