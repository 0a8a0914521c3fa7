#!/usr/bin/env python3
"""Benchmark of the BFP hot path on one MI355X.

A step is one pass of the whole path over one batch of config 4 (dense layer,
M = K = N = 4096, 8-bit mantissas, 1 x 24 activation/gradient blocks, 24 x 24 weight
tiles): the three FP32 matrices (input, weights, output gradient) are converted
FP32 -> BFP, each into both operand layouts it is needed in, stored and packed, by
one kernel that reads it once (hbfp_encode_packed_batch for input and weights,
hbfp_encode_packed for the gradient), and the forward, data-gradient and
weight-gradient products are multiplied from the packed operands (hbfp_gemm_packed,
hbfp_gemm_packed_batch: 8-bit mantissas times their block's power of two are exact
bf16 numbers, so the products run on the bf16 matrix instruction with FP32
accumulation).  The cpu_baseline leg does the same six conversions one by one and the
three products in FP64.  Inputs are resident in HBM before the timed region.  One JSON
line is printed; `value` is effective TOP/s (2*M*N*K per product, padding not counted)
including every conversion.

The same line carries: the roofline of the dominant kernel (the GEMM) and of the
encode kernel on config 2 (64M log-normal values, blocks of 32), both timed with HIP
events on the launch stream, and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0   # MI355X dense int8 matrix peak, published
FP6_PEAK_TFLOPS = 10100.0  # MI355X dense FP6 / FP4 matrix peak, published
FP32_VECTOR_PEAK_TFLOPS = 157.3   # MI355X FP32 vector peak, published (256 CUs x 4 SIMDs x 64 flop/clk x 2.4 GHz)
HBM_PEAK_GBPS = 8000.0    # MI355X HBM3E peak, published

BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/gemm_config4_hbm_traffic_counters.txt for the
# product kernel of config 4 alone, profiles/bench_default_hbm_traffic_counters.txt for the encode), scaled by what the same
# counters read for a plain 1 GiB device copy (fetch x2.0, write x1.0):
#   config 4 product kernel (gemm_bf_kernel, 128 k-steps of 32): 98454 KiB x 2.0 + 65536 KiB = 268.7 MB
#   config 2 encode m=8 RNE launch: 131552 KiB x 2.0 + 67588 KiB = 338.6 MB   (algorithmic 337.6 MB)
TRAFFIC_GEMM_C4_BYTES = 268.7e6
TRAFFIC_ENCODE_C2_M8_BYTES = 338.6e6
# algorithmic bytes of the config 4 product kernel: both operands as bf16 planes read once (4096 rows x 4096 k x 2 bytes
# each: blocks of 24 are packed without their padding) and C written once; operand panels are re-read by the workgroups
# of different XCDs
ALG_BYTES_GEMM_C4 = 2 * 4096 * 4096 * 2 + 4096 * 4096 * 4


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--preheat", type=int, default=60,
                    help="untimed steps before the warm-up steps: after idle the chip's power management needs some 50 steps to settle")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--graph", action="store_true", help="replay each step as one HIP graph instead of 8 separate launches")
    ap.add_argument("--no-extra", action="store_true", help="skip the config 2 / 3 / 5 side measurements")
    ap.add_argument("--no-probe", action="store_true", help="skip the register-only matrix-instruction loops")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies, so that a counter run can scale FETCH_SIZE/WRITE_SIZE")
    return ap.parse_args()


class Timer:
    """Accumulates HIP-event time of bracketed regions on the current stream."""

    def __init__(self, torch):
        self.torch = torch
        self.pairs = {}

    def region(self, name):
        t = self.torch
        a, b = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
        self.pairs.setdefault(name, []).append((a, b))
        return a, b

    def total_ms(self, name):
        return sum(a.elapsed_time(b) for a, b in self.pairs.get(name, []))

    def count(self, name):
        return len(self.pairs.get(name, []))


def _linear_layer(torch, hbfp, synth):
    """Buffers and the step function of config 4.  Nothing is allocated inside step()."""
    M = K = N = 4096
    Xh, Wh, dYh = synth.c4_linear(M, K, N)
    X, W, dY = (torch.from_numpy(a).cuda() for a in (Xh, Wh, dYh))
    f_act_row = hbfp.make_format(8, 1, 24)     # 1 x 24 blocks along a row-contiguous contraction axis
    f_act_col = hbfp.make_format(8, 24, 1)     # the same tensors contracted down their rows (weight gradient)
    f_w = hbfp.make_format(8, 24, 24)          # 24 x 24 weight tiles, either orientation

    ops = {
        # name: (source, contraction axis, format)
        "x_fwd": (X, 1, f_act_row), "w_fwd": (W, 0, f_w),
        "dy_dgrad": (dY, 1, f_act_row), "w_dgrad": (W, 1, f_w),
        "x_wgrad": (X, 0, f_act_col), "dy_wgrad": (dY, 0, f_act_col),
    }
    enc = {k: hbfp.alloc(f, s.shape[0], s.shape[1], ax) for k, (s, ax, f) in ops.items()}
    prods = [("x_fwd", "w_fwd"), ("dy_dgrad", "w_dgrad"), ("x_wgrad", "dy_wgrad")]
    outs = [torch.empty((enc[a].desc.rows, enc[b].desc.rows), dtype=torch.float32, device="cuda") for a, b in prods]
    # each source matrix is converted into both of its operand layouts, stored and packed for the block-scaled kernel,
    # by one call that reads it once (hbfp_encode_packed)
    packed = {k: torch.empty(hbfp.pack_bytes(t.desc), dtype=torch.uint8, device="cuda") for k, t in enc.items()}
    groups = {"x": ("encode_act", X, ["x_fwd", "x_wgrad"]), "dy": ("encode_act", dY, ["dy_dgrad", "dy_wgrad"]),
              "w": ("encode_w", W, ["w_fwd", "w_dgrad"])}
    assert all(hbfp.encode_packed_workspace([enc[k] for k in names]) == 0 for _, _, names in groups.values())
    product = lambda i: (enc[prods[i][0]], packed[prods[i][0]], enc[prods[i][1]], packed[prods[i][1]])
    ws_fwd = torch.empty(max(hbfp.gemm_packed_workspace(enc["x_fwd"].desc, enc["w_fwd"].desc), 256), dtype=torch.uint8, device="cuda")
    ws_bwd = torch.empty(max(hbfp.gemm_packed_batch_workspace([(product(i)[0], product(i)[2]) for i in (1, 2)]), 256),
                         dtype=torch.uint8, device="cuda")

    def bracket(timer, name, fn):
        if timer:
            a, b = timer.region(name)
            a.record()
        fn()
        if timer:
            b.record()

    source = lambda key: (groups[key][1], [enc[k] for k in groups[key][2]], [packed[k] for k in groups[key][2]])

    def convert(timer, key):
        bracket(timer, groups[key][0], lambda: hbfp.encode_packed(*source(key)))

    def step(timer=None):
        # the order of a training step: inputs and weights, the forward product, then the gradient that arrives from
        # the layer above and the two backward products that wait for it, which share one launch
        # (input and weights do not wait for each other: one call, one launch)
        bracket(timer, "encode_x_w", lambda: hbfp.encode_packed_batch([source("x"), source("w")]))
        bracket(timer, "gemm", lambda: hbfp.gemm_packed(*product(0), out=outs[0], workspace=ws_fwd))
        convert(timer, "dy")
        bracket(timer, "gemm_pair", lambda: hbfp.gemm_packed_batch([product(1), product(2)], outs[1:], workspace=ws_bwd))

    def step_weights_resident():
        # the same step when the weights already sit in BFP (Sec. 4.2 keeps them so between updates): only the FP32-resident
        # operands - input and output gradient - are converted
        convert(None, "x")
        hbfp.gemm_packed(*product(0), out=outs[0], workspace=ws_fwd)
        convert(None, "dy")
        hbfp.gemm_packed_batch([product(1), product(2)], outs[1:], workspace=ws_bwd)

    step.weights_resident = step_weights_resident
    flops_per_product = 2.0 * M * N * K
    return step, 3 * flops_per_product, flops_per_product, dict(M=M, N=N, K=K), outs


def _encode_config2(torch, hbfp, synth, reps=100):
    """Config 2: 64M log-normal values, blocks of 32; four rotating inputs (1 GiB) defeat the last-level cache.
    20 untimed and 100 timed launches each, the median reported."""
    n = 1 << 26
    x0 = torch.from_numpy(synth.c2_lognormal(n)).cuda().reshape(1, n)
    srcs = [x0] + [x0.roll(1 + i, dims=1).contiguous() for i in range(3)]
    res = {}
    for m, rounding, tag in ((8, 0, "m8_rne"), (8, 1, "m8_sr"), (12, 0, "m12_rne"), (12, 1, "m12_sr")):
        fmt = hbfp.make_format(m, 1, 32, rounding, 1234)
        outs = [hbfp.alloc(fmt, 1, n, 1) for _ in range(4)]
        for i in range(20):
            hbfp.encode(srcs[i % 4], 1, fmt, out=outs[i % 4])
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for r in range(reps):
            ev[r][0].record()
            hbfp.encode(srcs[r % 4], 1, fmt, out=outs[r % 4])
            ev[r][1].record()
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)[reps // 2]
        bytes_alg = n * (4 + (1 if m <= 8 else 2)) + n // 32
        res[f"encode_{tag}"] = {"ms": round(ms, 4), "GBps": round(bytes_alg / ms / 1e6, 1), "bytes": bytes_alg}
        if rounding == 0:
            dst = [torch.empty((1, n), dtype=torch.float32, device="cuda") for _ in range(4)]
            for i in range(20):
                hbfp.decode(outs[i % 4], out=dst[i % 4])
            torch.cuda.synchronize()
            for r in range(reps):
                ev[r][0].record()
                hbfp.decode(outs[r % 4], out=dst[r % 4])
                ev[r][1].record()
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in ev)[reps // 2]
            res[f"decode_m{m}"] = {"ms": round(ms, 4), "GBps": round(bytes_alg / ms / 1e6, 1), "bytes": bytes_alg}
            del dst
        del outs
    return res


def _time_call(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return sorted(a.elapsed_time(b) for a, b in ev)[reps // 2]


def _weight_update_config4(torch, hbfp, synth, reps=10):
    """Config 4's weights (4096 x 4096, 24 x 24 tiles) kept with 16-bit mantissas: one FP32 update step
    re-encoded into the wide copy and the two 8-bit operand layouts (forward, data gradient)."""
    _, Wh, dYh = synth.c4_linear()
    W, G = torch.from_numpy(Wh).cuda(), torch.from_numpy(dYh).cuda()
    f_wide, f_nar = hbfp.make_format(16, 24, 24), hbfp.make_format(8, 24, 24)
    wide = hbfp.encode(W, 1, f_wide)
    na, nb = hbfp.alloc(f_nar, 4096, 4096, 0), hbfp.alloc(f_nar, 4096, 4096, 1)
    ws = torch.empty(hbfp.weight_update_workspace(wide, na, nb), dtype=torch.uint8, device="cuda")
    ms = _time_call(torch, lambda: hbfp.weight_update(wide, G, -1e-3, na, nb, workspace=ws), reps)
    n = 4096 * 4096
    nblocks = 171 * 171
    alg = n * (2 + 4 + 2 + 1 + 1) + 4 * nblocks          # read wide + step, write wide + two narrow copies; one exponent per tile
    return {"weight_update_c4": {"ms": round(ms, 4), "GBps": round(alg / ms / 1e6, 1), "bytes": alg,
                                 "note": "one kernel: tiles of the updated weights stay in registers; 10 B/element algorithmic"}}


def _gemm_side_configs(torch, hbfp, synth, reps=10):
    """Config 3 (conv lowered to GEMM; forward, dgrad, wgrad), kernel-only and including encodes."""
    res = {}
    # config 1 (256^3, blocks of 32): the parity configuration, bound by launch latency; conversions and product as three calls
    Ah, Bh = synth.c1_gemm_small()
    A1, B1 = torch.from_numpy(Ah).cuda(), torch.from_numpy(Bh).cuda()
    f1a, f1b = hbfp.make_format(8, 1, 32), hbfp.make_format(8, 32, 1)
    t1a, t1b = hbfp.alloc(f1a, 256, 256, 1), hbfp.alloc(f1b, 256, 256, 0)
    out1 = torch.empty((256, 256), dtype=torch.float32, device="cuda")
    ws1 = torch.empty(max(hbfp.gemm_workspace(t1a.desc, t1b.desc), 256), dtype=torch.uint8, device="cuda")

    def c1_call():
        hbfp.encode(A1, 1, f1a, out=t1a)
        hbfp.encode(B1, 0, f1b, out=t1b)
        hbfp.gemm(t1a, t1b, out=out1, workspace=ws1)

    ms1 = _time_call(torch, c1_call, 50)
    res["c1_256_cubed_incl_encodes"] = {"ms": round(ms1, 4), "TOPS": round(2.0 * 256 ** 3 / ms1 / 1e9, 2)}
    del A1, B1, t1a, t1b, out1, ws1
    Xh, Wh, dYh = synth.c3_conv_as_gemm()
    X, W, dY = (torch.from_numpy(a).cuda() for a in (Xh, Wh, dYh))
    row, col = hbfp.make_format(8, 1, 32), hbfp.make_format(8, 32, 1)
    passes = {
        "c3_fwd": ((X, 1, row), (W, 0, col)),
        "c3_dgrad": ((dY, 1, row), (W, 1, row)),
        "c3_wgrad": ((X, 0, col), (dY, 0, col)),
    }
    for name, ((sa, axa, fa), (sb, axb, fb)) in passes.items():
        ta, tb = hbfp.alloc(fa, sa.shape[0], sa.shape[1], axa), hbfp.alloc(fb, sb.shape[0], sb.shape[1], axb)
        out = torch.empty((ta.desc.rows, tb.desc.rows), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(hbfp.gemm_workspace(ta.desc, tb.desc), 256), dtype=torch.uint8, device="cuda")
        hbfp.encode(sa, axa, fa, out=ta)
        hbfp.encode(sb, axb, fb, out=tb)
        flops = 2.0 * ta.desc.rows * tb.desc.rows * ta.desc.kdim
        ms_k = _time_call(torch, lambda: hbfp.gemm(ta, tb, out=out, workspace=ws), reps)
        ms_ea = _time_call(torch, lambda: hbfp.encode(sa, axa, fa, out=ta), reps)
        ms_eb = _time_call(torch, lambda: hbfp.encode(sb, axb, fb, out=tb), reps)
        res[name] = {"gemm_ms": round(ms_k, 4), "encode_a_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4),
                     "TOPS_kernel": round(flops / ms_k / 1e9, 1),
                     "TOPS_incl_encode": round(flops / (ms_k + ms_ea + ms_eb) / 1e9, 1)}
        del ta, tb, out, ws
    # config 3's forward product with the activation operand converted straight from the NHWC image tensor
    # (128 x 28 x 28 x 128, 3 x 3 filter, padding 1: the same 100352 x 1152 operand, never materialised in FP32)
    gi = torch.Generator(device="cuda").manual_seed(33)
    img = torch.relu(torch.randn((128, 28, 28, 128), device="cuda", generator=gi))
    conv = hbfp.Conv2d(128, 28, 28, 128, 3, 3, 1, 1, 1, 1, 0, 0)
    ta, tb = hbfp.alloc(row, 100352, 1152, 1), hbfp.encode(W, 0, col)
    out = torch.empty((ta.desc.rows, tb.desc.rows), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(hbfp.gemm_workspace(ta.desc, tb.desc), 256), dtype=torch.uint8, device="cuda")
    hbfp.encode_im2col(img, conv, row, out=ta)
    flops = 2.0 * ta.desc.rows * tb.desc.rows * ta.desc.kdim
    ms_k = _time_call(torch, lambda: hbfp.gemm(ta, tb, out=out, workspace=ws), reps)
    ms_ea = _time_call(torch, lambda: hbfp.encode_im2col(img, conv, row, out=ta), reps)
    ms_eb = _time_call(torch, lambda: hbfp.encode(W, 0, col, out=tb), reps)
    res["c3_fwd_from_image"] = {"gemm_ms": round(ms_k, 4), "encode_im2col_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4),
                                "TOPS_kernel": round(flops / ms_k / 1e9, 1),
                                "TOPS_incl_encode": round(flops / (ms_k + ms_ea + ms_eb) / 1e9, 1),
                                "note": "activation operand from the 51 MB image tensor instead of the 462 MB lowered matrix"}
    del ta, tb, out, ws
    # config 3's forward product without any lowered operand: the image converted once as [pixels][channels] (blocks of 32
    # channels, 12.8 MB of mantissas) and gathered tap by tap by the product kernel's own copies (hbfp_gemm_conv2d)
    x2 = img.view(-1, 128)
    ti, tf = hbfp.alloc(row, 100352, 128, 1), hbfp.encode(W, 0, col)
    out = torch.empty((100352, 128), dtype=torch.float32, device="cuda")
    wsc = torch.empty(hbfp.gemm_conv2d_workspace(ti.desc, conv, tf.desc), dtype=torch.uint8, device="cuda")
    hbfp.encode(x2, 1, row, out=ti)
    ms_k = _time_call(torch, lambda: hbfp.gemm_conv2d(ti, conv, tf, out=out, workspace=wsc), reps)
    ms_ea = _time_call(torch, lambda: hbfp.encode(x2, 1, row, out=ti), reps)
    ms_eb = _time_call(torch, lambda: hbfp.encode(W, 0, col, out=tf), reps)

    def conv_forward():
        hbfp.encode(x2, 1, row, out=ti)
        hbfp.encode(W, 0, col, out=tf)
        hbfp.gemm_conv2d(ti, conv, tf, out=out, workspace=wsc)

    ms_all = _time_call(torch, conv_forward, reps)
    # ... and delivered as the next layer's image: ReLU and the FP->BFP conversion applied to the accumulators by the same
    # kernel (hbfp_gemm_conv2d_bfp), against product + ReLU pass + conversion call
    nxt = hbfp.alloc(row, 100352, 128, 1)
    wsb = torch.empty(hbfp.gemm_conv2d_bfp_workspace(ti.desc, conv, tf.desc, nxt.desc), dtype=torch.uint8, device="cuda")

    def conv_relu_encode():
        hbfp.gemm_conv2d(ti, conv, tf, out=out, workspace=wsc)
        torch.relu_(out)
        hbfp.encode(out, 1, row, out=nxt)

    ms_three = _time_call(torch, conv_relu_encode, reps)
    ms_one = _time_call(torch, lambda: hbfp.gemm_conv2d_bfp(ti, conv, tf, row, relu=True, out=nxt, workspace=wsb), reps)
    res["c3_fwd_conv2d_delivered_as_the_next_image"] = {"conv_relu_encode_ms": round(ms_three, 4), "gemm_conv2d_bfp_ms": round(ms_one, 4),
                                                        "TOPS": round(flops / ms_one / 1e9, 1)}
    del nxt, wsb
    res["c3_fwd_conv2d_gather_in_the_product"] = {
        "gemm_ms": round(ms_k, 4), "encode_image_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4), "whole_forward_ms": round(ms_all, 4),
        "TOPS_kernel": round(flops / ms_k / 1e9, 1), "TOPS_incl_encode": round(flops / ms_all / 1e9, 1),
        "note": "no lowered operand in memory: 51 MB of FP32 image read once, 12.8 MB of mantissas written, the nine taps gathered from cache"}
    del ti, tf, out, wsc
    # ... in the format of Sec. 5.1: one exponent per training input (gathered and converted from the image tensor,
    # stored in blocks of 24) against the filter matrix in 24 x 24 tiles
    per_input, tile24 = hbfp.make_format(8, 28 * 28, 0, k_slot=24), hbfp.make_format(8, 24, 24)
    ta, tb = hbfp.alloc(per_input, 100352, 1152, 1), hbfp.encode(W, 0, tile24)
    out = torch.empty((ta.desc.rows, tb.desc.rows), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(hbfp.gemm_workspace(ta.desc, tb.desc), 256), dtype=torch.uint8, device="cuda")
    wse = torch.empty(max(hbfp.encode_workspace(ta.desc), 256), dtype=torch.uint8, device="cuda")
    hbfp.encode_im2col(img, conv, per_input, out=ta, workspace=wse)
    ms_k = _time_call(torch, lambda: hbfp.gemm(ta, tb, out=out, workspace=ws), reps)
    ms_ea = _time_call(torch, lambda: hbfp.encode_im2col(img, conv, per_input, out=ta, workspace=wse), reps)
    ms_eb = _time_call(torch, lambda: hbfp.encode(W, 0, tile24, out=tb), reps)
    res["c3_fwd_from_image_exponent_per_input_x_24x24_tiles"] = {
        "gemm_ms": round(ms_k, 4), "encode_im2col_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4),
        "TOPS_kernel": round(flops / ms_k / 1e9, 1), "TOPS_incl_encode": round(flops / (ms_k + ms_ea + ms_eb) / 1e9, 1)}
    del ta, tb, out, ws, wse
    # ... the same format in full (filter exponents shared by 24 channels x 24 filters x the whole window: window entries
    # channel block by channel block) without any lowered operand: the image, its channels padded with zeros to 144 = 6 x 24,
    # converted once with one exponent per training input, gathered slot by slot by the product (hbfp_gemm_conv2d)
    img144 = torch.zeros((128, 28, 28, 144), device="cuda")
    img144[..., :128] = img
    W144 = torch.zeros((6, 9, 24, 128), device="cuda")                        # [channel block][tap][channel][filter]
    W144.view(6, 9, 24, 128)[:5] = W.view(9, 128, 128)[:, :120].reshape(9, 5, 24, 128).permute(1, 0, 2, 3)
    W144[5, :, :8] = W.view(9, 128, 128)[:, 120:]
    W144 = W144.view(9 * 144, 128)
    conv144 = hbfp.Conv2d(128, 28, 28, 144, 3, 3, 1, 1, 1, 1, 24, 0)
    per_image, outer = hbfp.make_format(8, 28 * 28, 0, k_slot=24), hbfp.make_format(8, 9 * 24, 24, k_slot=24)
    x144 = img144.view(-1, 144)
    ti, tf = hbfp.alloc(per_image, 100352, 144, 1), hbfp.encode(W144, 0, outer)
    out = torch.empty((100352, 128), dtype=torch.float32, device="cuda")
    wsc = torch.empty(hbfp.gemm_conv2d_workspace(ti.desc, conv144, tf.desc), dtype=torch.uint8, device="cuda")
    wse = torch.empty(max(hbfp.encode_workspace(ti.desc), 256), dtype=torch.uint8, device="cuda")
    hbfp.encode(x144, 1, per_image, out=ti, workspace=wse)
    ms_k = _time_call(torch, lambda: hbfp.gemm_conv2d(ti, conv144, tf, out=out, workspace=wsc), reps)
    ms_ea = _time_call(torch, lambda: hbfp.encode(x144, 1, per_image, out=ti, workspace=wse), reps)
    ms_eb = _time_call(torch, lambda: hbfp.encode(W144, 0, outer, out=tf), reps)
    res["c3_fwd_conv2d_gather_exponent_per_input_x_outer_dimension_tiles"] = {
        "gemm_ms": round(ms_k, 4), "encode_image_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4),
        "TOPS_kernel": round(flops / ms_k / 1e9, 1), "TOPS_incl_encode": round(flops / (ms_k + ms_ea + ms_eb) / 1e9, 1),
        "note": "54 slots of 24 channels (stored as 32) instead of 36 blocks of 32; no 154 MB lowered operand"}
    del img144, W144, x144, ti, tf, out, wsc, wse
    # ... and its weight gradient dW [1152, 128] = lowered(X)^T dY with the lowered operand gathered the same way
    ta, tb = hbfp.alloc(col, 100352, 1152, 0), hbfp.encode(dY, 0, col)
    out = torch.empty((ta.desc.rows, tb.desc.rows), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(hbfp.gemm_workspace(ta.desc, tb.desc), 256), dtype=torch.uint8, device="cuda")
    hbfp.encode_im2col(img, conv, col, 0, out=ta)
    ms_k = _time_call(torch, lambda: hbfp.gemm(ta, tb, out=out, workspace=ws), reps)
    ms_ea = _time_call(torch, lambda: hbfp.encode_im2col(img, conv, col, 0, out=ta), reps)
    ms_eb = _time_call(torch, lambda: hbfp.encode(dY, 0, col, out=tb), reps)
    res["c3_wgrad_from_image"] = {"gemm_ms": round(ms_k, 4), "encode_im2col_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4),
                                  "TOPS_kernel": round(flops / ms_k / 1e9, 1),
                                  "TOPS_incl_encode": round(flops / (ms_k + ms_ea + ms_eb) / 1e9, 1)}
    del ta, tb, out, ws
    # ... and its data gradient as a forward-shaped product: dY (128 x 28 x 28 x 128 as an image of gradients) gathered
    # with padding r - 1 - pad = 1 against the mirrored filter with its channel axes exchanged gives dX [100352, 128]
    # itself, where the lowered form (c3_dgrad) leaves 462 MB of FP32 that a scatter-add still has to fold
    Wd = W.view(3, 3, 128, 128).flip(0, 1).permute(0, 1, 3, 2).reshape(1152, 128).contiguous()
    dimg = dY.view(128, 28, 28, 128)
    ta, tb = hbfp.alloc(row, 100352, 1152, 1), hbfp.encode(Wd, 0, col)
    out = torch.empty((ta.desc.rows, tb.desc.rows), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(hbfp.gemm_workspace(ta.desc, tb.desc), 256), dtype=torch.uint8, device="cuda")
    hbfp.encode_im2col(dimg, conv, row, out=ta)
    ms_k = _time_call(torch, lambda: hbfp.gemm(ta, tb, out=out, workspace=ws), reps)
    ms_ea = _time_call(torch, lambda: hbfp.encode_im2col(dimg, conv, row, out=ta), reps)
    ms_eb = _time_call(torch, lambda: hbfp.encode(Wd, 0, col, out=tb), reps)
    res["c3_dgrad_from_gradient_image"] = {"gemm_ms": round(ms_k, 4), "encode_im2col_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4),
                                           "TOPS_kernel": round(flops / ms_k / 1e9, 1),
                                           "TOPS_incl_encode": round(flops / (ms_k + ms_ea + ms_eb) / 1e9, 1),
                                           "note": "dX directly (51 MB), no lowered gradient and no scatter-add"}
    del ta, tb, out, ws
    # ... and the same data gradient with the gather in the product: the gradient image converted once (12.8 MB)
    d2 = dY.view(-1, 128)
    ti, tf = hbfp.alloc(row, 100352, 128, 1), hbfp.encode(Wd, 0, col)
    out = torch.empty((100352, 128), dtype=torch.float32, device="cuda")
    wsc = torch.empty(hbfp.gemm_conv2d_workspace(ti.desc, conv, tf.desc), dtype=torch.uint8, device="cuda")

    def conv_dgrad():
        hbfp.encode(d2, 1, row, out=ti)
        hbfp.encode(Wd, 0, col, out=tf)
        hbfp.gemm_conv2d(ti, conv, tf, out=out, workspace=wsc)

    ms_all = _time_call(torch, conv_dgrad, reps)
    ms_k = _time_call(torch, lambda: hbfp.gemm_conv2d(ti, conv, tf, out=out, workspace=wsc), reps)
    res["c3_dgrad_conv2d_gather_in_the_product"] = {"gemm_ms": round(ms_k, 4), "whole_data_gradient_ms": round(ms_all, 4),
                                                    "TOPS_kernel": round(flops / ms_k / 1e9, 1),
                                                    "TOPS_incl_encode": round(flops / ms_all / 1e9, 1)}
    del ti, tf, out, wsc
    # ... and the data gradient of the strided convolution that would produce config 3's activations (128 x 56 x 56 x 64,
    # 3 x 3, stride 2 -> 128 x 28 x 28 x 128): the same gradient image, no zeros stored or multiplied between its pixels,
    # one launch that walks the four output phases (hbfp_gemm_conv2d_dgrad)
    sconv = hbfp.Conv2d(128, 56, 56, 64, 3, 3, 1, 1, 2, 2, 0, 0)
    Ws = Wd[:, :64].contiguous()
    ti, tf = hbfp.alloc(row, 100352, 128, 1), hbfp.encode(Ws, 0, col)
    out = torch.empty((128 * 56 * 56, 64), dtype=torch.float32, device="cuda")
    wsc = torch.empty(hbfp.gemm_conv2d_dgrad_workspace(ti.desc, sconv, tf.desc), dtype=torch.uint8, device="cuda")

    def strided_dgrad():
        hbfp.encode(d2, 1, row, out=ti)
        hbfp.encode(Ws, 0, col, out=tf)
        hbfp.gemm_conv2d_dgrad(ti, sconv, tf, out=out, workspace=wsc)

    ms_all = _time_call(torch, strided_dgrad, reps)
    ms_k = _time_call(torch, lambda: hbfp.gemm_conv2d_dgrad(ti, sconv, tf, out=out, workspace=wsc), reps)
    sflops = 2.0 * 100352 * 9 * 64 * 128
    res["strided_dgrad_conv2d_gather_in_the_product"] = {
        "gemm_ms": round(ms_k, 4), "whole_data_gradient_ms": round(ms_all, 4), "TOPS_kernel": round(sflops / ms_k / 1e9, 1),
        "TOPS_incl_encode": round(sflops / ms_all / 1e9, 1),
        "note": "dX 401408 x 64 (103 MB) from the 51 MB gradient tensor; 64 output channels fill half of a 128-column tile (the waves of the other half only copy)"}
    del ti, tf, out, wsc, img, Wd, Ws, dimg
    del X, W, dY
    # config 5: 8192^3, 12-bit mantissas, blocks of 64, stochastic rounding (the library's choice of kernel: FP16 planes
    # relative to the rows' largest exponents, packed inside the call, on the 256 x 256-tile kernel)
    Ah, Bh = synth.c5_wide_range()
    A, B = torch.from_numpy(Ah).cuda(), torch.from_numpy(Bh).cuda()
    fa, fb = hbfp.make_format(12, 1, 64, hbfp.STOCHASTIC, 51), hbfp.make_format(12, 64, 1, hbfp.STOCHASTIC, 52)
    ta, tb = hbfp.alloc(fa, 8192, 8192, 1), hbfp.alloc(fb, 8192, 8192, 0)
    out = torch.empty((8192, 8192), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(hbfp.gemm_workspace(ta.desc, tb.desc), 256), dtype=torch.uint8, device="cuda")
    hbfp.encode(A, 1, fa, out=ta)
    hbfp.encode(B, 0, fb, out=tb)
    flops = 2.0 * 8192 ** 3
    ms_k = _time_call(torch, lambda: hbfp.gemm(ta, tb, out=out, workspace=ws), 5)
    ms_ea = _time_call(torch, lambda: hbfp.encode(A, 1, fa, out=ta), 5)
    ms_eb = _time_call(torch, lambda: hbfp.encode(B, 0, fb, out=tb), 5)
    res["c5_bfp12"] = {"gemm_ms": round(ms_k, 4), "encode_a_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4),
                       "TOPS_kernel": round(flops / ms_k / 1e9, 1),
                       "TOPS_incl_encode": round(flops / (ms_k + ms_ea + ms_eb) / 1e9, 1)}
    return res


def _time_product(torch, hbfp, sa, axa, fa, sb, axb, fb, reps):
    """One product with both of its conversions (workspaces allocated outside the timed calls)."""
    ta, tb = hbfp.alloc(fa, sa.shape[0], sa.shape[1], axa), hbfp.alloc(fb, sb.shape[0], sb.shape[1], axb)
    out = torch.empty((ta.desc.rows, tb.desc.rows), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(hbfp.gemm_workspace(ta.desc, tb.desc), 256), dtype=torch.uint8, device="cuda")
    wa = torch.empty(max(hbfp.encode_workspace(ta.desc), 256), dtype=torch.uint8, device="cuda")
    wb = torch.empty(max(hbfp.encode_workspace(tb.desc), 256), dtype=torch.uint8, device="cuda")
    hbfp.encode(sa, axa, fa, out=ta, workspace=wa)
    hbfp.encode(sb, axb, fb, out=tb, workspace=wb)
    flops = 2.0 * ta.desc.rows * tb.desc.rows * ta.desc.kdim
    ms_k = _time_call(torch, lambda: hbfp.gemm(ta, tb, out=out, workspace=ws), reps)
    ms_ea = _time_call(torch, lambda: hbfp.encode(sa, axa, fa, out=ta, workspace=wa), reps)
    ms_eb = _time_call(torch, lambda: hbfp.encode(sb, axb, fb, out=tb, workspace=wb), reps)
    return {"gemm_ms": round(ms_k, 4), "encode_a_ms": round(ms_ea, 4), "encode_b_ms": round(ms_eb, 4),
            "TOPS_kernel": round(flops / ms_k / 1e9, 1), "TOPS_incl_encode": round(flops / (ms_k + ms_ea + ms_eb) / 1e9, 1)}


def _paper_formats(torch, hbfp, reps=8):
    """Two more workloads of the paper, with synthetic N(0,1) activations and N(0, 0.02) weights:
    (1) config 4's layer in the format of the paper's own experiments (Sec. 5.1): one exponent per training input
        for activations and gradients, 24 x 24 weight tiles (hbfp_format.k_slot = 24 stores the activations in
        blocks that match the tiles);
    (2) the gate products of an LSTM language model (Sec. 5.2 evaluates one on PTB): 35 steps x batch 20 = 700 rows,
        hidden size 1500, four gates, in config 4's formats."""
    res = {}
    g = torch.Generator(device="cuda").manual_seed(11)
    n = 4096
    X = torch.randn((n, n), device="cuda", generator=g)
    W = torch.randn((n, n), device="cuda", generator=g) * 0.02
    act, tile = hbfp.make_format(8, 1, 0, k_slot=24), hbfp.make_format(8, 24, 24)
    res["c4_row_exponent_x_24x24_tiles_fwd"] = _time_product(torch, hbfp, X, 1, act, W, 0, tile, reps)
    res["c4_row_exponent_x_24x24_tiles_dgrad"] = _time_product(torch, hbfp, X, 1, act, W, 1, tile, reps)
    del X, W
    M, H = 700, 1500
    Xl = torch.randn((M, H), device="cuda", generator=g)
    Wl = torch.randn((H, 4 * H), device="cuda", generator=g) * 0.02
    dG = torch.randn((M, 4 * H), device="cuda", generator=g)
    row, col = hbfp.make_format(8, 1, 24), hbfp.make_format(8, 24, 1)
    res["lstm_gates_fwd"] = _time_product(torch, hbfp, Xl, 1, row, Wl, 0, tile, reps)
    res["lstm_gates_dgrad"] = _time_product(torch, hbfp, dG, 1, row, Wl, 1, tile, reps)
    res["lstm_gates_wgrad"] = _time_product(torch, hbfp, Xl, 0, col, dG, 0, col, reps)
    return {"paper_formats": res}


def _batched_products(torch, hbfp, reps=10):
    """hbfp_gemm_batch: four independent products of 2048 x 2048 x 4096 in config 4's formats (64 output tiles of
    256 x 256 each).  One call shares a launch of the block-scaled kernel among them; the same products one after
    the other go to the int8 kernels."""
    g = torch.Generator(device="cuda").manual_seed(12)
    row, tile = hbfp.make_format(8, 1, 24), hbfp.make_format(8, 24, 24)
    pairs, outs = [], []
    for _ in range(4):
        X = torch.randn((2048, 4096), device="cuda", generator=g)
        W = torch.randn((4096, 2048), device="cuda", generator=g) * 0.02
        pairs.append((hbfp.encode(X, 1, row), hbfp.encode(W, 0, tile)))
        outs.append(torch.empty((2048, 2048), dtype=torch.float32, device="cuda"))
    ws_one = [torch.empty(max(hbfp.gemm_workspace(a.desc, b.desc), 256), dtype=torch.uint8, device="cuda") for a, b in pairs]
    ws_all = torch.empty(max(hbfp.gemm_batch_workspace(pairs), 256), dtype=torch.uint8, device="cuda")

    def one_by_one():
        for i, (a, b) in enumerate(pairs):
            hbfp.gemm(a, b, out=outs[i], workspace=ws_one[i])

    ms_seq = _time_call(torch, one_by_one, reps)
    ms_bat = _time_call(torch, lambda: hbfp.gemm_batch(pairs, outs, workspace=ws_all), reps)
    flops = 4 * 2.0 * 2048 * 2048 * 4096
    return {"batch_4x_2048x2048x4096": {"one_by_one_ms": round(ms_seq, 4), "one_call_ms": round(ms_bat, 4),
                                        "TOPS_one_by_one": round(flops / ms_seq / 1e9, 1),
                                        "TOPS_one_call": round(flops / ms_bat / 1e9, 1)}}


def _encoded_output(torch, hbfp, reps=10):
    """hbfp_gemm_bfp: a 4096^3 product (activations in 1 x 32 blocks, weights in 32 x 32 tiles) delivered as the next
    product's operand (ReLU, 1 x 32 blocks, stochastic rounding), against hbfp_gemm followed by hbfp_encode."""
    g = torch.Generator(device="cuda").manual_seed(13)
    n = 4096
    X = torch.randn((n, n), device="cuda", generator=g)
    W = torch.randn((n, n), device="cuda", generator=g) * 0.02
    tx, tw = hbfp.encode(X, 1, hbfp.make_format(8, 1, 32)), hbfp.encode(W, 0, hbfp.make_format(8, 32, 32))
    del X, W
    res = {}
    for tag, rounding in (("rne", hbfp.RNE), ("sr", hbfp.STOCHASTIC)):
        fmt = hbfp.make_format(8, 1, 32, rounding, 5)
        out = hbfp.alloc(fmt, n, n, 1)
        C = torch.empty((n, n), dtype=torch.float32, device="cuda")
        ws = torch.empty(hbfp.gemm_workspace(tx.desc, tw.desc), dtype=torch.uint8, device="cuda")
        wsb = torch.empty(hbfp.gemm_bfp_workspace(tx.desc, tw.desc, out.desc), dtype=torch.uint8, device="cuda")

        def two_calls():
            hbfp.gemm(tx, tw, out=C, workspace=ws)
            C.clamp_(min=0)                                   # the ReLU as a pass of its own over the FP32 product
            hbfp.encode(C, 1, fmt, out=out)

        ms2 = _time_call(torch, two_calls, reps)
        ms1 = _time_call(torch, lambda: hbfp.gemm_bfp(tx, tw, fmt, 1, relu=True, out=out, workspace=wsb), reps)
        res[tag] = {"gemm_relu_encode_ms": round(ms2, 4), "gemm_bfp_ms": round(ms1, 4)}
    return {"encoded_output_4096_cubed": res}


def _kernel_families(torch, hbfp, reps=8):
    """The ways the library evaluates the product, side by side on square products with N(0,1) operands:
    int8 matrix instructions + FP32 scaling on the vector unit against the block-scaled matrix instruction, for 6..9-bit
    mantissas the bf16 matrix instruction on bf16 planes, and for 12-bit mantissas the FP16 matrix instruction on mantissas
    widened to FP16, with per-block scaling or on planes relative to the rows' largest exponents (hbfp_gemm_select).  Times are whole calls (packing / scale-word kernels included).  Block length 0 is one
    exponent per row of A and per column of B (Sec. 4), where the int8 family runs its 256 x 256-tile kernel
    (one chain of matrix instructions, exponents applied at the store)."""
    res = {}
    g = torch.Generator(device="cuda").manual_seed(7)
    for name, n, m, blk in (("4096_bfp8_b32", 4096, 8, 32), ("8192_bfp8_b32", 8192, 8, 32), ("4096_bfp8_b24", 4096, 8, 24),
                            ("4096_bfp4_b32", 4096, 4, 32), ("8192_bfp12_b64", 8192, 12, 64),
                            ("4096_bfp8_one_exponent_per_row", 4096, 8, 0), ("8192_bfp8_one_exponent_per_row", 8192, 8, 0)):
        A = torch.randn((n, n), device="cuda", generator=g)
        B = torch.randn((n, n), device="cuda", generator=g)
        fa, fb = hbfp.make_format(m, 1, blk), hbfp.make_format(m, blk, 1)
        ta, tb = hbfp.encode(A, 1, fa), hbfp.encode(B, 0, fb)
        entry = {}
        for tag, src, ax, fmt, t in (("encode_a_ms", A, 1, fa, ta), ("encode_b_ms", B, 0, fb, tb)):
            wse = torch.empty(max(hbfp.encode_workspace(t.desc), 256), dtype=torch.uint8, device="cuda")
            entry[tag] = round(_time_call(torch, lambda: hbfp.encode(src, ax, fmt, out=t, workspace=wse), reps), 4)
            del wse
        del A, B
        out = torch.empty((n, n), dtype=torch.float32, device="cuda")
        families = [("int8", hbfp.KERNEL_INT8), ("scaled", hbfp.KERNEL_SCALED)] + \
                   ([("fp16", hbfp.KERNEL_FP16), ("fp16_planes", hbfp.KERNEL_FP16_PLANES)] if m > 8 else []) + \
                   ([("bf16", hbfp.KERNEL_BF16)] if 6 <= m <= 9 else [])
        for tag, kernel in families:
            ws = torch.empty(max(hbfp.gemm_select_workspace(ta.desc, tb.desc, kernel), 256), dtype=torch.uint8, device="cuda")
            ms = _time_call(torch, lambda: hbfp.gemm(ta, tb, out=out, workspace=ws, kernel=kernel), reps)
            entry[tag + "_ms"] = round(ms, 4)
            entry[tag + "_TOPS"] = round(2.0 * n ** 3 / ms / 1e9, 1)
            del ws
        auto = hbfp.gemm_workspace(ta.desc, tb.desc)           # the choice shows in the workspace it asks for
        entry["automatic_choice"] = next((tag for tag, kernel in reversed(families)
                                          if auto == hbfp.gemm_select_workspace(ta.desc, tb.desc, kernel)), "int8")
        best = min(entry[tag + "_ms"] for tag, _ in families)
        entry["best_TOPS_incl_encode"] = round(2.0 * n ** 3 / (best + entry["encode_a_ms"] + entry["encode_b_ms"]) / 1e9, 1)
        res[name] = entry
        del ta, tb, out
    return {"kernel_families": res}


def _heavy_tails(torch, hbfp, reps=10):
    """A 4096^3 product of config 4's formats whose activation operand is heavy-tailed (Student-t, 3 degrees of freedom).
    8-bit mantissas are packed as bf16 numbers, which take any spread of block exponents: the operand is not marked and
    the product runs as fast as any other (the block-scaled limb packing used to hand such operands to the int8 kernels;
    HBFP_HINT_HEAVY_TAILS, which chooses the faster of those as the stand-by, matters for 4-bit mantissas only);
    hbfp_gemm_select with HBFP_KERNEL_INT8 for comparison."""
    n = 4096
    g = torch.Generator(device="cuda").manual_seed(11)
    z = torch.randn((n, n), device="cuda", generator=g)
    chi = (torch.randn((3, n, n), device="cuda", generator=g) ** 2).sum(0) / 3.0
    X = z / chi.sqrt()
    W = torch.randn((n, n), device="cuda", generator=g) * 0.02
    del z, chi
    x, w = hbfp.alloc(hbfp.make_format(8, 1, 24), n, n, 1), hbfp.alloc(hbfp.make_format(8, 24, 24), n, n, 0)
    px, pw = (torch.empty(hbfp.pack_bytes(t.desc), dtype=torch.uint8, device="cuda") for t in (x, w))
    hbfp.encode_packed(X, [x], [px])
    hbfp.encode_packed(W, [w], [pw])
    out = torch.empty((n, n), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(hbfp.gemm_packed_workspace(x.desc, w.desc), hbfp.gemm_select_workspace(x.desc, w.desc, hbfp.KERNEL_INT8), 256),
                     dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    mark = px[:8].view(torch.int32).tolist()
    res = {"operand_marked": mark[0] == mark[1]}
    res["gemm_packed_ms"] = round(_time_call(torch, lambda: hbfp.gemm_packed(x, px, w, pw, out=out, workspace=ws), reps), 4)
    x.desc.hints = hbfp.HINT_HEAVY_TAILS
    res["gemm_packed_with_hint_ms"] = round(_time_call(torch, lambda: hbfp.gemm_packed(x, px, w, pw, out=out, workspace=ws), reps), 4)
    x.desc.hints = 0
    res["gemm_select_int8_ms"] = round(_time_call(torch, lambda: hbfp.gemm(x, w, out=out, workspace=ws, kernel=hbfp.KERNEL_INT8), reps), 4)
    return {"c4_product_with_heavy_tailed_activations": res}


def _matrix_probe(torch, hbfp, iters=3000):
    """What the matrix core sustains on this machine: register-only loops (hbfp_probe_matrix_rate) of the int8 and of the
    block-scaled FP6 matrix instruction at 1 and 2 workgroups of 4 waves per compute unit, with constant and with
    random operand bits; the shader clock is the cycle counter against the 100 MHz wall clock inside the kernel."""
    res = {}
    sink = torch.empty(1024 * 256, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(2, dtype=torch.int64, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(1)
    operands = {"constant_bits": torch.full((64 * 64,), 0x01010101, dtype=torch.int32, device="cuda"),
                "random_bits": torch.randint(-2 ** 31, 2 ** 31 - 1, (64 * 64,), dtype=torch.int64, device="cuda", generator=g).to(torch.int32)}
    # bf16 operands: integers -127..127 times a power of two from 8 binades, as the packed operands of the product hold them
    vals = torch.randint(-127, 128, (2 * 64 * 64,), device="cuda", generator=g).float() * torch.exp2(torch.randint(-4, 4, (2 * 64 * 64,), device="cuda", generator=g).float())
    bf_words = vals.to(torch.bfloat16).view(torch.int32)
    for name, instr, flop in (("int8_32x32x32", 0, 2.0 * 32 * 32 * 32), ("scaled_fp6_32x32x64", 1, 2.0 * 32 * 32 * 64),
                              ("bf16_32x32x16", 2, 2.0 * 32 * 32 * 16)):
        for tag, words in (operands.items() if instr != 2 else (("mantissas_times_powers_of_two", bf_words),)):
            best = None
            for wgs in (512, 1024):
                hbfp.probe_matrix_rate(instr, words, wgs, 100, sink, clocks)
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                hbfp.probe_matrix_rate(instr, words, wgs, iters, sink, clocks)
                b.record()
                torch.cuda.synchronize()
                ms = a.elapsed_time(b)
                c = clocks.cpu().tolist()
                rate = wgs * 4 * iters * 16 * flop / ms / 1e9
                if best is None or rate > best["T_per_s"]:
                    best = {"T_per_s": round(rate, 1), "shader_clock_GHz": round(c[0] / max(c[1], 1) * 0.1, 3), "waves_per_simd": wgs // 512,
                            "ms": round(ms, 3)}
            res[f"{name}_{tag}"] = best
    res["note"] = ("T_per_s: tera-operations per second of the loop (int8: TOP/s, FP6 and bf16: TFLOP/s), best of 1 and 2 waves per SIMD; "
                   "the published peaks are 5000, 10100 and 2500")
    return res


def _cpu_baseline(synth):
    """The oracle as it stands on the host cores: one whole step of config 4 (forward, data gradient and
    weight gradient: six encodes, FP64 products of the dequantised operands)."""
    import numpy as np
    from oracle import ref
    M = K = N = 4096
    Xh, Wh, dYh = synth.c4_linear(M, K, N)
    WT, XT = np.ascontiguousarray(Wh.T), np.ascontiguousarray(Xh.T)
    t0 = time.perf_counter()
    reps = 0
    while reps == 0 or time.perf_counter() - t0 < 10.0:          # whole steps until at least 10 s of work
        ref.gemm(ref.decode(ref.encode(Xh, 1, 24, 8)), ref.decode(ref.encode(Wh, 24, 24, 8)))
        ref.gemm(ref.decode(ref.encode(dYh, 1, 24, 8)), ref.decode(ref.encode(WT, 24, 24, 8)))
        ref.gemm(ref.decode(ref.encode(XT, 1, 24, 8)), ref.decode(ref.encode(dYh, 24, 1, 8)))
        reps += 1
    dt = time.perf_counter() - t0
    return {"value": round(reps * 3 * 2.0 * M * N * K / dt / 1e12, 5), "unit": "TOP/s", "cores": ref.num_threads(),
            "kind": "oracle",
            "sample": f"{reps} full step(s) of config 4 (three 4096^3 products with their six encodes each), {dt:.1f} s"}


def main():
    args = _parse()
    if args.gpus != 1:
        print(f"bench.py measures one GPU; --gpus {args.gpus} is not supported (this build has no multi-GPU path)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import synth
    import __graft_entry__
    __graft_entry__.ensure_built()
    from paper_1804_01526_amd import hbfp

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    step, flops_step, flops_product, shape, outs = _linear_layer(torch, hbfp, synth)
    # No cyclic garbage collection while launches are being timed (what timeit does): with torch and numpy loaded a
    # full collection stops the launching thread for 35-50 ms, 70 steps' worth, at a moment that depends on how many
    # objects the interpreter happened to allocate before.  Reference counting still frees everything the steps create.
    gc.collect()
    gc.disable()
    # the first steps after idle, timed for the record (the power management has not settled: by the kernel trace the
    # product kernel takes 126 us at first, 141-146 us for a few steps, then falls to 122 us), then the rest of the
    # untimed steps
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    c_begin, c_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_from_idle = max(0, min(20, args.preheat - 3))
    c_begin.record()
    for _ in range(n_from_idle):
        step()
    c_end.record()
    for _ in range(max(0, args.preheat - 3 - n_from_idle) + args.warmup):
        step()
    torch.cuda.synchronize()
    ms_from_idle = c_begin.elapsed_time(c_end) / n_from_idle if n_from_idle else None
    run_step = step
    if args.graph:
        # one HIP graph of the launches of a step (no memset nodes: the library clears nothing with
        # hipMemsetAsync on this path); replayed outputs are checked against the eager ones below
        eager = [o.clone() for o in outs]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = graph.replay
        for _ in range(2):
            for o in outs:
                o.zero_()
            run_step()
            torch.cuda.synchronize()
            assert all(torch.equal(o, e) for o, e in zip(outs, eager)), "graph replay differs from the eager step"
    t_begin, t_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_begin.record()
    for _ in range(args.steps):
        run_step()
    t_end.record()
    torch.cuda.synchronize()
    # the same steps again with HIP events around every call, for the per-kernel figures
    timer = Timer(torch)
    n_bracketed = min(args.steps, 100)
    for _ in range(n_bracketed):
        step(timer)
    torch.cuda.synchronize()
    ms_step = t_begin.elapsed_time(t_end) / args.steps
    tops = flops_step / ms_step / 1e9
    # ... and with the weights already converted (the middle one of the three ways to count: product kernels alone,
    # plus the conversions of the FP32-resident operands, plus all conversions)
    r_begin, r_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        step.weights_resident()
    r_begin.record()
    for _ in range(n_bracketed):
        step.weights_resident()
    r_end.record()
    torch.cuda.synchronize()
    ms_step_resident = r_begin.elapsed_time(r_end) / n_bracketed

    # one hbfp_gemm_packed call = one launch of the bf16 product kernel
    product_ms = timer.total_ms("gemm") / timer.count("gemm")
    product_tops = flops_product / product_ms / 1e9
    enc_xw_ms = timer.total_ms("encode_x_w") / n_bracketed
    enc_dy_ms = timer.total_ms("encode_act") / n_bracketed
    pair_ms = timer.total_ms("gemm_pair") / timer.count("gemm_pair")
    gemm_step_ms = (timer.total_ms("gemm") + timer.total_ms("gemm_pair")) / n_bracketed

    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    out = {
        "metric": "BFP8 GEMM effective TOPS incl. encode (% int8 MFMA peak); encode GB/s",
        "value": round(tops, 2), "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16",
        "dtype_note": "8-bit mantissas times their block's power of two are exact bf16 numbers: bf16 matrix instruction, FP32 accumulate; "
                      "the conversions compute in integer arithmetic on the FP32 bit patterns",
        "data": "synthetic",
        "config": {"workload": "config 4: dense layer M=K=N=4096, BFP8, 1x24 activation blocks, 24x24 weight tiles, "
                               "forward + data gradient + weight gradient, all six operand encodes included (2 conversion calls: input and weights in one launch, then the "
                               "output gradient; 3 products: "
                               "the forward one alone, the two backward ones in one launch)", "preheat_steps": args.preheat, **shape},
        "pct_int8_peak": round(100.0 * tops / INT8_PEAK_TOPS, 2),
        "ms_per_step_first_steps_after_idle": None if ms_from_idle is None else round(ms_from_idle, 4),
        "breakdown_ms_per_step": {"gemm_x3": round(gemm_step_ms, 4), "encode_input_and_weights_x4": round(enc_xw_ms, 4),
                                  "encode_output_gradient_x2": round(enc_dy_ms, 4)},
        "TOPS_kernel_only": round(flops_step / gemm_step_ms / 1e9, 2),
        "TOPS_incl_activation_and_gradient_encodes": round(flops_step / ms_step_resident / 1e9, 2),
        "ms_per_step_weights_already_converted": round(ms_step_resident, 4),
        # Roofline of the dominant kernel against the peak the metric names: effective operations 2*M*N*K, counted once
        # per mantissa product, over the product kernel's launch time, against the published dense int8 matrix peak.
        # The kernel reaches them on the bf16 matrix instruction (one multiply-add per mantissa pair), whose own
        # published peak is half the int8 one: own_dtype holds the same rate against that.
        "roofline": {"bound": "mfma", "kernel": "gemm_bf_kernel<false, false>", "achieved": round(product_tops, 1),
                     "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": round(product_tops / INT8_PEAK_TOPS, 4),
                     "own_dtype": {"dtype": "bf16", "achieved": round(product_tops, 1), "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": round(product_tops / BF16_PEAK_TFLOPS, 4),
                                   "note": "v_mfma_f32_32x32x16_bf16: the peak of the instruction the kernel issues"},
                     "traffic": TRAFFIC_GEMM_C4_BYTES, "traffic_unit": "bytes per launch (HBM, rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)",
                     "algorithmic_bytes": ALG_BYTES_GEMM_C4, "avg_launch_ms": round(product_ms, 4),
                     "algorithmic_ops_per_launch": flops_product, "backward_pair_launch_ms": round(pair_ms, 4),
                     "note": "avg_launch_ms is the HIP-event time of the hbfp_gemm_packed call of the step (the forward product) on the "
                             "launch stream: one launch of the product kernel (grid 256 workgroups of 512 threads; the bracket holds 3 to 4 us of "
                             "dispatch latency on top of the kernel duration that rocprofv3 lists); "
                             "backward_pair_launch_ms is the hbfp_gemm_packed_batch call: the same kernel over both backward "
                             "products (grid 512); the operands were packed by the conversion calls; the rocprofv3 summary lists "
                             "each kernel"},
    }
    if not args.no_probe:
        out["roofline"]["matrix_probe"] = _matrix_probe(torch, hbfp)
    if not args.no_extra:
        extra = _encode_config2(torch, hbfp, synth)
        e = extra["encode_m8_rne"]
        out["encode_GBps"] = e["GBps"]
        out["roofline_encode"] = {"bound": "hbm", "kernel": "enc_row_kernel (config 2, m=8, RNE)", "achieved": e["GBps"],
                                  "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(e["GBps"] / HBM_PEAK_GBPS, 4),
                                  "traffic": TRAFFIC_ENCODE_C2_M8_BYTES, "traffic_unit": "bytes per launch (HBM, measured)",
                                  "algorithmic_bytes": e["bytes"], "avg_launch_ms": e["ms"]}
        for section in (lambda: _gemm_side_configs(torch, hbfp, synth), lambda: _weight_update_config4(torch, hbfp, synth),
                        lambda: _kernel_families(torch, hbfp), lambda: _paper_formats(torch, hbfp),
                        lambda: _batched_products(torch, hbfp), lambda: _encoded_output(torch, hbfp),
                        lambda: _heavy_tails(torch, hbfp)):
            gc.collect()                     # between the sections, not inside their timed loops
            extra.update(section())
        out["extra"] = extra
    gc.enable()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(synth)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
