#!/usr/bin/env python3
"""Benchmark of the 4/6 NVFP4 hot path on one MI355X.

One step = one pass of the whole path over one 8192x8192 BF16 weight-like tensor
(workload c2): tensor scale (Eq. 1) -> 4/6 rowwise quantize, round to nearest
(Eq. 2-3, Table 3) -> dequantize.  Inputs are resident in HBM before the timed
region.  Steps rotate over several independent buffer sets so that no step finds
its input in the 256 MB memory-side cache left there by the previous step.

Prints ONE JSON line (see the keys below).  `roofline` describes the dominant
kernel, the rowwise quantize: algorithmic bytes (2 B read + 0.5 B codes + 1/16 B
scale per element) over its average duration measured with events on the launch
stream inside the timed region.  `cpu_baseline` is the CPU oracle on the same
tensor on the host's cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2512_02010_amd import binding as B  # noqa: E402
from paper_2512_02010_amd import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0
# fp32 vector rate of the chip in lane-operations/s: 157.3 TFLOP/s counts a fused
# multiply-add as two, i.e. 256 CUs x 128 lanes x 2.4 GHz.  Measured issue rates
# (profiles/valu_issue_rates.txt): the plain (unpacked) v_fma/v_mul/v_add and the two-operand
# logic operations do issue at about this rate (a wave's instruction in two passes) while
# conversions, comparisons, selects, min/max, integer multiplies, three-operand integer
# operations and any fp32 instruction with a scalar-register source take four passes, the
# FP4/FP8 packing conversions eight and the stochastic-rounding FP4 conversion twelve.
VALU_PEAK_TOPS = 256 * 128 * 2.4e9 / 1e12
# VALU wave-instructions per block of 16 elements in the rowwise 4/6 kernel, from
# rocprofv3 --pmc SQ_INSTS_VALU (profiles/c2_step_counters.txt): 14,730,144 per 4,194,304/64 wave-blocks
VALU_INSTS_PER_BLOCK_46 = 14730144.0 / (4194304.0 / 64.0)
# the same for the kernels of c4 (both orientations, per 16 elements;
# profiles/c4_both_and_fake_quant_counters.txt) and c5 (Hadamard + stochastic rounding;
# profiles/c5_rowwise_rht_sr_counters.txt)
VALU_INSTS_PER_BLOCK_C4 = 31557668.0 / (4194304.0 / 64.0)
VALU_INSTS_PER_BLOCK_C5 = 46169804.0 / (4194304.0 / 64.0)
# HBM bytes per element of the same kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled
# by a plain copy's readings (same file): (65665.8 * 2.000 + 36891.5 * 1.000) KiB per 67,108,864
HBM_TRAFFIC_PER_ELEM_46 = (65665.8 * 2.0 + 36891.5) * 1024.0 / 67108864.0
BYTES_PER_ELEM_QUANT = 2.0 + 0.5 + 1.0 / 16.0        # read x, write codes, write scales
BYTES_PER_ELEM_AMAX = 2.0
BYTES_PER_ELEM_DEQUANT = 0.5 + 1.0 / 16.0 + 2.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--rows", type=int, default=8192)
    ap.add_argument("--cols", type=int, default=8192)
    ap.add_argument("--buffers", type=int, default=4, help="independent buffer sets rotated over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gemm", action="store_true",
                    help="skip the consumer-side leg (NVFP4 x NVFP4 matrix product, 8192^3)")
    ap.add_argument("--other-workloads", action="store_true",
                    help="also time the c3 (fake-quant), c4 (both orientations) and c5 "
                         "(Hadamard + stochastic rounding) steps at their full sizes and add "
                         "them to the JSON line as `other_workloads`")
    ap.add_argument("--counter-pass", action="store_true",
                    help="launch a calibration copy and each kernel of the step a few times and "
                         "exit (for `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE -- python3 bench.py "
                         "--counter-pass`); prints no benchmark line")
    ap.add_argument("--counter-pass-gemm", nargs="?", const=8192, type=int, default=None, metavar="M",
                    help="launch nvfp4_46_gemm (M x 8192 x 8192, M = 8192 unless given; random "
                         "codes, scale bytes 0x30..0x47; eight rotating weight operands) sixteen "
                         "times (four when M = 8192) and exit (for `rocprofv3 --pmc ... -- python3 "
                         "bench.py --counter-pass-gemm [M]`); prints no benchmark line")
    ap.add_argument("--layer-pass", action="store_true",
                    help="run five steps of the Fig. 3 linear layer (8192 tokens, 8192 -> 8192) and "
                         "exit (for `rocprofv3 --kernel-trace --stats -- python3 bench.py "
                         "--layer-pass`); prints no benchmark line")
    return ap.parse_args()


class HipEvents:
    """Timing events of the HIP runtime itself, recorded on a given stream.

    They are created with hipEventDisableSystemFence: the event's completion then carries
    no system-scope cache flush, which an event made through torch adds to the interval it
    closes (about 2-4 us per event on this kernel, against a 30 us dispatch)."""
    DISABLE_SYSTEM_FENCE = 0x20000000

    def __init__(self):
        import ctypes as C
        self.C = C
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def _check(self, rc, what):
        if rc != 0:
            raise RuntimeError(f"{what} failed with HIP error {rc}")

    def new(self):
        e = self.C.c_void_p()
        self._check(self.hip.hipEventCreateWithFlags(self.C.byref(e), self.DISABLE_SYSTEM_FENCE),
                    "hipEventCreateWithFlags")
        return e

    def record(self, e, stream):
        self._check(self.hip.hipEventRecord(e, self.C.c_void_p(stream.cuda_stream)), "hipEventRecord")

    def elapsed_ms(self, a, b):
        ms = self.C.c_float()
        self._check(self.hip.hipEventElapsedTime(self.C.byref(ms), a, b), "hipEventElapsedTime")
        return ms.value

    def free(self, events):
        for e in events:
            self.hip.hipEventDestroy(e)


_EV = None


def hip_events():
    global _EV
    if _EV is None:
        _EV = HipEvents()
    return _EV


class BufferSet:
    def __init__(self, x_host: torch.Tensor):
        rows, cols = x_host.shape
        self.rows, self.cols = rows, cols
        self.x = x_host.cuda()
        self.alpha = torch.empty(1, dtype=torch.float32, device="cuda")
        self.out = B.alloc_outputs(rows, cols, B.ROWWISE, "cuda", want_choice=False)
        self.deq = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
        self.params = B.make_params(rows, cols)
        self.workspace = B.new_workspace()      # zeroed once; nvfp4_46_tensor_scale_ws keeps it so
        self.stream = torch.cuda.current_stream()


def step(bs: BufferSet, ev=None, quantize_params=None):
    """tensor_scale -> quantize -> dequantize, all on the current stream.  `ev`: two events
    recorded around the quantize call, or four around all three calls.  `quantize_params`
    replaces the 4/6 options of the quantize call (context measurements only)."""
    st = bs.stream
    he = hip_events() if ev else None
    every = ev is not None and len(ev) == 4
    if every:
        he.record(ev[0], st)
    rc = B.tensor_scale_ws_raw(bs.x, bs.params, bs.alpha, bs.workspace, B.TENSOR_SCALE_WS_BYTES, st)
    if ev:
        he.record(ev[1] if every else ev[0], st)
    rc |= B.quantize_raw(bs.x, quantize_params or bs.params, bs.alpha, bs.out["codes_row"],
                         bs.out["scales_row"], None, None, None, None, st)
    if ev:
        he.record(ev[2] if every else ev[1], st)
    rc |= B.dequantize_raw(bs.out["codes_row"], bs.out["scales_row"], bs.alpha, bs.rows, bs.cols,
                           B.ROWWISE, bs.deq, st)
    if every:
        he.record(ev[3], st)
    if rc:
        raise RuntimeError(f"library call failed with status {rc}")


def time_single(fn, sets, iters):
    """Average duration (ms) of one library call, rotating over the buffer sets."""
    for i in range(4):
        fn(sets[i % len(sets)])
    he, st = hip_events(), torch.cuda.current_stream()
    evs = [(he.new(), he.new()) for _ in range(iters)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(evs):
        he.record(a, st)
        fn(sets[i % len(sets)])
        he.record(b, st)
    torch.cuda.synchronize()
    ts = sorted(he.elapsed_ms(a, b) for a, b in evs)
    for pair in evs:
        he.free(pair)
    return sum(ts) / len(ts), ts[len(ts) // 2], ts[0]


def cpu_baseline(x_host):
    """The CPU oracle on the host's cores: full passes over the same tensor for about ten
    seconds with all threads, then one pass over a slice of rows on a single thread."""
    import ctypes as C
    from oracle import ref
    xb = wl.bf16_bits(x_host)
    rows, cols = xb.shape
    ref.lib()

    def one_pass(bits):
        alpha = ref.tensor_scale(bits)
        codes, scales, _ = ref.quantize(bits, alpha)
        ref.dequantize(codes, scales, alpha, bits.shape[0], bits.shape[1])

    t0 = time.perf_counter()
    reps = 0
    while True:
        one_pass(xb)
        reps += 1
        dt = time.perf_counter() - t0
        if dt > 10.0 or reps >= 100:      # about ten seconds of host work
            break
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    out = {"value": rows * cols * reps / dt / 1e9, "unit": "G elem/s", "cores": cores,
           "kind": "oracle",
           "sample": f"{reps} full passes (tensor scale + quantize + dequantize) over the same "
                     f"{rows}x{cols} tensor in {dt:.1f} s, OpenMP over rows"}
    try:
        omp = C.CDLL("libgomp.so.1")
        omp.omp_set_num_threads(1)
        srows = min(rows, 1024)
        sl = xb[:srows].copy()
        t0 = time.perf_counter()
        one_pass(sl)
        dt1 = time.perf_counter() - t0
        omp.omp_set_num_threads(cores)
        out["single_thread"] = {"value": srows * cols / dt1 / 1e9, "unit": "G elem/s",
                                "sample": f"one pass over the first {srows} rows in {dt1:.1f} s"}
    except OSError:
        pass
    return out


MFMA_F16_PEAK_TFLOPS = 2500.0
# HBM-side bytes of one 8192^3 product from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (profiles/gemm_8192_counters.txt): (221,602.7 KiB x 2.000 + 131,120.0 KiB x 1.000)
GEMM_8192_TRAFFIC_BYTES = (221602.7 * 2.0 + 131120.0) * 1024.0


def time_gemm(w_host, iters=20):
    """The consumer of the quantizer's output (Fig. 3, FPROP): y = x W^T with x a c3-like
    activation batch [8192][8192] and W the c2 weight matrix, both quantized rowwise (along
    the contraction axis) by this library, multiplied by nvfp4_46_gemm into BF16.  For
    context the same product of the dequantized FP16 operands by the vendor library
    (torch.matmul): what the matrix units sustain here without any operand expansion."""
    st = torch.cuda.current_stream()
    he = hip_events()
    n, k = w_host.shape
    m = 8192
    ops = []
    for x in (wl.make("c3", m, k).cuda(), w_host.cuda()):
        alpha = B.nvfp4_46_tensor_scale(x)
        o = B.nvfp4_46_quantize(x, alpha, want_choice=False)
        ops += [o["codes_row"], o["scales_row"], alpha]
        del x
    out = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")

    def timed(fn):
        for _ in range(3):
            fn()
        evs = [(he.new(), he.new()) for _ in range(iters)]
        torch.cuda.synchronize()
        for a, b in evs:
            he.record(a, st)
            fn()
            he.record(b, st)
        torch.cuda.synchronize()
        ts = sorted(he.elapsed_ms(a, b) for a, b in evs)
        for pair in evs:
            he.free(pair)
        return sum(ts) / len(ts), ts[len(ts) // 2]

    def ours():
        rc = B.gemm_raw(*ops, m, n, k, B.OUT_BF16, out, st)
        if rc:
            raise RuntimeError(f"nvfp4_46_gemm failed with status {rc}")

    t_avg, t_med = timed(ours)
    one = torch.ones(1, dtype=torch.float32, device="cuda")
    a16 = B.nvfp4_46_dequantize(ops[0], ops[1], one, m, k).to(torch.float16)
    b16 = B.nvfp4_46_dequantize(ops[3], ops[4], one, n, k).to(torch.float16)
    lib_avg, lib_med = timed(lambda: torch.matmul(a16, b16.t(), out=out.view(torch.float16)))
    flops = 2.0 * m * n * k
    return {
        "what": f"{m}x{n}x{k}: c3-like activations x c2 weights, both 4/6-quantized rowwise, "
                "BF16 output",
        "us_avg": t_avg * 1e3, "us_median": t_med * 1e3,
        "roofline": {"bound": "mfma", "kernel": "k_gemm_dma (v_mfma_f32_32x32x16_f16)",
                     "achieved": flops / (t_avg * 1e-3) / 1e12, "peak": MFMA_F16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (t_avg * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS,
                     "traffic": GEMM_8192_TRAFFIC_BYTES if (m, n, k) == (8192, 8192, 8192) else None,
                     "traffic_note": "from rocprofv3 counters at this shape (profiles/"
                                     "gemm_8192_counters.txt), not re-measured in this run"},
        "operand_bytes": (m + n) * (k // 2 + k // 16), "output_bytes": m * n * 2,
        "library_fp16_gemm_on_expanded_operands": {
            "us_median": lib_med * 1e3, "tflops": flops / (lib_avg * 1e-3) / 1e12,
            "note": "torch.matmul on the same operands expanded to FP16 (4x the operand bytes)"},
    }


def time_other_workloads(iters=30):
    """Median event-timed duration of the tensor-scale call and of the main call of
    workloads c3, c4, c5 (full size, two rotating buffer sets each)."""
    import statistics
    res = {}
    st = torch.cuda.current_stream()

    def med(fn):
        for i in range(4):
            fn(i)
        he = hip_events()
        evs = [(he.new(), he.new()) for _ in range(iters)]
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(evs):
            he.record(a, st)
            fn(i)
            he.record(b, st)
        torch.cuda.synchronize()
        m = statistics.median(he.elapsed_ms(a, b) for a, b in evs) * 1e3
        for pair in evs:
            he.free(pair)
        return m

    def entry(n, bpe, t_scale, t_main, what, valu_per_block=None):
        e = {"what": what, "elements": n, "tensor_scale_us": t_scale, "main_us": t_main,
             "main_g_elem_s": n / t_main / 1e3, "main_algorithmic_gb_s": n * bpe / t_main / 1e3,
             "main_frac_of_8tbs": n * bpe / t_main / 1e3 / HBM_PEAK_GBS}
        if valu_per_block is not None:
            # the vector-ALU roof: lane-operations (rocprofv3 SQ_INSTS_VALU per block) / s
            tops = valu_per_block * (n / 16.0) / (t_main * 1e-6) / 1e12
            e["main_alu"] = {"bound": "alu", "achieved": tops, "peak": VALU_PEAK_TOPS,
                             "unit": "T lane-op/s", "frac": tops / VALU_PEAK_TOPS,
                             "valu_insts_per_16_elements": valu_per_block}
        return e

    # variants of the rowwise quantizer on the c2 tensor: the other selection rules, the
    # stochastic-rounding modes, 16x16 tiles
    xs = [wl.make("c2").cuda() for _ in range(2)]
    r, c = xs[0].shape
    alpha = B.nvfp4_46_tensor_scale(xs[0])
    os_ = [B.alloc_outputs(r, c, B.ROWWISE, "cuda", want_choice=False) for _ in range(2)]
    variants = {
        "mse (default)": dict(),
        "always 6 (standard NVFP4)": dict(select=B.SEL_FORCE6),
        "mean absolute error rule": dict(select=B.SEL_46_MAE),
        "largest absolute error rule": dict(select=B.SEL_46_ABSMAX),
        "stochastic rounding": dict(rounding=B.SR, sr_seed=wl.C5_SR_SEED),
        "SR after RTN selection": dict(rounding=B.SR_AFTER_RTN_SELECT, sr_seed=wl.C5_SR_SEED),
        "always 6 + SR": dict(rounding=B.SR, select=B.SEL_FORCE6, sr_seed=wl.C5_SR_SEED),
        "16x16 tiles": dict(block2d=1),
        "16x16 tiles, MAE rule": dict(block2d=1, select=B.SEL_46_MAE),
    }
    res["c2_variants_main_us"] = {}
    for name, kw in variants.items():
        p = B.make_params(r, c, **kw)
        res["c2_variants_main_us"][name] = med(
            lambda i: B.quantize_raw(xs[i % 2], p, alpha, os_[i % 2]["codes_row"],
                                     os_[i % 2]["scales_row"], None, None, None, None, st))
    # 16x16 tiles with the packing for the transposed matrix written in the same pass (what the
    # layer's weight quantization runs): 3.125 B/elem, back-to-back launches
    ob = [B.alloc_outputs(r, c, B.BOTH, "cuda", want_choice=False, block2d=1) for _ in range(2)]
    p = B.make_params(r, c, layout=B.BOTH, block2d=1)
    res["c2_variants_main_us"]["16x16 tiles, both packings"] = med(
        lambda i: B.quantize_raw(xs[i % 2], p, alpha, ob[i % 2]["codes_row"], ob[i % 2]["scales_row"],
                                 ob[i % 2]["codes_col"], ob[i % 2]["scales_col"], None, None, st))
    del ob
    # quantization error of each block-scale rule on the same tensor (what Tables 2 and 4 of the
    # paper measure in perplexity, here as normalised mean squared / mean absolute error)
    xf = xs[0].double()
    ref_sq, ref_abs = float((xf ** 2).mean()), float(xf.abs().mean())
    res["c2_error_by_rule"] = {}
    for name, sel in (("always 6 (standard NVFP4)", B.SEL_FORCE6), ("always 4", B.SEL_FORCE4),
                      ("4/6 by squared error", B.SEL_46_MSE), ("4/6 by absolute error", B.SEL_46_MAE),
                      ("4/6 by largest error", B.SEL_46_ABSMAX)):
        d = B.nvfp4_46_fake_quant(xs[0], alpha, select=sel).double() - xf
        res["c2_error_by_rule"][name] = {"nmse": float((d ** 2).mean()) / ref_sq,
                                         "nmae": float(d.abs().mean()) / ref_abs}
    del xf, d
    del xs, os_
    # c2 held as FP32 master weights (Fig. 3): 4 B read per element
    xh = wl.make("c2", dtype=torch.float32)
    xs = [xh.cuda() for _ in range(2)]
    os_ = [B.alloc_outputs(r, c, B.BOTH, "cuda", want_choice=False) for _ in range(2)]
    p_row = B.make_params(r, c, x_dtype=B.X_F32)
    p_both = B.make_params(r, c, layout=B.BOTH, x_dtype=B.X_F32)
    t_s = med(lambda i: B.tensor_scale_raw(xs[i % 2], p_row, alpha, st))
    t_m = med(lambda i: B.quantize_raw(xs[i % 2], p_row, alpha, os_[i % 2]["codes_row"],
                                       os_[i % 2]["scales_row"], None, None, None, None, st))
    res["c2_fp32_rowwise"] = entry(r * c, 4.0 + 0.5625, t_s, t_m,
                                   "8192x8192 FP32 weights, rowwise RTN 4/6")
    t_m = med(lambda i: B.quantize_raw(xs[i % 2], p_both, alpha, os_[i % 2]["codes_row"],
                                       os_[i % 2]["scales_row"], os_[i % 2]["codes_col"],
                                       os_[i % 2]["scales_col"], None, None, st))
    res["c2_fp32_both"] = entry(r * c, 4.0 + 1.125, t_s, t_m,
                                "8192x8192 FP32 weights, both orientations, RTN 4/6")
    del xs, os_
    # one training step of an 8192 -> 8192 linear layer on 8192 tokens as in Fig. 3: the weight
    # matrix (FP32, 16x16 tiles, both packings), three activations / gradient quantizations in
    # four orientations, three NVFP4 products; against the three BF16 products of the vendor
    # library on the unquantized tensors
    from paper_2512_02010_amd import linear
    xa = wl.make("c3", 8192, 8192).cuda()
    wf = xh.cuda()
    dy = wl.make("c1", 8192, 8192).cuda()

    ws = B.new_workspace()       # the five tensor scales of a step: one launch each

    def layer_step():
        qw = linear.quantize_weight(wf, workspace=ws)
        linear.fprop(xa, qw, workspace=ws)
        linear.dgrad(dy, qw, sr_seed=wl.C5_SR_SEED, workspace=ws)
        linear.wgrad(dy, xa, sr_seed=wl.C5_SR_SEED, rht_seed=wl.C5_RHT_SEED, workspace=ws)

    def wall(fn, n=10):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e6

    wb = wf.to(torch.bfloat16)
    t_layer = wall(layer_step)
    t_bf16 = wall(lambda: (xa @ wb.t(), dy @ wb, dy.t() @ xa))
    res["linear_layer_step"] = {
        "what": "8192 tokens x (8192 -> 8192) linear layer, forward + both backward products "
                "(Fig. 3): 1 weight + 4 activation/gradient quantizations, 3 NVFP4 products",
        "us": t_layer, "tflops": 3 * 2.0 * 8192 ** 3 / t_layer / 1e6,
        "bf16_products_only_us": t_bf16,
        "note": "gfx950 has no NVFP4 matrix instruction (its FP4 MFMA takes E8M0 scales per 32), "
                "so the NVFP4 products run at the FP16 MFMA rate after exact expansion"}
    del xa, wf, dy, wb, xh
    torch.cuda.empty_cache()
    # few rows of A against the 8192 x 8192 weight matrix (a small batch at inference): bound by
    # reading the weights once; rotating weight buffers keep them out of the memory-side cache
    g = torch.Generator(device="cuda")
    g.manual_seed(2)
    u8 = dict(dtype=torch.uint8, device="cuda", generator=g)
    ws = [(torch.randint(0, 256, (8192, 4096), **u8), torch.randint(0x30, 0x48, (8192, 512), **u8))
          for _ in range(8)]
    w16 = [torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16) for _ in range(3)]
    one = torch.ones(1, dtype=torch.float32, device="cuda")
    res["small_batch_products"] = {}
    for m in (1, 16, 64, 128):
        ca, sa = torch.randint(0, 256, (m, 4096), **u8), torch.randint(0x30, 0x48, (m, 512), **u8)
        a16 = torch.randn(m, 8192, device="cuda", dtype=torch.bfloat16)
        o = torch.empty((m, 8192), dtype=torch.bfloat16, device="cuda")
        t_n = med(lambda i: B.gemm_raw(ca, sa, one, ws[i % 8][0], ws[i % 8][1], one, m, 8192, 8192,
                                       B.OUT_BF16, o, st))
        t_l = med(lambda i: torch.matmul(a16, w16[i % 3].t(), out=o))
        wbytes = 8192 * (4096 + 512)
        res["small_batch_products"][f"M={m}"] = {
            "nvfp4_us": t_n, "weight_gb_s": wbytes / t_n / 1e3,
            "frac_of_8tbs": wbytes / t_n / 1e3 / HBM_PEAK_GBS, "library_bf16_us": t_l}
    del ws, w16
    torch.cuda.empty_cache()
    # c3: activation batch, fake-quant round trip in one kernel (2 B read + 2 B written)
    xs = [wl.make("c3").cuda() for _ in range(2)]
    r, c = xs[0].shape
    alpha = torch.empty(1, dtype=torch.float32, device="cuda")
    outs = [torch.empty_like(xs[0]) for _ in range(2)]
    p = B.make_params(r, c)
    t_s = med(lambda i: B.tensor_scale_raw(xs[i % 2], p, alpha, st))
    t_m = med(lambda i: B.fake_quant_raw(xs[i % 2], p, alpha, outs[i % 2], st))
    res["c3"] = entry(r * c, 4.0, t_s, t_m, "16384x4096 fake-quant, rowwise RTN 4/6")
    del xs, outs
    # c4: rowwise + columnwise outputs from one read (2 B read + 1.125 B written)
    xs = [wl.make("c4").cuda() for _ in range(2)]
    r, c = xs[0].shape
    os_ = [B.alloc_outputs(r, c, B.BOTH, "cuda", want_choice=False) for _ in range(2)]
    p = B.make_params(r, c, layout=B.BOTH)
    t_s = med(lambda i: B.tensor_scale_raw(xs[i % 2], p, alpha, st))
    t_m = med(lambda i: B.quantize_raw(xs[i % 2], p, alpha, os_[i % 2]["codes_row"],
                                       os_[i % 2]["scales_row"], os_[i % 2]["codes_col"],
                                       os_[i % 2]["scales_col"], None, None, st))
    res["c4"] = entry(r * c, 3.125, t_s, t_m, "8192x8192 quantize, both orientations, RTN 4/6",
                      VALU_INSTS_PER_BLOCK_C4)
    del xs, os_
    # c5: gradient tensor, Hadamard transform + stochastic rounding (arithmetic-bound)
    xs = [wl.make("c5").cuda() for _ in range(2)]
    r, c = xs[0].shape
    os_ = [B.alloc_outputs(r, c, B.ROWWISE, "cuda", want_choice=False) for _ in range(2)]
    p = B.make_params(r, c, rounding=B.SR, rht=1, sr_seed=wl.C5_SR_SEED, rht_seed=wl.C5_RHT_SEED)
    t_s = med(lambda i: B.tensor_scale_raw(xs[i % 2], p, alpha, st))
    t_m = med(lambda i: B.quantize_raw(xs[i % 2], p, alpha, os_[i % 2]["codes_row"],
                                       os_[i % 2]["scales_row"], None, None, None, None, st))
    res["c5"] = entry(r * c, BYTES_PER_ELEM_QUANT, t_s, t_m,
                      "32768x8192 quantize, rowwise, Hadamard + stochastic rounding, 4/6",
                      VALU_INSTS_PER_BLOCK_C5)
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU part); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    B.lib()
    if args.counter_pass_gemm:
        g = torch.Generator(device="cuda")
        g.manual_seed(1)
        m, nk = args.counter_pass_gemm, 8192
        u8 = dict(dtype=torch.uint8, device="cuda", generator=g)

        def operand(rows):
            return [torch.randint(0, 256, (rows, nk // 2), **u8),
                    torch.randint(0x30, 0x48, (rows, nk // 16), **u8)]

        one = torch.ones(1, dtype=torch.float32, device="cuda")
        a = operand(m)
        ws = [operand(nk) for _ in range(1 if m == nk else 8)]
        out = torch.empty((m, nk), dtype=torch.bfloat16, device="cuda")
        launches = 4 if m == nk else 16
        for i in range(launches):
            w = ws[i % len(ws)]
            rc = B.gemm_raw(*a, one, *w, one, m, nk, nk, B.OUT_BF16, out, torch.cuda.current_stream())
            if rc:
                raise RuntimeError(f"nvfp4_46_gemm failed with status {rc}")
        torch.cuda.synchronize()
        print(f"counter pass done: {launches} products {m} x {nk} x {nk}")
        return
    if args.layer_pass:
        from paper_2512_02010_amd import linear
        xa = wl.make("c3", 8192, 8192).cuda()
        wf = wl.make("c2", dtype=torch.float32).cuda()
        dy = wl.make("c1", 8192, 8192).cuda()
        ws = B.new_workspace()
        for _ in range(5):
            qw = linear.quantize_weight(wf, workspace=ws)
            linear.fprop(xa, qw, workspace=ws)
            linear.dgrad(dy, qw, sr_seed=wl.C5_SR_SEED, workspace=ws)
            linear.wgrad(dy, xa, sr_seed=wl.C5_SR_SEED, rht_seed=wl.C5_RHT_SEED, workspace=ws)
        torch.cuda.synchronize()
        print("layer pass done: 5 steps")
        return
    rows, cols = args.rows, args.cols
    n = rows * cols
    x_host = wl.make("c2", rows, cols)
    sets = [BufferSet(x_host) for _ in range(max(1, args.buffers))]
    torch.cuda.synchronize()

    if args.counter_pass:
        # a plain copy of known size (rows*cols*2 bytes read, the same written) calibrates
        # the byte counters; then every kernel of the step runs on rotating buffer sets
        for i in range(3):
            sets[i % len(sets)].deq.copy_(sets[(i + 1) % len(sets)].x)
        for i in range(6):
            step(sets[i % len(sets)])
        if args.other_workloads:
            # the kernels that stage data in LDS: both orientations in one pass (c4 recipe)
            # and the fake-quant round trip, on tensors of the same shape
            x4 = wl.make("c4", rows, cols).cuda()
            o4 = B.alloc_outputs(rows, cols, B.BOTH, "cuda", want_choice=False)
            p4 = B.make_params(rows, cols, layout=B.BOTH)
            st = torch.cuda.current_stream()
            for i in range(4):
                B.quantize_raw(x4, p4, sets[0].alpha, o4["codes_row"], o4["scales_row"],
                               o4["codes_col"], o4["scales_col"], None, None, st)
                B.fake_quant_raw(x4, sets[0].params, sets[0].alpha, sets[0].deq, st)
            # the arithmetic-bound rowwise kernel: Hadamard transform + stochastic rounding
            # on the c5 recipe (same per-block work as the full 32768x8192 tensor)
            x5 = wl.make("c5", rows, cols).cuda()
            p5 = B.make_params(rows, cols, rounding=B.SR, rht=1, sr_seed=wl.C5_SR_SEED,
                               rht_seed=wl.C5_RHT_SEED)
            a5 = torch.empty(1, dtype=torch.float32, device="cuda")
            B.tensor_scale_raw(x5, p5, a5, st)
            for i in range(4):
                B.quantize_raw(x5, p5, a5, o4["codes_row"], o4["scales_row"], None, None, None,
                               None, st)
            # one scale per 16x16 tile on the c2 tensor: the rowwise packing alone, and with the
            # packing for the transposed matrix from the same pass
            ob = B.alloc_outputs(rows, cols, B.BOTH, "cuda", want_choice=False, block2d=1)
            pr = B.make_params(rows, cols, block2d=1)
            pb = B.make_params(rows, cols, layout=B.BOTH, block2d=1)
            for i in range(4):
                xs_ = sets[i % len(sets)]
                B.quantize_raw(xs_.x, pr, xs_.alpha, ob["codes_row"], ob["scales_row"], None, None,
                               None, None, st)
                B.quantize_raw(xs_.x, pb, xs_.alpha, ob["codes_row"], ob["scales_row"],
                               ob["codes_col"], ob["scales_col"], None, None, st)
        torch.cuda.synchronize()
        print("counter pass done: 3 copies of %d bytes, 6 steps" % (n * 2))
        return

    for i in range(args.warmup):
        step(sets[i % len(sets)])
    he = hip_events()
    evs = [[he.new() for _ in range(2)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % len(sets)], evs[i])        # two events per step, around the quantize call
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    t_quant_all = sorted(he.elapsed_ms(e[0], e[1]) for e in evs)
    t_quant = sum(t_quant_all) / len(t_quant_all)
    quant_gbs = n * BYTES_PER_ELEM_QUANT / (t_quant * 1e-3) / 1e9

    # ---- everything below is outside the timed region -------------------------------------
    import statistics

    # every call of the step between its own events (context for `value`)
    evs4 = [[he.new() for _ in range(4)] for _ in range(max(args.steps, 50))]
    torch.cuda.synchronize()
    for i, e in enumerate(evs4):
        step(sets[i % len(sets)], e)
    torch.cuda.synchronize()
    t_scale = statistics.median(he.elapsed_ms(e[0], e[1]) for e in evs4)
    t_quant_med = statistics.median(he.elapsed_ms(e[1], e[2]) for e in evs4)
    t_deq = statistics.median(he.elapsed_ms(e[2], e[3]) for e in evs4)

    # what this memory system gives a pure stream of the quantizer's shape (2 B read +
    # 0.5625 B written per element), from two things that ship: the read-only pass of the
    # tensor scale (reads all of x, writes nothing) and a plain device copy (reads and writes
    # 2 B per element); their difference prices written bytes, of which the quantizer has
    # 0.5625 / 2 as many.  Same rotation over buffer sets, same events.
    st = torch.cuda.current_stream()

    def scale_only(bs):
        B.tensor_scale_ws_raw(bs.x, bs.params, bs.alpha, bs.workspace, B.TENSOR_SCALE_WS_BYTES, st)

    def copy_only(bs):
        bs.deq.copy_(bs.x)

    t_read = time_single(scale_only, sets, 60)[1]
    t_copy = time_single(copy_only, sets, 60)[1]
    t_ceiling = t_read + (BYTES_PER_ELEM_QUANT - 2.0) / 2.0 * (t_copy - t_read)

    # 4/6 against standard NVFP4 (always 6): launches of the two alternate, so that clock
    # drift over the run hits both alike; medians over 60 launches each, every launch on a
    # buffer set whose data is not in the memory-side cache
    p6 = B.make_params(rows, cols, select=B.SEL_FORCE6)

    def q46(bs):
        B.quantize_raw(bs.x, bs.params, bs.alpha, bs.out["codes_row"], bs.out["scales_row"], None,
                       None, None, None)

    def q6(bs):
        B.quantize_raw(bs.x, p6, bs.alpha, bs.out["codes_row"], bs.out["scales_row"], None, None,
                       None, None)

    pair = [(he.new(), he.new(), he.new()) for _ in range(60)]
    for i in range(8):
        q46(sets[i % len(sets)])
        q6(sets[(i + 1) % len(sets)])
    torch.cuda.synchronize()
    for i, (e0, e1, e2) in enumerate(pair):
        he.record(e0, st)
        q46(sets[(2 * i) % len(sets)])
        he.record(e1, st)
        q6(sets[(2 * i + 1) % len(sets)])
        he.record(e2, st)
    torch.cuda.synchronize()
    t46 = sorted(he.elapsed_ms(e[0], e[1]) for e in pair)
    t6 = sorted(he.elapsed_ms(e[1], e[2]) for e in pair)
    t46 = (sum(t46) / len(t46), t46[len(t46) // 2], t46[0])
    t6 = (sum(t6) / len(t6), t6[len(t6) // 2], t6[0])
    hot = time_single(q46, sets[:1], 100)
    # the same comparison inside the step (the quantize call follows the tensor-scale pass over
    # the same tensor, as in the timed region): steps alternate between the two quantizers
    evs_alt = [[he.new() for _ in range(2)] for _ in range(120)]
    torch.cuda.synchronize()
    for i, e in enumerate(evs_alt):
        step(sets[i % len(sets)], e, p6 if i % 2 else None)
    torch.cuda.synchronize()
    t46_step = statistics.median(he.elapsed_ms(e[0], e[1]) for e in evs_alt[0::2])
    t6_step = statistics.median(he.elapsed_ms(e[0], e[1]) for e in evs_alt[1::2])

    # what the method buys on this tensor (config 2 asks for it): squared error of 4/6 against
    # always-6 under both tensor-scale constants, and how often 4 is chosen; the sums run in
    # fp64 on the device over the library's fake-quant outputs
    bs = sets[0]
    xf = bs.x.double()
    ref_sq = float((xf * xf).mean())

    def mse(**kw):
        a = B.nvfp4_46_tensor_scale(bs.x, fp8_max=kw.get("fp8_max", 256.0))
        d = B.nvfp4_46_fake_quant(bs.x, a, **kw).double() - xf
        return float((d * d).mean())

    choice = B.nvfp4_46_quantize(bs.x, bs.alpha)["choice_row"]
    quality = {
        "mse_46": mse(), "mse_always6_at_256": mse(select=B.SEL_FORCE6),
        "mse_always6_at_448": mse(select=B.SEL_FORCE6, fp8_max=448.0),
        "mean_x_squared": ref_sq, "share_of_blocks_scaled_to_4": float(choice.float().mean()),
        "note": "fp64 mean squared error of dequantize(quantize(x)) on this tensor: 4/6 (tensor "
                "scale with 256), standard NVFP4 with the same tensor scale, and standard NVFP4 "
                "as usually run (448)",
    }
    del xf, choice

    # the same step replayed from HIP graphs (one per buffer set): what launch gaps cost
    graphs = []
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for bs in sets:
            bs.stream = side
            step(bs)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                bs.stream = torch.cuda.current_stream()
                step(bs)
            graphs.append(g)
        for i in range(args.warmup):
            graphs[i % len(graphs)].replay()
        side.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[i % len(graphs)].replay()
        side.synchronize()
        graph_ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    result = {
        "metric": "4/6 NVFP4 quantize G elem/s + achieved HBM GB/s (% of peak), 8192x8192 bf16",
        "value": n / (ms_per_step * 1e-3) / 1e9,
        "unit": "G elem/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"c2: {rows}x{cols} BF16, 0.02*Student-t(3) with 1% outlier columns x50, "
                        "seed 4602; step = tensor_scale (one launch, workspace form) + rowwise 4/6 "
                        "RTN quantize + dequantize",
            "buffer_sets": len(sets),
            "generator": f"torch.Generator(cpu) of torch {torch.__version__} "
                         "(paper_2512_02010_amd/workloads.py)",
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "k_flat<RTN, 4/6-MSE> (rowwise quantize)",
            "achieved": quant_gbs,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": quant_gbs / HBM_PEAK_GBS,
            "traffic": n * HBM_TRAFFIC_PER_ELEM_46,
            "timing": "average over the timed steps of the interval between two HIP events "
                      "(hipEventDisableSystemFence) recorded on the launch stream around the call; "
                      "a pair of events reads about 3 us more than the dispatch duration that "
                      "rocprofv3 reports for the kernel (profiles/c2_step_kernel_trace.txt)",
            "us_avg_median_min": [t_quant * 1e3, t_quant_all[len(t_quant_all) // 2] * 1e3,
                                  t_quant_all[0] * 1e3],
            "stream_ceiling": {
                "read_only_pass_us": t_read * 1e3, "device_copy_us": t_copy * 1e3,
                "ceiling_us": t_ceiling * 1e3,
                "ceiling_gbs": n * BYTES_PER_ELEM_QUANT / (t_ceiling * 1e-3) / 1e9,
                "frac_of_ceiling": t_ceiling / t_quant,
                "note": "a pure stream of this shape, priced in this run from the read-only pass of "
                        "the tensor scale (2 B/elem read) and a device copy (2 B read + 2 B "
                        "written): read time + 0.5625/2 of the copy's extra time; cold medians of "
                        "60 launches each, against the timed region's average",
            },
            "traffic_note": "bytes per launch from rocprofv3 FETCH_SIZE/WRITE_SIZE at this "
                            "shape (profiles/c2_step_counters.txt), not re-measured in this run",
        },
        "roofline_alu": {
            "bound": "alu",
            "note": "the same kernel against the chip's fp32 vector rate (157.3 TFLOP/s = 78.6 T "
                    "fused multiply-adds/s; reached by plain instructions, packed fp32 is not "
                    "used): lane-operations = wave-instructions per block (rocprofv3 "
                    "SQ_INSTS_VALU) x blocks; half of this kernel's instructions are of classes "
                    "that issue at half or a quarter of that rate "
                    "(profiles/valu_issue_rates.txt)",
            "achieved": VALU_INSTS_PER_BLOCK_46 * (n / 16.0) / (t_quant * 1e-3) / 1e12,
            "peak": VALU_PEAK_TOPS,
            "unit": "T lane-op/s",
            "frac": VALU_INSTS_PER_BLOCK_46 * (n / 16.0) / (t_quant * 1e-3) / 1e12 / VALU_PEAK_TOPS,
        },
        "kernels_us": {
            "note": "medians of a separate pass with events around every call of the step",
            "tensor_scale": t_scale * 1e3,
            "quantize": t_quant_med * 1e3,
            "dequantize": t_deq * 1e3,
        },
        "kernels_gbs": {
            "tensor_scale": n * BYTES_PER_ELEM_AMAX / (t_scale * 1e-3) / 1e9,
            "quantize": n * BYTES_PER_ELEM_QUANT / (t_quant_med * 1e-3) / 1e9,
            "dequantize": n * BYTES_PER_ELEM_DEQUANT / (t_deq * 1e-3) / 1e9,
        },
        "c2_quality": quality,
        "graph_replay": {
            "ms_per_step": graph_ms_per_step,
            "g_elem_s": n / (graph_ms_per_step * 1e-3) / 1e9,
            "note": "the same step replayed from one HIP graph per buffer set (context; `value` "
                    "is the eagerly launched loop above)",
        },
        "quantize_only": {
            "g_elem_s_in_step": n / (t_quant * 1e-3) / 1e9,
            "cold_us_avg_median_min": [t * 1e3 for t in t46],
            "hot_us_avg_median_min": [t * 1e3 for t in hot],
            "force6_cold_us_avg_median_min": [t * 1e3 for t in t6],
            "t46_over_t6": t46_step / t6_step,
            "t46_over_t6_note": "ratio of the medians of the quantize call inside 60 + 60 steps that "
                                "alternate between 4/6 and always-6 (the call follows the "
                                "tensor-scale pass over the same tensor, as in the timed region)",
            "in_step_us_46_and_always6": [t46_step * 1e3, t6_step * 1e3],
            "t46_over_t6_cold": t46[1] / t6[1],
            "t46_over_t6_cold_note": "the same for 60 + 60 alternating launches on their own, each "
                                     "on a tensor that no recent kernel touched",
            "paper_context": "the paper reports <15% overhead of 4/6 over plain NVFP4 "
                             "quantization on NVIDIA Blackwell (Sections 1, 3.2)",
        },
    }
    del sets, graphs
    torch.cuda.empty_cache()
    if not args.no_gemm and (rows, cols) == (8192, 8192):
        result["gemm"] = time_gemm(x_host)
    if args.other_workloads:
        torch.cuda.empty_cache()
        result["other_workloads"] = time_other_workloads()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(x_host)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
