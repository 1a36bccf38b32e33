#!/usr/bin/env python3
"""Benchmark of the SBP matmul + boxing hot path on one MI355X.

One step = one pass of the whole path over the Megatron-style MLP workload (k = 8 logical
devices as 8 shard sets in one GPU's HBM):

    H  = gelu(X W1)     X [8192,4096] bf16 B,  W1 [4096,16384] bf16 S(1)  -> H S(1) bf16
    Y  = H W2           W2 [16384,4096] bf16 S(0)                         -> Y P(sum), 8 fp32 partials
    Yb = boxing(Y)      P(sum) -> B (all-reduce): 8 partials -> 8 identical fp32 copies

Inputs are seeded synthetic tensors, resident in HBM before the timed region.  Before the warm-up steps the step
runs for --preroll-ms (default 100 ms, reported as "preroll_ms" / "preroll_steps") so that the device has left its
idle clocks; then exactly --warmup untimed and --steps timed steps.  Prints ONE JSON line.
`value` is the matmul work of a step (2.199 TFLOP) divided by the time of the whole step (boxing
included); the per-kernel figures are in "kernels", "roofline" (dominant kernel) and
"roofline_boxing".  The CPU oracle is timed on a bounded sample of the same workload.

`--workload dp_grad | classifier | relayout | uvw | zero` times the other full-size workloads the same way
(one JSON line each, per-kernel times in "kernels", no oracle leg): the data-parallel weight gradient
with its reduce-scatter / all-reduce, the model-parallel classifier head with its softmax statistics,
the pure relayout chain S(0) -> S(1) -> B -> S(0) on 16 logical devices, Y = U V W with the boxing
deferred to the end against boxing right after the first product, and (`zero`) the two cast-fused
boxings of a sharded optimizer state.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak, TFLOP/s
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E peak, GB/s
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs, scaled by the
# calibration copy; summary in profiles/bench_mlp_k8_counters.md).  Offline figures, not re-measured here.
TRAFFIC_SOURCE = "constant from an earlier rocprofv3 --pmc run of this command (profiles/bench_mlp_k8_counters.md), not measured by this run"
TRAFFIC_BYTES = {"gemm1": 1.853e9, "gemm2": 2.683e9, "boxing_p2b": 2.099e9}


def shard_range(n, k, i):
    """[begin, end) of shard i when n indices are split over k devices: the library's own balanced split
    (sbp_local_shape), so that the harness holds no split rule of its own"""
    import paper_2110_15032_amd as sbp
    lens = [sbp.sbp_local_shape(n, 1, sbp.S(0), k, j)[0] for j in range(i + 1)]
    return sum(lens[:-1]), sum(lens)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--preroll-ms", type=float, default=100.0,
                    help="before the warm-up steps, run the step for about this long (wall clock) so that the device has left its "
                         "idle clocks: after idling (input generation) the part needs some 30 ms of work to reach the clock it "
                         "then holds, more than a few 2 ms steps; 0 = off.  The timed region is not touched")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--cpu-rows", type=int, default=4096, help="token rows in the oracle's sample")
    ap.add_argument("--variant", type=int, default=0, help="GEMM kernel variant knob (0 = default)")
    ap.add_argument("--tile-order", type=int, default=0, help="GEMM tile walk knob (0 = the library's choice)")
    ap.add_argument("--layout", default="separate", choices=["separate", "contiguous", "staggered"],
                    help="how the k shard buffers of a tensor lie in HBM: k allocations (default), back to back in one, or --stagger bytes apart in one")
    ap.add_argument("--stagger", type=int, default=4096, help="bytes between consecutive shard buffers with --layout staggered")
    ap.add_argument("--workload", default="mlp", choices=["mlp", "dp_grad", "classifier", "relayout", "uvw", "zero", "across", "clock_probe", "mfma_probe", "vendor_gemm", "tiny", "grid"],
                    help="mlp (default) is the workload the headline metric is quoted on")
    ap.add_argument("--dense-logits", action="store_true",
                    help="classifier workload: logits and gradient rows back to back (pitch 125000) instead of padded to 128 bytes")
    ap.add_argument("--calibrate", action="store_true",
                    help="before the timed region run ONE plain copy of known size (identity boxing B->B of the "
                         "1 GiB fp32 tensor: 1 GiB read + 1 GiB written) so that a counter run has a reference dispatch")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the k logical devices are k shard buffers in one HBM); "
              "--gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2110_15032_amd as sbp
    import workloads as wl
    from workloads import CONFIGS

    PREROLL["ms"] = args.preroll_ms
    sbp.lib()   # fail loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload != "mlp":
        sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, args.variant)
        sbp.sbp_set_knob(sbp.KNOB_TILE_ORDER, args.tile_order)
        out = OTHER_WORKLOADS[args.workload](args, CONFIGS.get(args.workload), sbp, wl, torch, np)
        print(json.dumps(out), flush=True)
        return
    cfg = CONFIGS["mlp"]
    k = cfg["k"]
    T, D = cfg["X"]["shape"]          # 8192 tokens, 4096 model width
    F = cfg["W1"]["shape"][1]         # 16384 hidden width
    seed = wl.SEED_BASE

    def bf16_dev(spec, rows=None, cols=None):
        x = wl.normal(seed, spec["id"], spec["shape"], spec["dist"][1], rows, cols, dtype=np.float32)
        return torch.from_numpy(wl.to_bf16_bits(x).view(np.int16)).to(dev)

    # The k shard buffers of a tensor stand for memory on k different devices; here they are k allocations
    # (--layout separate, the default), or k pieces of one allocation back to back (contiguous) or with
    # --stagger bytes between them (staggered).
    arena = make_arena(torch, np, args)

    t0 = time.time()
    x_full = bf16_dev(cfg["X"])
    x_sh = arena([(T, D)] * k, torch.int16)                                      # B: k physical copies
    for t in x_sh:
        t.copy_(x_full)
    w1_sh = arena([(D, F // k)] * k, torch.int16)                                # [4096, 2048] each
    w2_sh = arena([(F // k, D)] * k, torch.int16)                                # [2048, 4096] each
    for i in range(k):
        w1_sh[i].copy_(bf16_dev(cfg["W1"], cols=np.arange(*shard_range(F, k, i))))
        w2_sh[i].copy_(bf16_dev(cfg["W2"], rows=np.arange(*shard_range(F, k, i))))
    h_sh = arena([(T, F // k)] * k, torch.int16)
    y_sh = arena([(T, D)] * k, torch.float32)
    yb_sh = arena([(T, D)] * k, torch.float32)
    gen_s = time.time() - t0

    X = sbp.SbpTensor(x_sh, T, D, sbp.BF16)
    W1 = sbp.SbpTensor(w1_sh, D, F, sbp.BF16)
    W2 = sbp.SbpTensor(w2_sh, F, D, sbp.BF16)
    H = sbp.SbpTensor(h_sh, T, F, sbp.BF16)
    Y = sbp.SbpTensor(y_sh, T, D, sbp.F32)
    Yb = sbp.SbpTensor(yb_sh, T, D, sbp.F32)
    stream = torch.cuda.current_stream()
    sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, args.variant)
    sbp.sbp_set_knob(sbp.KNOB_TILE_ORDER, args.tile_order)

    def step(ev=None):
        if ev:
            ev[0].record(stream)
        sbp.sbp_matmul_ex(X, sbp.B, W1, sbp.S(1), H, sbp.S(1), k, stream, sbp.EPI_GELU)
        if ev:
            ev[1].record(stream)
        sbp.sbp_matmul(H, sbp.S(1), W2, sbp.S(0), Y, sbp.P_SUM, k, stream)
        if ev:
            ev[2].record(stream)
        sbp.sbp_boxing(Y, sbp.P_SUM, Yb, sbp.B, k, stream)
        if ev:
            ev[3].record(stream)

    if args.calibrate:
        # Yb -> Y as a B -> B identity: k contiguous copies of 128 MiB, 1 GiB in + 1 GiB out in total
        sbp.sbp_boxing(Yb, sbp.B, Y, sbp.B, k, stream)
        torch.cuda.synchronize()
    preroll_steps = preroll(torch, step, args.preroll_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps, HIP events on the launch stream around every kernel
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_begin) * 1e3
    ms_per_step = wall_ms / args.steps
    k_ms = [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i in range(3)]

    # the boxing alone on each of the three buffer layouts (outside the timed region): fresh buffers, the
    # partials copied from the step's, 10 calls each
    box_layouts = {}
    for layout in ("separate", "contiguous", "staggered"):
        ar = make_arena(torch, np, args, layout)
        yi, yo = ar([(T, D)] * k, torch.float32), ar([(T, D)] * k, torch.float32)
        for a, b in zip(yi, y_sh):
            a.copy_(b)
        Yi, Yo = sbp.SbpTensor(yi, T, D, sbp.F32), sbp.SbpTensor(yo, T, D, sbp.F32)
        for _ in range(3):
            sbp.sbp_boxing(Yi, sbp.P_SUM, Yo, sbp.B, k, stream)
        e = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
        e[0].record(stream)
        for i in range(10):
            sbp.sbp_boxing(Yi, sbp.P_SUM, Yo, sbp.B, k, stream)
            e[i + 1].record(stream)
        torch.cuda.synchronize()
        box_layouts[layout] = 2.0 * k * T * D * 4 / (e[0].elapsed_time(e[10]) / 10 * 1e-3) / 1e9
        del yi, yo, Yi, Yo
    torch.cuda.empty_cache()

    flops_gemm = 2.0 * T * D * F                      # per GEMM, summed over the 8 shards
    bytes_box = 2.0 * k * T * D * 4                   # P->B: read k partials, write k copies
    gemm1_tf = flops_gemm / (k_ms[0] * 1e-3) / 1e12
    gemm2_tf = flops_gemm / (k_ms[1] * 1e-3) / 1e12
    box_gbps = bytes_box / (k_ms[2] * 1e-3) / 1e9
    value = 2.0 * flops_gemm / (ms_per_step * 1e-3) / 1e12
    dom = 0 if k_ms[0] >= k_ms[1] else 1
    dom_name = ["sbp_matmul (B,S1)->S1 bf16 + GeLU", "sbp_matmul (S1,S0)->P(sum) fp32 partials"][dom]
    dom_tf = [gemm1_tf, gemm2_tf][dom]

    out = {
        "metric": "SBP matmul TFLOP/s (% MFMA peak) + boxing GB/s (% HBM peak), k=8",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "preroll_ms": args.preroll_ms,
        "preroll_steps": preroll_steps,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "Megatron-style MLP block, k=8: X[8192,4096] bf16 B; W1[4096,16384] S(1) -> H S(1) "
                               "(GeLU); W2[16384,4096] S(0) -> Y P(sum); boxing P->B of 8 fp32 8192x4096 partials",
                   "k": k, "gemm_variant": args.variant, "shard_buffer_layout": args.layout},
        "kernels": {
            "gemm1_gelu_ms": round(k_ms[0], 4), "gemm1_tflops": round(gemm1_tf, 2),
            "gemm2_psum_ms": round(k_ms[1], 4), "gemm2_tflops": round(gemm2_tf, 2),
            "boxing_p2b_ms": round(k_ms[2], 4), "boxing_gbps": round(box_gbps, 1),
            "matmul_pct_mfma_peak": round(100 * 2 * flops_gemm / ((k_ms[0] + k_ms[1]) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
            "boxing_pct_hbm_peak": round(100 * box_gbps / PEAK_HBM_GBPS, 2),
            "boxing_gbps_separate": round(box_layouts["separate"], 1),
            "boxing_gbps_contiguous": round(box_layouts["contiguous"], 1),
            "boxing_gbps_staggered": round(box_layouts["staggered"], 1),
            "input_gen_s": round(gen_s, 2),
        },
        "roofline": {"bound": "mfma", "kernel": dom_name, "achieved": round(dom_tf, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(dom_tf / PEAK_BF16_TFLOPS, 4),
                     "traffic": TRAFFIC_BYTES["gemm1" if dom == 0 else "gemm2"], "traffic_unit": "bytes per launch",
                     "traffic_source": TRAFFIC_SOURCE},
        "roofline_boxing": {"bound": "hbm", "kernel": "sbp_boxing P(sum)->B", "achieved": round(box_gbps, 1),
                            "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(box_gbps / PEAK_HBM_GBPS, 4),
                            "traffic": TRAFFIC_BYTES["boxing_p2b"], "traffic_unit": "bytes per launch",
                            "traffic_source": TRAFFIC_SOURCE},
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, k, args.cpu_rows, seed)
    print(json.dumps(out), flush=True)


# ------------------------------------------------------------------------------------------------
# The other full-size workloads
# ------------------------------------------------------------------------------------------------
def make_arena(torch, np, args, layout=None):
    """arena(shapes, dtype) -> one buffer per shape: separate allocations, or pieces of one allocation back to
    back (contiguous) or --stagger bytes apart (staggered).  Equal offsets in equally sized back-to-back
    buffers fall on the same memory channel, which k real devices would not share; the stagger removes that
    artefact of holding k devices' shards in one HBM."""
    layout = layout or args.layout
    gap = {"separate": None, "contiguous": 0, "staggered": args.stagger}[layout]

    def arena(shapes, dtype):
        if gap is None:
            return [torch.empty(*sh, dtype=dtype, device="cuda") for sh in shapes]
        esz = torch.empty((), dtype=dtype).element_size()
        sizes = [int(np.prod(sh)) for sh in shapes]
        step = [((n * esz + gap + 255) // 256 * 256) // esz for n in sizes]
        buf = torch.empty(sum(step) + 64, dtype=dtype, device="cuda")
        out, off = [], 0
        for sh, n, st in zip(shapes, sizes, step):
            out.append(buf[off:off + n].view(*sh))
            off += st
        return out
    return arena


PREROLL = {"ms": 0.0, "steps": 0}     # set from --preroll-ms in main(); steps: what the last run needed


def preroll(torch, step, ms):
    """Runs step() back to back for about `ms` of wall clock (in batches, synchronised) before any warm-up or timed
    step: the device leaves its idle clocks.  Returns the number of steps run."""
    n = 0
    if ms > 0:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(4):
                step()
            n += 4
            torch.cuda.synchronize()
    return n


def time_stages(torch, stages_of, steps, warmup):
    """stages_of(s) -> list of callables for step s.  Returns (avg ms per stage, wall ms per step)."""
    stream = torch.cuda.current_stream()

    def one_step():
        for f in stages_of(0):
            f(stream)
    PREROLL["steps"] = preroll(torch, one_step, PREROLL["ms"])
    for s in range(warmup):
        for f in stages_of(s):
            f(stream)
    torch.cuda.synchronize()
    n = len(stages_of(0))
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(n + 1)] for _ in range(steps)]
    t0 = time.perf_counter()
    for s in range(steps):
        evs[s][0].record(stream)
        for i, f in enumerate(stages_of(warmup + s)):
            f(stream)
            evs[s][i + 1].record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / steps for i in range(n)], wall


def result_line(args, workload, k, value, unit, wall_ms, kernels, roofline, dtype="bf16"):
    return {"metric": f"SBP matmul TFLOP/s (% MFMA peak) + boxing GB/s (% HBM peak), k={k}",
            "value": round(value, 3), "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "preroll_ms": PREROLL["ms"], "preroll_steps": PREROLL["steps"],
            "ms_per_step": round(wall_ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": dtype, "data": "synthetic", "config": {"workload": workload, "k": k, "gemm_variant": args.variant},
            "kernels": kernels, "roofline": roofline}


def bench_dp_grad(args, cfg, sbp, wl, torch, np):
    """dW = X^T dY on 8 token shards -> 8 fp32 partials; P(sum) -> S(0) and P(sum) -> B.  The
    tensors are about the size of the memory-side cache, so the step rotates over three buffer sets."""
    k = cfg["k"]
    Tk, Din = cfg["X"]["shape"]
    Dout = cfg["dY"]["shape"][1]
    arena = make_arena(torch, np, args)
    seed = wl.SEED_BASE
    sets = []
    for r in range(3):
        x_sh = arena([(Tk // k, Din)] * k, torch.int16)
        dy_sh = arena([(Tk // k, Dout)] * k, torch.int16)
        for i in range(k):
            rows = np.arange(*shard_range(Tk, k, i))
            for dst, spec in ((x_sh[i], cfg["X"]), (dy_sh[i], cfg["dY"])):
                v = wl.normal(seed + r, spec["id"], spec["shape"], spec["dist"][1], rows, None, dtype=np.float32)
                dst.copy_(torch.from_numpy(wl.to_bf16_bits(v).view(np.int16)))
        XT = sbp.SbpTensor(x_sh, Din, Tk, sbp.BF16, trans=1)
        DY = sbp.SbpTensor(dy_sh, Tk, Dout, sbp.BF16)
        DW = sbp.SbpTensor(arena([(Din, Dout)] * k, torch.float32), Din, Dout, sbp.F32)
        DWS = sbp.SbpTensor(arena([(Din // k, Dout)] * k, torch.float32), Din, Dout, sbp.F32)
        DWB = sbp.SbpTensor(arena([(Din, Dout)] * k, torch.float32), Din, Dout, sbp.F32)
        sets.append((XT, DY, DW, DWS, DWB))

    def stages_of(s):
        XT, DY, DW, DWS, DWB = sets[s % 3]
        return [lambda st: sbp.sbp_matmul(XT, sbp.S(1), DY, sbp.S(0), DW, sbp.P_SUM, k, st),
                lambda st: sbp.sbp_boxing(DW, sbp.P_SUM, DWS, sbp.S(0), k, st),
                lambda st: sbp.sbp_boxing(DW, sbp.P_SUM, DWB, sbp.B, k, st)]

    ms, wall = time_stages(torch, stages_of, args.steps, args.warmup)
    flops = 2.0 * Din * Tk * Dout
    b_p2s, b_p2b = (k + 1) * Din * Dout * 4.0, 2.0 * k * Din * Dout * 4.0
    tf = flops / (ms[0] * 1e-3) / 1e12
    kernels = {"gemm_tn_psum_ms": round(ms[0], 4), "gemm_tflops": round(tf, 2),
               "boxing_p2s_ms": round(ms[1], 4), "boxing_p2s_gbps": round(b_p2s / ms[1] / 1e6, 1),
               "boxing_p2b_ms": round(ms[2], 4), "boxing_p2b_gbps": round(b_p2b / ms[2] / 1e6, 1),
               "buffer_sets_rotated": 3}
    roof = {"bound": "mfma", "kernel": "sbp_matmul (S1,S0)->P(sum), transposed X", "achieved": round(tf, 2),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4), "traffic": None}
    return result_line(args, "data-parallel weight gradient, k=8: dW = X^T dY, X[16384,1024] S(0) stored by tokens, "
                             "dY[16384,4096] S(0) -> 8 fp32 partials [1024,4096]; boxing P->S(0) and P->B",
                       k, flops / (wall * 1e-3) / 1e12, "TFLOP/s", wall, kernels, roof)


def bench_classifier(args, cfg, sbp, wl, torch, np):
    """logits = F W on 8 class shards (bf16), local row max -> P(max) -> B, local sum of exp -> P(sum) -> B,
    then the sparse cross entropy: loss partials -> P(sum) -> B and the gradient of the logits (S(1))."""
    k = cfg["k"]
    R, Dm = cfg["F"]["shape"]
    C = cfg["W"]["shape"][1]
    Ci = C // k
    arena = make_arena(torch, np, args)
    seed = wl.SEED_BASE

    def bits(spec, rows=None, cols=None):
        v = wl.normal(seed, spec["id"], spec["shape"], spec["dist"][1], rows, cols, dtype=np.float32)
        return torch.from_numpy(wl.to_bf16_bits(v).view(np.int16))

    f_sh = arena([(R, Dm)] * k, torch.int16)
    f0 = bits(cfg["F"])
    for t in f_sh:
        t.copy_(f0)
    w_sh = arena([(Dm, Ci)] * k, torch.int16)
    for i in range(k):
        w_sh[i].copy_(bits(cfg["W"], cols=np.arange(*shard_range(C, k, i))))
    # Row pitch of the logits and of their gradient: 125000 bf16 = 250000 bytes would put seven of eight rows across
    # cache-line boundaries; the buffers are allocated with the pitch rounded up to 128 bytes (125056 elements) and
    # passed with that leading dimension.  --dense-logits times the unpadded layout.
    P = Ci if args.dense_logits else (Ci + 63) // 64 * 64
    LD = 0 if P == Ci else P
    l_sh = arena([(R, P)] * k, torch.int16)
    vec = lambda: arena([(R, 1)] * k, torch.float32)      # noqa: E731
    Ft, Wt = sbp.SbpTensor(f_sh, R, Dm, sbp.BF16), sbp.SbpTensor(w_sh, Dm, C, sbp.BF16)
    L = sbp.SbpTensor(l_sh, R, C, sbp.BF16, 0, LD)
    MP, MP2, MB, SP, SB, LP, LB, GR = (sbp.SbpTensor(vec(), R, 1, sbp.F32) for _ in range(8))
    for t in GR.keep:
        t.fill_(1.0 / R)
    labels = torch.from_numpy((wl.uniform(seed, 7, (R, 1), 0.0, float(C)).astype(np.int64) % C).astype(np.int32)).cuda()
    Y = sbp.SbpTensor([labels] * k, R, 1, sbp.I32)
    DL = sbp.SbpTensor(arena([(R, P)] * k, torch.int16), R, C, sbp.BF16, 0, LD)

    def stages_of(s):
        return [lambda st: sbp.sbp_matmul_rowmax(Ft, sbp.B, Wt, sbp.S(1), L, sbp.S(1), MP, k, st),     # logits + local row max
                lambda st: sbp.sbp_row_max(L, sbp.S(1), MP2, k, st),      # the separate pass, timed for comparison only
                lambda st: sbp.sbp_boxing(MP, sbp.P_MAX, MB, sbp.B, k, st),
                lambda st: sbp.sbp_row_sumexp(L, sbp.S(1), MB, SP, k, st),
                lambda st: sbp.sbp_boxing(SP, sbp.P_SUM, SB, sbp.B, k, st),
                lambda st: sbp.sbp_xent_loss(L, sbp.S(1), Y, MB, SB, LP, k, st),
                lambda st: sbp.sbp_boxing(LP, sbp.P_SUM, LB, sbp.B, k, st),
                lambda st: sbp.sbp_xent_grad(L, sbp.S(1), Y, MB, SB, GR, DL, k, st)]

    ms, wall = time_stages(torch, stages_of, args.steps, args.warmup)
    flops = 2.0 * R * Dm * C
    lbytes = 2.0 * R * C
    gbytes = lbytes + 2.0 * Dm * C + 2.0 * R * Dm       # logits written, W and F read once
    tf = flops / (ms[0] * 1e-3) / 1e12
    same = all(bool(torch.equal(a, b)) for a, b in zip(MP.keep, MP2.keep))
    kernels = {"gemm_logits_rowmax_ms": round(ms[0], 4), "gemm_tflops": round(tf, 2),
               "gemm_algorithmic_gbps": round(gbytes / ms[0] / 1e6, 1),
               "separate_row_max_ms_not_in_step": round(ms[1], 4), "separate_row_max_gbps": round(lbytes / ms[1] / 1e6, 1),
               "fused_equals_separate_row_max": same,
               "boxing_pmax_us": round(ms[2] * 1e3, 1),
               "row_sumexp_ms": round(ms[3], 4), "row_sumexp_gbps": round(lbytes / ms[3] / 1e6, 1),
               "boxing_psum_us": round(ms[4] * 1e3, 1),
               "xent_loss_us": round(ms[5] * 1e3, 1), "boxing_loss_us": round(ms[6] * 1e3, 1),
               "xent_grad_ms": round(ms[7], 4), "xent_grad_gbps": round(2 * lbytes / ms[7] / 1e6, 1),
               "mean_loss": float(LB.keep[0].mean()), "logits_row_pitch_elements": P}
    roof = {"bound": "mfma", "kernel": "sbp_matmul (B,S1)->S1 bf16 logits", "achieved": round(tf, 2),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4), "traffic": None}
    wall -= ms[1]     # the comparison pass is not part of the step
    return result_line(args, "model-parallel classifier head, k=8: F[1024,512] B x W[512,1000000] S(1) -> bf16 logits S(1) with fused "
                             "row max P(max)->B; sum exp(L - max) P(sum)->B; sparse cross entropy loss P(sum)->B and gradient S(1); "
                             f"logits row pitch {P} elements",
                       k, flops / (wall * 1e-3) / 1e12, "TFLOP/s", wall, kernels, roof)


def bench_relayout(args, cfg, sbp, wl, torch, np):
    """S(0) -> S(1) (all2all), S(1) -> B (all-gather), B -> S(0) (local slice) on 16 logical devices."""
    k = cfg["k"]
    R, C = cfg["T"]["shape"]
    Rk, Ck = R // k, C // k
    arena = make_arena(torch, np, args)
    s0 = arena([(Rk, C)] * k, torch.int16)
    for i in range(k):
        s0[i].copy_(torch.from_numpy(wl.pattern_u16((R, C), rows=np.arange(i * Rk, (i + 1) * Rk)).view(np.int16)))
    s1 = arena([(R, Ck)] * k, torch.int16)
    b = arena([(R, C)] * k, torch.int16)
    o = arena([(Rk, C)] * k, torch.int16)
    T0, T1, TB, TO = (sbp.SbpTensor(x, R, C, sbp.BF16) for x in (s0, s1, b, o))

    def stages_of(s):
        return [lambda st: sbp.sbp_boxing(T0, sbp.S(0), T1, sbp.S(1), k, st),
                lambda st: sbp.sbp_boxing(T1, sbp.S(1), TB, sbp.B, k, st),
                lambda st: sbp.sbp_boxing(TB, sbp.B, TO, sbp.S(0), k, st)]

    ms, wall = time_stages(torch, stages_of, args.steps, args.warmup)
    t = 2.0 * R * C
    by = [2 * t, (1 + k) * t, 2 * t]
    g = [by[i] / ms[i] / 1e6 for i in range(3)]
    kernels = {"s0_to_s1_ms": round(ms[0], 4), "s0_to_s1_gbps": round(g[0], 1),
               "s1_to_b_ms": round(ms[1], 4), "s1_to_b_gbps": round(g[1], 1),
               "b_to_s0_ms": round(ms[2], 4), "b_to_s0_gbps": round(g[2], 1)}
    roof = {"bound": "hbm", "kernel": "sbp_boxing S(1)->B (1 GiB read, 16 GiB written)", "achieved": round(g[1], 1),
            "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(g[1] / PEAK_HBM_GBPS, 4), "traffic": None}
    return result_line(args, "relayout boxing, k=16: T[65536,8192] 16-bit words, S(0)->S(1), S(1)->B, B->S(0)",
                       k, sum(by) / (wall * 1e-3) / 1e9, "GB/s", wall, kernels, roof)


def bench_uvw(args, cfg, sbp, wl, torch, np):
    """Y = U V W with U S(1), V S(0), W B (Sec. 3.3), bf16 inputs, k = 8.  Deferred boxing: (UV) stays
    8 fp32 partials, each multiplied by W (Table 1 row 4), one P->B on Y.  Immediate boxing: P->B on
    (UV), then the row-6 product.  Same matmul work either way; the boxed tensor is [M,N1] or [M,N2]."""
    k = 8
    M, K1, N1, N2 = 4096, 16384, 4096, 1024
    arena = make_arena(torch, np, args)
    seed = wl.SEED_BASE

    def bits(tid, shape, std, rows=None, cols=None):
        v = wl.normal(seed, tid, shape, std, rows, cols, dtype=np.float32)
        return torch.from_numpy(wl.to_bf16_bits(v).view(np.int16))

    u_sh = arena([(M, K1 // k)] * k, torch.int16)
    v_sh = arena([(K1 // k, N1)] * k, torch.int16)
    w_sh = arena([(N1, N2)] * k, torch.int16)
    w0 = bits(102, (N1, N2), 0.02)
    for i in range(k):
        u_sh[i].copy_(bits(100, (M, K1), 1.0, cols=np.arange(*shard_range(K1, k, i))))
        v_sh[i].copy_(bits(101, (K1, N1), 0.02, rows=np.arange(*shard_range(K1, k, i))))
        w_sh[i].copy_(w0)
    U, V, W = sbp.SbpTensor(u_sh, M, K1, sbp.BF16), sbp.SbpTensor(v_sh, K1, N1, sbp.BF16), sbp.SbpTensor(w_sh, N1, N2, sbp.BF16)
    f32 = lambda r, c: sbp.SbpTensor(arena([(r, c)] * k, torch.float32), r, c, sbp.F32)      # noqa: E731
    UV, UVB, YP, YL, YE = f32(M, N1), f32(M, N1), f32(M, N2), f32(M, N2), f32(M, N2)

    def stages_of(s):
        return [lambda st: sbp.sbp_matmul(U, sbp.S(1), V, sbp.S(0), UV, sbp.P_SUM, k, st),
                lambda st: sbp.sbp_matmul(UV, sbp.P_SUM, W, sbp.B, YP, sbp.P_SUM, k, st),      # deferred
                lambda st: sbp.sbp_boxing(YP, sbp.P_SUM, YL, sbp.B, k, st),
                lambda st: sbp.sbp_boxing(UV, sbp.P_SUM, UVB, sbp.B, k, st),                   # immediate
                lambda st: sbp.sbp_matmul(UVB, sbp.B, W, sbp.B, YE, sbp.B, k, st)]

    ms, wall = time_stages(torch, stages_of, args.steps, args.warmup)
    f1, f2 = 2.0 * M * K1 * N1, 2.0 * k * M * N1 * N2
    late, early = ms[0] + ms[1] + ms[2], ms[0] + ms[3] + ms[4]
    kernels = {"gemm_uv_ms": round(ms[0], 4), "gemm_uv_tflops": round(f1 / ms[0] / 1e9, 2),
               "late_gemm_partial_x_w_ms": round(ms[1], 4), "late_gemm_tflops": round(f2 / ms[1] / 1e9, 2),
               "late_boxing_ms": round(ms[2], 4), "late_boxing_gbps": round(2.0 * k * M * N2 * 4 / ms[2] / 1e6, 1),
               "early_boxing_ms": round(ms[3], 4), "early_boxing_gbps": round(2.0 * k * M * N1 * 4 / ms[3] / 1e6, 1),
               "early_gemm_b_x_w_ms": round(ms[4], 4), "early_gemm_tflops": round(f2 / ms[4] / 1e9, 2),
               "late_total_ms": round(late, 4), "early_total_ms": round(early, 4),
               "max_abs_diff_late_vs_early": float((YL.keep[0] - YE.keep[0]).abs().max())}
    tf = f2 / ms[1] / 1e9
    roof = {"bound": "mfma", "kernel": "sbp_matmul (P(sum) fp32, B bf16)->P(sum): three bf16 MFMAs per product term",
            "achieved": round(tf, 2), "peak": PEAK_BF16_TFLOPS / 3, "unit": "TFLOP/s (fp32-operand products)",
            "frac": round(3 * tf / PEAK_BF16_TFLOPS, 4), "traffic": None}
    return result_line(args, "Y = U V W, k=8: U[4096,16384] S(1), V[16384,4096] S(0), W[4096,1024] B, bf16; boxing deferred "
                             "(one P->B on Y) against immediate (P->B on UV)",
                       k, (f1 + f2) / (late * 1e-3) / 1e12, "TFLOP/s", wall, kernels, roof)


def bench_zero(args, cfg, sbp, wl, torch, np):
    """Sharded optimizer state with mixed precision (Sec. 6.4), k = 8, 2^28 parameters: fp32 master
    weights S(0) -> bf16 B (cast fused into the all-gather), and bf16 partial gradients P(sum) -> fp32
    S(0) (cast fused into the reduce-scatter)."""
    k = 8
    R, C = 16384, 16384
    arena = make_arena(torch, np, args)
    w32 = arena([(R // k, C)] * k, torch.float32)
    for i in range(k):
        rows = np.arange(*shard_range(R, k, i))
        w32[i].copy_(torch.from_numpy(wl.normal(wl.SEED_BASE, 200, (R, C), 0.02, rows, None, dtype=np.float32)))
    w16 = arena([(R, C)] * k, torch.int16)
    g16 = arena([(R, C)] * k, torch.int16)
    for i in range(k):
        g16[i].view(torch.bfloat16).normal_(0.0, 1.0)   # partial gradients, N(0, 1) rounded to bf16
    g32 = arena([(R // k, C)] * k, torch.float32)
    W32, W16 = sbp.SbpTensor(w32, R, C, sbp.F32), sbp.SbpTensor(w16, R, C, sbp.BF16)
    G16, G32 = sbp.SbpTensor(g16, R, C, sbp.BF16), sbp.SbpTensor(g32, R, C, sbp.F32)

    def stages_of(s):
        return [lambda st: sbp.sbp_boxing_cast(W32, sbp.S(0), W16, sbp.B, k, st),
                lambda st: sbp.sbp_boxing_cast(G16, sbp.P_SUM, G32, sbp.S(0), k, st)]

    ms, wall = time_stages(torch, stages_of, args.steps, args.warmup)
    n = float(R) * C
    by = [4 * n + 2 * n * k, 2 * n * k + 4 * n]
    g = [by[i] / ms[i] / 1e6 for i in range(2)]
    kernels = {"cast_all_gather_ms": round(ms[0], 4), "cast_all_gather_gbps": round(g[0], 1),
               "cast_reduce_scatter_ms": round(ms[1], 4), "cast_reduce_scatter_gbps": round(g[1], 1)}
    roof = {"bound": "hbm", "kernel": "sbp_boxing_cast fp32 S(0) -> bf16 B (1 GiB read, 4 GiB written)", "achieved": round(g[0], 1),
            "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(g[0] / PEAK_HBM_GBPS, 4), "traffic": None}
    return result_line(args, "sharded optimizer state, k=8, 2^28 parameters: fp32 S(0) -> bf16 B and bf16 P(sum) -> fp32 S(0)",
                       k, sum(by) / (wall * 1e-3) / 1e9, "GB/s", wall, kernels, roof)


def bench_across(args, cfg, sbp, wl, torch, np):
    """Boxing between disjoint placements (Sec. 3.2, Table 2 column "disjoint"): a pipeline-stage
    boundary where the producer runs on 8 logical devices and the consumer on 4 others.  Activations
    T[16384,16384] 16-bit words: S(0) on 8 -> S(0) on 4, S(0) on 8 -> B on 4; partial results
    [8192,4096] fp32: P(sum) on 8 -> B on 4, P(sum) on 8 -> S(0) on 4."""
    ki, ko = 8, 4
    R, C = 16384, 16384
    arena = make_arena(torch, np, args)
    a8 = arena([(R // ki, C)] * ki, torch.int16)
    for i in range(ki):
        a8[i].copy_(torch.from_numpy(wl.pattern_u16((R, C), rows=np.arange(i * (R // ki), (i + 1) * (R // ki))).view(np.int16)))
    a4 = arena([(R // ko, C)] * ko, torch.int16)
    b4 = arena([(R, C)] * ko, torch.int16)
    PR, PC = 8192, 4096
    p8 = arena([(PR, PC)] * ki, torch.float32)
    for i in range(ki):
        p8[i].normal_(0.0, 0.02)
    pb4 = arena([(PR, PC)] * ko, torch.float32)
    ps4 = arena([(PR // ko, PC)] * ko, torch.float32)
    A8, A4, B4 = (sbp.SbpTensor(x, R, C, sbp.BF16) for x in (a8, a4, b4))
    P8, PB4, PS4 = (sbp.SbpTensor(x, PR, PC, sbp.F32) for x in (p8, pb4, ps4))

    def stages_of(s):
        return [lambda st: sbp.sbp_boxing_across(A8, sbp.S(0), ki, A4, sbp.S(0), ko, st),
                lambda st: sbp.sbp_boxing_across(A8, sbp.S(0), ki, B4, sbp.B, ko, st),
                lambda st: sbp.sbp_boxing_across(P8, sbp.P_SUM, ki, PB4, sbp.B, ko, st),
                lambda st: sbp.sbp_boxing_across(P8, sbp.P_SUM, ki, PS4, sbp.S(0), ko, st)]

    ms, wall = time_stages(torch, stages_of, args.steps, args.warmup)
    t, pt = 2.0 * R * C, 4.0 * PR * PC
    by = [2 * t, (1 + ko) * t, (ki + ko) * pt, (ki + 1) * pt]
    g = [by[i] / ms[i] / 1e6 for i in range(4)]
    names = ["s0x8_to_s0x4", "s0x8_to_bx4", "psumx8_to_bx4", "psumx8_to_s0x4"]
    kernels = {}
    for n, m, r in zip(names, ms, g):
        kernels[n + "_ms"] = round(m, 4)
        kernels[n + "_gbps"] = round(r, 1)
    roof = {"bound": "hbm", "kernel": "sbp_boxing_across P(sum) on 8 -> B on 4 (8 x 128 MiB read, 4 x 128 MiB written)",
            "achieved": round(g[2], 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(g[2] / PEAK_HBM_GBPS, 4), "traffic": None}
    return result_line(args, "boxing between placements, 8 -> 4 logical devices: T[16384,16384] 16-bit words S(0)->S(0), S(0)->B; "
                             "[8192,4096] fp32 partials P(sum)->B, P(sum)->S(0)",
                       ki, sum(by) / (wall * 1e-3) / 1e9, "GB/s", wall, kernels, roof)


class ClockSampler:
    """Samples the shader clock with `rocm-smi --showclocks` on a thread while a sustained GPU loop runs."""

    def __init__(self):
        import threading
        self.clocks, self._stop = [], threading.Event()
        self._th = threading.Thread(target=self._run)

    def _run(self):
        import subprocess
        while not self._stop.is_set():
            try:
                txt = subprocess.run(["/opt/rocm/bin/rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=10).stdout
                for ln in txt.splitlines():
                    if "sclk" in ln and "Mhz" in ln:
                        self.clocks.append(int(ln.split("(")[1].split("Mhz")[0]))
            except Exception:
                pass
            self._stop.wait(0.3)

    def __enter__(self):
        self._th.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._th.join()

    def median(self):
        c = sorted(self.clocks[1:]) if len(self.clocks) > 2 else sorted(self.clocks)
        return c[len(c) // 2] if c else None


def sustained(torch, call, seconds, batch):
    """Runs call() back to back for about `seconds`, the shader clock sampled beside it.
    Returns (ms per call, calls, median sclk MHz)."""
    for _ in range(3):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with ClockSampler() as cs:
        t0, n = time.perf_counter(), 0
        e0.record()
        while time.perf_counter() - t0 < seconds:
            for _ in range(batch):
                call()
            n += batch
            torch.cuda.synchronize()
        e1.record()
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n, n, cs.median()


def bench_mfma_probe(args, cfg, sbp, wl, torch, np):
    """Diagnostic, not a workload of the paper: what the matrix pipes sustain on this chip with the GEMM kernels'
    instruction (v_mfma_f32_16x16x32_bf16, 8 waves per compute unit), alone (mode 0), with the operand fragment
    reads of the lockstep GEMM schedule (mode 1) and of the ping-pong schedule (mode 2), each with pseudo-random
    and with all-zero operands, run for about 1.5 seconds each with the shader clock sampled.  The kernels
    count shader cycles themselves: cycles per round of 32 matrix instructions per wave (two waves share a
    SIMD, so 64 instructions of 16 cycles = 1024 cycles is the floor), and cycles / time = the clock that was
    actually granted."""
    iters = 2000
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    scratch = torch.zeros((16 << 20) + (3 << 29), dtype=torch.uint8, device="cuda")   # 16 MiB + 1.5 GiB: what modes 7 and 8 walk
    scratch.random_(0, 256)
    flop = cus * 8.0 * iters * 32 * (2 * 16 * 16 * 32)
    kernels, best = {}, 0.0
    for mode, name in ((0, "mfma_only"), (3, "mfma_only_32x32x16"), (1, "lockstep_reads"), (2, "pingpong_reads"), (4, "pingpong_12_reads"), (5, "pingpong_8_reads"), (6, "pingpong_12_reads_l2_operand_stream"),
                       (7, "pingpong_12_reads_operand_stream_quarter_from_hbm"), (8, "pingpong_12_reads_operand_stream_and_stores")):
        for zero, zname in ((0, "random"), (1, "zeros")):
            ms, n, sclk = sustained(torch, lambda: sbp.sbp_probe_mfma(mode, iters, zero, scratch), 1.5, 100)
            cyc = scratch[:64].cpu().view(torch.int64).numpy()
            per_round = float(cyc.max()) / iters
            tf = flop / ms / 1e9
            kernels[f"{name}_{zname}"] = {"ms": round(ms, 4), "tflops": round(tf, 1), "cycles_per_round": round(per_round, 1),
                                          "granted_clock_mhz": round(float(cyc.max()) / ms / 1e3, 0), "sclk_mhz_smi": sclk, "calls": n}
            if zero == 0:
                best = max(best, tf)
    roof = {"bound": "mfma", "kernel": "probe_mfma_kernel, pseudo-random operands, best of the three schedules", "achieved": round(best, 1),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(best / PEAK_BF16_TFLOPS, 4), "traffic": None}
    return result_line(args, "diagnostic: v_mfma_f32_16x16x32_bf16 alone / with lockstep fragment reads / in ping-pong, 8 waves per CU, "
                             "random and zero operands, sustained 1.5 s each", 1, best, "TFLOP/s", kernels["mfma_only_random"]["ms"], kernels, roof)


def bench_vendor_gemm(args, cfg, sbp, wl, torch, np):
    """Diagnostic, not part of the path: the vendor GEMM library (through torch.bmm / torch.matmul, bf16 in, bf16 out)
    on the three GEMM shapes of the workloads and on the unsharded logical products, N(0, 0.02) operands, sustained
    two seconds each with the shader clock sampled.  Context for the hand-written kernels' rate on the same chip;
    its outputs are bf16 where the path writes fp32 partials, so it moves fewer bytes than the path does.  The path's
    own kernels then run on the same operand tensors, timed the same way ("ours_" entries): a like-for-like
    comparison on one box in one run (the workload benches time the kernels inside their steps instead, between
    other kernels and on rotating buffers)."""
    g = torch.Generator(device="cuda").manual_seed(1234)

    def rnd(*shape):
        return (torch.randn(*shape, generator=g, device="cuda") * 0.02).to(torch.bfloat16)

    cases = []
    x, w1 = rnd(8192, 4096), rnd(8, 4096, 2048)
    cases.append(("mlp_gemm1_8x[8192,4096]x[4096,2048]", lambda: torch.matmul(x, w1), 2.0 * 8 * 8192 * 4096 * 2048))
    h, w2 = rnd(8, 8192, 2048), rnd(8, 2048, 4096)
    cases.append(("mlp_gemm2_8x[8192,2048]x[2048,4096]", lambda: torch.bmm(h, w2), 2.0 * 8 * 8192 * 2048 * 4096))
    W1f, W2f, hf = rnd(4096, 16384), rnd(16384, 4096), rnd(8192, 16384)
    cases.append(("mlp_gemm1_unsharded_[8192,4096]x[4096,16384]", lambda: torch.matmul(x, W1f), 2.0 * 8192 * 4096 * 16384))
    cases.append(("mlp_gemm2_unsharded_[8192,16384]x[16384,4096]", lambda: torch.matmul(hf, W2f), 2.0 * 8192 * 16384 * 4096))
    xs, dy = rnd(8, 2048, 1024), rnd(8, 2048, 4096)
    cases.append(("dp_grad_tn_8x[2048,1024]^T x[2048,4096]", lambda: torch.bmm(xs.transpose(1, 2), dy), 2.0 * 8 * 2048 * 1024 * 4096))
    f, wc = rnd(1024, 512), rnd(8, 512, 125000)
    cases.append(("classifier_8x[1024,512]x[512,125000]", lambda: torch.matmul(f, wc), 2.0 * 8 * 1024 * 512 * 125000))
    # the path's own kernels on the very same operand tensors, timed the same way in the same run (GEMM1 with and
    # without its GeLU; GEMM2 and the weight gradient write fp32 partials, the classifier bf16 logits on rows padded to
    # 128 bytes with the row maximum fused): "ours_" entries
    def shards(t):
        return [t[i] for i in range(t.shape[0])]

    k = 8
    hs = torch.empty(8, 8192, 2048, dtype=torch.bfloat16, device="cuda")
    y2 = torch.empty(8, 8192, 4096, dtype=torch.float32, device="cuda")
    dw = torch.empty(8, 1024, 4096, dtype=torch.float32, device="cuda")
    PL = (125000 + 63) // 64 * 64
    lg = torch.empty(8, 1024, PL, dtype=torch.bfloat16, device="cuda")
    mx = torch.empty(8, 1024, 1, dtype=torch.float32, device="cuda")
    Xb, W1 = sbp.SbpTensor([x] * k, 8192, 4096, sbp.BF16), sbp.SbpTensor(shards(w1), 4096, 16384, sbp.BF16)
    Hs = sbp.SbpTensor(shards(hs), 8192, 16384, sbp.BF16)
    H2, W2, Y2 = sbp.SbpTensor(shards(h), 8192, 16384, sbp.BF16), sbp.SbpTensor(shards(w2), 16384, 4096, sbp.BF16), sbp.SbpTensor(shards(y2), 8192, 4096, sbp.F32)
    XT, DY, DW = sbp.SbpTensor(shards(xs), 1024, 16384, sbp.BF16, 1), sbp.SbpTensor(shards(dy), 16384, 4096, sbp.BF16), sbp.SbpTensor(shards(dw), 1024, 4096, sbp.F32)
    Fc, Wc = sbp.SbpTensor([f] * k, 1024, 512, sbp.BF16), sbp.SbpTensor(shards(wc), 512, 1000000, sbp.BF16)
    Lg, Mx = sbp.SbpTensor(shards(lg), 1024, 1000000, sbp.BF16, 0, PL), sbp.SbpTensor(shards(mx), 1024, 1, sbp.F32)
    ours = [("ours_mlp_gemm1_no_epilogue", lambda: sbp.sbp_matmul(Xb, sbp.B, W1, sbp.S(1), Hs, sbp.S(1), k), cases[0][2]),
            ("ours_mlp_gemm1_gelu", lambda: sbp.sbp_matmul_ex(Xb, sbp.B, W1, sbp.S(1), Hs, sbp.S(1), k, None, sbp.EPI_GELU), cases[0][2]),
            ("ours_mlp_gemm2_fp32_partials", lambda: sbp.sbp_matmul(H2, sbp.S(1), W2, sbp.S(0), Y2, sbp.P_SUM, k), cases[1][2]),
            ("ours_dp_grad_tn_fp32_partials", lambda: sbp.sbp_matmul(XT, sbp.S(1), DY, sbp.S(0), DW, sbp.P_SUM, k), cases[4][2]),
            ("ours_classifier_rowmax_padded_rows", lambda: sbp.sbp_matmul_rowmax(Fc, sbp.B, Wc, sbp.S(1), Lg, sbp.S(1), Mx, k), cases[5][2])]
    kernels, best = {}, 0.0
    for name, call, flop in cases + ours:
        ms, n, sclk = sustained(torch, call, 2.0, 50)
        tf = flop / ms / 1e9
        kernels[name] = {"ms": round(ms, 4), "tflops": round(tf, 1), "sclk_mhz_smi": sclk, "calls": n}
        if not name.startswith("ours_"):
            best = max(best, tf)
    roof = {"bound": "mfma", "kernel": "vendor library GEMM through torch (bf16 out), best shape", "achieved": round(best, 1),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(best / PEAK_BF16_TFLOPS, 4), "traffic": None}
    return result_line(args, "diagnostic: vendor-library bf16 GEMM (torch.matmul / torch.bmm) on the workloads' GEMM shapes, sustained 2 s each",
                       8, best, "TFLOP/s", kernels[cases[0][0]]["ms"], kernels, roof)


def bench_clock_probe(args, cfg, sbp, wl, torch, np):
    """Diagnostic, not a workload of the paper: GEMM2 of the MLP block, (S1,S0)->P(sum), run back to back for
    three seconds with N(0, 0.02) operands and again with all-zero operands, with the lockstep kernel (the
    default for this shape) and with the ping-pong kernel (variant 21), while `rocm-smi --showclocks` samples
    the shader clock.  Same kernels, same launches: the difference between the operand sets is what the chip's
    power management does with the operand data."""
    k, M, N, K = 8, 8192, 4096, 16384
    arena = make_arena(torch, np, args)
    kernels, res = {}, {}
    for mode in ("normal", "zero"):
        xs = arena([(M, K // k)] * k, torch.bfloat16)
        ws = arena([(K // k, N)] * k, torch.bfloat16)
        ys = arena([(M, N)] * k, torch.float32)
        for t in xs + ws:
            t.zero_() if mode == "zero" else t.normal_(0.0, 0.02)
        X, W, Y = sbp.SbpTensor(xs, M, K, sbp.BF16), sbp.SbpTensor(ws, K, N, sbp.BF16), sbp.SbpTensor(ys, M, N, sbp.F32)
        for variant, vname in ((args.variant, "gemm2"), (21, "gemm2_pingpong")):
            sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, variant)
            ms, n, sclk = sustained(torch, lambda: sbp.sbp_matmul(X, sbp.S(1), W, sbp.S(0), Y, sbp.P_SUM, k), 3.0, 50)
            res[(vname, mode)] = (ms, 2.0 * M * N * K / ms / 1e9)
            kernels[f"{vname}_{mode}_ms"] = round(ms, 4)
            kernels[f"{vname}_{mode}_tflops"] = round(res[(vname, mode)][1], 1)
            kernels[f"{vname}_{mode}_sclk_mhz"] = sclk
            kernels[f"{vname}_{mode}_calls"] = n
        sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, args.variant)
        del xs, ws, ys, X, W, Y
        torch.cuda.empty_cache()
    ms, tf = res[("gemm2", "normal")]
    roof = {"bound": "mfma", "kernel": "sbp_matmul (S1,S0)->P(sum), N(0,0.02) operands, sustained", "achieved": round(tf, 1),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4), "traffic": None}
    return result_line(args, "diagnostic: sustained GEMM2 of the MLP block with N(0,0.02) and with all-zero operands, lockstep and ping-pong kernels, "
                             "shader clock sampled", k, tf, "TFLOP/s", ms, kernels, roof)


def bench_tiny(args, cfg, sbp, wl, torch, np):
    """The small fp32 configuration (k = 2): latency only.  X[64,128] S(1) x W[128,96] S(0) -> 2 fp32 partials
    [64,96]; boxing P(sum)->B and P(sum)->S(0).  Reported in microseconds per call."""
    k = cfg["k"]
    (M, K), N = cfg["X"]["shape"], cfg["W"]["shape"][1]
    x = [torch.from_numpy(wl.uniform(wl.SEED_BASE, cfg["X"]["id"], (M, K), -1.0, 1.0, None, np.arange(*shard_range(K, k, i)))
                          .astype(np.float32)).cuda().contiguous() for i in range(k)]
    w = [torch.from_numpy(wl.uniform(wl.SEED_BASE, cfg["W"]["id"], (K, N), -1.0, 1.0, np.arange(*shard_range(K, k, i)), None)
                          .astype(np.float32)).cuda().contiguous() for i in range(k)]
    y = [torch.empty(M, N, dtype=torch.float32, device="cuda") for _ in range(k)]
    yb = [torch.empty(M, N, dtype=torch.float32, device="cuda") for _ in range(k)]
    ys = [torch.empty(shard_range(M, k, i)[1] - shard_range(M, k, i)[0], N, dtype=torch.float32, device="cuda") for i in range(k)]
    X, W = sbp.SbpTensor(x, M, K, sbp.F32), sbp.SbpTensor(w, K, N, sbp.F32)
    Y, YB, YS = (sbp.SbpTensor(t, M, N, sbp.F32) for t in (y, yb, ys))

    def stages_of(s):
        return [lambda st: sbp.sbp_matmul(X, sbp.S(1), W, sbp.S(0), Y, sbp.P_SUM, k, st),
                lambda st: sbp.sbp_boxing(Y, sbp.P_SUM, YB, sbp.B, k, st),
                lambda st: sbp.sbp_boxing(Y, sbp.P_SUM, YS, sbp.S(0), k, st)]

    ms, wall = time_stages(torch, stages_of, max(args.steps, 200), max(args.warmup, 20))
    ref = sum(a.double() @ b.double() for a, b in zip(x, w))
    err = float((yb[0].double() - ref).abs().max() / ref.abs().max())
    kernels = {"matmul_us": round(ms[0] * 1e3, 2), "boxing_p2b_us": round(ms[1] * 1e3, 2), "boxing_p2s_us": round(ms[2] * 1e3, 2),
               "max_rel_err_after_p2b": err, "timed_calls": max(args.steps, 200)}
    roof = {"bound": "latency", "kernel": "sbp_matmul fp32 64x128x96 on 2 devices", "achieved": round(ms[0] * 1e3, 2), "peak": None,
            "unit": "us per call", "frac": None, "traffic": None}
    flops = 2.0 * M * K * N
    return result_line(args, "small fp32 configuration, k=2: X[64,128] S(1) x W[128,96] S(0) -> P(sum); boxing P->B, P->S(0); latency only",
                       k, flops / (wall * 1e-3) / 1e12, "TFLOP/s", wall, kernels, roof, dtype="f32")


def bench_grid(args, cfg, sbp, wl, torch, np):
    """Two-dimensional SBP (Sec. 3.3, Table 3) on a 2 x 4 grid of logical devices, at the MLP block's sizes:
    row 1: X[8192,4096] (S(0),B) x W[4096,16384] (B,S(1)) -> Y (S(0),S(1)) bf16;
    row 2: X[8192,16384] (S(0),S(1)) x W[16384,4096] (B,S(0)) -> Y (S(0),P(sum)) fp32, then boxing along the
    inner axis (S(0),P) -> (S(0),B): an all-reduce inside each group of 4."""
    k0, k1 = 2, 4
    k = k0 * k1
    S0, S1, B_, P = sbp.S(0), sbp.S(1), sbp.B, sbp.P_SUM
    arena = make_arena(torch, np, args)

    def fill(ts, std):
        for t in ts:
            t.view(torch.bfloat16).normal_(0.0, std)
        return ts

    M, D, F = 8192, 4096, 16384
    x1 = fill(arena([(M // k0, D)] * k, torch.int16), 1.0)            # (S0, B): rows by group, copies inside
    w1 = fill(arena([(D, F // k1)] * k, torch.int16), 0.02)           # (B, S1): columns by device inside every group
    y1 = arena([(M // k0, F // k1)] * k, torch.int16)
    x2 = fill(arena([(M // k0, F // k1)] * k, torch.int16), 1.0)      # (S0, S1)
    w2 = fill(arena([(F // k1, D)] * k, torch.int16), 0.02)           # (B, S0): rows by device inside every group
    y2 = arena([(M // k0, D)] * k, torch.float32)                     # (S0, P)
    y2b = arena([(M // k0, D)] * k, torch.float32)                    # (S0, B)
    X1, W1, Y1 = sbp.SbpTensor(x1, M, D, sbp.BF16), sbp.SbpTensor(w1, D, F, sbp.BF16), sbp.SbpTensor(y1, M, F, sbp.BF16)
    X2, W2 = sbp.SbpTensor(x2, M, F, sbp.BF16), sbp.SbpTensor(w2, F, D, sbp.BF16)
    Y2, Y2B = sbp.SbpTensor(y2, M, D, sbp.F32), sbp.SbpTensor(y2b, M, D, sbp.F32)

    def stages_of(s):
        return [lambda st: sbp.sbp_matmul_2d(X1, (S0, B_), W1, (B_, S1), Y1, (S0, S1), k0, k1, st),
                lambda st: sbp.sbp_matmul_2d(X2, (S0, S1), W2, (B_, S0), Y2, (S0, P), k0, k1, st),
                lambda st: sbp.sbp_boxing_2d(Y2, (S0, P), Y2B, (S0, B_), k0, k1, st)]

    ms, wall = time_stages(torch, stages_of, args.steps, args.warmup)
    flops = 2.0 * M * D * F
    box_bytes = 2.0 * k * (M // k0) * D * 4
    kernels = {"row1_s0b_x_bs1_ms": round(ms[0], 4), "row1_tflops": round(flops / ms[0] / 1e9, 2),
               "row2_s0s1_x_bs0_ms": round(ms[1], 4), "row2_tflops": round(flops / ms[1] / 1e9, 2),
               "boxing_inner_p2b_ms": round(ms[2], 4), "boxing_inner_p2b_gbps": round(box_bytes / ms[2] / 1e6, 1)}
    tf = flops / ms[1] / 1e9
    roof = {"bound": "mfma", "kernel": "sbp_matmul_2d (S(0),S(1)) x (B,S(0)) -> (S(0),P(sum))", "achieved": round(tf, 2),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4), "traffic": None}
    return result_line(args, "two-dimensional SBP on a 2 x 4 grid: Table 3 row 1 and row 2 at the MLP block's sizes, "
                             "all-reduce of the partial results inside every group",
                       k, 2 * flops / (wall * 1e-3) / 1e12, "TFLOP/s", wall, kernels, roof)


OTHER_WORKLOADS = {"mfma_probe": bench_mfma_probe, "vendor_gemm": bench_vendor_gemm, "grid": bench_grid, "tiny": bench_tiny, "clock_probe": bench_clock_probe, "across": bench_across, "dp_grad": bench_dp_grad, "classifier": bench_classifier, "relayout": bench_relayout, "uvw": bench_uvw,
                   "zero": bench_zero}


def cpu_baseline(cfg, k, rows, seed):
    """The oracle, as it stands, on the first `rows` tokens of the same workload: per-shard GEMM1,
    GeLU, bf16 rounding, per-shard GEMM2 partials, P(sum)->B.  Same algorithmic FLOP count per
    token as the GPU step."""
    import numpy as np

    import oracle as orc
    import workloads as wl

    T, D = cfg["X"]["shape"]
    F = cfg["W1"]["shape"][1]
    r = np.arange(rows)
    Xs = orc.bf16_to_f64(wl.to_bf16_bits(wl.normal(seed, cfg["X"]["id"], (T, D), 1.0, rows=r)))
    W1 = orc.bf16_to_f64(wl.to_bf16_bits(wl.normal(seed, cfg["W1"]["id"], (D, F), cfg["W1"]["dist"][1])))
    W2 = orc.bf16_to_f64(wl.to_bf16_bits(wl.normal(seed, cfg["W2"]["id"], (F, D), cfg["W2"]["dist"][1])))
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    t0 = time.perf_counter()
    Hs, s_h = orc.matmul_sbp(orc.scatter(Xs, orc.B, k), orc.B, orc.scatter(W1, orc.S1, k), orc.S1)
    Hs = [orc.bf16_to_f64(orc.bf16_round(orc.gelu(h))) for h in Hs]
    Ys, s_y = orc.matmul_sbp(Hs, orc.S1, orc.scatter(W2, orc.S0, k), orc.S0)
    Yb = orc.boxing(Ys, s_y, orc.B, k)
    dt = time.perf_counter() - t0
    flops = 2 * 2.0 * rows * D * F
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"first {rows} of {T} tokens through the whole step (GEMM1+GeLU, GEMM2 partials, P->B), "
                      f"{flops / 1e9:.1f} GFLOP in {dt:.2f} s",
            "checksum": float(np.sum(Yb[0]))}


if __name__ == "__main__":
    main()
