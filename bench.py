#!/usr/bin/env python3
"""Benchmark of the group-quantized linear hot path on one MI355X.

Workload (benchmark configs[1]): the four linears of one BERT-base encoder layer
(QKV 768->2304, out 768->768, FFN 768->3072, 3072->768) on 32x128 = 4096 tokens, 128 groups per
matrix, weight bit-widths {2,3,4,8}, forward only, synthetic seeded data.

One step = one pass of the forward hot path over that batch for every bit-width of the sweep:
  16 x quantize/pack of fp32 master weights (16 distinct matrices, one batched launch), 4 x 8-bit activation
  quantize (one batched launch), 16 x int8 MFMA GEMM with the scale epilogue (one batched call: per bit-width one
  persistent launch walks the 2304 tiles of QKV, attention-out, FFN-up and FFN-down: 4 launches).
All inputs are resident in HBM before the timed region.  `value` = int8 GEMM operations of the
step (2*T*N*K summed) divided by the wall time of the whole step, in TOPS.

The timed region replays captured HIP graphs that hold nothing but the 6 kernels of a step, five whole steps per
graph (--steps-per-graph; consecutive replays of a one-step graph leave the GPU idle for about 8 us in between);
--no-graph launches every kernel eagerly instead.  Before the warm-up steps the step is
replayed for at least 60 ms so that the clocks have settled whatever --warmup says.  The per-kernel
averages in `roofline` and `kernels` come from a second pass in the same run, on the same stream: the GEMM
launches (and the 4 activation quantizers, four times over) as one graph, replayed ten times between two
HIP events; the quantize/pack kernel on three distinct copies of the step's matrices (339 MB, one launch), so that
no repetition finds its weights in the 256 MB last-level cache.

Also printed on the same JSON line: every GEMM shape on its own (one launch, and four independent problems of
the shape in one batched call), the STE backward (configs[2]), one iteration of the 12-layer stack
(configs[3]: quantize/pack + act-quant + forward + backward at 12288 tokens with per-layer bits), BERT-large
(configs[4]: GEMMs at 32768 tokens, the 24-layer quantize/pack aggregate over 1.2 GB of distinct weights, the
embedding path), all timed outside the K steps, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, published
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
T_TOKENS = 4096
GROUPS = 128
CLIP = 6.0
BITS_SWEEP = (2, 3, 4, 8)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-graph", action="store_true", help="launch kernels eagerly instead of replaying HIP graphs")
    ap.add_argument("--steps-per-graph", type=int, default=5,
                    help="whole steps captured back to back in one HIP graph (1: one graph replay per step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--single-launches", action="store_true",
                    help="one launch per GEMM (16 qb_qlinear_fwd calls) instead of the batched call")
    ap.add_argument("--no-extras", action="store_true", help="skip the backward and embedding timings")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy three times (reference dispatch for HBM byte counters)")
    ap.add_argument("--gemm-only", type=str, default=None, metavar="T,N,K,BITS",
                    help="run only this GEMM shape (30 single launches of qb_qlinear_fwd, then 10 batched calls of four "
                         "independent problems) and print its timing: the command profiled for per-shape counters")
    ap.add_argument("--stack-only", action="store_true",
                    help="run only the 12-layer iteration (configs[3]) and print its result: the command profiled for the "
                         "split of a fine-tuning iteration over its kernels")
    ap.add_argument("--backward-only", action="store_true",
                    help="run only the STE-backward leg (configs[2]) and print its result: the command profiled for "
                         "the backward kernels")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1909_05840_amd as qb
    from paper_1909_05840_amd import workloads as wl

    qb.load_library()   # raises if the HIP library is not built: there is no other path
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    linears = wl.BERT_BASE_LINEARS
    T = T_TOKENS
    if args.backward_only:
        print(json.dumps({"backward": backward_leg(torch, qb, wl, dev)}))
        return
    if args.stack_only:
        print(json.dumps({"stack_12_layers": stack_leg(torch, qb, wl, dev)}))
        return
    if args.gemm_only:
        print(json.dumps({"gemm": gemm_only_leg(torch, qb, wl, dev, [int(v) for v in args.gemm_only.split(",")])}))
        return

    # ---- inputs, resident in HBM ---------------------------------------------------------------
    # one fp32 master matrix per (bit-width, linear): 16 distinct matrices, 113 MB, so that no quantize/pack
    # job finds its input in a cache because another job of the launch has just read it
    Ws = {(b, i): wl.weight(N, K, seed=wl.config_seed(1, 100 * b + i)).to(dev)
          for b in BITS_SWEEP for i, (_, N, K) in enumerate(linears)}
    Xs = [wl.activation(T, K, seed=wl.config_seed(1, 10 + i)).to(dev) for i, (_, N, K) in enumerate(linears)]
    # ---- outputs, allocated once -----------------------------------------------------------------
    q = {}
    for b in BITS_SWEEP:
        for i, (_, N, K) in enumerate(linears):
            q[(b, i)] = dict(packed=torch.empty(qb.qb_packed_nbytes(N, K, b), dtype=torch.uint8, device=dev),
                             h=torch.empty(GROUPS, dtype=torch.float32, device=dev),
                             m=torch.empty(GROUPS, dtype=torch.float32, device=dev),
                             rs_w=torch.empty(N, dtype=torch.int32, device=dev))
    acts = [dict(Xq=torch.empty((T, K), dtype=torch.int8, device=dev),
                 rs_x=torch.empty(T, dtype=torch.int32, device=dev)) for (_, N, K) in linears]
    # the 16 GEMMs of a step are independent jobs of one batched call: each has its own output
    Ys = {(b, i): torch.empty((T, N), dtype=torch.float32, device=dev)
          for b in BITS_SWEEP for i, (_, N, K) in enumerate(linears)}

    quant_jobs = [dict(W=Ws[(b, i)], bits=b, groups=GROUPS, **q[(b, i)]) for b in BITS_SWEEP for i in range(len(linears))]
    gemm_jobs = [dict(Xq=acts[i]["Xq"], rs_x=acts[i]["rs_x"], clip=CLIP, packed=q[(b, i)]["packed"], h=q[(b, i)]["h"],
                      rs_w=q[(b, i)]["rs_w"], bits=b, groups=GROUPS, N=N, Y=Ys[(b, i)])
                 for b in BITS_SWEEP for i, (_, N, K) in enumerate(linears)]

    def stage_quantize():
        qb.qb_quantize_groupwise_batched(quant_jobs)   # all 16 matrices of the step, one launch

    act_jobs = [dict(X=Xs[i], clip=CLIP, Xq=acts[i]["Xq"], rs_x=acts[i]["rs_x"]) for i in range(len(linears))]

    def stage_act():
        if args.single_launches:
            for i in range(len(linears)):
                qb.qb_quantize_act(Xs[i], CLIP, acts[i]["Xq"], acts[i]["rs_x"])
        else:
            qb.qb_quantize_act_batched(act_jobs)   # the layer's four input tensors, one launch

    def stage_gemm():
        if args.single_launches:   # one launch per linear, as separate qb_qlinear_fwd calls
            for j in gemm_jobs:
                qb.qb_qlinear_fwd(j["Xq"], j["rs_x"], CLIP, j["packed"], j["h"], j["rs_w"], j["bits"], GROUPS, j["N"], Y=j["Y"])
        else:
            qb.qb_qlinear_fwd_batched(gemm_jobs)   # one persistent launch per bit-width

    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    stages = [stage_quantize, stage_act, stage_gemm]
    n_quant = 1                            # kernels per stage
    n_act = 4 if args.single_launches else 1
    n_gemm = 16 if args.single_launches else len(BITS_SWEEP)   # one persistent launch per bit-width walks all four linears
    stream = torch.cuda.Stream(device=dev)   # default priority
    use_graph = not args.no_graph

    def whole_step():
        for s in stages:
            s()

    def capture(fn):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            fn()
        return g.replay

    with torch.cuda.stream(stream):
        whole_step()
        stream.synchronize()
        one_step = capture(whole_step) if use_graph else whole_step
        # Consecutive replays of a one-step graph leave the GPU idle for about 8 us between them (the host's graph launch,
        # seen in the kernel trace as the only gap of a step).  A training loop captures more than one layer's step at a
        # time; here a second graph holds GRAPH_STEPS whole steps back to back, and K steps are K // GRAPH_STEPS replays of
        # it plus K % GRAPH_STEPS replays of the one-step graph.
        many_steps = None
        if use_graph and args.steps_per_graph > 1:
            def several():
                for _ in range(args.steps_per_graph):
                    whole_step()
            many_steps = capture(several)

        def run_steps(k):
            if many_steps is not None:
                for _ in range(k // args.steps_per_graph):
                    many_steps()
                k %= args.steps_per_graph
            for _ in range(k):
                one_step()
        # settle the clocks: the first tens of milliseconds after idle run at other clocks than the steady state
        t_w = time.perf_counter()
        while time.perf_counter() - t_w < 0.06:
            run_steps(20)
            stream.synchronize()
        run_steps(args.warmup)
        stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(args.steps)
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()

        # ---- per-kernel pass: each stage on its own, thirty replays between two events.
        # The quantize/pack stage of the step is one launch over 113 MB of weights, which would stay in the 256 MB
        # last-level cache from one repetition to the next (inside a step the GEMM outputs evict them).  Its
        # figure is therefore taken on THREE distinct copies of the step's 16 matrices (48 jobs, 339 MB of weights,
        # still one launch of the same kernel): every repetition then reads its weights from HBM.  For reference
        # the step's own launch is also timed behind a 512 MiB fill, as the difference to the fill alone; that
        # way charges the quantizer with the write-back of the fill's dirty lines.
        def timed(run, n=30, settle_ms=25.0):
            # the stage is first repeated for settle_ms: after a change of kernel mix the chip's clocks take tens of
            # milliseconds to settle (a GEMM stage timed right behind the memory-bound stages came out 13 % slow)
            t_s = time.perf_counter()
            while True:
                for _ in range(5):
                    run()
                stream.synchronize()
                if (time.perf_counter() - t_s) * 1e3 >= settle_ms:
                    break
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(n):
                run()
            e1.record(stream)
            stream.synchronize()
            return e0.elapsed_time(e1) / n

        seg_ms = []
        big_jobs = list(quant_jobs)
        for rep in range(2):
            for j in quant_jobs:
                big_jobs.append(dict(W=j["W"].clone(), bits=j["bits"], groups=GROUPS,
                                     **{k: torch.empty_like(j[k]) for k in ("packed", "h", "m", "rs_w")}))

        def quant_big():
            qb.qb_quantize_groupwise_batched(big_jobs)
        seg_ms.append(timed(capture(quant_big) if use_graph else quant_big) / 3.0)   # per 16 matrices
        flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)

        def fill_only():
            flush.zero_()

        def fill_quant():
            flush.zero_()
            stage_quantize()
        if use_graph:
            quant_after_fill_ms = timed(capture(fill_quant)) - timed(capture(fill_only))
        else:
            quant_after_fill_ms = timed(fill_quant) - timed(fill_only)
        del flush, big_jobs
        for fn, nk in zip(stages[1:], (n_act, n_gemm)):
            reps = max(1, 16 // nk) if fn is stage_act else 1   # the short activation stage is repeated inside its graph

            def many(fn=fn, reps=reps):
                for _ in range(reps):
                    fn()
            run = capture(many) if use_graph else many
            seg_ms.append(timed(run) / reps)   # one pass over the stage

    wall = t1 - t0
    ms_per_step = wall * 1e3 / args.steps

    # ---- algorithmic work of one step ----------------------------------------------------------------
    gemm_ops = sum(2.0 * T * N * K for (_, N, K) in linears) * len(BITS_SWEEP)
    quant_bytes = sum(N * K * (4.0 + b / 8.0) + GROUPS * 8 + N * 4 for b in BITS_SWEEP for (_, N, K) in linears)
    act_bytes = sum(T * K * 5.0 + T * 4 for (_, N, K) in linears)
    gemm_bytes = sum(T * K + N * K * b / 8.0 + 4.0 * T * N + 4 * T + 4 * N for b in BITS_SWEEP for (_, N, K) in linears)
    gemm_tops = gemm_ops / (seg_ms[2] * 1e-3) / 1e12
    mfma_peak = measured_mfma_peak(torch, qb, dev)
    quant_gbs = quant_bytes / (seg_ms[0] * 1e-3) / 1e9
    act_gbs = act_bytes / (seg_ms[1] * 1e-3) / 1e9
    value = gemm_ops / (wall / args.steps) / 1e12

    out = {
        "metric": "group-quant int8 GEMM TOPS & % int8 MFMA peak; quantize/pack GB/s",
        "value": round(value, 3), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "configs[1]: BERT-base encoder layer, 4 linears (QKV 768->2304, out 768->768, "
                               "FFN 768->3072, 3072->768), tokens 32x128=4096, 128 groups, bits {2,3,4,8}, fwd only; "
                               "step = 16 quantize/pack (16 distinct fp32 matrices, 1 launch) + 4 act-quant (1 launch) + 16 int8 GEMM+epilogue",
                   "tokens": T, "groups": GROUPS, "bits": list(BITS_SWEEP), "hip_graph": use_graph,
                   "steps_per_graph": args.steps_per_graph if use_graph else 0,
                   "gemm_launches_per_step": n_gemm},
        "roofline": {"kernel": "qgemm_i8_ws_kernel (int8 MFMA GEMM + scale epilogue; per bit-width one persistent launch "
                               "walks the 128x96 tiles of QKV, attention-out, FFN-up and FFN-down), "
                               "%d launches per step" % n_gemm,
                     "bound": "mfma", "achieved": round(gemm_tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": round(gemm_tops / PEAK_INT8_TOPS, 4), "traffic": measured_traffic("qgemm_i8"),
                     "avg_launch_us": round(seg_ms[2] * 1e3 / n_gemm, 3),
                     "ops_per_launch": gemm_ops / n_gemm,
                     # with fp32 outputs the step's GEMMs sit below the machine balance (625 op/B): by the roofline
                     # model their bound is HBM; both fractions are given
                     "hbm_side": {"bytes_per_launch": gemm_bytes / n_gemm,
                                  "achieved_gbs": round(gemm_bytes / (seg_ms[2] * 1e-3) / 1e9, 1),
                                  "frac_hbm_peak": round(gemm_bytes / (seg_ms[2] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                  "intensity_op_per_byte": round(gemm_ops / gemm_bytes, 1),
                                  "machine_balance_op_per_byte": PEAK_INT8_TOPS * 1e3 / PEAK_HBM_GBS},
                     "peak_measured": round(mfma_peak, 1), "frac_of_measured": round(gemm_tops / mfma_peak, 4),
                     "peak_measured_note": "issue rate of v_mfma_i32_32x32x32_i8 alone (registers only, 2 wavefronts "
                                           "per SIMD), measured in this run at the clock the chip holds under it"},
        "kernels": {
            "quantize_pack": {"bound": "hbm", "achieved": round(quant_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                              "frac": round(quant_gbs / PEAK_HBM_GBS, 4),
                              "avg_launch_us": round(seg_ms[0] * 3e3, 3), "bytes_per_launch": quant_bytes * 3,
                              "launch": "48 distinct matrices (three copies of the step's 16, 339 MB of fp32 weights), one launch",
                              "step_launch_after_512MiB_fill_gbs": round(quant_bytes / (quant_after_fill_ms * 1e-3) / 1e9, 1),
                              "step_launch_after_512MiB_fill_us": round(quant_after_fill_ms * 1e3, 3)},
            "quantize_act": {"bound": "hbm", "achieved": round(act_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": round(act_gbs / PEAK_HBM_GBS, 4),
                             "avg_launch_us": round(seg_ms[1] * 1e3 / n_act, 3),
                             "bytes_per_launch": act_bytes / n_act},
        },
    }

    if not args.no_extras:
        out["shapes"] = per_shape(torch, qb, wl, dev)
        out["q8_output"] = q8_output_leg(torch, qb, wl, dev)
        out["dynamic_range"] = dynamic_range_leg(torch, qb, wl, dev)
        out["asymmetric_ranges"] = asymmetric_leg(torch, qb, wl, dev)
        out["backward"] = backward_leg(torch, qb, wl, dev)
        out["stack_12_layers"] = stack_leg(torch, qb, wl, dev)
        out["bert_large"] = bert_large_leg(torch, qb, wl, dev)
        out["embedding"] = embedding_leg(torch, qb, wl, dev)
        out["copy_gbs_measured"] = copy_ceiling(torch, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` on this workload, from the committed rocprofv3 counter
    summary (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known size); None if not measured."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_config2.json")
    try:
        with open(path) as f:
            return json.load(f)[kernel]["bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def measured_mfma_peak(torch, qb, dev):
    """TOP/s of the int8 matrix-core instruction issued back to back with nothing else (the published peak assumes a
    clock the chip may not hold): two wavefronts per SIMD on every CU, warmed up, best of three."""
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    wgs = 2 * torch.cuda.get_device_properties(0).multi_processor_count
    best = 0.0
    qb.qb_probe_mfma_i8(wgs, 20000, sink)
    torch.cuda.synchronize()
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ops = qb.qb_probe_mfma_i8(wgs, 20000, sink)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, ops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best


def time_launches(torch, fn, iters=100, warm=30, per=10):
    """Seconds per call of fn: `per` calls captured in a HIP graph (the Python binding costs more per call than a
    small kernel runs), the graph replayed between two events on its stream."""
    s = torch.cuda.Stream()   # default priority
    with torch.cuda.stream(s):
        for _ in range(warm):
            fn()
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            for _ in range(per):
                fn()
        g.replay()
        s.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(1, iters // per)
        e0.record(s)
        for _ in range(reps):
            g.replay()
        e1.record(s)
        s.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / (reps * per)


def per_shape(torch, qb, wl, dev):
    """Each GEMM shape on its own, against min(int8 MFMA peak, HBM peak x intensity) for its algorithmic bytes:
    `us` / `tops` = back-to-back single launches (qb_qlinear_fwd) between two events; `us_batched4` / `tops_batched4`
    = four independent problems of the shape (own weights, activations and outputs) in one qb_qlinear_fwd_batched
    call, per problem.  BERT-base at T = 4096 and, as the asymptotic case, BERT-large FFN at T = 32768."""
    res = []
    cases = [(T_TOKENS, N, K, 4) for (_, N, K) in wl.BERT_BASE_LINEARS] + [(T_TOKENS, 768, 3072, b) for b in (2, 3, 8)]
    cases += [(32768, 1024, 4096, 2), (32768, 4096, 1024, 3)]
    # configs[0]; few-token inference batches (launch-bound: a batched call runs its four problems in one launch)
    cases += [(1024, 768, 768, 4), (128, 768, 3072, 4), (128, 2304, 768, 4), (16, 3072, 768, 2)]
    for (T, N, K, b) in cases:
        nprob = 4 if T <= 4096 else 1
        jobs = []
        for c in range(nprob):
            W = wl.weight(N, K, seed=N + K + c).to(dev)
            X = wl.activation(T, K, seed=T + K + c).to(dev)
            packed, h, m, rs_w = qb.qb_quantize_groupwise(W, b, GROUPS)
            Xq, rs_x = qb.qb_quantize_act(X, CLIP)
            jobs.append(dict(Xq=Xq, rs_x=rs_x, clip=CLIP, packed=packed, h=h, rs_w=rs_w, bits=b, groups=GROUPS, N=N,
                             Y=torch.empty((T, N), dtype=torch.float32, device=dev)))
            del W, X
        j0 = jobs[0]
        sec = time_launches(torch, lambda: qb.qb_qlinear_fwd(j0["Xq"], j0["rs_x"], CLIP, j0["packed"], j0["h"], j0["rs_w"], b,
                                                             GROUPS, N, Y=j0["Y"]))
        ops = 2.0 * T * N * K
        byts = T * K + N * K * b / 8.0 + 4.0 * T * N + 4 * T + 4 * N
        roof = min(PEAK_INT8_TOPS, PEAK_HBM_GBS * 1e9 * (ops / byts) / 1e12)
        row = {"T": T, "N": N, "K": K, "bits": b, "us": round(sec * 1e6, 2), "tops": round(ops / sec / 1e12, 1),
               "frac_int8_peak": round(ops / sec / 1e12 / PEAK_INT8_TOPS, 4),
               "roofline_tops": round(roof, 1), "frac_roofline": round(ops / sec / 1e12 / roof, 4),
               "gbs": round(byts / sec / 1e9, 1)}
        if nprob > 1:
            secb = time_launches(torch, lambda: qb.qb_qlinear_fwd_batched(jobs)) / nprob
            row.update({"us_batched4": round(secb * 1e6, 2), "tops_batched4": round(ops / secb / 1e12, 1),
                        "frac_int8_peak_batched4": round(ops / secb / 1e12 / PEAK_INT8_TOPS, 4),
                        "frac_roofline_batched4": round(ops / secb / 1e12 / roof, 4)})
        res.append(row)
        del jobs, j0
    return res


def gemm_only_leg(torch, qb, wl, dev, shape):
    """One GEMM shape, eagerly launched (every launch is its own dispatch for the profiler): 30 single launches, then 10
    batched calls of four independent problems."""
    T, N, K, b = shape
    jobs = []
    for c in range(4):
        W = wl.weight(N, K, seed=N + K + c).to(dev)
        X = wl.activation(T, K, seed=T + K + c).to(dev)
        packed, h, m, rs_w = qb.qb_quantize_groupwise(W, b, GROUPS)
        Xq, rs_x = qb.qb_quantize_act(X, CLIP)
        jobs.append(dict(Xq=Xq, rs_x=rs_x, clip=CLIP, packed=packed, h=h, rs_w=rs_w, bits=b, groups=GROUPS, N=N,
                         Y=torch.empty((T, N), dtype=torch.float32, device=dev)))
    j0 = jobs[0]
    torch.cuda.synchronize()
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    e[0].record()
    for _ in range(30):
        qb.qb_qlinear_fwd(j0["Xq"], j0["rs_x"], CLIP, j0["packed"], j0["h"], j0["rs_w"], b, GROUPS, N, Y=j0["Y"])
    e[1].record()
    for _ in range(10):
        qb.qb_qlinear_fwd_batched(jobs)
    e[2].record()
    torch.cuda.synchronize()
    return {"T": T, "N": N, "K": K, "bits": b, "single_us_eager": round(e[0].elapsed_time(e[1]) * 1e3 / 30, 2),
            "batched4_us_per_problem_eager": round(e[1].elapsed_time(e[2]) * 1e3 / 40, 2)}


def q8_output_leg(torch, qb, wl, dev):
    """The forward with 8-bit output (the next layer's input written instead of fp32 Y) on the BERT-base shapes at
    4 bits, next to the fp32-output call on the same inputs; FFN-up also with GELU in the epilogue."""
    res = []
    for (name, N, K) in wl.BERT_BASE_LINEARS:
        T, b = T_TOKENS, 4
        W = wl.weight(N, K, seed=N + K).to(dev)
        X = wl.activation(T, K, seed=T + K).to(dev)
        packed, h, m, rs_w = qb.qb_quantize_groupwise(W, b, GROUPS)
        Xq, rs_x = qb.qb_quantize_act(X, CLIP)
        Y = torch.empty((T, N), dtype=torch.float32, device=dev)
        Yq = torch.empty((T, N), dtype=torch.int8, device=dev)
        rs_y = torch.empty(T, dtype=torch.int32, device=dev)
        s32 = time_launches(torch, lambda: qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, b, GROUPS, N, Y=Y))
        s_act = time_launches(torch, lambda: qb.qb_quantize_act(Y, CLIP, Yq, rs_y))  # what the next layer needs, two-step route
        acts = (0, 1) if name == "ffn_up" else (0,)
        for act in acts:
            s8 = time_launches(torch, lambda: qb.qb_qlinear_fwd_q8(Xq, rs_x, CLIP, packed, h, rs_w, b, GROUPS, N, CLIP,
                                                                   act=act, Yq=Yq, rs_y=rs_y))
            ops = 2.0 * T * N * K
            byts = T * K + N * K * b / 8.0 + 1.0 * T * N + 8 * T + 4 * N
            roof = min(PEAK_INT8_TOPS, PEAK_HBM_GBS * 1e9 * (ops / byts) / 1e12)
            res.append({"linear": name, "T": T, "N": N, "K": K, "bits": b, "act": "gelu" if act else "none",
                        "us_fp32_out": round(s32 * 1e6, 2), "us_quantize_act_of_it": round(s_act * 1e6, 2),
                        "us": round(s8 * 1e6, 2), "tops": round(ops / s8 / 1e12, 1),
                        "frac_int8_peak": round(ops / s8 / 1e12 / PEAK_INT8_TOPS, 4),
                        "roofline_tops": round(roof, 1), "frac_roofline": round(ops / s8 / 1e12 / roof, 4)})
        del W, X, Y, Yq, Xq
    return res


def dynamic_range_leg(torch, qb, wl, dev):
    """Dynamic activation range, per token and per tensor: the quantizers and the forward that takes per-token
    scales, next to the static-clip calls on the same shapes (4 bits, T = 4096)."""
    res = []
    for (name, N, K) in wl.BERT_BASE_LINEARS:
        T, b = T_TOKENS, 4
        W = wl.weight(N, K, seed=N + K).to(dev)
        X = wl.activation(T, K, seed=T + K).to(dev)
        packed, h, m, rs_w = qb.qb_quantize_groupwise(W, b, GROUPS)
        Xq, rs_x = qb.qb_quantize_act(X, CLIP)
        hx = torch.empty(T, dtype=torch.float32, device=dev)
        Y = torch.empty((T, N), dtype=torch.float32, device=dev)
        sa = time_launches(torch, lambda: qb.qb_quantize_act(X, CLIP, Xq, rs_x))
        sad = time_launches(torch, lambda: qb.qb_quantize_act_dyn(X, Xq, rs_x, hx))
        c = torch.empty(1, dtype=torch.float32, device=dev)
        sat = time_launches(torch, lambda: qb.qb_quantize_act_dyn_tensor(X, Xq, rs_x, hx, c))  # reads X twice
        sf = time_launches(torch, lambda: qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, b, GROUPS, N, Y=Y))
        sfd = time_launches(torch, lambda: qb.qb_qlinear_fwd_dyn(Xq, rs_x, hx, packed, h, rs_w, b, GROUPS, N, Y=Y))
        res.append({"linear": name, "act_quant_us": round(sa * 1e6, 2), "act_quant_dyn_us": round(sad * 1e6, 2),
                    "act_quant_dyn_tensor_us": round(sat * 1e6, 2),
                    "fwd_us": round(sf * 1e6, 2), "fwd_dyn_us": round(sfd * 1e6, 2)})
        del W, X, Y, Xq
    return res


def asymmetric_leg(torch, qb, wl, dev):
    """Asymmetric group ranges [min, max]: quantize/pack and the forward next to the symmetric calls (4 bits, T = 4096)."""
    res = []
    for (name, N, K) in wl.BERT_BASE_LINEARS:
        T, b = T_TOKENS, 4
        W = wl.weight(N, K, seed=N + K).to(dev)
        X = wl.activation(T, K, seed=T + K).to(dev)
        packed, h, m, rs_w = qb.qb_quantize_groupwise(W, b, GROUPS)
        pa, delta, q0, rs_a = qb.qb_quantize_groupwise_asym(W, b, GROUPS)
        Xq, rs_x = qb.qb_quantize_act(X, CLIP)
        Y = torch.empty((T, N), dtype=torch.float32, device=dev)
        sq = time_launches(torch, lambda: qb.qb_quantize_groupwise(W, b, GROUPS, packed, h, m, rs_w))
        sqa = time_launches(torch, lambda: qb.qb_quantize_groupwise_asym(W, b, GROUPS, pa, delta, q0, rs_a))
        sf = time_launches(torch, lambda: qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, b, GROUPS, N, Y=Y))
        sfa = time_launches(torch, lambda: qb.qb_qlinear_fwd_asym(Xq, rs_x, CLIP, pa, delta, q0, rs_a, b, GROUPS, N, Y=Y))
        res.append({"linear": name, "quantize_us": round(sq * 1e6, 2), "quantize_asym_us": round(sqa * 1e6, 2),
                    "fwd_us": round(sf * 1e6, 2), "fwd_asym_us": round(sfa * 1e6, 2)})
        del W, X, Y, Xq
    return res


def backward_leg(torch, qb, wl, dev):
    """configs[2]: STE backward of the same layer, 3-bit weights, dY bf16; flops = 4*T*N*K."""
    T, b = T_TOKENS, 3
    tot_sec, tot_flops, tot_masked, rows = 0.0, 0.0, 0.0, []
    for i, (name, N, K) in enumerate(wl.BERT_BASE_LINEARS):
        W = wl.weight(N, K, seed=wl.config_seed(2, i)).to(dev)
        X = wl.activation(T, K, seed=wl.config_seed(2, 10 + i)).to(dev)
        dY = wl.grad_output_bf16(T, N, seed=wl.config_seed(2, 20 + i)).to(dev)
        packed, h, m, rs_w = qb.qb_quantize_groupwise(W, b, GROUPS)
        Xq, rs_x = qb.qb_quantize_act(X, CLIP)
        dX = torch.empty((T, K), dtype=torch.bfloat16, device=dev)
        dW = torch.empty((N, K), dtype=torch.float32, device=dev)
        ws = torch.empty(qb.qb_bwd_workspace_nbytes(T, N, K), dtype=torch.uint8, device=dev)
        sec = time_launches(torch, lambda: qb.qb_qlinear_bwd_ste(dY, Xq, CLIP, packed, h, b, GROUPS, dX=dX, dW=dW,
                                                                 workspace=ws), iters=20)
        secm = time_launches(torch, lambda: qb.qb_qlinear_bwd_ste_masked(dY, Xq, CLIP, packed, h, b, GROUPS, X=X, W=W, m=m,
                                                                         dX=dX, dW=dW, workspace=ws), iters=20)
        fl = 4.0 * T * N * K
        rows.append({"linear": name, "us": round(sec * 1e6, 1), "tflops": round(fl / sec / 1e12, 1),
                     "clamp_masked_us": round(secm * 1e6, 1)})
        tot_sec += sec
        tot_masked += secm
        tot_flops += fl
    return {"workload": "configs[2]: dX and dW for the four linears, T=4096, 3-bit, bf16 MFMA / fp32 accumulate",
            "tflops": round(tot_flops / tot_sec / 1e12, 1), "frac_bf16_peak": round(tot_flops / tot_sec / 1e12 / PEAK_BF16_TFLOPS, 4),
            "us_per_layer": round(tot_sec * 1e6, 1), "clamp_masked_us_per_layer": round(tot_masked * 1e6, 1),
            "per_linear": rows}


def embedding_leg(torch, qb, wl, dev):
    """configs[4]: 8-bit grouped embedding table 30522 x 1024 and a 32768-id de-quantized gather."""
    V, d, n = 30522, 1024, 32768
    E = wl.embedding_table(V, d, seed=wl.config_seed(4, 0)).to(dev)
    ids = wl.token_ids(n, V, seed=wl.config_seed(4, 1)).to(dev)
    codes = torch.empty((V, d), dtype=torch.uint8, device=dev)
    h = torch.empty(GROUPS, dtype=torch.float32, device=dev)
    m = torch.empty(GROUPS, dtype=torch.float32, device=dev)
    out = torch.empty((n, d), dtype=torch.float32, device=dev)
    sq = time_launches(torch, lambda: qb.qb_embedding_quantize(E, GROUPS, codes, h, m), iters=20)
    sg = time_launches(torch, lambda: qb.qb_embedding_gather(codes, h, GROUPS, ids, out), iters=20)
    # the paper's mixed-precision embedding: BERT-base word embeddings (30522 x 768) at 4 bits
    V4, d4 = 30522, 768
    E4 = wl.embedding_table(V4, d4, seed=wl.config_seed(4, 2)).to(dev)
    c4 = torch.empty((V4, d4 // 2), dtype=torch.uint8, device=dev)
    out4 = torch.empty((n, d4), dtype=torch.float32, device=dev)
    sq4 = time_launches(torch, lambda: qb.qb_embedding_quantize_bits(E4, 4, GROUPS, c4, h, m), iters=20)
    sg4 = time_launches(torch, lambda: qb.qb_embedding_gather_bits(c4, h, 4, GROUPS, ids, out4), iters=20)
    four = {"table": "30522 x 768, 4-bit", "quantize_us": round(sq4 * 1e6, 1), "quantize_gbs": round(V4 * d4 * 4.5 / sq4 / 1e9, 1),
            "gather_us": round(sg4 * 1e6, 1), "gather_gbs": round(n * d4 * 4.5 / sg4 / 1e9, 1)}
    return {"quantize_us": round(sq * 1e6, 1), "quantize_gbs": round(V * d * 5.0 / sq / 1e9, 1), "four_bit": four,
            "gather_us": round(sg * 1e6, 1), "gather_gbs": round(n * d * 5.0 / sg / 1e9, 1),
            "note": "algorithmic bytes: 4 read + 1 written per table element (the kernels read the table twice: column-group "
                    "max over all rows, then codes); 1 read + 4 written per gathered element"}


def stack_leg(torch, qb, wl, dev):
    """configs[3]: one iteration of the 12-layer BERT-base linear stack at 32 x 384 = 12288 tokens, per-layer weight
    bits drawn by seed: 48 quantize/pack (batched, 48 distinct master matrices), per layer 4 activation quantizers,
    4 forward GEMMs (one batched call) and 4 STE backwards (dX and dW)."""
    T = 12288
    bits = wl.layer_bits(12, seed=wl.config_seed(3, 0))
    lin = wl.BERT_BASE_LINEARS
    Ws = [[wl.weight(N, K, seed=wl.config_seed(3, 10 * l + i)).to(dev) for i, (_, N, K) in enumerate(lin)] for l in range(12)]
    Xs = [wl.activation(T, K, seed=wl.config_seed(3, 500 + i)).to(dev) for i, (_, N, K) in enumerate(lin)]
    dYs = [wl.grad_output_bf16(T, N, seed=wl.config_seed(3, 600 + i)).to(dev) for i, (_, N, K) in enumerate(lin)]
    qs = [[dict(packed=torch.empty(qb.qb_packed_nbytes(N, K, bits[l]), dtype=torch.uint8, device=dev),
                h=torch.empty(GROUPS, dtype=torch.float32, device=dev), m=torch.empty(GROUPS, dtype=torch.float32, device=dev),
                rs_w=torch.empty(N, dtype=torch.int32, device=dev)) for (_, N, K) in lin] for l in range(12)]
    acts = [dict(Xq=torch.empty((T, K), dtype=torch.int8, device=dev), rs_x=torch.empty(T, dtype=torch.int32, device=dev))
            for (_, N, K) in lin]
    Ys = [torch.empty((T, N), dtype=torch.float32, device=dev) for (_, N, K) in lin]
    dXs = [torch.empty((T, K), dtype=torch.bfloat16, device=dev) for (_, N, K) in lin]
    dWs = [torch.empty((N, K), dtype=torch.float32, device=dev) for (_, N, K) in lin]
    ws = torch.empty(max(qb.qb_bwd_workspace_nbytes(T, N, K) for (_, N, K) in lin), dtype=torch.uint8, device=dev)
    qjobs = [dict(W=Ws[l][i], bits=bits[l], groups=GROUPS, **qs[l][i]) for l in range(12) for i in range(4)]

    def quant():
        qb.qb_quantize_groupwise_batched(qjobs)

    def fwd():
        for l in range(12):
            qb.qb_quantize_act_batched([dict(X=Xs[i], clip=CLIP, Xq=acts[i]["Xq"], rs_x=acts[i]["rs_x"]) for i in range(4)])
            qb.qb_qlinear_fwd_batched([dict(Xq=acts[i]["Xq"], rs_x=acts[i]["rs_x"], clip=CLIP, packed=qs[l][i]["packed"],
                                            h=qs[l][i]["h"], rs_w=qs[l][i]["rs_w"], bits=bits[l], groups=GROUPS, N=lin[i][1],
                                            Y=Ys[i]) for i in range(4)])

    def bwd():
        for l in range(12):
            for i in range(4):
                qb.qb_qlinear_bwd_ste(dYs[i], acts[i]["Xq"], CLIP, qs[l][i]["packed"], qs[l][i]["h"], bits[l], GROUPS,
                                      dX=dXs[i], dW=dWs[i], workspace=ws)

    tq, tf, tb = (time_launches(torch, f, iters=5, warm=2, per=1) for f in (quant, fwd, bwd))
    ops = 12 * sum(2.0 * T * N * K for (_, N, K) in lin)
    qbytes = sum(N * K * (4.0 + bits[l] / 8.0) + GROUPS * 8 + N * 4 for l in range(12) for (_, N, K) in lin)
    return {"workload": "configs[3]: 12 layers x 4 linears, T=12288, bits per layer " + str(list(bits)) +
                        ", per iteration: 48 quantize/pack + 48 act-quant + 48 fwd GEMM + 48 STE bwd",
            "ms_per_iteration": round((tq + tf + tb) * 1e3, 3), "quantize_pack_ms": round(tq * 1e3, 3),
            "quantize_pack_gbs": round(qbytes / tq / 1e9, 1), "fwd_ms": round(tf * 1e3, 3),
            "fwd_tops_incl_act_quant": round(ops / tf / 1e12, 1), "bwd_ms": round(tb * 1e3, 3),
            "bwd_tflops": round(2.0 * ops / tb / 1e12, 1)}


def bert_large_leg(torch, qb, wl, dev):
    """configs[4], the linear layers: the four GEMMs of a BERT-large layer at 64 x 512 = 32768 tokens at 2 and 3 bits,
    and quantize/pack of all 24 layers (96 matrices, 1.2 GB of distinct fp32 master weights: nothing fits a cache)."""
    T = 32768
    lin = wl.BERT_LARGE_LINEARS
    rows = []
    for b in (2, 3):
        jobs = []
        for i, (name, N, K) in enumerate(lin):
            W = wl.weight(N, K, seed=wl.config_seed(4, 10 + i)).to(dev)
            X = wl.activation(T, K, seed=wl.config_seed(4, 20 + i)).to(dev)
            packed, h, m, rs_w = qb.qb_quantize_groupwise(W, b, GROUPS)
            Xq, rs_x = qb.qb_quantize_act(X, CLIP)
            jobs.append(dict(Xq=Xq, rs_x=rs_x, clip=CLIP, packed=packed, h=h, rs_w=rs_w, bits=b, groups=GROUPS, N=N,
                             Y=torch.empty((T, N), dtype=torch.float32, device=dev)))
            del W, X
        sec = time_launches(torch, lambda: qb.qb_qlinear_fwd_batched(jobs), iters=20, warm=5)
        ops = sum(2.0 * T * N * K for (_, N, K) in lin)
        rows.append({"bits": b, "us_per_layer": round(sec * 1e6, 1), "tops": round(ops / sec / 1e12, 1),
                     "frac_int8_peak": round(ops / sec / 1e12 / PEAK_INT8_TOPS, 4)})
        del jobs
    masters = [wl.weight(N, K, seed=wl.config_seed(4, 30 + i)).to(dev) for i, (_, N, K) in enumerate(lin)]
    res = {"gemm_per_layer": rows}
    for b in (2, 3):
        qjobs = []
        for l in range(24):
            for i, (_, N, K) in enumerate(lin):
                qjobs.append(dict(W=masters[i].clone(), bits=b, groups=GROUPS,
                                  packed=torch.empty(qb.qb_packed_nbytes(N, K, b), dtype=torch.uint8, device=dev),
                                  h=torch.empty(GROUPS, dtype=torch.float32, device=dev),
                                  m=torch.empty(GROUPS, dtype=torch.float32, device=dev),
                                  rs_w=torch.empty(N, dtype=torch.int32, device=dev)))
        sec = time_launches(torch, lambda: qb.qb_quantize_groupwise_batched(qjobs), iters=10, warm=2)
        byts = 24 * sum(N * K * (4.0 + b / 8.0) + GROUPS * 8 + N * 4 for (_, N, K) in lin)
        res["quantize_pack_24_layers_%dbit" % b] = {"ms": round(sec * 1e3, 3), "gbs": round(byts / sec / 1e9, 1),
                                                     "frac_hbm_peak": round(byts / sec / 1e9 / PEAK_HBM_GBS, 4),
                                                     "bytes": byts, "launches": (len(qjobs) + 15) // 16}
        del qjobs
    return res


def copy_ceiling(torch, dev):
    """GB/s (read + written) of a plain 1 GiB device-to-device copy on this machine: what HBM sustains for a kernel
    that only moves bytes, to set beside the published 8 TB/s."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    sec = time_launches(torch, lambda: dst.copy_(src), iters=20, warm=5)
    return round(2.0 * (1 << 30) / sec / 1e9, 1)


def cpu_baseline(wl):
    """The CPU oracle (the same source, untuned) on a bounded sample of the step.  All threads (its OpenMP build): the
    whole step, all 4096 token rows, four linears, four bit-widths, including the quantize steps.  One thread (the
    serial build): the same step on the first 256 token rows."""
    import numpy as np
    import oracle
    Ts = T_TOKENS
    linears = wl.BERT_BASE_LINEARS
    Ws = {(b, i): wl.weight(N, K, seed=wl.config_seed(1, 100 * b + i)).numpy()
          for b in BITS_SWEEP for i, (_, N, K) in enumerate(linears)}
    Xs = [wl.activation(Ts, K, seed=wl.config_seed(1, 10 + i)).numpy() for i, (_, N, K) in enumerate(linears)]

    def run(rows, omp):
        t0 = time.perf_counter()
        acts = [oracle.quantize_act(X[:rows], CLIP) for X in Xs]
        ops = 0.0
        for b in BITS_SWEEP:
            for i, (_, N, K) in enumerate(linears):
                codes, h, m, rs_w = oracle.quantize_groupwise(Ws[(b, i)], b, GROUPS)
                oracle.qlinear_fwd(acts[i][0], CLIP, codes, h, b, openmp=omp)
                ops += 2.0 * rows * N * K
        return ops, time.perf_counter() - t0
    threads = oracle.num_threads(True)
    ops, sec = run(Ts, True)
    ops1, sec1 = run(256, False)
    return {"value": round(ops / sec / 1e12, 5), "unit": "TOPS", "cores": threads, "kind": "oracle",
            "sample": "one whole step: 4096 token rows, 4 linears x 4 bit-widths, incl. the quantize steps; %.1f s" % sec,
            "single_thread": {"value": round(ops1 / sec1 / 1e12, 6), "unit": "TOPS", "cores": 1,
                              "sample": "the same step on the first 256 token rows (weights quantized in full); %.1f s" % sec1},
            "host_cpus": os.cpu_count(), "cpu_model": cpu_model()}


def cpu_model():
    """Model string of the host CPU with what /proc/cpuinfo tells about it (family / model / stepping, logical CPUs)."""
    info = {}
    n = 0
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if ":" not in line:
                    continue
                k, v = [x.strip() for x in line.split(":", 1)]
                if k == "processor":
                    n += 1
                elif k in ("model name", "vendor_id", "cpu family", "model", "stepping") and k not in info:
                    info[k] = v
    except OSError:
        return "unknown"
    return "%s (%s, family %s model %s stepping %s, %d logical CPUs visible)" % (
        info.get("model name", "unknown"), info.get("vendor_id", "?"), info.get("cpu family", "?"), info.get("model", "?"),
        info.get("stepping", "?"), n)


if __name__ == "__main__":
    main()
