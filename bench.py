#!/usr/bin/env python3
"""Benchmark of the MSD hot path on one MI355X.

Headline workload (``config.workload``): the W8A16 decode shapes, M in {1,8,32,128}, K=4096,
N in {4096,14336}.  One step = the whole hot path (decomposition, dual INT8 GEMM, dual-scale
epilogue) once for each of the eight shapes.  Weights are replicated so that the working set a
step cycles through exceeds twice the 256 MB last-level cache: every weight byte comes from HBM.
Inputs are resident in HBM before the timed region.  ``value`` is algorithmic bytes per second.

Prints ONE JSON line (rank 0).  ``--gpus`` above 1 is refused: this build is single-GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
INT8_PEAK_TOPS = 5000.0
FP4_PEAK_TFLOPS = 10100.0
BF16_PEAK_TFLOPS = 2500.0
LLC_BYTES = 256 << 20


def w8_bytes(M, K, N):
    """Algorithmic HBM bytes of one W8A16 call: W once, BF16 x, s_W, fp32 y."""
    return K * N + 2 * M * K + 4 * N + 4 * M * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=48)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", default="all", help="comma list of extra legs: cfg0,prefill,w4,attn,cmp,variants,nq,moe,mla | all | none")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one 1 GiB device copy (the calibration kernel), then "
                         "three cold-cache eager calls of each decode shape in the order of 'shapes'; no timing")
    ap.add_argument("--counter-probe", default="", choices=["", "w8_prefill", "w4_prefill", "attn", "mla16", "mla128"],
                    help="for rocprofv3 --pmc runs: three eager calls of one compute-heavy shape (W8A16 "
                         "2048x8192x8192, W4A16 4096x8192x28672, attention L=32768, latent-cache attention with 16 heads "
                         "at L=32768 or 128 heads at L=4096), nothing else; no timing")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_13915_amd import binding as msd, synth

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    msd.lib()

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    if args.counter_probe:
        g = torch.Generator(device=dev)
        g.manual_seed(7)
        if args.counter_probe == "w8_prefill":
            M, K, N = 2048, 8192, 8192
            x = dev_bf16(synth.activations(synth.seed_for(2, 0), M, K, outliers=True))
            W = torch.randint(-127, 128, (N, K), dtype=torch.int8, device=dev, generator=g)
            sc = torch.rand(N, device=dev) * 0.009 + 0.001
            call = lambda: msd.msd_gemm_w8a16(x, W, sc)
        elif args.counter_probe == "w4_prefill":
            M, K, N = 4096, 8192, 28672
            x = dev_bf16(synth.activations(synth.seed_for(3, 2), M, K, outliers=True))
            codes = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device=dev, generator=g)
            exps = torch.randint(118, 124, (N, K // 32), dtype=torch.uint8, device=dev, generator=g)
            call = lambda: msd.msd_gemm_w4a16(x, codes, exps)
        elif args.counter_probe in ("mla16", "mla128"):
            B, Hq, L = (32, 16, 32768) if args.counter_probe == "mla16" else (32, 128, 4096)
            q = dev_bf16(synth.queries(synth.seed_for(9, Hq), B, Hq, 576))
            Cl = torch.randint(-127, 128, (B, L, 576), dtype=torch.int8, device=dev, generator=g)
            sl = torch.rand((B, L), device=dev) * 0.02 + 0.02
            call = lambda: msd.msd_mla_decode_int8kv(q, Cl, sl, msd.MSD_PER_TOKEN, 1.0 / 192.0 ** 0.5)
        else:
            B, Hq, Hkv, d, L = 16, 32, 8, 128, 32768
            q = dev_bf16(synth.queries(synth.seed_for(4, 0), B, Hq, d))
            Kc = torch.randint(-127, 128, (B, Hkv, L, d), dtype=torch.int8, device=dev, generator=g)
            Vc = torch.randint(-127, 128, (B, Hkv, L, d), dtype=torch.int8, device=dev, generator=g)
            ks = torch.rand((B, Hkv, L), device=dev) * 0.02 + 0.02
            vs = torch.rand((B, Hkv, L), device=dev) * 0.02 + 0.02
            call = lambda: msd.msd_attn_decode_int8kv(q, Kc, Vc, ks, vs, msd.MSD_PER_TOKEN)
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        print(json.dumps({"counter_probe": args.counter_probe, "calls": 3}))
        return

    K = 4096
    Ms = [1, 8, 32, 128]
    Ns = [4096, 14336]
    # ---- inputs, resident in HBM
    acts = {}
    for i, M in enumerate(Ms):
        acts[M] = dev_bf16(synth.activations(synth.seed_for(1, i), M, K, outliers=True))
    weights = {}
    for j, N in enumerate(Ns):
        W, s = synth.int8_weights(synth.seed_for(1, 10 + j), N, K)
        copies = max(2, -(-2 * LLC_BYTES // (N * K)) + 1)
        Wd = torch.from_numpy(W).to(dev)
        reps = [Wd] + [Wd.clone() for _ in range(copies - 1)]
        weights[N] = (reps, torch.from_numpy(s).to(dev))
    outs = {(M, N): torch.empty((M, N), dtype=torch.float32, device=dev) for M in Ms for N in Ns}
    ws_bytes = max(msd.lib().msd_gemm_w8a16_workspace_bytes(M, K, N) for M in Ms for N in Ns)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    shapes = [(M, N) for N in Ns for M in Ms]
    step_bytes = sum(w8_bytes(M, K, N) for M, N in shapes)

    if args.traffic_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # calibration: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        for (M, N) in shapes:
            reps, s = weights[N]
            for i in range(3):
                msd.msd_gemm_w8a16(acts[M], reps[(5 * i + 1) % len(reps)], s, y=outs[(M, N)], ws=ws)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": [{"M": M, "K": K, "N": N, "calls": 3} for (M, N) in shapes],
                          "calibration_copy_bytes": 1 << 30}))
        return

    # ---- every call is marshalled once (binding.Prepared) and the timed region replays HIP graphs of
    # whole steps, so that the GPU, not the Python interpreter (~10 us per ctypes call), sets the pace
    side = torch.cuda.Stream()
    CH = 12  # steps per graph; consecutive steps use different weight copies (cold HBM)

    def step_calls(i):
        calls = []
        for (M, N) in shapes:
            reps, s = weights[N]
            idx = (i * 3) % len(reps) if N == 4096 else i % len(reps)
            calls.append(msd.msd_gemm_w8a16(acts[M], reps[idx], s, y=outs[(M, N)], ws=ws, prepare=True))
        return calls

    def capture(call_list):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for c in call_list:
                c()
        return g

    with torch.cuda.stream(side):
        all_calls = [step_calls(i) for i in range(CH)]
        for c in all_calls[0]:
            c()  # first launches outside capture (module load, function attributes)
        torch.cuda.synchronize()
        g_full = capture([c for st in all_calls for c in st])
        rem = args.steps % CH
        g_rem = capture([c for st in all_calls[:rem] for c in st]) if rem else None
    torch.cuda.synchronize()
    for _ in range(max(1, -(-args.warmup // CH))):
        g_full.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps // CH):
        g_full.replay()
    if g_rem is not None:
        g_rem.replay()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-shape device time: HIP events on the launch stream around graph replays of cold-cache calls
    def time_calls(make_call, n_calls, replays=3):
        """make_call(i) -> binding.Prepared for call i; returns microseconds per call."""
        with torch.cuda.stream(side):
            calls = [make_call(i) for i in range(n_calls)]
            calls[0]()
            torch.cuda.synchronize()
            g = capture(calls)
            g.replay()
            torch.cuda.synchronize()
            best = float("inf")
            for _ in range(replays):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(side)
                g.replay()
                e1.record(side)
                e1.synchronize()
                best = min(best, e0.elapsed_time(e1) * 1e3 / n_calls)
        return best

    per_shape = []
    stream_us = {}
    for (M, N) in shapes:
        reps, s = weights[N]

        def mk(i, M=M, N=N, reps=reps, s=s):
            return msd.msd_gemm_w8a16(acts[M], reps[i % len(reps)], s, y=outs[(M, N)], ws=ws, prepare=True)

        us = time_calls(mk, 2 * len(reps))
        if N not in stream_us:
            # a bare read of the same weight bytes (no arithmetic, one launch), same cold-cache protocol:
            # what this GPU charges for the stream alone at this size
            stream_us[N] = time_calls(lambda i, reps=reps: msd.msd_stream_read(reps[i % len(reps)], prepare=True),
                                      2 * len(reps))
        # the same call on one weight copy over and over (cache-resident weights), labelled warm
        warm = time_calls(lambda i, M=M, N=N, reps=reps, s=s: msd.msd_gemm_w8a16(acts[M], reps[0], s, y=outs[(M, N)],
                                                                             ws=ws, prepare=True), 16)
        b = w8_bytes(M, K, N)
        per_shape.append({"M": M, "K": K, "N": N, "us_per_call": round(us, 2), "warm_us_per_call": round(warm, 2),
                          "GBps": round(b / us / 1e3, 1), "hbm_frac": round(b / us / 1e3 / HBM_PEAK_GBS, 3),
                          "exec_TOPS": round(4.0 * M * K * N / us / 1e6, 2),
                          "bare_weight_read_us": round(stream_us[N], 2),
                          "bare_read_over_call": round(stream_us[N] / us, 3)})
    # measured streaming-read rate of this GPU: a bare read of 1 GiB (four launches of 256 MiB, cold)
    big = torch.empty((4, 65536, 4096), dtype=torch.uint8, device=dev)
    big.fill_(1)
    rd_us = time_calls(lambda i: msd.msd_stream_read(big[i % 4], prepare=True), 8)
    measured_stream_GBps = (65536 * 4096) / rd_us / 1e3
    del big
    torch.cuda.empty_cache()
    dom = max(per_shape, key=lambda r: r["us_per_call"] )
    # HBM bytes per call from the committed counter summary (FETCH_SIZE / WRITE_SIZE runs of
    # `bench.py --traffic-probe`, scaled by a copy of known size); null when the file has no line for it
    traffic = None
    try:
        import re
        with open(os.path.join(ROOT, "profiles", "w8a16_decode_hbm_traffic_pmc.txt")) as fh:
            mt = re.search(r"^traffic M=%d N=%d total_bytes=(\d+)" % (dom["M"], dom["N"]), fh.read(), re.M)
        traffic = int(mt.group(1)) if mt else None
    except OSError:
        traffic = None
    roofline = {"bound": "hbm", "kernel": "msd_gemm_w8a16 M=%d K=%d N=%d (all launches of one call)" %
                (dom["M"], dom["K"], dom["N"]),
                "achieved": dom["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(dom["GBps"] / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_unit": "bytes per call (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)",
                "algorithmic_bytes": w8_bytes(dom["M"], K, dom["N"]),
                "measured_stream_read_GBps": round(measured_stream_GBps, 1),
                "bare_weight_read_us_same_shape": dom["bare_weight_read_us"]}

    extras = {}
    want = set(args.extras.split(",")) if args.extras not in ("all", "none") else (
        {"cfg0", "prefill", "w4", "attn", "cmp", "variants", "nq", "moe", "mla"} if args.extras == "all" else set())
    try:
        import bench_extras
        extras = bench_extras.run(want, msd, synth, time_calls, dev)
    except ImportError:
        extras = {}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        # the whole eight-shape step, repeated until about 10 s of CPU work have been timed
        data = []
        for j, N in enumerate(Ns):
            W, s = synth.int8_weights(synth.seed_for(1, 10 + j), N, K)
            for i, M in enumerate(Ms):
                data.append((synth.activations(synth.seed_for(1, i), M, K, outliers=True), W, s, M, N))
        oracle.gemm_w8a16(data[0][0], data[0][1][:64], data[0][2][:64])  # load the library first
        reps = 0
        c0 = time.perf_counter()
        while True:
            for x, W, s, M, N in data:
                oracle.gemm_w8a16(x, W, s)
            reps += 1
            if time.perf_counter() - c0 > 10.0 or reps >= 20:
                break
        c1 = time.perf_counter()
        cpu = {"value": round(reps * step_bytes / (c1 - c0) / 1e9, 4), "unit": "GB/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "oracle W8A16 MSD GEMM (Alg. 1), full outputs of all 8 decode shapes, %d pass(es), %.1f s"
                         % (reps, c1 - c0)}

    line = {
        "metric": "MSD W8A16 decode GEMM, algorithmic HBM GB/s (decompose + dual INT8 GEMM + epilogue)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "W8A16 MSD GEMM decode shapes: M in {1,8,32,128}, K=4096, N in {4096,14336}; "
                               "one step = all 8 shapes, weights cycled through >512 MB of copies (cold HBM)",
                   "bytes_per_step": step_bytes},
        "roofline": roofline, "cpu_baseline": cpu, "shapes": per_shape, "extras": extras,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
