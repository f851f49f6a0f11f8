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


def kernel_sources_sha():
    """sha256 over the HIP sources of the library: the counter summaries under profiles/ carry the value they
    were measured at, and a summary taken at other sources is not reported as this build's traffic."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2605_13915_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hpp")):
            with open(os.path.join(d, name), "rb") as fh:
                h.update(name.encode() + b"\0" + fh.read())
    return h.hexdigest()[:16]


def w8_bytes(M, K, N):
    """Algorithmic HBM bytes of one W8A16 call: W once, BF16 x, s_W, fp32 y."""
    return K * N + 2 * M * K + 4 * N + 4 * M * N


def cpu_other_configs(oracle, synth, np):
    """Oracle time for the configurations besides the headline one, on the host cores: full outputs where that
    takes about a second, otherwise a sample of complete activation rows / batch entries (rows and batch entries
    are independent, so the time scales linearly) extrapolated to the full shape and labelled so.  About 15 s."""
    out = {}

    def clock(fn):
        t0 = time.perf_counter()
        fn()
        return time.perf_counter() - t0

    rng = np.random.default_rng(7)
    # cfg0: full
    x = synth.activations(synth.seed_for(0), 16, 1024, outliers=False)
    W, s = synth.int8_weights(synth.seed_for(0), 1024, 1024)
    out["cfg0"] = {"oracle_s": round(clock(lambda: oracle.gemm_w8a16(x, W, s)), 5), "extrapolated": False, "sample": "full output"}
    # cfg2: 8 complete activation rows against the full weight matrix
    K = 8192
    Wb = rng.integers(-127, 128, (28672, K), dtype=np.int8)
    sb = rng.random(28672, dtype=np.float32) * 0.009 + 0.001
    xr = synth.activations(synth.seed_for(2, 0), 8, K, outliers=True)
    rows = {}
    for N in (8192, 28672):
        t8 = clock(lambda: oracle.gemm_w8a16(xr, Wb[:N], sb[:N]))
        for M in (2048, 8192):
            rows["M%d_N%d" % (M, N)] = {"oracle_s": round(t8 * M / 8, 2), "extrapolated": True,
                                        "sample": "8 complete rows, %.3f s" % t8}
    out["cfg2"] = rows
    del Wb
    # cfg3: MXFP4 weights (one 2048-channel slab repeated along N, as in the GPU leg)
    codes, exps = synth.mxfp4_weights(synth.seed_for(3, 0), 2048, K)
    codes, exps = np.tile(codes, (14, 1)), np.tile(exps, (14, 1))
    x1 = synth.activations(synth.seed_for(3, 1), 1, K, outliers=True)
    x4 = synth.activations(synth.seed_for(3, 32), 4, K, outliers=True)
    t1 = clock(lambda: oracle.gemm_w4a16(x1, codes, exps))
    t4 = clock(lambda: oracle.gemm_w4a16(x4, codes, exps))
    # the oracle decodes the weight matrix once per call: time = a + b*M, fitted to the two samples
    b_row = max(t4 - t1, 0.0) / 3.0
    a_call = max(t1 - b_row, 0.0)
    fit = "a + b*M fitted to M=1 (%.3f s) and M=4 (%.3f s)" % (t1, t4)
    out["cfg3"] = {"M1": {"oracle_s": round(t1, 3), "extrapolated": False, "sample": "full output"},
                   "M32": {"oracle_s": round(a_call + 32 * b_row, 2), "extrapolated": True, "sample": fit},
                   "M4096": {"oracle_s": round(a_call + 4096 * b_row, 1), "extrapolated": True, "sample": fit}}
    del codes, exps
    # cfg4: one batch entry (32 query heads on 8 KV heads) of 16
    for L in (4096, 32768):
        q = synth.queries(synth.seed_for(4, L), 1, 32, 128)
        Kc, ks, Vc, vs = synth.kv_cache_per_token(synth.seed_for(4, 1), 1, 8, 4096, 128)
        rep = L // 4096
        Kc, Vc, ks, vs = np.tile(Kc, (1, 1, rep, 1)), np.tile(Vc, (1, 1, rep, 1)), np.tile(ks, (1, 1, rep)), np.tile(vs, (1, 1, rep))
        tb = clock(lambda: oracle.attn_decode(q, Kc, Vc, ks, vs, oracle.PER_TOKEN))
        out.setdefault("cfg4", {})["L%d" % L] = {"oracle_s": round(tb * 16, 3), "extrapolated": True,
                                                 "sample": "1 of 16 batch entries, %.3f s" % tb}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=48)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--weights", default="packed", choices=["packed", "canonical"],
                    help="weight layout of the timed decode step: packed once by msd_pack_weights_w8 before the "
                         "timed region (default), or the canonical row-major [N][K] array; the per-shape table "
                         "reports both")
    ap.add_argument("--extras", default="all", help="comma list of extra legs: mfma_rate,lds_fill,cfg0,prefill,w4,attn,cmp,variants,nq,moe,mla | all | none")
    ap.add_argument("--one-layout", action="store_true",
                    help="time the --weights layout only (kernel traces then hold one layout per kernel name); the "
                         "other layout's fields are null")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one 1 GiB device copy (the calibration kernel), then "
                         "three cold-cache eager calls of each decode shape in the order of 'shapes'; no timing")
    ap.add_argument("--counter-probe", default="",
                    choices=["", "w8_prefill", "w4_prefill", "attn", "attn4k", "mla16", "mla128", "w4_m1", "w4_m32",
                             "probe_w8", "probe_w8_const", "probe_w4", "rate_w8", "rate_w8_const", "rate_w4", "rate_w4_const",
                             "fill_l2", "fill_mix", "fill_hbm"],
                    help="for rocprofv3 --pmc runs: three eager calls of one shape (W8A16 2048x8192x8192, W4A16 "
                         "4096 / 1 / 32 x 8192 x 28672 (both on packed weights), attention L=32768 / 4096, latent-cache attention with 16 heads "
                         "at L=32768 or 128 heads at L=4096, the MFMA-only probes of the two prefill kernels with random "
                         "or constant operands, the matrix-instruction-only kernel msd_probe_mfma_rate on random or constant "
                         "bits, the fill-instruction-only kernel msd_probe_lds_fill_rate on an L2-resident window, "
                         "half and half, or streamed ranges), nothing else; no timing")
    ap.add_argument("--with-copy", action="store_true",
                    help="with --counter-probe: first one 1 GiB device copy, the calibration kernel of the "
                         "FETCH_SIZE / WRITE_SIZE counters")
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
        if args.with_copy:
            src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
            dst = torch.empty_like(src)
            torch.cuda.synchronize()
            dst.copy_(src)  # calibration: reads 1 GiB, writes 1 GiB
            torch.cuda.synchronize()
            del src, dst
            torch.cuda.empty_cache()
        if args.counter_probe.startswith("rate_"):
            # the matrix pipe alone (msd_probe_mfma_rate) on random or constant operand bits
            if args.counter_probe.endswith("_const"):
                buf = torch.full((16384,), 0x01010101, dtype=torch.int32, device=dev)
            else:
                buf = torch.randint(-2 ** 31, 2 ** 31 - 1, (16384,), dtype=torch.int32, device=dev, generator=g)
            fmt = msd.MSD_MXFP4 if "w4" in args.counter_probe else msd.MSD_INT8
            call = lambda: msd.msd_probe_mfma_rate(fmt, buf, 4000)
        elif args.counter_probe.startswith("fill_"):
            # the tile kernels' LDS fill instructions alone (msd_probe_lds_fill_rate): from a 1 MB window every
            # workgroup shares, half and half, or from disjoint ranges of a 1 GiB buffer
            buf = torch.empty(((1 << 30) + (1 << 20),), dtype=torch.int8, device=dev)
            buf.random_(-128, 127)
            parts = {"fill_l2": 4, "fill_mix": 2, "fill_hbm": 0}[args.counter_probe]
            call = lambda: msd.msd_probe_lds_fill_rate(buf, 1 << 20, parts, 128)
        elif args.counter_probe in ("w8_prefill", "probe_w8", "probe_w8_const"):
            M, K, N = 2048, 8192, 8192
            x = dev_bf16(synth.activations(synth.seed_for(2, 0), M, K, outliers=True))
            W = torch.randint(-127, 128, (N, K), dtype=torch.int8, device=dev, generator=g)
            sc = torch.rand(N, device=dev) * 0.009 + 0.001
            if args.counter_probe == "probe_w8_const":   # the same instruction stream on constant operand bits
                x = torch.ones_like(x)
                W = torch.ones_like(W)
            if args.counter_probe == "w8_prefill":
                Wp = msd.msd_pack_weights_w8(W)  # the layout the timed runs use
                call = lambda: msd.msd_gemm_w8a16_packed(x, Wp, sc)
            else:
                call = lambda: msd.msd_probe_mfma_w8a16(x, W, sc)
        elif args.counter_probe in ("w4_prefill", "w4_m1", "w4_m32", "probe_w4"):
            M = {"w4_m1": 1, "w4_m32": 32}.get(args.counter_probe, 4096)
            K, N = 8192, 28672
            x = dev_bf16(synth.activations(synth.seed_for(3, 2), M, K, outliers=True))
            codes = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device=dev, generator=g)
            exps = torch.randint(118, 124, (N, K // 32), dtype=torch.uint8, device=dev, generator=g)
            if args.counter_probe == "probe_w4":
                call = lambda: msd.msd_probe_mfma_w4a16(x, codes, exps)
            else:
                Wp4, Ep4 = msd.msd_pack_weights_w4(codes, exps)  # the layout the timed runs use
                call = lambda: msd.msd_gemm_w4a16_packed(x, Wp4, Ep4, N)
        elif args.counter_probe in ("mla16", "mla128"):
            B, Hq, L = (32, 16, 32768) if args.counter_probe == "mla16" else (32, 128, 4096)
            q = dev_bf16(synth.queries(synth.seed_for(9, Hq), B, Hq, 576))
            Cl = torch.randint(-127, 128, (B, L, 576), dtype=torch.int8, device=dev, generator=g)
            sl = torch.rand((B, L), device=dev) * 0.02 + 0.02
            call = lambda: msd.msd_mla_decode_int8kv(q, Cl, sl, msd.MSD_PER_TOKEN, 1.0 / 192.0 ** 0.5)
        else:
            B, Hq, Hkv, d, L = 16, 32, 8, 128, (4096 if args.counter_probe == "attn4k" else 32768)
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
    packed = {}
    for j, N in enumerate(Ns):
        W, s = synth.int8_weights(synth.seed_for(1, 10 + j), N, K)
        copies = max(2, -(-2 * LLC_BYTES // (N * K)) + 1)
        Wd = torch.from_numpy(W).to(dev)
        reps = [Wd] + [Wd.clone() for _ in range(copies - 1)]
        weights[N] = (reps, torch.from_numpy(s).to(dev))
        packed[N] = [msd.msd_pack_weights_w8(w) for w in reps]  # one-time repack, outside every timed region
    outs = {(M, N): torch.empty((M, N), dtype=torch.float32, device=dev) for M in Ms for N in Ns}
    ws_bytes = max(msd.lib().msd_gemm_w8a16_workspace_bytes(M, K, N) for M in Ms for N in Ns)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    shapes = [(M, N) for N in Ns for M in Ms]
    step_bytes = sum(w8_bytes(M, K, N) for M, N in shapes)

    def gemm(M, N, idx, layout=None, prepare=True):
        """The decode call of shape (M, N) on weight copy idx in the given layout (default: --weights)."""
        reps, s = weights[N]
        if (layout or args.weights) == "packed":
            return msd.msd_gemm_w8a16_packed(acts[M], packed[N][idx % len(reps)], s, y=outs[(M, N)], ws=ws, prepare=prepare)
        return msd.msd_gemm_w8a16(acts[M], reps[idx % len(reps)], s, y=outs[(M, N)], ws=ws, prepare=prepare)

    if args.traffic_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # calibration: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        for (M, N) in shapes:
            reps, s = weights[N]
            for i in range(3):
                gemm(M, N, 5 * i + 1, prepare=False)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": [{"M": M, "K": K, "N": N, "calls": 3} for (M, N) in shapes],
                          "weights": args.weights,
                          "calibration_copy_bytes": 1 << 30}))
        return

    # ---- every call is marshalled once (binding.Prepared) and the timed region replays HIP graphs of
    # whole steps, so that the GPU, not the Python interpreter (~10 us per ctypes call), sets the pace
    side = torch.cuda.Stream()
    CH = 12  # steps per graph; consecutive steps use different weight copies (cold HBM)

    def step_calls(i):
        # every call reads a weight copy that no call of the last 500 MB of traffic has touched: the copies of
        # one N are walked round-robin across steps AND across the four M of a step
        calls = []
        for pos, (M, N) in enumerate(shapes):
            reps, s = weights[N]
            idx = (i * len(Ms) + pos % len(Ms)) % len(reps)
            calls.append(gemm(M, N, idx))
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
    def time_calls(make_call, n_calls, replays=10):
        """make_call(i) -> binding.Prepared for call i.  Captures the n_calls calls into one HIP graph and replays
        it `replays` times; returns the MEDIAN microseconds per call (HIP events on the launch stream) and leaves
        {"median", "min"} in time_calls.last."""
        with torch.cuda.stream(side):
            calls = [make_call(i) for i in range(n_calls)]
            calls[0]()
            torch.cuda.synchronize()
            g = capture(calls)
            g.replay()
            torch.cuda.synchronize()
            ts = []
            for _ in range(replays):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(side)
                g.replay()
                e1.record(side)
                e1.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3 / n_calls)
        ts.sort()
        time_calls.last = {"median": ts[len(ts) // 2], "min": ts[0]}
        return ts[len(ts) // 2]

    per_shape = []
    stream_us = {}
    linear_us = {}
    for (M, N) in shapes:
        reps, s = weights[N]

        us = time_calls(lambda i, M=M, N=N: gemm(M, N, i), 2 * len(reps))
        us_min = time_calls.last["min"]
        other = "canonical" if args.weights == "packed" else "packed"
        us_other = None if args.one_layout else time_calls(lambda i, M=M, N=N: gemm(M, N, i, layout=other), 2 * len(reps))
        if N not in stream_us:
            # a bare read of the same weight bytes (no arithmetic, one launch), same cold-cache protocol:
            # what this GPU charges for the stream alone at this size
            stream_us[N] = time_calls(lambda i, reps=reps: msd.msd_stream_read(reps[i % len(reps)], prepare=True),
                                      2 * len(reps))
            # and as one linear array (contiguous kilobytes per wave instruction, 16 in flight per lane): the
            # pattern the packed layout is read in
            linear_us[N] = time_calls(lambda i, reps=reps: msd.msd_stream_read_linear(reps[i % len(reps)], prepare=True),
                                      2 * len(reps))
        # the same call on one weight copy over and over (cache-resident weights), labelled warm
        warm = time_calls(lambda i, M=M, N=N: gemm(M, N, 0), 16)
        b = w8_bytes(M, K, N)
        per_shape.append({"M": M, "K": K, "N": N, "us_per_call": round(us, 2), "us_per_call_min": round(us_min, 2),
                          "warm_us_per_call": round(warm, 2), "weights": args.weights,
                          other + "_weights_us_per_call": None if us_other is None else round(us_other, 2),
                          "GBps": round(b / us / 1e3, 1), "hbm_frac": round(b / us / 1e3 / HBM_PEAK_GBS, 3),
                          "exec_TOPS": round(4.0 * M * K * N / us / 1e6, 2),
                          "bare_weight_read_us": round(stream_us[N], 2),
                          "bare_linear_read_us": round(linear_us[N], 2),
                          "bare_read_over_call": round(min(stream_us[N], linear_us[N]) / us, 3)})
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
    traffic_note = "no counter summary"
    try:
        import re
        with open(os.path.join(ROOT, "profiles", "w8a16_decode_hbm_traffic_pmc.txt")) as fh:
            txt = fh.read()
        ms = re.search(r"^kernel_sources_sha256_16=([0-9a-f]+)", txt, re.M)
        mt = re.search(r"^traffic M=%d N=%d total_bytes=(\d+)" % (dom["M"], dom["N"]), txt, re.M)
        if ms and ms.group(1) == kernel_sources_sha() and mt:
            traffic = int(mt.group(1))
            traffic_note = "profiles/w8a16_decode_hbm_traffic_pmc.txt, taken at these kernel sources"
        else:
            traffic_note = "profiles/w8a16_decode_hbm_traffic_pmc.txt was taken at other kernel sources: not reported"
    except OSError:
        traffic = None
    roofline = {"bound": "hbm", "kernel": "%s M=%d K=%d N=%d (all launches of one call)" %
                ("msd_gemm_w8a16_packed" if args.weights == "packed" else "msd_gemm_w8a16", dom["M"], dom["K"], dom["N"]),
                "achieved": dom["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(dom["GBps"] / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_unit": "bytes per call (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)",
                "traffic_source": traffic_note,
                "algorithmic_bytes": w8_bytes(dom["M"], K, dom["N"]),
                "measured_stream_read_GBps": round(measured_stream_GBps, 1),
                "bare_weight_read_us_same_shape": dom["bare_weight_read_us"],
                "bare_linear_read_us_same_shape": dom["bare_linear_read_us"]}

    extras = {}
    want = set(args.extras.split(",")) if args.extras not in ("all", "none") else (
        {"mfma_rate", "lds_fill", "cfg0", "prefill", "w4", "attn", "cmp", "variants", "nq", "moe", "mla"} if args.extras == "all" else set())
    try:
        import bench_extras
        extras = bench_extras.run(want, msd, synth, time_calls, dev)
    except ImportError:
        extras = {}

    # ---- decomposition kernels alone (a1 / a4): 2*M*K bytes in, 2*M*K + 4*M out (INT8); HBM/L2-bound
    dec = []
    for (Md, Kd) in [(128, 4096), (8192, 8192)]:
        xg = torch.randn((Md, Kd), device=dev).to(torch.bfloat16)
        q1 = torch.empty((Md, Kd), dtype=torch.int8, device=dev)
        q2 = torch.empty_like(q1)
        al = torch.empty((Md,), dtype=torch.float32, device=dev)
        L_ = msd.lib()
        import ctypes as C_
        argsd = (msd.MSD_INT8, C_.c_void_p(xg.data_ptr()), Md, Kd, Kd, C_.c_void_p(q1.data_ptr()), C_.c_void_p(q2.data_ptr()),
                 C_.c_void_p(al.data_ptr()), C_.c_void_p(side.cuda_stream))
        us_d = time_calls(lambda i: msd.Prepared(L_.msd_decompose, argsd, (xg, q1, q2, al), "msd_decompose", None), 8)
        bd = 4 * Md * Kd + 4 * Md
        dec.append({"M": Md, "K": Kd, "us": round(us_d, 2), "us_min": round(time_calls.last["min"], 2),
                    "GBps": round(bd / us_d / 1e3, 1), "hbm_frac": round(bd / us_d / 1e3 / HBM_PEAK_GBS, 4)})
        del xg, q1, q2, al
    torch.cuda.empty_cache()

    # ---- every configuration in one compact table (kept inside `roofline` so that it travels with the line)
    def _r(v, n=3):
        return None if v is None else round(v, n)
    per_config = {"cfg1_w8a16_decode": [
        {"M": r["M"], "N": r["N"], "us": r["us_per_call"], "us_min": r["us_per_call_min"],
         ("canonical" if args.weights == "packed" else "packed") + "_weights_us":
             r[("canonical" if args.weights == "packed" else "packed") + "_weights_us_per_call"], "bound": "hbm",
         "frac": r["hbm_frac"], "vs_bare_read": r["bare_read_over_call"]} for r in per_shape],
        "decomposition_alone": dec}
    ex = extras if isinstance(extras, dict) else {}
    if isinstance(ex.get("cmp"), list):
        cm = {(c["M"], c["N"]): c for c in ex["cmp"]}
        for e_ in per_config["cfg1_w8a16_decode"]:
            c = cm.get((e_["M"], e_["N"]))
            if c:
                e_["vs_dequant"] = c["speedup_vs_dequant"]
    if isinstance(ex.get("cfg0"), dict) and "msd_us" in ex["cfg0"]:
        per_config["cfg0_w8a16_16x1024x1024"] = {"us": ex["cfg0"]["msd_us"], "bound": "launch latency",
                                                 "vs_dequant": _r(ex["cfg0"]["dequant_us"] / ex["cfg0"]["msd_us"])}
    if isinstance(ex.get("prefill"), list):
        per_config["cfg2_w8a16_prefill"] = [
            {"M": r["M"], "N": r["N"], "us": r["us"], "bound": "mfma_int8", "frac": r["int8_mfma_frac"],
             "exec_TOPS": r["exec_TOPS"], "vs_dequant": r.get("speedup_vs_dequant"),
             "frac_of_mfma_only_probe": r.get("frac_of_mfma_only")} for r in ex["prefill"]]
    if isinstance(ex.get("w4"), list):
        per_config["cfg3_w4a16"] = [
            {"M": r["M"], "us": r["us"], "bound": "hbm" if r["M"] <= 32 else "mfma_fp4",
             "frac": r["hbm_frac"] if r["M"] <= 32 else r["fp4_mfma_frac"], "vs_dequant": r.get("speedup_vs_dequant")}
            for r in ex["w4"]]
    if isinstance(ex.get("attn"), list):
        per_config["cfg4_attention"] = [
            {"L": r["L"], "us": r["us"], "bound": "hbm", "frac": r["hbm_frac"], "vs_dequant": r["speedup_vs_dequant"],
             "per_channel_us": r["per_channel"]["us"], "lowprec_us": r.get("lowprec_us")} for r in ex["attn"]]
    if isinstance(ex.get("mfma_rate"), dict) and "error" not in ex["mfma_rate"]:
        # the matrix pipe alone on random and on constant operand bits (msd_probe_mfma_rate): the ceiling of the
        # MFMA-bound rows on this machine is the random-bits figure, not the datasheet peak
        per_config["matrix_pipe_alone"] = {k: {"random_bits_Tops": v["random_bits"]["Tops"],
                                               "constant_bits_Tops": v["constant_bits"]["Tops"],
                                               "random_bits_frac_of_datasheet": v["random_bits"]["frac_of_datasheet"]}
                                           for k, v in ex["mfma_rate"].items()}
    if isinstance(ex.get("lds_fill"), dict) and "error" not in ex["lds_fill"]:
        # the tile kernels' LDS fill instructions alone (msd_probe_lds_fill_rate): what a CU can pull into LDS
        per_config["lds_fill_alone"] = {k: v["TBps"] for k, v in ex["lds_fill"].items() if isinstance(v, dict)}
        per_config["lds_fill_alone"]["unit"] = "TB/s over 256 CUs"
    roofline["per_config"] = per_config

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
            if time.perf_counter() - c0 > 6.0 or reps >= 20:
                break
        c1 = time.perf_counter()
        cpu = {"value": round(reps * step_bytes / (c1 - c0) / 1e9, 4), "unit": "GB/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "oracle W8A16 MSD GEMM (Alg. 1), full outputs of all 8 decode shapes, %d pass(es), %.1f s"
                         % (reps, c1 - c0)}
        cpu["per_config"] = cpu_other_configs(oracle, synth, np)

    line = {
        "metric": "MSD W8A16 decode GEMM, algorithmic HBM GB/s (decompose + dual INT8 GEMM + epilogue)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "W8A16 MSD GEMM decode shapes: M in {1,8,32,128}, K=4096, N in {4096,14336}; "
                               "one step = all 8 shapes, weights cycled through >512 MB of copies (cold HBM); "
                               + ("weights repacked once by msd_pack_weights_w8 before the timed region"
                                  if args.weights == "packed" else "weights in the canonical [N][K] layout"),
                   "weights": args.weights,
                   "bytes_per_step": step_bytes},
        "roofline": roofline, "cpu_baseline": cpu, "shapes": per_shape, "extras": extras,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
