#!/usr/bin/env python3
"""Regenerate the rocprofv3 summaries under profiles/ (run from the repository root on one MI355X).

    python3 bench_profiles.py trace      kernel trace of bench.py's headline run
    python3 bench_profiles.py traffic    FETCH_SIZE / WRITE_SIZE of the W8A16 decode shapes, W4A16 decode, prefill, attention
    python3 bench_profiles.py counters   SQ / TCC / GRBM counters of the compute-heavy kernels and of the MFMA-only probes
    python3 bench_profiles.py all

Every rocprofv3 pass is a child process of its own with its own time limit (`rocprofv3 ... -- python3 bench.py ...`:
the profiled program is the interpreter itself), counters are collected without any trace domain, and at most the
number of counters per hardware block that one pass can hold.  Raw output goes to gpurun_out/ (scratch); the text
summaries go to profiles/ and carry the sha256 of the kernel sources they were measured at.
"""
import collections
import csv
import json
import os
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(ROOT, "gpurun_out")
PROF = os.path.join(ROOT, "profiles")
sys.path.insert(0, ROOT)
from bench import kernel_sources_sha  # noqa: E402  (host-side helper, no GPU work at import)


def run_pass(name, rocprof_args, bench_args, limit=240):
    """One rocprofv3 run; returns the output directory.  Raises on a non-zero exit or a timeout."""
    d = os.path.join(OUT, name)
    shutil.rmtree(d, ignore_errors=True)
    os.makedirs(OUT, exist_ok=True)
    cmd = ["rocprofv3", *rocprof_args, "-d", d, "-o", "p", "--output-format", "csv", "--",
           "python3", os.path.join(ROOT, "bench.py"), *bench_args]
    env = dict(os.environ, TMPDIR="/tmp")
    print("[bench_profiles] " + " ".join(cmd), flush=True)
    with open(os.path.join(OUT, name + ".log"), "w") as log:
        r = subprocess.run(cmd, cwd="/tmp", env=env, stdout=log, stderr=subprocess.STDOUT, timeout=limit)
    if r.returncode != 0:
        raise RuntimeError("rocprofv3 pass %s failed (rc %d), see gpurun_out/%s.log" % (name, r.returncode, name))
    print("[bench_profiles] pass %s done" % name, flush=True)
    return d


def find_csv(d, suffix):
    for base, _, files in os.walk(d):
        for f in files:
            if f.endswith(suffix):
                return os.path.join(base, f)
    raise FileNotFoundError("%s under %s" % (suffix, d))


def short(name):
    return name.replace("(anonymous namespace)::", "").split("(")[0].replace("void ", "")


def stamp():
    return "kernel_sources_sha256_16=%s\n" % kernel_sources_sha()


def write_summary(name, text):
    """profiles/<name>, and a copy under gpurun_out/profiles/ (the scratch folder is the one that travels back from
    a remote GPU machine)"""
    for d in (PROF, os.path.join(OUT, "profiles")):
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, name), "w") as fh:
            fh.write(text)


# ------------------------------------------------------------------ kernel trace of the headline run
def do_trace():
    d = run_pass("prof_bench", ["--kernel-trace", "--stats"], ["--extras", "none", "--no-cpu-baseline", "--one-layout"], limit=400)
    line = None
    with open(os.path.join(OUT, "prof_bench.log")) as fh:
        for ln in fh:
            if ln.startswith("{") and '"metric"' in ln:
                line = json.loads(ln)
    out = ["W8A16 decode bench: rocprofv3 kernel-trace summary\n",
           "===================================================\n",
           "Command (from the repository root, on one MI355X):  python3 bench_profiles.py trace\n",
           "  = rocprofv3 --kernel-trace --stats -d gpurun_out/prof_bench -o p --output-format csv -- \\\n",
           "        python3 bench.py --extras none --no-cpu-baseline --one-layout        (cwd /tmp, TMPDIR=/tmp)\n", stamp(),
           "Workload: bench.py's headline step (8 W8A16 decode shapes, M in {1,8,32,128}, K=4096, N in {4096,14336}),\n",
           "warm-up + timed steps replayed from HIP graphs, then the per-shape timing graphs (cold and warm weights,\n",
           "bare weight reads, decomposition alone), all on weights packed once at set-up (the repack dispatches are left\n",
           "out).  The trace records the kernels inside graph replays.\n\n",
           "Per kernel and grid size (one template instantiation serves several shapes); columns: kernel, grid threads,\n",
           "workgroup, VGPRs, LDS bytes (static), scratch, dispatches, avg / min / median / max us:\n"]
    rows = list(csv.DictReader(open(find_csv(d, "kernel_trace.csv"))))
    g = collections.defaultdict(list)
    for r in rows:
        if "msd::" not in r["Kernel_Name"] or "pack_weights" in r["Kernel_Name"]:
            continue
        g[(short(r["Kernel_Name"]), int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1), r["Workgroup_Size_X"],
           r["VGPR_Count"], r["LDS_Block_Size"], r["Scratch_Size"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    avg = {}
    for k, v in sorted(g.items()):
        v2 = sorted(v)
        avg[(k[0], k[1])] = sum(v) / len(v) / 1e3
        out.append("  %-58s grid %8d wg %4s vgpr %3s lds %6s scratch %s  n %4d  avg %7.2f  min %7.2f  med %7.2f  max %7.2f\n"
                   % (k[0], k[1], k[2], k[3], k[4], k[5], len(v), sum(v) / len(v) / 1e3, v2[0] / 1e3, v2[len(v) // 2] / 1e3,
                      v2[-1] / 1e3))
    if line:
        out.append("\nbench.py's own line from the same (profiled) run: value %.1f GB/s, %.4f ms/step; per shape, HIP-event\n"
                   "time per call on the launch stream (all launches of a call), median of 10 graph replays:\n"
                   % (line["value"], line["ms_per_step"]))
        for r in line["shapes"]:
            out.append("  M=%-4d N=%-6d %6.2f us/call (min %6.2f, warm %6.2f)  %7.1f GB/s  (%.3f of 8 TB/s)  bare weight read %5.2f us\n"
                       % (r["M"], r["N"], r["us_per_call"], r["us_per_call_min"], r["warm_us_per_call"], r["GBps"], r["hbm_frac"],
                          r["bare_weight_read_us"]))
        rf = line["roofline"]
        out.append("\nroofline entry of that line: %s: %.1f GB/s = %.4f of %.0f GB/s.\n" % (rf["kernel"], rf["achieved"], rf["frac"], rf["peak"]))
        m = [int(t.split("=")[1]) for t in rf["kernel"].split() if t.startswith("M=")][0]
        dk = [a for k, a in avg.items() if "decompose_int8" in k[0] and k[1] == m * 256]
        if dk:
            out.append("Its decomposition launch (grid %d) averages %.2f us in the trace; add the GEMM kernel of that shape from the\n"
                       "table above to compare with the event time per call.\n" % (m * 256, dk[0]))
    write_summary("w8a16_decode_bench_kernel_stats.txt", "".join(out))
    print("".join(out))


# ------------------------------------------------------------------ kernel trace of the other configurations
def do_trace_extras():
    legs = "prefill,w4,attn,mla,moe"
    d = run_pass("prof_extras", ["--kernel-trace", "--stats"], ["--extras", legs, "--no-cpu-baseline", "--one-layout"], limit=500)
    out = ["Prefill, W4, attention, latent-cache and grouped legs: rocprofv3 kernel-trace summary\n",
           "=====================================================================================\n",
           "Command (from the repository root, on one MI355X):  python3 bench_profiles.py trace_extras\n",
           "  = rocprofv3 --kernel-trace --stats -d gpurun_out/prof_extras -o p --output-format csv -- \\\n",
           "        python3 bench.py --extras %s --no-cpu-baseline --one-layout        (cwd /tmp, TMPDIR=/tmp)\n" % legs, stamp(),
           "Workload: bench.py's legs for cfg2 (W8A16 prefill), cfg3 (W4A16, M = 1 / 32 / 4096), cfg4 (attention decode,\n",
           "L = 4096 / 32768), attention over a latent cache and the grouped GEMMs, each with its comparison kernel,\n",
           "replayed from HIP graphs; the headline step runs first (its kernels are in w8a16_decode_bench_kernel_stats.txt\n",
           "too).  One template instantiation serves several shapes: the grid size tells them apart.\n\n",
           "Columns: kernel, grid threads, workgroup, VGPRs, scratch, dispatches, avg / min / median / max us:\n"]
    rows = list(csv.DictReader(open(find_csv(d, "kernel_trace.csv"))))
    g = collections.defaultdict(list)
    for r in rows:
        if "msd::" not in r["Kernel_Name"] or "pack_weights" in r["Kernel_Name"]:
            continue
        g[(short(r["Kernel_Name"]), int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1), r["Workgroup_Size_X"],
           r["VGPR_Count"], r["Scratch_Size"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    for k, v in sorted(g.items()):
        v2 = sorted(v)
        out.append("  %-66s grid %8d wg %4s vgpr %3s scratch %s  n %4d  avg %8.2f  min %8.2f  med %8.2f  max %8.2f\n"
                   % (k[0][:66], k[1], k[2], k[3], k[4], len(v), sum(v) / len(v) / 1e3, v2[0] / 1e3, v2[len(v) // 2] / 1e3,
                      v2[-1] / 1e3))
    write_summary("prefill_w4_attn_kernel_stats.txt", "".join(out))
    print("".join(out))


# ------------------------------------------------------------------ HBM traffic
def counter_rows(d):
    """dispatches of the counter run, without the one-time weight repack kernels of the set-up (the probes run on
    packed weights, whose repack includes the rearrangement of the MXFP4 scale bytes)"""
    return [r for r in csv.DictReader(open(find_csv(d, "counter_collection.csv")))
            if "pack_weights" not in r["Kernel_Name"] and "transpose_w_scales" not in r["Kernel_Name"]]


def calib(rows):
    """counter value of the calibration dispatch: the runtime's device-to-device copy kernel of 1 GiB"""
    big = [float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"]]
    if not big:
        raise RuntimeError("calibration copy not found among the dispatches")
    return max(big)


def do_traffic():
    o = ["HBM traffic of the MSD kernels from rocprofv3 counters\n",
         "======================================================\n",
         "Command (from the repository root, on one MI355X):  python3 bench_profiles.py traffic\n",
         "  = for C in FETCH_SIZE, WRITE_SIZE (one counter per run, no trace domain):\n",
         "      rocprofv3 --pmc C -d gpurun_out/pmc_C_W -o p --output-format csv -- python3 bench.py --traffic-probe\n",
         "      rocprofv3 --pmc C ... -- python3 bench.py --counter-probe W --with-copy   (W = w4_m1, w4_m32, w8_prefill, w4_prefill, attn4k, attn)\n",
         stamp(),
         "The decode shapes and the W8 / W4 probes run on weights packed once at set-up (msd_pack_weights_w8 / _w4; those\n",
         "dispatches are left out).  Every probe first runs one 1 GiB device-to-device copy: the counters read in KiB per dispatch up to a constant\n",
         "factor that the copy (1048576 KiB read, 1048576 KiB written) fixes.  Then three eager calls of each shape; values\n",
         "are the median over the three dispatches of a kernel, scaled to bytes.\n\n"]
    F = counter_rows(run_pass("pmc_fetch_decode", ["--pmc", "FETCH_SIZE"], ["--traffic-probe"]))
    W = counter_rows(run_pass("pmc_write_decode", ["--pmc", "WRITE_SIZE"], ["--traffic-probe"]))
    ff, fw = 1048576.0 / calib(F), 1048576.0 / calib(W)
    o.append("Calibration: FETCH_SIZE reads %.2f for the copy -> factor %.4f;  WRITE_SIZE reads %.2f -> factor %.4f\n\n"
             % (calib(F), ff, calib(W), fw))
    o.append("W8A16 decode (cfg1), per call: 'alg' = K*N + 2*M*K + 4*N + 4*M*N bytes; calls with a decomposition launch list it as 'dec'\n")
    shapes = [(M, N) for N in (4096, 14336) for M in (1, 8, 32, 128)]

    def seq(rows):
        rows = [r for r in rows if "msd::" in r["Kernel_Name"]]
        res, i = [], 0
        for _ in shapes:
            calls = []
            for _c in range(3):
                dec = None
                if "decompose" in rows[i]["Kernel_Name"]:
                    dec = float(rows[i]["Counter_Value"])
                    i += 1
                calls.append((dec, float(rows[i]["Counter_Value"]), short(rows[i]["Kernel_Name"])))
                i += 1
            res.append(calls)
        return res

    med = lambda l: sorted(l)[len(l) // 2]  # noqa: E731
    for (M, N), fc, wc in zip(shapes, seq(F), seq(W)):
        K = 4096
        alg = K * N + 2 * M * K + 4 * N + 4 * M * N
        gf, gw = med([c[1] for c in fc]) * ff * 1024, med([c[1] for c in wc]) * fw * 1024
        df, dw = med([c[0] or 0 for c in fc]) * ff * 1024, med([c[0] or 0 for c in wc]) * fw * 1024
        tot = gf + gw + df + dw
        o.append("  M=%-4d N=%-6d %-52s gemm fetch %10.0f B write %9.0f B | dec fetch %8.0f B write %8.0f B\n"
                 % (M, N, fc[0][2], gf, gw, df, dw))
        o.append("traffic M=%d N=%d total_bytes=%d alg_bytes=%d ratio=%.3f\n" % (M, N, tot, alg, tot / alg))
    alg_of = {"w4_m1": 8192 * 28672 // 2 + 8192 * 28672 // 32 + 2 * 8192 + 4 * 28672,
              "w4_m32": 8192 * 28672 // 2 + 8192 * 28672 // 32 + 32 * (2 * 8192 + 4 * 28672),
              "w8_prefill": 8192 * 8192 + 2048 * (2 * 8192 + 4 * 8192),
              "w4_prefill": 8192 * 28672 // 2 + 8192 * 28672 // 32 + 4096 * (2 * 8192 + 4 * 28672),
              "attn4k": 2 * 16 * 8 * 4096 * 128 + 8 * 16 * 8 * 4096 + 6 * 16 * 32 * 128,
              "attn": 2 * 16 * 8 * 32768 * 128 + 8 * 16 * 8 * 32768 + 6 * 16 * 32 * 128}
    o.append("\nOther configurations, per call (sum over the launches of a call; 'alg' as DESIGN.md states per kernel):\n")
    for w in ("w4_m1", "w4_m32", "w8_prefill", "w4_prefill", "attn4k", "attn"):
        Fw = counter_rows(run_pass("pmc_fetch_" + w, ["--pmc", "FETCH_SIZE"], ["--counter-probe", w, "--with-copy"]))
        Ww = counter_rows(run_pass("pmc_write_" + w, ["--pmc", "WRITE_SIZE"], ["--counter-probe", w, "--with-copy"]))
        f2, w2 = 1048576.0 / calib(Fw), 1048576.0 / calib(Ww)
        per = collections.OrderedDict()
        for rows, fac, key in ((Fw, f2, "f"), (Ww, w2, "w")):
            for r in rows:
                if "msd::" in r["Kernel_Name"]:
                    per.setdefault(short(r["Kernel_Name"]), {"f": [], "w": []})[key].append(float(r["Counter_Value"]) * fac * 1024)
        tot = 0.0
        for nm, v in per.items():
            f_, w_ = med(v["f"]), med(v["w"])
            tot += f_ + w_
            o.append("  %-10s %-52s fetch %11.0f B  write %11.0f B\n" % (w, nm, f_, w_))
        o.append("traffic %s total_bytes=%d alg_bytes=%d ratio=%.3f\n" % (w, tot, alg_of[w], tot / alg_of[w]))
    write_summary("w8a16_decode_hbm_traffic_pmc.txt", "".join(o))
    print("".join(o))


# ------------------------------------------------------------------ SQ / TCC / GRBM counters
PASSES = [["SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES", "SQ_WAIT_INST_ANY", "SQ_WAIT_ANY", "SQ_INSTS_LDS", "SQ_VALU_MFMA_BUSY_CYCLES",
           "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_LDS"],
          ["SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE", "SQ_INSTS_MFMA", "SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_ACTIVE_INST_VALU",
           "SQ_ACTIVE_INST_SCA", "SQ_INSTS_VMEM_RD"],
          ["TCC_HIT_sum", "TCC_MISS_sum"],
          ["GRBM_GUI_ACTIVE", "GRBM_COUNT"]]
WORKLOADS = ["rate_w8", "rate_w8_const", "rate_w4", "rate_w4_const", "fill_l2", "fill_mix", "fill_hbm", "w8_prefill", "probe_w8", "probe_w8_const", "w4_prefill",
             "probe_w4", "w4_m1", "w4_m32", "attn", "attn4k", "mla16", "mla128"]


def do_counters(workloads=None):
    workloads = workloads or WORKLOADS
    out = ["Compute-heavy kernels and the MFMA-only probes: rocprofv3 hardware counters\n",
           "===========================================================================\n",
           "Command (from the repository root, on one MI355X):  python3 bench_profiles.py counters\n",
           "  = for W in %s,\n" % ", ".join(WORKLOADS),
           "    four passes each (8 SQ counters | 8 SQ counters | TCC_HIT_sum TCC_MISS_sum | GRBM_GUI_ACTIVE GRBM_COUNT):\n",
           "      rocprofv3 --pmc <counters> -d gpurun_out/pmcx_W_i -o p --output-format csv -- python3 bench.py --counter-probe W\n",
           stamp(),
           "rate_w8 / rate_w8_const / rate_w4 / rate_w4_const = msd_probe_mfma_rate, 2048 waves x 32000 matrix instructions\n",
           "(INT8 32x32x32 resp. FP6 x FP4 32x32x64) on random resp. constant operand bits and nothing else: equal cycle\n",
           "counts, while bench.py's mfma_rate leg times the random-bits run 1.4x longer -- the clock under load differs.\n",
           "fill_l2 / fill_mix / fill_hbm = msd_probe_lds_fill_rate, 256 workgroups x 128 rounds x 32 KB of LDS fills and nothing\n",
           "else, from a 1 MB window every workgroup shares / half from the window, half from disjoint ranges of 1 GiB / all\n",
           "from those ranges (the L2 hit rates say which is which).\n",
           "bench.py --counter-probe W runs three eager calls of one shape: w8_prefill = msd_gemm_w8a16_packed 2048x8192x8192;\n",
           "probe_w8 / probe_w8_const = msd_probe_mfma_w8a16 on the same shape (the prefill kernel's MFMA sequence, tile schedule\n",
           "and epilogue with no tile fill, no barrier, no LDS traffic after the first K step) with the benchmark's random operands\n",
           "resp. all-ones operands; w4_prefill = msd_gemm_w4a16_packed 4096x8192x28672, probe_w4 its MFMA-only probe; w4_m1 / w4_m32 the\n",
           "same weights with 1 / 32 rows; attn / attn4k = msd_attn_decode_int8kv B=16, 32/8 heads, d=128, L=32768 / 4096;\n",
           "mla16 / mla128 = msd_mla_decode_int8kv B=32 with 16 heads at L=32768 / 128 heads at L=4096.\n",
           "Values are the median over the three dispatches of a kernel.  Derived: kernel cycles = GRBM_GUI_ACTIVE / 8 (the\n",
           "counter sums the 8 XCDs); MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x kernel cycles); vector ALU =\n",
           "4 x SQ_ACTIVE_INST_VALU / (1024 x kernel cycles), a lower bound; LDS busy = SQ_LDS_IDX_ACTIVE / (256 CUs x kernel\n",
           "cycles); waiting = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES; L2 hit = TCC_HIT / (TCC_HIT + TCC_MISS); LDS conflict share =\n",
           "SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE; MFMA cycles per instruction = SQ_VALU_MFMA_BUSY_CYCLES / SQ_INSTS_MFMA\n",
           "(per-wave instruction count; what the counter charges one instruction).\n\n"]
    for w in workloads:
        vals = {}
        for i, ctrs in enumerate(PASSES, 1):
            d = run_pass("pmcx_%s_%d" % (w, i), ["--pmc", *ctrs], ["--counter-probe", w])
            acc = collections.defaultdict(lambda: collections.defaultdict(list))
            for r in counter_rows(d):
                if "msd::" in r["Kernel_Name"]:
                    acc[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
            for nm, c in acc.items():
                for k, v in c.items():
                    vals.setdefault(nm, {})[k] = sorted(v)[len(v) // 2]
        out.append("%s\n" % w)
        for nm, c in vals.items():
            cyc = c.get("GRBM_GUI_ACTIVE", 0.0) / 8
            if cyc < 20000:
                continue
            out.append("  %s\n" % nm)
            out.append("    kernel cycles %.0f   MFMA instructions %.0f   VALU %.0f   SALU %.0f   LDS %.0f   vector memory reads %.0f (per-wave counts)\n"
                       % (cyc, c["SQ_INSTS_MFMA"], c["SQ_INSTS_VALU"], c["SQ_INSTS_SALU"], c["SQ_INSTS_LDS"], c["SQ_INSTS_VMEM_RD"]))
            out.append("    MFMA busy %.3f (%.1f busy cycles per instruction)   vector ALU %.3f   LDS busy %.3f   waiting %.3f (on LDS %.3f)   L2 hit %.3f   LDS conflict share %.3f\n"
                       % (c["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024 * cyc), c["SQ_VALU_MFMA_BUSY_CYCLES"] / max(c["SQ_INSTS_MFMA"], 1),
                          4 * c["SQ_ACTIVE_INST_VALU"] / (1024 * cyc), c["SQ_LDS_IDX_ACTIVE"] / (256 * cyc),
                          c["SQ_WAIT_INST_ANY"] / max(c["SQ_WAVE_CYCLES"], 1), c["SQ_WAIT_INST_LDS"] / max(c["SQ_WAVE_CYCLES"], 1),
                          c["TCC_HIT_sum"] / max(c["TCC_HIT_sum"] + c["TCC_MISS_sum"], 1),
                          c["SQ_LDS_BANK_CONFLICT"] / max(c["SQ_LDS_IDX_ACTIVE"], 1)))
        out.append("\n")
        write_summary("prefill_attn_counters_pmc.txt", "".join(out))  # written as it grows
    print("".join(out))


if __name__ == "__main__":
    what = sys.argv[1] if len(sys.argv) > 1 else "all"
    os.makedirs(PROF, exist_ok=True)
    if what in ("trace", "all"):
        do_trace()
    if what in ("trace_extras", "all"):
        do_trace_extras()
    if what in ("traffic", "all"):
        do_traffic()
    if what in ("counters", "all"):
        # an optional comma list restricts the workloads (the summary file then holds only those)
        do_counters(sys.argv[2].split(",") if len(sys.argv) > 2 else None)
