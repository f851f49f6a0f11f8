"""Secondary benchmark legs printed inside bench.py's JSON line under "extras".

Each leg times one C-ABI entry point on the shapes the benchmark spec lists for it, with HIP events
on the launch stream, inputs resident in HBM and (for memory-bound shapes) weight / KV copies
cycled so that the working set exceeds twice the 256 MB last-level cache.  Microsecond-scale calls
are marshalled once and replayed as HIP graphs (time_calls); millisecond-scale ones run eagerly.  Figures: time per
call, algorithmic GB/s or executed/effective TOP/s, and the fraction of the MI355X peak that
bounds the leg.  The comparison kernels (dequantise-then-BF16-MFMA) run beside the MSD kernels.
"""
import numpy as np
import torch

HBM = 8000.0
INT8_TOPS = 5000.0
FP4_TFLOPS = 10100.0
LLC = 256 << 20


def _eager_us(fn, n):
    """HIP-event time per call of n eager calls on the current stream (for millisecond-scale kernels)."""
    st = torch.cuda.current_stream()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(st)
    for i in range(n):
        fn(i)
    e1.record(st)
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def _bf16(bits, dev):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)


def _copies(t, nbytes):
    n = max(2, -(-2 * LLC // max(nbytes, 1)) + 1)
    n = min(n, 48)
    return [t] + [t.clone() for _ in range(n - 1)]


def _rand_i8(shape, dev, seed):
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    return torch.randint(-127, 128, shape, dtype=torch.int8, device=dev, generator=g)


def leg_prefill(msd, synth, time_calls, dev):
    """W8A16 prefill shapes (MFMA-bound): executed ops 4MKN against the INT8 peak."""
    out = []
    for (M, K, N) in [(2048, 8192, 8192), (8192, 8192, 8192), (2048, 8192, 28672), (8192, 8192, 28672)]:
        # M distinct rows, N(0,1) with 1 % of the channels scaled by 50, drawn on the device (set-up time)
        gx = torch.Generator(device=dev)
        gx.manual_seed(synth.seed_for(2, M))
        xf = torch.randn((M, K), device=dev, generator=gx)
        xf[:, torch.randperm(K, device=dev, generator=gx)[:round(0.01 * K)]] *= 50.0
        x = xf.to(torch.bfloat16)
        del xf
        W = _rand_i8((N, K), dev, 5)
        s = torch.rand(N, device=dev) * 0.009 + 0.001
        y = torch.empty((M, N), dtype=torch.float32, device=dev)
        ws = torch.empty(msd.lib().msd_gemm_w8a16_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
        Wp = msd.msd_pack_weights_w8(W)  # one-time repack, not timed
        f = lambda i: msd.msd_gemm_w8a16_packed(x, Wp, s, y=y, ws=ws)
        f(0)
        us = sorted(_eager_us(f, 2) for _ in range(5))[2]   # median of five timings of two calls each
        fc = lambda i: msd.msd_gemm_w8a16(x, W, s, y=y, ws=ws)
        fc(0)
        us_canon = sorted(_eager_us(fc, 2) for _ in range(5))[2]
        rec = {"M": M, "K": K, "N": N, "us": round(us, 1), "weights": "packed", "canonical_weights_us": round(us_canon, 1),
               "exec_TOPS": round(4.0 * M * K * N / us / 1e6, 1),
               "eff_TOPS": round(2.0 * M * K * N / us / 1e6, 1),
               "int8_mfma_frac": round(4.0 * M * K * N / us / 1e6 / INT8_TOPS, 4)}
        try:  # the matrix pipe alone on the same shape and data (no fill, no barriers, no LDS traffic)
            h = lambda i: msd.msd_probe_mfma_w8a16(x, W, s, y=y, ws=ws)
            h(0)
            us3 = _eager_us(h, 3)
            rec["mfma_only_us"] = round(us3, 1)
            rec["mfma_only_TOPS"] = round(4.0 * M * K * N / us3 / 1e6, 1)
            rec["frac_of_mfma_only"] = round(us3 / us, 3)
        except Exception as e:  # noqa: BLE001
            rec["probe_error"] = str(e)
        ws2 = g = None
        try:
            ws2 = torch.empty(msd.lib().msd_dequant_gemm_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
            g = lambda i: msd.msd_dequant_gemm_w8a16(x, W, s, y=y, ws=ws2)
            g(0)
            us2 = _eager_us(g, 2)
            rec["cmp_dequant_us"] = round(us2, 1)
            rec["speedup_vs_dequant"] = round(us2 / us, 3)
            rec["canonical_speedup_vs_dequant"] = round(us2 / us_canon, 3)
        except Exception as e:  # noqa: BLE001
            rec["cmp_error"] = str(e)
        out.append(rec)
        del x, W, Wp, y, ws, ws2, f, fc, g
        torch.cuda.empty_cache()
    return out


def leg_w4(msd, synth, time_calls, dev):
    out = []
    K, N = 8192, 28672
    codes, exps = synth.mxfp4_weights(synth.seed_for(3, 0), 2048, K)
    codes = torch.from_numpy(codes).to(dev).repeat(N // 2048, 1).contiguous()
    exps = torch.from_numpy(exps).to(dev).repeat(N // 2048, 1).contiguous()
    wbytes = K * N // 2 + K * N // 32
    reps = [(codes, exps)] + [(codes.clone(), exps.clone()) for _ in range(-(-2 * LLC // wbytes))]
    preps = [msd.msd_pack_weights_w4(c, e) for (c, e) in reps]  # one-time repack, not timed
    for M in (1, 32, 4096):
        x = _bf16(synth.activations(synth.seed_for(3, M), min(M, 64), K), dev)
        if M > 64:
            x = x.repeat(M // 64, 1).contiguous()
        y = torch.empty((M, N), dtype=torch.float32, device=dev)
        ws = torch.empty(msd.lib().msd_gemm_w4a16_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
        f = lambda i: msd.msd_gemm_w4a16_packed(x, *preps[i % len(reps)], N, y=y, ws=ws, prepare=M <= 32)
        fc = lambda i: msd.msd_gemm_w4a16(x, *reps[i % len(reps)], y=y, ws=ws, prepare=M <= 32)
        if M <= 32:
            us = time_calls(f, 2 * len(reps))
            us_canon = time_calls(fc, 2 * len(reps))
        else:
            f(0)
            us = _eager_us(f, 3)
            fc(0)
            us_canon = _eager_us(fc, 3)
        b = wbytes + 2 * M * K + 4 * M * N
        if M == 1:  # bare read of the same weight bytes (codes + scale bytes), two launches, cold
            def rd(i):
                c, e = reps[i % len(reps)]
                return [msd.msd_stream_read(c, prepare=True), msd.msd_stream_read(e, prepare=True)]
            class _Both:
                def __init__(self, ps): self.ps = ps
                def __call__(self):
                    for p_ in self.ps: p_()
            bare_us = time_calls(lambda i: _Both(rd(i)), 2 * len(reps))
            # the same number of bytes as one linear array in one launch (cold copies of a plain buffer)
            lin = [torch.empty(wbytes, dtype=torch.uint8, device=dev).fill_(i_) for i_ in range(len(reps))]
            bare_lin_us = time_calls(lambda i: msd.msd_stream_read_linear(lin[i % len(lin)], prepare=True), 2 * len(lin))
            del lin
        rec = {"M": M, "K": K, "N": N, "us": round(us, 1), "weights": "packed", "canonical_weights_us": round(us_canon, 1),
               "GBps": round(b / us / 1e3, 1),
               "hbm_frac": round(b / us / 1e3 / HBM, 4), "exec_TFLOPS": round(4.0 * M * K * N / us / 1e6, 1),
               "fp4_mfma_frac": round(4.0 * M * K * N / us / 1e6 / FP4_TFLOPS, 4)}
        if M <= 32:
            rec["bare_weight_read_us"] = round(bare_us, 1)
            rec["bare_linear_read_us"] = round(bare_lin_us, 1)
        else:  # the matrix pipe alone on the same shape and data
            try:
                h = lambda i: msd.msd_probe_mfma_w4a16(x, *reps[i % len(reps)], y=y, ws=ws)
                h(0)
                us3 = _eager_us(h, 3)
                rec["mfma_only_us"] = round(us3, 1)
                rec["mfma_only_TFLOPS"] = round(4.0 * M * K * N / us3 / 1e6, 1)
                rec["frac_of_mfma_only"] = round(us3 / us, 3)
            except Exception as e:  # noqa: BLE001
                rec["probe_error"] = str(e)
        try:
            ws2 = torch.empty(msd.lib().msd_dequant_gemm_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
            g = lambda i: msd.msd_dequant_gemm_w4a16(x, *reps[i % len(reps)], y=y, ws=ws2, prepare=M <= 32)
            if M <= 32:
                us2 = time_calls(g, 2 * len(reps))
            else:
                g(0)
                us2 = _eager_us(g, 2)
            rec["cmp_dequant_us"] = round(us2, 1)
            rec["speedup_vs_dequant"] = round(us2 / us, 3)
            rec["canonical_speedup_vs_dequant"] = round(us2 / us_canon, 3)
        except Exception as e:  # noqa: BLE001
            rec["cmp_error"] = str(e)
        out.append(rec)
    return out


def leg_attn(msd, synth, time_calls, dev):
    out = []
    B, Hq, Hkv, d = 16, 32, 8, 128
    q = _bf16(synth.queries(synth.seed_for(4, 0), B, Hq, d), dev)
    for L in (4096, 32768):
        kvbytes = 2 * B * Hkv * L * d
        n = max(2, min(6, -(-2 * LLC // kvbytes) + 1)) if L <= 4096 else 2
        sets = []
        for r in range(n):
            Kc = _rand_i8((B, Hkv, L, d), dev, 11 + r)
            Vc = _rand_i8((B, Hkv, L, d), dev, 31 + r)
            ks = torch.rand((B, Hkv, L), device=dev) * 0.02 + 0.02
            vs = torch.rand((B, Hkv, L), device=dev) * 0.02 + 0.02
            sets.append((Kc, Vc, ks, vs))
        o = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
        ws = torch.empty(msd.lib().msd_attn_decode_int8kv_workspace_bytes(B, Hq, Hkv, d, L), dtype=torch.uint8,
                         device=dev)
        f = lambda i: msd.msd_attn_decode_int8kv(q, *sets[i % n], msd.MSD_PER_TOKEN, out=o, ws=ws, prepare=True)
        us = time_calls(f, 4 * n)
        # the comparison kernel (K, V lifted to BF16 in registers) and the paper's per-channel scale mode
        fc = lambda i: msd.msd_dequant_attn_decode_int8kv(q, *sets[i % n], msd.MSD_PER_TOKEN, out=o, ws=ws,
                                                          prepare=True)
        us_cmp = time_calls(fc, 4 * n)
        kc = torch.rand((Hkv, d), device=dev) * 0.02 + 0.02
        vc = torch.rand((Hkv, d), device=dev) * 0.02 + 0.02
        fch = lambda i: msd.msd_attn_decode_int8kv(q, sets[i % n][0], sets[i % n][1], kc, vc, msd.MSD_PER_CHANNEL,
                                                   out=o, ws=ws, prepare=True)
        us_ch = time_calls(fch, 4 * n)
        fcc = lambda i: msd.msd_dequant_attn_decode_int8kv(q, sets[i % n][0], sets[i % n][1], kc, vc,
                                                           msd.MSD_PER_CHANNEL, out=o, ws=ws, prepare=True)
        us_ch_cmp = time_calls(fcc, 4 * n)
        us_low = time_calls(lambda i: msd.msd_attn_decode_int8kv_variant(msd.MSD_VARIANT_ATTN_LOWPREC, q, *sets[i % n],
                                                                         msd.MSD_PER_TOKEN, out=o, ws=ws, prepare=True), 4 * n)
        # accuracy of both kernels against an fp64 attention over the exactly dequantised cache (two batch
        # entries; the quantity of the paper's flash-attention error table, Sec. 6.4, on this workload)
        acc = None
        if L <= 4096:
            def truth(Kc, Vc, sk_, sv_, per_token, nb=2):
                Kd, Vd = Kc[:nb].double(), Vc[:nb].double()
                if per_token:
                    Kd, Vd = Kd * sk_[:nb, :, :, None].double(), Vd * sv_[:nb, :, :, None].double()
                else:
                    Kd, Vd = Kd * sk_[None, :, None, :].double(), Vd * sv_[None, :, None, :].double()
                qg = q[:nb].double().view(nb, Hkv, Hq // Hkv, d)
                P = torch.softmax(torch.einsum("bhgd,bhld->bhgl", qg, Kd) / d ** 0.5, dim=-1)
                return torch.einsum("bhgl,bhld->bhgd", P, Vd).reshape(nb, Hq, d)

            def rel(t):
                return float(((o[:2].double() - t).norm() / t.norm()).item())

            Kc0, Vc0, ks0, vs0 = sets[0]
            acc = {}
            t_tok, t_ch = truth(Kc0, Vc0, ks0, vs0, True), truth(Kc0, Vc0, kc, vc, False)
            low = lambda *a_, **k_: msd.msd_attn_decode_int8kv_variant(msd.MSD_VARIANT_ATTN_LOWPREC, *a_, **k_)
            for name, fn, args_, t in (("msd_per_token", msd.msd_attn_decode_int8kv, (ks0, vs0, msd.MSD_PER_TOKEN), t_tok),
                                       ("msd_lowprec_per_token", low, (ks0, vs0, msd.MSD_PER_TOKEN), t_tok),
                                       ("msd_lowprec_per_channel", low, (kc, vc, msd.MSD_PER_CHANNEL), t_ch),
                                       ("dequant_per_token", msd.msd_dequant_attn_decode_int8kv, (ks0, vs0, msd.MSD_PER_TOKEN), t_tok),
                                       ("msd_per_channel", msd.msd_attn_decode_int8kv, (kc, vc, msd.MSD_PER_CHANNEL), t_ch),
                                       ("dequant_per_channel", msd.msd_dequant_attn_decode_int8kv, (kc, vc, msd.MSD_PER_CHANNEL), t_ch)):
                fn(q, Kc0, Vc0, *args_, out=o, ws=ws)
                torch.cuda.synchronize()
                acc[name] = float("%.3g" % rel(t))
            del t_tok, t_ch
        b = kvbytes + 8 * B * Hkv * L + 2 * B * Hq * d + 4 * B * Hq * d
        # bare read of the same K and V bytes (one launch each), same cold-cache protocol
        class _Both:
            def __init__(self, ps): self.ps = ps
            def __call__(self):
                for p_ in self.ps: p_()
        bare_us = time_calls(lambda i: _Both([msd.msd_stream_read(sets[i % n][0].view(-1, 4096), prepare=True),
                                              msd.msd_stream_read(sets[i % n][1].view(-1, 4096), prepare=True)]), 4 * n)
        out.append({"B": B, "Hq": Hq, "Hkv": Hkv, "d": d, "L": L, "us": round(us, 1),
                    "GBps": round(b / us / 1e3, 1), "hbm_frac": round(b / us / 1e3 / HBM, 4),
                    "bare_kv_read_us": round(bare_us, 1), "dequant_us": round(us_cmp, 1),
                    "speedup_vs_dequant": round(us_cmp / us, 3), "lowprec_us": round(us_low, 1),
                    "per_channel": {"us": round(us_ch, 1), "dequant_us": round(us_ch_cmp, 1),
                                    "GBps": round((kvbytes + 6 * B * Hq * d) / us_ch / 1e3, 1),
                                    "speedup_vs_dequant": round(us_ch_cmp / us_ch, 3)}})
        if acc is not None:
            out[-1]["rel_l2_vs_fp64"] = acc
        del sets
        torch.cuda.empty_cache()
    return out


def leg_nq_sweep(msd, synth, time_calls, dev):
    """Query rows per KV head (the paper's Nq, Sec. 4.4): MSD against the dequantising comparison kernel at
    B = 16, Hkv = 8, L = 4096, d = 128, per-channel scales (the paper's setting) and per-token scales, cold KV.
    The paper's cost model puts the crossover N* at about 20 to 32 rows on its hardware."""
    B, Hkv, d, L = 16, 8, 128, 4096
    kvbytes = 2 * B * Hkv * L * d
    n = 5
    sets = []
    for r in range(n):
        sets.append((_rand_i8((B, Hkv, L, d), dev, 51 + r), _rand_i8((B, Hkv, L, d), dev, 71 + r),
                     torch.rand((B, Hkv, L), device=dev) * 0.02 + 0.02, torch.rand((B, Hkv, L), device=dev) * 0.02 + 0.02))
    kc = torch.rand((Hkv, d), device=dev) * 0.02 + 0.02
    vc = torch.rand((Hkv, d), device=dev) * 0.02 + 0.02
    rows = []
    for G in (1, 2, 4, 8, 12, 16, 24, 32, 48):
        Hq = Hkv * G
        q = _bf16(synth.queries(synth.seed_for(4, G), B, Hq, d), dev)
        o = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
        ws = torch.empty(msd.lib().msd_attn_decode_int8kv_workspace_bytes(B, Hq, Hkv, d, L), dtype=torch.uint8,
                         device=dev)
        row = {"Nq": G}
        for mode, name in ((msd.MSD_PER_CHANNEL, "per_channel"), (msd.MSD_PER_TOKEN, "per_token")):
            def args(i):
                K_, V_, ks_, vs_ = sets[i % n]
                return (q, K_, V_, kc, vc, mode) if mode == msd.MSD_PER_CHANNEL else (q, K_, V_, ks_, vs_, mode)
            us = time_calls(lambda i: msd.msd_attn_decode_int8kv(*args(i), out=o, ws=ws, prepare=True), 2 * n)
            us_c = time_calls(lambda i: msd.msd_dequant_attn_decode_int8kv(*args(i), out=o, ws=ws, prepare=True), 2 * n)
            # the low-precision arithmetic of Sec. 4.4 (integer S / O merge, FP16 decomposition of P)
            us_l = time_calls(lambda i: msd.msd_attn_decode_int8kv_variant(msd.MSD_VARIANT_ATTN_LOWPREC, *args(i), out=o,
                                                                           ws=ws, prepare=True), 2 * n)
            row[name] = {"msd_us": round(us, 1), "dequant_us": round(us_c, 1), "speedup_vs_dequant": round(us_c / us, 3),
                         "msd_lowprec_us": round(us_l, 1), "lowprec_speedup_vs_dequant": round(us_c / us_l, 3)}
        rows.append(row)
    return {"B": B, "Hkv": Hkv, "d": d, "L": L, "kv_bytes": kvbytes, "rows": rows}


def leg_moe(msd, synth, time_calls, dev):
    """Grouped W8A16 GEMM (paper Sec. 7.5): E = 64 experts of N = 2048, K = 4096 (537 MB of INT8 weights, beyond
    the last-level cache), decode batches routed at random (multinomial counts); one grouped call against one
    msd_gemm_w8a16 call per active expert.  GB/s counts the weights of the active experts only."""
    E, N, K = 64, 2048, 4096
    W = _rand_i8((E, N, K), dev, 91)
    sc = torch.rand((E, N), device=dev) * 0.009 + 0.001
    rng = np.random.default_rng(91)
    out = []
    for T in (16, 64, 256):
        counts = rng.multinomial(T, np.ones(E) / E)
        # four routings that are rotations of each other: consecutive calls touch different experts, so that
        # the weights come from HBM even when one call's active set would fit the last-level cache
        rolls = [np.roll(counts, 16 * r) for r in range(4)]
        offs_np = [np.concatenate([[0], np.cumsum(c)]) for c in rolls]
        offs = [torch.from_numpy(o.astype(np.int32)).to(dev) for o in offs_np]
        x = _bf16(synth.activations(synth.seed_for(8, T), T, K), dev)
        y = torch.empty((T, N), dtype=torch.float32, device=dev)
        ws = torch.empty(msd.lib().msd_gemm_w8a16_workspace_bytes(T, K, N), dtype=torch.uint8, device=dev)
        us = time_calls(lambda i: msd.msd_moe_gemm_w8a16(x, offs[i % 4], W, sc, y=y, ws=ws, prepare=True), 8)
        active = [e for e in range(E) if counts[e] > 0]

        class _PerExpert:
            def __init__(self, o, c):
                self.ps = [msd.msd_gemm_w8a16(x[o[e]:o[e + 1]], W[e], sc[e], y=y[o[e]:o[e + 1]], ws=ws, prepare=True)
                           for e in range(E) if c[e] > 0]
            def __call__(self):
                for p_ in self.ps: p_()
        us_loop = time_calls(lambda i: _PerExpert(offs_np[i % 4], rolls[i % 4]), 4)
        wbytes = len(active) * N * K
        out.append({"fmt": "w8a16", "T": T, "E": E, "active_experts": len(active),
                    "max_rows_per_expert": int(counts.max()),
                    "K": K, "N": N, "grouped_us": round(us, 1), "per_expert_calls_us": round(us_loop, 1),
                    "GBps_active_weights": round(wbytes / us / 1e3, 1),
                    "hbm_frac": round(wbytes / us / 1e3 / HBM, 4)})
    del W
    torch.cuda.empty_cache()
    # MXFP4 experts, twice as many so that the weights still exceed the last-level cache
    E = 128
    g = torch.Generator(device=dev)
    g.manual_seed(92)
    codes = torch.randint(0, 256, (E, N, K // 2), dtype=torch.uint8, device=dev, generator=g)
    exps = torch.randint(118, 124, (E, N, K // 32), dtype=torch.uint8, device=dev, generator=g)
    for T in (16, 64, 256):
        counts = rng.multinomial(T, np.ones(E) / E)
        rolls = [np.roll(counts, 32 * r) for r in range(4)]
        offs = [torch.from_numpy(np.concatenate([[0], np.cumsum(c)]).astype(np.int32)).to(dev) for c in rolls]
        x = _bf16(synth.activations(synth.seed_for(8, T + 1), T, K), dev)
        y = torch.empty((T, N), dtype=torch.float32, device=dev)
        ws = torch.empty(msd.lib().msd_gemm_w4a16_workspace_bytes(T, K, N), dtype=torch.uint8, device=dev)
        us = time_calls(lambda i: msd.msd_moe_gemm_w4a16(x, offs[i % 4], codes, exps, y=y, ws=ws, prepare=True), 8)
        n_act = int((counts > 0).sum())
        wbytes = n_act * (N * K // 2 + N * K // 32)
        out.append({"fmt": "w4a16", "T": T, "E": E, "active_experts": n_act, "max_rows_per_expert": int(counts.max()),
                    "K": K, "N": N, "grouped_us": round(us, 1), "GBps_active_weights": round(wbytes / us / 1e3, 1),
                    "hbm_frac": round(wbytes / us / 1e3 / HBM, 4)})
    return out


def leg_mfma_rate(msd, synth, time_calls, dev):
    """The matrix pipe alone (msd_probe_mfma_rate: nothing but matrix instructions, operands read once) on random
    operand bits, the benchmark's kind of data, and on constant ones: same instruction stream, same cycles per
    instruction; what differs is the clock the chip sustains.  The random-bits figure is the ceiling of any GEMM
    kernel on this machine for such data."""
    out = {}
    g = torch.Generator(device=dev)
    g.manual_seed(11)
    rnd = torch.randint(-2 ** 31, 2 ** 31 - 1, (16384,), dtype=torch.int32, device=dev, generator=g)
    ones = torch.full((16384,), 0x01010101, dtype=torch.int32, device=dev)
    for name, fmt, peak, iters in (("int8_32x32x32", msd.MSD_INT8, INT8_TOPS, 20000), ("fp6xfp4_32x32x64", msd.MSD_MXFP4, FP4_TFLOPS, 20000)):
        rec = {}
        for label, buf in (("random_bits", rnd), ("constant_bits", ones)):
            msd.msd_probe_mfma_rate(fmt, buf, 100)
            torch.cuda.synchronize()
            ts = []
            for _ in range(3):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                ops = msd.msd_probe_mfma_rate(fmt, buf, iters)
                e1.record()
                e1.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e-3)
            t = sorted(ts)[1]
            rec[label] = {"ms": round(t * 1e3, 3), "Tops": round(ops / t / 1e12, 1), "frac_of_datasheet": round(ops / t / 1e12 / peak, 3)}
        out[name] = rec
    return out


def leg_lds_fill(msd, synth, time_calls, dev):
    """The LDS fill path alone (msd_probe_lds_fill_rate: the tile kernels' asynchronous fill instructions, ring and
    barriers with no fragment reads and no matrix instructions), one eight-wave workgroup per CU: from a 1 MB window
    every workgroup shares (L2 hits, like the activation codes), from disjoint ranges of a 1 GB buffer (HBM, like the
    weights), and half and half -- the mix of the batched-decode tiles.  Bytes a tile kernel moves into LDS divided
    by these rates bound its time from below whatever its arithmetic."""
    buf = torch.empty(((1 << 30) + (1 << 20),), dtype=torch.int8, device=dev)
    buf.random_(-128, 127)
    out = {"workgroups": 256, "waves_per_workgroup": 8, "bytes_in_flight_per_cu": 65536}
    rounds = 128
    for label, parts in (("l2_window", 4), ("half_window_half_stream", 2), ("hbm_stream", 0)):
        msd.msd_probe_lds_fill_rate(buf, 1 << 20, parts, rounds)
        torch.cuda.synchronize()
        ts = []
        for r in (rounds, 0):  # the empty launch is subtracted
            tt = []
            for _ in range(5):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                nbytes = msd.msd_probe_lds_fill_rate(buf, 1 << 20, parts, r)
                e1.record()
                e1.synchronize()
                tt.append(e0.elapsed_time(e1) * 1e-3)
            ts.append(sorted(tt)[2])
        moved = 256 * rounds * 32768
        t = ts[0] - ts[1]
        out[label] = {"us": round(t * 1e6, 1), "TBps": round(moved / t / 1e12, 2), "GBps_per_cu": round(moved / t / 1e9 / 256, 1)}
    del buf
    torch.cuda.empty_cache()
    return out


def leg_cfg0(msd, synth, time_calls, dev):
    """The correctness configuration (M = 16, K = 1024, N = 1024, 1 MB of weights): launch-latency scale,
    time only, MSD and comparison kernel."""
    M, K, N = 16, 1024, 1024
    x = _bf16(synth.activations(synth.seed_for(0, 0), M, K), dev)
    W = _rand_i8((N, K), dev, 5)
    sc = torch.rand(N, device=dev) * 0.009 + 0.001
    y = torch.empty((M, N), dtype=torch.float32, device=dev)
    ws = torch.empty(msd.lib().msd_gemm_w8a16_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
    us = time_calls(lambda i: msd.msd_gemm_w8a16(x, W, sc, y=y, ws=ws, prepare=True), 16)
    us_c = time_calls(lambda i: msd.msd_dequant_gemm_w8a16(x, W, sc, y=y, ws=ws, prepare=True), 16)
    return {"M": M, "K": K, "N": N, "msd_us": round(us, 2), "dequant_us": round(us_c, 2),
            "exec_TOPS": round(4.0 * M * K * N / us / 1e6, 2)}


def leg_mla(msd, synth, time_calls, dev):
    """Attention over a latent KV cache (576-channel keys, 512-channel values from the same rows; paper Sec. 4.4 /
    Sec. 7.3): B = 32 batch entries, Hq query heads on the one latent, per-token scales, cold cache.  Bytes = the
    cached rows once; ops = executed INT8 multiply-adds x 2 (both components, key and value products)."""
    B, d = 32, 576
    out = []
    for L in (4096, 32768):
        n = 3 if L <= 4096 else 2
        sets = [(_rand_i8((B, L, d), dev, 201 + r), torch.rand((B, L), device=dev) * 0.02 + 0.02) for r in range(n)]
        for Hq in (16, 128):
            if L > 4096 and Hq > 16:
                continue
            q = _bf16(synth.queries(synth.seed_for(9, Hq), B, Hq, d), dev)
            o = torch.empty((B, Hq, 512), dtype=torch.float32, device=dev)
            ws = torch.empty(msd.lib().msd_mla_decode_int8kv_workspace_bytes(B, Hq, L), dtype=torch.uint8, device=dev)
            f = lambda i: msd.msd_mla_decode_int8kv(q, sets[i % n][0], sets[i % n][1], msd.MSD_PER_TOKEN,
                                                    1.0 / 192.0 ** 0.5, out=o, ws=ws, prepare=True)
            us = time_calls(f, 2 * n)
            fc = lambda i: msd.msd_dequant_mla_decode_int8kv(q, sets[i % n][0], sets[i % n][1], msd.MSD_PER_TOKEN,
                                                             1.0 / 192.0 ** 0.5, out=o, ws=ws, prepare=True)
            us_c = time_calls(fc, 2 * n)  # the dequantise-then-BF16 comparison kernel, same protocol
            byts = B * L * d + 4 * B * L
            ops = 2.0 * 2 * B * Hq * L * (576 + 512)
            out.append({"B": B, "Hq": Hq, "L": L, "us": round(us, 1), "GBps": round(byts / us / 1e3, 1),
                        "hbm_frac": round(byts / us / 1e3 / HBM, 4), "exec_TOPS": round(ops / us / 1e6, 1),
                        "int8_mfma_frac": round(ops / us / 1e6 / INT8_TOPS, 4), "dequant_us": round(us_c, 1),
                        "speedup_vs_dequant": round(us_c / us, 3)})
            if L <= 4096:  # accuracy against an fp64 attention over the dequantised rows (two batch entries)
                C0, s0 = sets[0]
                msd.msd_mla_decode_int8kv(q, C0, s0, msd.MSD_PER_TOKEN, 1.0 / 192.0 ** 0.5, out=o, ws=ws)
                torch.cuda.synchronize()
                Cd = C0[:2].double() * s0[:2, :, None].double()
                P = torch.softmax(torch.einsum("bhd,bld->bhl", q[:2].double(), Cd) / 192.0 ** 0.5, dim=-1)
                t = torch.einsum("bhl,bld->bhd", P, Cd[:, :, :512])
                out[-1]["rel_l2_vs_fp64"] = float("%.3g" % ((o[:2].double() - t).norm() / t.norm()).item())
                del Cd, P, t
        if L == 4096:
            # head-count sweep on the same cache (Sec. 4.4's crossover question on the latent shape): MSD against the
            # comparison kernel
            sweep = []
            for Hq in (1, 2, 4, 8, 16, 32, 64, 128):
                q = _bf16(synth.queries(synth.seed_for(9, 100 + Hq), B, Hq, d), dev)
                o = torch.empty((B, Hq, 512), dtype=torch.float32, device=dev)
                ws = torch.empty(msd.lib().msd_mla_decode_int8kv_workspace_bytes(B, Hq, L), dtype=torch.uint8, device=dev)
                us = time_calls(lambda i: msd.msd_mla_decode_int8kv(q, sets[i % n][0], sets[i % n][1], msd.MSD_PER_TOKEN,
                                                                    1.0 / 192.0 ** 0.5, out=o, ws=ws, prepare=True), 2 * n)
                us_c = time_calls(lambda i: msd.msd_dequant_mla_decode_int8kv(q, sets[i % n][0], sets[i % n][1],
                                                                              msd.MSD_PER_TOKEN, 1.0 / 192.0 ** 0.5, out=o,
                                                                              ws=ws, prepare=True), 2 * n)
                sweep.append({"Hq": Hq, "msd_us": round(us, 1), "dequant_us": round(us_c, 1),
                              "speedup_vs_dequant": round(us_c / us, 3)})
            out.append({"B": B, "L": L, "heads_sweep": sweep})
        del sets
        torch.cuda.empty_cache()
    return out


def leg_cmp_decode(msd, synth, time_calls, dev):
    """Dequant comparison kernel on the W8A16 decode shapes (same cold-cache protocol)."""
    out = []
    K = 4096
    for N in (4096, 14336):
        W = _rand_i8((N, K), dev, 3)
        reps = _copies(W, N * K)
        preps = [msd.msd_pack_weights_w8(w) for w in reps]  # one-time repack, not timed
        s = torch.rand(N, device=dev) * 0.009 + 0.001
        for M in (1, 8, 32, 128):
            x = _bf16(synth.activations(synth.seed_for(1, M), M, K), dev)
            y = torch.empty((M, N), dtype=torch.float32, device=dev)
            ws = torch.empty(msd.lib().msd_gemm_w8a16_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
            f = lambda i: msd.msd_gemm_w8a16(x, reps[i % len(reps)], s, y=y, ws=ws, prepare=True)
            ws2 = torch.empty(msd.lib().msd_dequant_gemm_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
            g = lambda i: msd.msd_dequant_gemm_w8a16(x, reps[i % len(reps)], s, y=y, ws=ws2, prepare=True)
            fp = lambda i: msd.msd_gemm_w8a16_packed(x, preps[i % len(reps)], s, y=y, ws=ws, prepare=True)
            us_msd = time_calls(f, 2 * len(reps))
            us_pk = time_calls(fp, 2 * len(reps))
            us_cmp = time_calls(g, 2 * len(reps))
            # like for like first: both paths on the canonical layout; then MSD on its packed layout
            out.append({"M": M, "K": K, "N": N, "msd_us": round(us_msd, 2), "msd_packed_us": round(us_pk, 2),
                        "dequant_us": round(us_cmp, 2), "speedup_vs_dequant": round(us_cmp / us_msd, 3),
                        "packed_speedup_vs_dequant": round(us_cmp / us_pk, 3)})
        del reps, preps, W
        torch.cuda.empty_cache()
    return out


def leg_variants(msd, synth, time_calls, dev):
    """Decomposition-constant variants (paper Sec. 3.3) on a 2048 x 2048 x 2048 GEMM: relative L2 error of
    the GPU output against an fp64 product of the same activations and exactly dequantised weights, and
    time per call -- the variants change constants only, so the times should agree.  The MXFP4 rows are
    the quantities of the paper's design-evolution table (Gaussian activations, MXFP4 weights)."""
    M = K = N = 2048
    out = {"shape": [M, K, N]}

    def rel(y, truth):
        return float(torch.linalg.norm(y.double() - truth) / torch.linalg.norm(truth))

    xb = synth.activations(synth.seed_for(7, 0), M, K, outliers=False)
    x = _bf16(xb, dev)
    xd = x.double()
    # INT8 weights
    Wn, sn = synth.int8_weights(synth.seed_for(7, 1), N, K)
    W, sc = torch.from_numpy(Wn).to(dev), torch.from_numpy(sn).to(dev)
    truth = (xd @ W.double().T) * sc.double()[None, :]
    y = torch.empty((M, N), dtype=torch.float32, device=dev)
    ws = torch.empty(max(msd.lib().msd_gemm_w8a16_workspace_bytes(M, K, N),
                         msd.lib().msd_dequant_gemm_workspace_bytes(M, K, N)), dtype=torch.uint8, device=dev)
    w8 = {}
    for name, fn in (("main", lambda i: msd.msd_gemm_w8a16(x, W, sc, y=y, ws=ws)),
                     ("fractional", lambda i: msd.msd_gemm_w8a16_variant(msd.MSD_VARIANT_INT8_FRACTIONAL, x, W, sc,
                                                                         y=y, ws=ws)),
                     ("dequant_bf16", lambda i: msd.msd_dequant_gemm_w8a16(x, W, sc, y=y, ws=ws))):
        fn(0)
        torch.cuda.synchronize()
        w8[name] = {"rel_l2_vs_fp64": float("%.4g" % rel(y, truth)), "us": round(_eager_us(fn, 20), 1)}
    out["w8a16"] = w8
    del truth, W
    # MXFP4 weights
    cn, en = synth.mxfp4_weights(synth.seed_for(7, 2), N, K)
    codes, exps = torch.from_numpy(cn).to(dev), torch.from_numpy(en).to(dev)
    truth = xd @ torch.from_numpy(synth.dequantize_mxfp4(cn, en).astype(np.float64)).to(dev).T
    ws = torch.empty(max(msd.lib().msd_gemm_w4a16_workspace_bytes(M, K, N),
                         msd.lib().msd_dequant_gemm_workspace_bytes(M, K, N)), dtype=torch.uint8, device=dev)
    w4 = {}
    for name, var in (("v1", msd.MSD_VARIANT_MXFP4_V1), ("v2", msd.MSD_VARIANT_MXFP4_V2),
                      ("v3_main", msd.MSD_VARIANT_MAIN), ("e2m1_grid_ablation", msd.MSD_VARIANT_MXFP4_E2M1)):
        fn = lambda i, var=var: msd.msd_gemm_w4a16_variant(var, x, codes, exps, y=y, ws=ws)
        fn(0)
        torch.cuda.synchronize()
        w4[name] = {"rel_l2_vs_fp64": float("%.4g" % rel(y, truth)), "us": round(_eager_us(fn, 20), 1)}
    out["w4a16"] = w4
    out["paper_table_l2"] = {"v1": 0.0182, "v2": 0.0107, "v3": 0.0101}
    return out


def run(want, msd, synth, time_calls, dev):
    res = {}
    legs = {"mfma_rate": leg_mfma_rate, "lds_fill": leg_lds_fill, "cfg0": leg_cfg0, "prefill": leg_prefill, "w4": leg_w4, "attn": leg_attn, "cmp": leg_cmp_decode,
            "variants": leg_variants, "nq": leg_nq_sweep, "moe": leg_moe, "mla": leg_mla}
    for name, fn in legs.items():
        if name in want:
            try:
                res[name] = fn(msd, synth, time_calls, dev)
            except Exception as e:  # noqa: BLE001
                res[name] = {"error": repr(e)}
            torch.cuda.empty_cache()
    return res
