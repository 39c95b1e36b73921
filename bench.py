#!/usr/bin/env python3
"""Benchmark of the HieraSparse hot path on one MI355X.

A step = one pass of the whole path on the Llama-3.1-8B-shaped workload
(B=1, 32 query heads / 8 KV heads, head dim 128, context 32768, bf16):
  compress K,V to 2:4 (fused prune + pack)  ->  causal prefill attention over the
  packed cache  ->  one decode-attention token against the packed cache.
Inputs are synthetic (seeded; keys with outlier channels) and resident in HBM
before the timed region.  The packed cache rotates through several buffers so
that the decode stage of a step reads a cache that was written several steps
(> 512 MB of other traffic) earlier: its bytes come from HBM, not from the
256 MB last-level cache.

Prints ONE JSON line: metric / value / unit / stages, the roofline objects of the three kernels, the extra
legs (stages_extra) and the oracle timed on the host (cpu_baseline).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_DENSE_PEAK_TFLOPS = 2500.0
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "bench_cfg1_hbm_traffic.md")


def traffic_from_profile(kernel_prefix):
    """HBM bytes per launch of a kernel of the headline step, as the last committed rocprofv3 counter run
    measured them: the "fetched MB (scaled)" + "written MB (scaled)" columns of the summary table (two --pmc
    runs, FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a 256 MiB copy).  None
    if the summary is missing or has no row for the kernel: a reading, never a constant of this file."""
    try:
        for line in open(TRAFFIC_SUMMARY):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) >= 6 and cells[1].startswith(kernel_prefix):
                return (float(cells[3]) + float(cells[5])) * 1e6
    except (OSError, ValueError):
        pass
    return None


def packed_bytes(B, Hkv, T, counts):
    n_skip, ndk, nsk, ndv, nsv = counts
    per_row = (ndk + ndv) * 16384 + (nsk + nsv) * 9216 + 2 * T * 4
    return B * Hkv * per_row


def cpu_baseline(cfg):
    """The oracle, as it stands, timed on the host on the same workload (same seeded inputs):
    prune + pack of the whole cache, decode attention over all heads, and causal prefill
    attention for a bounded sample of query rows.  `value` is the decode leg in the metric's
    unit (packed GB/s); the other legs are quoted in `sample`."""
    import numpy as np
    from oracle import hs_oracle as orc
    from paper_2604_16864_amd import workloads as wl
    # threads: the attention legs are numpy matrix products (the BLAS pool); prune + pack is Python loops
    # over tiles on one thread
    host_cpus = os.cpu_count() or 1
    blas = None
    try:
        from threadpoolctl import threadpool_info
        pools = [p.get("num_threads") for p in threadpool_info() if p.get("user_api") == "blas"]
        blas = max(pools) if pools else None
    except ImportError:
        pass
    if blas is None:
        blas = int(os.environ.get("OMP_NUM_THREADS", host_cpus))
    cores = int(blas)
    n_rows = 48
    Q, K, V = wl.make_qkv(cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["L"], cfg["D"], cfg["L"], cfg["seed"], cfg["k_outliers"])
    q = Q[:, :, -1, :].copy()
    t0 = time.perf_counter()
    pk, pv, _ = orc.compress_kv(K, V, Bt=64)
    t_c = time.perf_counter() - t0
    t0 = time.perf_counter()
    orc.attention_decode(q, pk, pv)
    t_d = time.perf_counter() - t0
    rows = wl.sample_rows(cfg["B"], cfg["Hq"], cfg["L"], n_rows, seed=cfg["seed"] + 4)
    t0 = time.perf_counter()
    orc.attention_rows(Q, pk, pv, rows, causal=True)
    t_p = time.perf_counter() - t0
    nbytes = pk.nbytes() + pv.nbytes()
    return {"value": nbytes / t_d / 1e9, "unit": "GB/s", "cores": int(cores), "host_cpus": int(host_cpus),
            "threads_note": "decode and prefill legs: BLAS pool of `cores` threads; prune+pack: 1 thread", "kind": "oracle",
            "sample": f"same workload and inputs: oracle decode attention over all {cfg['Hkv']} KV heads "
                      f"({nbytes / 1e6:.1f} MB packed) {t_d:.2f} s; prune+pack of the whole cache {t_c:.2f} s; "
                      f"causal prefill attention for {n_rows} sampled query rows {t_p:.2f} s "
                      f"({t_p / n_rows * 1e3:.0f} ms per row incl. one unpack of the cache)",
            "compress_s": t_c, "decode_s": t_d, "prefill_rows": n_rows, "prefill_rows_s": t_p,
            "prefill_full_s_extrapolated": t_p / n_rows * cfg["B"] * cfg["Hq"] * cfg["L"]}


def _time(torch, fn, reps, warm=1):
    for _ in range(warm):
        fn(0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


LEGS = ("sk0_sv1", "block_sparsity_sweep", "decode_b8_128k", "prefill_64k", "prefill_16k", "chunked_prefill_128k",
        "paper_kernel_shape_b8_32k", "fp16_same_shape")
PREFILL_REPS = 5          # timed repetitions of every prefill leg (after one warm-up)


def prefill_floor_s(flops_dense_tiles, flops_sparse_tiles_dense_equiv):
    """Time the matrix pipes need at their published peak: dense tile pairs at the dense bf16 rate, 2:4
    tile pairs at twice that (half the multiplications are executed) -- the prefill model of Sec. III-D."""
    return flops_dense_tiles / (MFMA_BF16_DENSE_PEAK_TFLOPS * 1e12) + flops_sparse_tiles_dense_equiv / (2 * MFMA_BF16_DENSE_PEAK_TFLOPS * 1e12)


def extra_legs(hb, torch, Q, K, V, qd, sh, args):
    """Context numbers beside the headline: other sparsity settings of the same path.  Inputs of the
    large shapes are N(0,1) drawn on the device (seeded torch generator); everything else as in the step.
    args.legs / args.cases select legs and cases (profiling runs take one at a time)."""
    res = {}
    legs = LEGS if args.legs == "all" else tuple(x for x in args.legs.split(",") if x)
    cases = None if args.cases == "all" else set(args.cases.split(","))
    want = lambda case: cases is None or case in cases
    B, Hq, Hkv, L = sh.B, sh.Hq, sh.Hkv, sh.L
    T = L // 64
    ws_c = torch.empty(max(16, hb.workspace_bytes(sh, 0)), dtype=torch.uint8, device="cuda")
    n = hb.decode_auto_splits(sh)
    ws_d = torch.empty(hb.workspace_bytes(sh, 2, n), dtype=torch.uint8, device="cuda")
    Od = torch.empty_like(qd)
    flops1 = 4.0 * 128 * Hq * B * (L * (L + 1) / 2.0)
    if "sk0_sv1" in legs:
        # the paper's quality-preserving point: keys dense, values 2:4 (S_K = 0, S_V = 1), same workload
        pol = hb.make_policy(sparse_frac_k=0.0, sparse_frac_v=1.0)
        cts = hb.tile_counts(sh, pol)
        kvm = [hb.compress_kv(sh, pol, K, V, workspace=ws_c) for _ in range(6)]
        O = torch.empty_like(Q)
        t_p = _time(torch, lambda i: hb.prefill_attn(sh, Q, kvm[i % 6], causal=True, want_lse=False, out=O), PREFILL_REPS)
        t_d = _time(torch, lambda i: hb.decode_attn(sh, qd, kvm[i % 6], n_splits=n, want_lse=False, out=Od, workspace=ws_d), 24, warm=6)
        res["sk0_sv1_same_workload"] = {"prefill_ms": t_p * 1e3, "decode_us": t_d * 1e6,
                                        "prefill_mfma_frac": prefill_floor_s(flops1 / 2, flops1 / 2) / t_p,
                                        "decode_GBps": packed_bytes(B, Hkv, T, cts) / t_d / 1e9,
                                        "ideal_prefill_speedup": 4.0 / 3.0, "ideal_decode_speedup": 1.0 / (1.0 - 0.21875)}
        # differentiated sparsity: that prefill cache pruned further to S_K = S_V = 1 for decode
        # (the dense key pool is read, pruned and packed; the 2:4 value pool is copied)
        pol1 = hb.make_policy()
        cts1 = hb.tile_counts(sh, pol1)
        kv_dec = [hb.recompress_kv(sh, kvm[i], pol1) for i in range(6)]
        t_r = _time(torch, lambda i: hb.recompress_kv(sh, kvm[i % 6], pol1, out=kv_dec[i % 6]), 12, warm=2)
        t_d2 = _time(torch, lambda i: hb.decode_attn(sh, qd, kv_dec[i % 6], n_splits=n, want_lse=False, out=Od, workspace=ws_d), 24, warm=6)
        res["sk0_sv1_prefill_then_sk1_sv1_decode"] = {
            "recompress_us": t_r * 1e6,
            "recompress_GBps": (packed_bytes(B, Hkv, T, cts) + packed_bytes(B, Hkv, T, cts1)) / t_r / 1e9,
            "decode_us": t_d2 * 1e6, "decode_GBps": packed_bytes(B, Hkv, T, cts1) / t_d2 / 1e9}
        del kvm, kv_dec, O
    if "block_sparsity_sweep" in legs:
        # block-sparsity sweep S_K = S_V = S with the paper's pruning-loss ranking (Eq. 2c-d), against
        # the analytical curves of Sec. III-D: decode 1/(1 - 0.4375 S), prefill 4/(4 - 2S)
        O = torch.empty_like(Q)
        sweep_s = []
        for S in (0.0, 0.25, 0.5, 0.75, 1.0):
            pol = hb.make_policy(sparse_frac_k=S, sparse_frac_v=S)
            cts = hb.tile_counts(sh, pol)
            kvs_ = [hb.compress_kv(sh, pol, K, V, workspace=ws_c) for _ in range(6)]
            t_p = _time(torch, lambda i: hb.prefill_attn(sh, Q, kvs_[i % 6], causal=True, want_lse=False, out=O), PREFILL_REPS)
            t_d = _time(torch, lambda i: hb.decode_attn(sh, qd, kvs_[i % 6], n_splits=n, want_lse=False, out=Od, workspace=ws_d), 24, warm=6)
            sweep_s.append({"S": S, "prefill_ms": t_p * 1e3, "decode_us": t_d * 1e6, "packed_MB": packed_bytes(B, Hkv, T, cts) / 1e6,
                            "ideal_prefill_speedup": 4.0 / (4.0 - 2 * S), "ideal_decode_speedup": 1.0 / (1.0 - 0.4375 * S)})
            del kvs_
        for r in sweep_s:
            r["prefill_speedup_vs_S0"] = sweep_s[0]["prefill_ms"] / r["prefill_ms"]
            r["decode_speedup_vs_S0"] = sweep_s[0]["decode_us"] / r["decode_us"]
        res["block_sparsity_sweep_same_workload"] = sweep_s
        del O
    torch.cuda.empty_cache()
    g = torch.Generator(device="cuda")
    g.manual_seed(3000)
    if "decode_b8_128k" in legs:
        # hierarchical decode sweep: B8, 32/8 heads, L131072; skip {0, .25, .5, .75} of the tiles + 2:4 in the rest
        B3, L3 = 8, 131072
        sh3 = hb.make_shape(B3, Hq, Hkv, L3)
        K3 = torch.randn((B3, Hkv, L3, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        V3 = torch.randn((B3, Hkv, L3, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        q3 = torch.randn((B3, Hq, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        ws3 = torch.empty(hb.workspace_bytes(sh3, 0), dtype=torch.uint8, device="cuda")
        n3 = hb.decode_auto_splits(sh3)
        wsd3 = torch.empty(hb.workspace_bytes(sh3, 2, n3), dtype=torch.uint8, device="cuda")
        O3 = torch.empty_like(q3)
        sweep = []
        for name3, kw in (("dense", dict(sparse_frac_k=0.0, sparse_frac_v=0.0)), ("skip0", dict(skip_frac=0.0)),
                          ("skip0.25", dict(skip_frac=0.25)), ("skip0.5", dict(skip_frac=0.5)), ("skip0.75", dict(skip_frac=0.75))):
            if not want(name3):
                continue
            p3 = hb.make_policy(**kw)
            c3 = hb.tile_counts(sh3, p3)
            kv3 = hb.PackedKV(sh3, c3)
            t_c = _time(torch, lambda i: hb.compress_kv(sh3, p3, K3, V3, out=kv3, workspace=ws3), 5)
            t = _time(torch, lambda i: hb.decode_attn(sh3, q3, kv3, n_splits=n3, want_lse=False, out=O3, workspace=wsd3), 8, warm=2)
            nb = packed_bytes(B3, Hkv, L3 // 64, c3)
            dense_b = 2 * B3 * Hkv * L3 * 128 * 2
            ranked = kw.get("skip_frac", 0.0) > 0
            sweep.append({"case": name3, "decode_us": t * 1e6, "decode_GBps": nb / t / 1e9, "hbm_frac": nb / t / 1e9 / HBM_PEAK_GBPS,
                          "packed_MB": nb / 1e6, "compress_us": t_c * 1e6,
                          "compress_GBps": (dense_b + nb) / t_c / 1e9,
                          # floors: K, V read once + packed bytes written once at the HBM peak; a ranked policy has to
                          # read K, V once to score every tile and the kept tiles once more to pack them
                          "compress_frac_of_single_read_floor": (dense_b + nb) / (HBM_PEAK_GBPS * 1e9) / t_c,
                          "compress_frac_of_two_read_floor": ((dense_b * (2 - kw.get("skip_frac", 0.0)) if ranked else dense_b) + nb)
                                                             / (HBM_PEAK_GBPS * 1e9) / t_c})
            del kv3
        for r in sweep:
            if sweep[0]["case"] == "dense":
                r["speedup_vs_dense"] = sweep[0]["decode_us"] / r["decode_us"]
        res["decode_b8_128k"] = sweep
        del K3, V3, ws3
        torch.cuda.empty_cache()
    for leg, L4, key in (("prefill_64k", 65536, "prefill_64k"), ("prefill_16k", 16384, "prefill_16k")):
        if leg not in legs:
            continue
        # causal prefill with tile skipping: B1, 32/8 heads, N(0,1) inputs (L 65536: the long-prefill workload at the
        # highest hierarchical sparsity; L 16384: the 16K prefill workload)
        sh4 = hb.make_shape(1, Hq, Hkv, L4)
        K4 = torch.randn((1, Hkv, L4, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        V4 = torch.randn((1, Hkv, L4, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        Q4 = torch.randn((1, Hq, L4, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        O4 = torch.empty_like(Q4)
        ws4 = torch.empty(hb.workspace_bytes(sh4, 0), dtype=torch.uint8, device="cuda")
        flops4 = 4.0 * 128 * Hq * (L4 * (L4 + 1) / 2.0)
        pf = []
        for name4, kw in (("dense", dict(sparse_frac_k=0.0, sparse_frac_v=0.0)), ("2:4", dict()), ("2:4+skip0.75", dict(skip_frac=0.75))):
            if not want(name4):
                continue
            kv4 = hb.compress_kv(sh4, hb.make_policy(**kw), K4, V4, workspace=ws4)
            t = _time(torch, lambda i: hb.prefill_attn(sh4, Q4, kv4, causal=True, want_lse=False, out=O4), PREFILL_REPS)
            # tile pairs a causal query tile visits: those of kept tiles only (read back from the map; not timed)
            kept = (kv4.k_map != 0).double()                                      # [1, Hkv, T]
            pairs = float((kept * torch.arange(L4 // 64, 0, -1, device="cuda", dtype=torch.float64)).sum().item())
            # dense-equivalent flops of the visited pairs: 4 heads per kv head, 64 x 64 x 128 x 4 per pair, the
            # diagonal pair counted as half
            fl = 4.0 * 64 * 64 * 128 * (Hq // Hkv) * (pairs - 0.5 * float(kept.sum().item()))
            floor = prefill_floor_s(fl, 0.0) if name4 == "dense" else prefill_floor_s(0.0, fl)
            pf.append({"case": name4, "prefill_ms": t * 1e3, "dense_equiv_TFLOPs_of_full_causal": flops4 / t / 1e12,
                       "dense_equiv_TFLOPs_of_visited_tiles": fl / t / 1e12, "mfma_frac": floor / t})
            del kv4
        for r in pf:
            if pf[0]["case"] == "dense":
                r["speedup_vs_dense"] = pf[0]["prefill_ms"] / r["prefill_ms"]
        res[key] = pf
        del K4, V4, Q4, O4, ws4
        torch.cuda.empty_cache()
    if "chunked_prefill_128k" in legs:
        # chunked prefill as in the paper's end-to-end runs (Sec. V-B: 32K-token chunks): a cache allocated
        # for 128K tokens; per chunk one append (compress the chunk's K, V into the next pool slots) and one
        # causal attention call with the chunk's queries at their position
        Lc, chunk = 131072, 32768
        shc = hb.make_shape(1, Hq, Hkv, Lc)
        Tc, nct = Lc // 64, chunk // 64
        Kc = torch.randn((1, Hkv, Lc, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        Vc = torch.randn((1, Hkv, Lc, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        Qc = torch.randn((1, Hq, chunk, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        Oc = torch.empty_like(Qc)
        flops_c = 4.0 * 128 * Hq * (Lc * (Lc + 1) / 2.0)
        cp = []
        for name_c, stk, stv in (("dense", hb.DENSE, hb.DENSE), ("sk0_sv1", hb.DENSE, hb.SPARSE24), ("2:4", hb.SPARSE24, hb.SPARSE24)):
            kvc = hb.PackedKV(shc, [0, Tc if stk == hb.DENSE else 0, Tc if stk == hb.SPARSE24 else 0,
                                    Tc if stv == hb.DENSE else 0, Tc if stv == hb.SPARSE24 else 0])
            kvc.uniform = 0

            def run_chunks(_):
                kvc.k_map.zero_()
                kvc.v_map.zero_()
                for c in range(Lc // chunk):
                    hb.append_tile(shc, kvc, nct * c, Kc[:, :, chunk * c:chunk * (c + 1)], Vc[:, :, chunk * c:chunk * (c + 1)],
                                   state_k=stk, state_v=stv)
                    hb.prefill_attn(shc, Qc, kvc, causal=True, want_lse=False, out=Oc, q_start=chunk * c)
            t = _time(torch, run_chunks, PREFILL_REPS)
            cp.append({"case": name_c, "total_ms": t * 1e3, "dense_equiv_TFLOPs_of_full_causal": flops_c / t / 1e12})
            del kvc
        for r in cp:
            r["speedup_vs_dense"] = cp[0]["total_ms"] / r["total_ms"]
        res["chunked_prefill_128k_in_32k_chunks"] = cp
        del Kc, Vc, Qc, Oc
        torch.cuda.empty_cache()
    if "paper_kernel_shape_b8_32k" in legs:
        # the shape of the paper's own kernel benchmarks (Sec. V-B: batch 8, 32K tokens), 32/8 heads: context only
        B5, L5 = 8, 32768
        sh5 = hb.make_shape(B5, Hq, Hkv, L5)
        K5 = torch.randn((B5, Hkv, L5, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        V5 = torch.randn((B5, Hkv, L5, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        Q5 = torch.randn((B5, Hq, L5, 128), device="cuda", dtype=torch.bfloat16, generator=g)
        q5 = Q5[:, :, -1, :].contiguous()
        O5 = torch.empty_like(Q5)
        o5 = torch.empty_like(q5)
        ws5 = torch.empty(hb.workspace_bytes(sh5, 0), dtype=torch.uint8, device="cuda")
        n5 = hb.decode_auto_splits(sh5)
        wsd5 = torch.empty(hb.workspace_bytes(sh5, 2, n5), dtype=torch.uint8, device="cuda")
        flops5 = 4.0 * 128 * Hq * B5 * (L5 * (L5 + 1) / 2.0)
        b8 = []
        for name5, kw in (("dense", dict(sparse_frac_k=0.0, sparse_frac_v=0.0)), ("sk0_sv1", dict(sparse_frac_k=0.0)), ("2:4", dict())):
            p5 = hb.make_policy(**kw)
            c5 = hb.tile_counts(sh5, p5)
            kv5 = hb.compress_kv(sh5, p5, K5, V5, workspace=ws5)
            t_p = _time(torch, lambda i: hb.prefill_attn(sh5, Q5, kv5, causal=True, want_lse=False, out=O5), PREFILL_REPS)
            t_d = _time(torch, lambda i: hb.decode_attn(sh5, q5, kv5, n_splits=n5, want_lse=False, out=o5, workspace=wsd5), 10, warm=2)
            nb = packed_bytes(B5, Hkv, L5 // 64, c5)
            b8.append({"case": name5, "prefill_ms": t_p * 1e3, "prefill_dense_equiv_TFLOPs": flops5 / t_p / 1e12,
                       "decode_us": t_d * 1e6, "decode_GBps": nb / t_d / 1e9, "hbm_frac": nb / t_d / 1e9 / HBM_PEAK_GBPS})
            del kv5
        for r in b8:
            r["prefill_speedup_vs_dense"] = b8[0]["prefill_ms"] / r["prefill_ms"]
            r["decode_speedup_vs_dense"] = b8[0]["decode_us"] / r["decode_us"]
        res["paper_kernel_shape_b8_32k"] = b8
        del K5, V5, Q5, O5, ws5
        torch.cuda.empty_cache()
    if "fp16_same_shape" in legs:
        # the paper's element type: fp16 at the benchmark workload's shape (N(0,1) inputs), one term of P in GEMM2
        sh6 = hb.make_shape(B, Hq, Hkv, L, dtype=hb.FP16)
        K6 = torch.randn((B, Hkv, L, 128), device="cuda", dtype=torch.float16, generator=g)
        V6 = torch.randn((B, Hkv, L, 128), device="cuda", dtype=torch.float16, generator=g)
        Q6 = torch.randn((B, Hq, L, 128), device="cuda", dtype=torch.float16, generator=g)
        q6 = Q6[:, :, -1, :].contiguous()
        O6 = torch.empty_like(Q6)
        o6 = torch.empty_like(q6)
        f16 = []
        for name6, kw in (("dense", dict(sparse_frac_k=0.0, sparse_frac_v=0.0)), ("sk0_sv1", dict(sparse_frac_k=0.0)), ("2:4", dict())):
            p6 = hb.make_policy(**kw)
            c6 = hb.tile_counts(sh6, p6)
            kv6 = [hb.compress_kv(sh6, p6, K6, V6, workspace=ws_c) for _ in range(6)]
            t_p = _time(torch, lambda i: hb.prefill_attn(sh6, Q6, kv6[i % 6], causal=True, want_lse=False, out=O6), PREFILL_REPS)
            t_d = _time(torch, lambda i: hb.decode_attn(sh6, q6, kv6[i % 6], n_splits=n, want_lse=False, out=o6, workspace=ws_d), 24, warm=6)
            nb = packed_bytes(B, Hkv, T, c6)
            f16.append({"case": name6, "prefill_ms": t_p * 1e3, "prefill_dense_equiv_TFLOPs": flops1 / t_p / 1e12,
                        "decode_us": t_d * 1e6, "decode_GBps": nb / t_d / 1e9})
            del kv6
        for r in f16:
            r["prefill_speedup_vs_dense"] = f16[0]["prefill_ms"] / r["prefill_ms"]
            r["decode_speedup_vs_dense"] = f16[0]["decode_us"] / r["decode_us"]
        res["fp16_same_shape"] = f16
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--copies", type=int, default=8, help="packed-cache buffers to rotate through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense-KV baseline legs")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the extra legs (hierarchical decode sweep at B8 x 128K, long prefill with tile "
                         "skipping, the paper's S_K=0/S_V=1 point)")
    ap.add_argument("--legs", default="all", help="comma-separated extra legs to run (default all): " + ", ".join(LEGS))
    ap.add_argument("--cases", default="all", help="comma-separated cases of the swept legs to run, e.g. skip0.5 (default all)")
    ap.add_argument("--only-legs", action="store_true",
                    help="run only the selected extra legs (no headline step): what the per-leg rocprofv3 runs use")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (reference kernel of known traffic for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2604_16864_amd.binding as hb
    from paper_2604_16864_amd import workloads as wl

    hb.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    name = "cfg1_decode_llama8b_32k"
    cfg = dict(wl.CONFIGS[name])
    B, Hq, Hkv, L, D = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["L"], cfg["D"]
    T = L // 64
    Qh, Kh, Vh = wl.make_qkv(B, Hq, Hkv, L, D, L, cfg["seed"], cfg["k_outliers"])
    Q = hb.bits_to_bf16_tensor(Qh)
    K = hb.bits_to_bf16_tensor(Kh)
    V = hb.bits_to_bf16_tensor(Vh)
    qd = Q[:, :, -1, :].contiguous()
    del Qh, Kh, Vh
    sh = hb.make_shape(B, Hq, Hkv, L)
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.only_legs:
        print(json.dumps({"legs_only": True, "data": "synthetic", "n_gpus": 1,
                          "stages_extra": extra_legs(hb, torch, Q, K, V, qd, sh, args)}))
        return
    pol = hb.make_policy()                       # 2:4 on every K and V tile, no skipping
    counts = hb.tile_counts(sh, pol)
    kvs = [hb.PackedKV(sh, counts) for _ in range(args.copies)]
    ws_c = torch.empty(max(16, hb.workspace_bytes(sh, 0)), dtype=torch.uint8, device="cuda")
    n_splits = hb.decode_auto_splits(sh)
    ws_d = torch.zeros(hb.workspace_bytes(sh, 2, n_splits), dtype=torch.uint8, device="cuda")
    O = torch.empty_like(Q)
    Od = torch.empty_like(qd)
    lse_d = torch.empty((B, Hq), dtype=torch.float32, device="cuda")
    for kv in kvs:                                # every buffer holds a valid cache before timing
        hb.compress_kv(sh, pol, K, V, out=kv, workspace=ws_c)
    torch.cuda.synchronize()

    def step(i, ev=None):
        kv_w = kvs[i % args.copies]               # compressed + prefilled this step
        kv_r = kvs[(i + 1) % args.copies]         # decoded this step: written copies-1 steps ago
        if ev: ev[0].record()
        hb.compress_kv(sh, pol, K, V, out=kv_w, workspace=ws_c)
        if ev: ev[1].record()
        hb.prefill_attn(sh, Q, kv_w, causal=True, want_lse=False, out=O)
        if ev: ev[2].record()
        hb.decode_attn(sh, qd, kv_r, n_splits=n_splits, out=Od, lse=lse_d, workspace=ws_d)
        if ev: ev[3].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_c = np.array([e[0].elapsed_time(e[1]) for e in evs]) * 1e-3
    t_p = np.array([e[1].elapsed_time(e[2]) for e in evs]) * 1e-3
    t_d = np.array([e[2].elapsed_time(e[3]) for e in evs]) * 1e-3
    # The split-KV kernel alone (the kernel that streams the cache): the same launch, over the same rotation
    # of cold buffers, back to back between two events, the merge kernel left out (phases = 1).
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_rep = max(args.steps, 16)
    for i in range(args.copies):
        hb.decode_attn(sh, qd, kvs[i], n_splits=n_splits, out=Od, lse=lse_d, workspace=ws_d, phases=1)
    e0.record()
    for i in range(n_rep):
        hb.decode_attn(sh, qd, kvs[i % args.copies], n_splits=n_splits, out=Od, lse=lse_d, workspace=ws_d, phases=1)
    e1.record()
    torch.cuda.synchronize()
    t_ds = np.array([e0.elapsed_time(e1) / n_rep]) * 1e-3
    e0.record()
    for i in range(n_rep):
        hb.decode_attn(sh, qd, kvs[i % args.copies], n_splits=n_splits, out=Od, lse=lse_d, workspace=ws_d, phases=2)
    e1.record()
    torch.cuda.synchronize()
    t_dm = e0.elapsed_time(e1) / n_rep * 1e-3
    # whole decode calls back to back, as a decode loop issues them (still one cold cache per call)
    e0.record()
    for i in range(n_rep):
        hb.decode_attn(sh, qd, kvs[i % args.copies], n_splits=n_splits, out=Od, lse=lse_d, workspace=ws_d)
    e1.record()
    torch.cuda.synchronize()
    t_dc = e0.elapsed_time(e1) / n_rep * 1e-3
    # the compress kernel alone, the same way: back-to-back launches into rotating output buffers, reading from
    # rotating copies of K and V (one copy of them would stay in the 256 MB last-level cache between launches)
    n_in = 4
    K_in = [K] + [K.clone() for _ in range(n_in - 1)]
    V_in = [V] + [V.clone() for _ in range(n_in - 1)]
    for i in range(n_in):
        hb.compress_kv(sh, pol, K_in[i], V_in[i], out=kvs[i % args.copies], workspace=ws_c)
    e0.record()
    for i in range(n_rep):
        hb.compress_kv(sh, pol, K_in[i % n_in], V_in[i % n_in], out=kvs[i % args.copies], workspace=ws_c)
    e1.record()
    torch.cuda.synchronize()
    t_ck = e0.elapsed_time(e1) / n_rep * 1e-3
    del K_in, V_in
    # what the memory system gives the split kernel's access pattern with nothing else in the kernel: a load-only
    # kernel of the same launch shape, pools, tile order and depth (with a combine through LDS and a partial
    # store per workgroup), over rotating cold buffers of the same size
    n_tiles = B * Hkv * T
    arena = torch.empty(args.copies * n_tiles * 18432, dtype=torch.uint8, device="cuda").fill_(1)
    probe_sink = torch.zeros(16 + 512 * n_splits * Hkv * B, dtype=torch.float32, device="cuda")
    views = [arena[i * n_tiles * 18432:(i + 1) * n_tiles * 18432] for i in range(args.copies)]
    for v in views:
        hb.probe_stream_read(v, n_tiles, n_splits * Hkv * B, True, probe_sink)
    e0.record()
    for i in range(n_rep):
        hb.probe_stream_read(views[i % args.copies], n_tiles, n_splits * Hkv * B, True, probe_sink)
    e1.record()
    torch.cuda.synchronize()
    t_probe = e0.elapsed_time(e1) / n_rep * 1e-3
    del arena, views
    # rate of the matrix pipes on this chip, register-resident (no memory, no LDS, no vector-ALU work)
    sink = torch.zeros(4, dtype=torch.int64, device="cuda")
    mfma_meas = {}
    for kind, label in ((0, "dense_16x16x32_bf16"), (1, "sparse_16x16x64_bf16_dense_equiv")):
        hb.probe_mfma_rate(kind, 2000, sink)
        e0.record()
        flop = hb.probe_mfma_rate(kind, 40000, sink)
        e1.record()
        torch.cuda.synchronize()
        mfma_meas[label] = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
        clk = sink.cpu().tolist()
        mfma_meas[label + "_sustained_GHz"] = clk[0] / max(clk[1], 1) * 0.1

    kv_bytes = packed_bytes(B, Hkv, T, counts)
    q_bytes = B * Hq * D * 2
    part_bytes = B * Hq * n_splits * (D + 1) * 4
    decode_bytes = kv_bytes + q_bytes + part_bytes          # algorithmic bytes of the split kernel (read KV once, write partials)
    compress_bytes = 2 * B * Hkv * L * D * 2 + kv_bytes     # read dense K,V once + write packed
    prefill_flops = 4.0 * D * Hq * B * (L * (L + 1) / 2.0)  # dense-equivalent causal FLOPs
    dec_s, pre_s, cmp_s = float(t_d.mean()), float(t_p.mean()), float(t_c.mean())
    dec_split_s = float(t_ds.mean())

    stages = {
        "compress_us": cmp_s * 1e6, "compress_GBps": compress_bytes / cmp_s / 1e9,
        "compress_frac_of_prefill": cmp_s / pre_s,
        "prefill_ms": pre_s * 1e3, "prefill_dense_equiv_TFLOPs": prefill_flops / pre_s / 1e12,
        "decode_us": dec_s * 1e6, "decode_us_min": float(t_d.min()) * 1e6, "decode_us_median": float(np.median(t_d)) * 1e6,
        "prefill_ms_median": float(np.median(t_p)) * 1e3, "compress_us_median": float(np.median(t_c)) * 1e6,
        "decode_GBps": decode_bytes / dec_s / 1e9,
        "decode_split_kernel_us": dec_split_s * 1e6, "decode_split_kernel_GBps": decode_bytes / dec_split_s / 1e9,
        # back-to-back merge-only calls: bounded by the host's launch rate, not by the 4 us kernel
        # (its own duration is in profiles/bench_cfg1_kernel_trace.md)
        "decode_merge_call_us_host_bound": t_dm * 1e6,
        "decode_call_us_back_to_back": t_dc * 1e6, "decode_call_GBps_back_to_back": decode_bytes / t_dc / 1e9,
        "decode_n_splits": n_splits, "packed_MB": kv_bytes / 1e6, "dense_MB": 2 * B * Hkv * L * D * 2 / 1e6,
        "compression_ratio": 2 * B * Hkv * L * D * 2 / kv_bytes,
        "ideal_decode_speedup": 1.0 / (1.0 - 0.21875 * 2), "ideal_prefill_speedup": 2.0,
    }

    if not args.no_dense:
        # same-build dense-KV baseline (every tile DENSE), same inputs, same run
        del kvs[1:]
        torch.cuda.empty_cache()
        pol_d = hb.make_policy(sparse_frac_k=0.0, sparse_frac_v=0.0)
        cd = hb.tile_counts(sh, pol_d)
        n_d = 5
        kvd = [hb.PackedKV(sh, cd) for _ in range(n_d)]
        for kv in kvd:
            hb.compress_kv(sh, pol_d, K, V, out=kv, workspace=ws_c)
        torch.cuda.synchronize()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        reps = max(3, args.steps // 4)
        hb.prefill_attn(sh, Q, kvd[0], causal=True, want_lse=False, out=O)
        e[0].record()
        for i in range(reps):
            hb.prefill_attn(sh, Q, kvd[i % n_d], causal=True, want_lse=False, out=O)
        e[1].record()
        torch.cuda.synchronize()
        pre_dense = e[0].elapsed_time(e[1]) * 1e-3 / reps
        # decode: each launch reads a buffer last touched >= 4 x 134 MB ago
        for i in range(n_d):
            hb.decode_attn(sh, qd, kvd[i], n_splits=n_splits, out=Od, lse=lse_d, workspace=ws_d)
        reps = max(10, args.steps)
        e[0].record()
        for i in range(reps):
            hb.decode_attn(sh, qd, kvd[i % n_d], n_splits=n_splits, out=Od, lse=lse_d, workspace=ws_d)
        e[1].record()
        torch.cuda.synchronize()
        dec_dense = e[0].elapsed_time(e[1]) * 1e-3 / reps
        dense_bytes = packed_bytes(B, Hkv, T, cd) + q_bytes + part_bytes
        stages.update({
            "prefill_dense_ms": pre_dense * 1e3, "prefill_dense_TFLOPs": prefill_flops / pre_dense / 1e12,
            "prefill_speedup_vs_dense": pre_dense / pre_s,
            "decode_dense_us": dec_dense * 1e6, "decode_dense_GBps": dense_bytes / dec_dense / 1e9,
            "decode_speedup_vs_dense": dec_dense / dec_s,
        })

    extra = None
    if not args.no_extra:
        del kvs
        if not args.no_dense:
            del kvd
        torch.cuda.empty_cache()
        extra = extra_legs(hb, torch, Q, K, V, qd, sh, args)

    out = {
        "metric": "decode_attn_hbm_GBps_on_packed_kv", "value": decode_bytes / dec_s / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "B": B, "Hq": Hq, "Hkv": Hkv, "L": L, "D": D, "tile": 64,
                   "sparsity": "2:4 on every K and V tile (S_K = S_V = 1), no skipping",
                   "step": "compress -> causal prefill (Lq = L) -> decode (1 token)"},
        "stages": stages,
        # dominant kernel of the metric: the split-KV kernel alone (back-to-back launches with the merge kernel
        # left out); `value` above is the whole decode call (split + merge + launch gap) inside the step
        "roofline": {"bound": "hbm", "kernel": "decode_split_kernel<0, 0, 1>", "achieved": decode_bytes / dec_split_s / 1e9,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": decode_bytes / dec_split_s / 1e9 / HBM_PEAK_GBPS,
                     "traffic": traffic_from_profile("decode_split_kernel<0, 0, 1"), "traffic_source": "profiles/bench_cfg1_hbm_traffic.md",
                     "algorithmic_bytes": decode_bytes, "avg_launch_us": dec_split_s * 1e6,
                     # load-only kernel with the same access pattern and launch shape (hs_probe_stream_read)
                     "load_only_probe_us": t_probe * 1e6, "load_only_probe_frac": n_tiles * 18432 / t_probe / 1e9 / HBM_PEAK_GBPS,
                     "whole_call_us": dec_s * 1e6, "whole_call_frac": decode_bytes / dec_s / 1e9 / HBM_PEAK_GBPS},
        # prefill against the matrix pipes: every tile is 2:4, so half of the dense-equivalent multiplications are
        # executed; `achieved` counts the executed ones and `peak` is the dense bf16 rate, i.e. frac = t_floor / t with
        # t_floor = dense-equivalent FLOPs of 2:4 tile pairs / (2 x dense peak) (Sec. III-D prefill model)
        "roofline_prefill": {"bound": "mfma", "kernel": "prefill_kernel<0, 0, 2>", "achieved": 0.5 * prefill_flops / pre_s / 1e12,
                             "peak": MFMA_BF16_DENSE_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": prefill_floor_s(0.0, prefill_flops) / pre_s,
                             "floor_ms": prefill_floor_s(0.0, prefill_flops) * 1e3,
                             "dense_equiv_TFLOPs": prefill_flops / pre_s / 1e12,
                             "traffic": traffic_from_profile("prefill_kernel<0, 0, 2"), "traffic_source": "profiles/bench_cfg1_hbm_traffic.md",
                             "note": "executed multiply-adds (half of the dense-equivalent ones on 2:4 tiles) over the dense bf16 peak; "
                                     "issued-instruction utilisation from counters: profiles/prefill_l32768_mfma_counters.md",
                             "measured_peak_TFLOPs": mfma_meas,
                             "frac_of_measured_sparse_rate": prefill_flops / pre_s / 1e12 / mfma_meas["sparse_16x16x64_bf16_dense_equiv"]},
        # the pack kernel alone (back-to-back launches); the stage inside the step (one launch between two events,
        # launch latency included) is whole_call_*
        "roofline_compress": {"bound": "hbm", "kernel": "pack_kernel", "achieved": compress_bytes / t_ck / 1e9,
                              "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": compress_bytes / t_ck / 1e9 / HBM_PEAK_GBPS,
                              "avg_launch_us": t_ck * 1e6, "whole_call_us": cmp_s * 1e6,
                              "whole_call_frac": compress_bytes / cmp_s / 1e9 / HBM_PEAK_GBPS, "algorithmic_bytes": compress_bytes,
                              "traffic": traffic_from_profile("pack_kernel"), "traffic_source": "profiles/bench_cfg1_hbm_traffic.md"},
    }
    if not args.no_dense:
        out["roofline_prefill"]["same_build_dense_frac"] = prefill_floor_s(prefill_flops, 0.0) / pre_dense
    if extra is not None:
        out["stages_extra"] = extra
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
