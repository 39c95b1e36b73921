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

Prints ONE JSON line (see README / DESIGN notes for the fields).
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
# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE on this workload (summary, commands and
# the copy-kernel calibration: profiles/bench_cfg1_hbm_traffic.md).  Only valid for cfg1 with 2:4 on all tiles.
TRAFFIC_BYTES = {"decode": (36949.8 * 2.000 + 544.0) * 1024, "compress": (65851.7 * 2.000 + 73728.0) * 1024,
                 "prefill": (823241.6 * 2.000 + 262144.0) * 1024}


def packed_bytes(B, Hkv, T, counts):
    n_skip, ndk, nsk, ndv, nsv = counts
    per_row = (ndk + ndv) * 16384 + (nsk + nsv) * 9216 + 2 * T * 4
    return B * Hkv * per_row


def cpu_baseline(cfg, sample_heads):
    """The oracle, as it stands, timed on the host on a bounded sample of the same
    workload: decode attention (unpack + fp64 softmax attention) over `sample_heads`
    of the KV heads.  Reported in the metric's unit (compressed GB/s)."""
    import numpy as np
    from oracle import hs_oracle as orc
    from paper_2604_16864_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    G = cfg["Hq"] // cfg["Hkv"]
    Q, K, V = wl.make_qkv(cfg["B"], sample_heads * G, sample_heads, cfg["L"], cfg["D"], 1, cfg["seed"], cfg["k_outliers"])
    q = Q[:, :, 0, :].copy()
    pk, pv, _ = orc.compress_kv(K, V, Bt=64)
    t0 = time.perf_counter()
    orc.attention_decode(q, pk, pv)
    dt = time.perf_counter() - t0
    nbytes = pk.nbytes() + pv.nbytes()
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle decode attention (unpack + fp64 attention) over {sample_heads} of {cfg['Hkv']} KV heads "
                      f"of the same workload, {nbytes / 1e6:.1f} MB packed, {dt:.2f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--copies", type=int, default=8, help="packed-cache buffers to rotate through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense-KV baseline legs")
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

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

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

    kv_bytes = packed_bytes(B, Hkv, T, counts)
    q_bytes = B * Hq * D * 2
    part_bytes = B * Hq * n_splits * (D + 1) * 4
    decode_bytes = kv_bytes + q_bytes + part_bytes          # algorithmic bytes of the split kernel (read KV once, write partials)
    compress_bytes = 2 * B * Hkv * L * D * 2 + kv_bytes     # read dense K,V once + write packed
    prefill_flops = 4.0 * D * Hq * B * (L * (L + 1) / 2.0)  # dense-equivalent causal FLOPs
    dec_s, pre_s, cmp_s = float(t_d.mean()), float(t_p.mean()), float(t_c.mean())

    stages = {
        "compress_us": cmp_s * 1e6, "compress_GBps": compress_bytes / cmp_s / 1e9,
        "compress_frac_of_prefill": cmp_s / pre_s,
        "prefill_ms": pre_s * 1e3, "prefill_dense_equiv_TFLOPs": prefill_flops / pre_s / 1e12,
        "decode_us": dec_s * 1e6, "decode_us_min": float(t_d.min()) * 1e6, "decode_GBps": decode_bytes / dec_s / 1e9,
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

    out = {
        "metric": "decode_attn_hbm_GBps_on_packed_kv", "value": decode_bytes / dec_s / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "B": B, "Hq": Hq, "Hkv": Hkv, "L": L, "D": D, "tile": 64,
                   "sparsity": "2:4 on every K and V tile (S_K = S_V = 1), no skipping",
                   "step": "compress -> causal prefill (Lq = L) -> decode (1 token)"},
        "stages": stages,
        "roofline": {"bound": "hbm", "kernel": "decode_split_kernel<0> (+ merge)", "achieved": decode_bytes / dec_s / 1e9,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": decode_bytes / dec_s / 1e9 / HBM_PEAK_GBPS,
                     "traffic": TRAFFIC_BYTES["decode"]},
        "roofline_prefill": {"bound": "mfma", "kernel": "prefill_kernel<0>", "achieved": prefill_flops / pre_s / 1e12,
                             "peak": MFMA_BF16_DENSE_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": prefill_flops / pre_s / 1e12 / MFMA_BF16_DENSE_PEAK_TFLOPS, "traffic": TRAFFIC_BYTES["prefill"],
                             "note": "dense-equivalent causal FLOPs over the dense bf16 peak"},
        "roofline_compress": {"bound": "hbm", "kernel": "pack_kernel", "achieved": compress_bytes / cmp_s / 1e9,
                              "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": compress_bytes / cmp_s / 1e9 / HBM_PEAK_GBPS,
                              "traffic": TRAFFIC_BYTES["compress"]},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, sample_heads=2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
