"""Seeded synthetic inputs for the HieraSparse hot path.

Holds none of the method's arithmetic: only random draws, the per-channel key
scales that mimic the outlier channels the paper observes in key caches
(Sec. II, key/value magnitude figure), and round-to-nearest-even conversion of
fp32 to bf16 bit patterns.  Both the CPU oracle's tests and the HIP path's
tests feed on these arrays, so both see identical bits.

Shapes follow the Llama-3.1-8B attention geometry the paper benchmarks
(32 query heads, 8 KV heads, head dim 128, 64-token blocks; Sec. V-B).
"""
import numpy as np

# name -> (phase, B, Hq, Hkv, L, D, k_outlier_channels)
CONFIGS = {
    "cfg0_decode_small": dict(phase="decode", B=1, Hq=4, Hkv=1, L=2048, D=128, k_outliers=False, seed=0),
    "cfg1_decode_llama8b_32k": dict(phase="decode", B=1, Hq=32, Hkv=8, L=32768, D=128, k_outliers=True, seed=1000),
    "cfg2_prefill_llama8b_16k": dict(phase="prefill", B=1, Hq=32, Hkv=8, L=16384, D=128, k_outliers=False, seed=2000),
    "cfg3_decode_b8_128k": dict(phase="decode", B=8, Hq=32, Hkv=8, L=131072, D=128, k_outliers=False, seed=3000),
    "cfg4_prefill_64k": dict(phase="prefill", B=1, Hq=32, Hkv=8, L=65536, D=128, k_outliers=False, seed=4000),
}


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16).  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def f32_to_f16_bits(x):
    """Round-to-nearest-even fp32 -> IEEE fp16 bit patterns (uint16)."""
    return np.asarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(bits):
    return np.ascontiguousarray(np.asarray(bits, dtype=np.uint16)).view(np.float16).astype(np.float32)


def bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng, shape, chunk=1 << 24, dtype="bf16"):
    """N(0,1) draws rounded to bf16 (or fp16), generated in chunks to bound host memory."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    rnd = f32_to_bf16_bits if dtype == "bf16" else f32_to_f16_bits
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = rnd(rng.standard_normal(e - s, dtype=np.float32))
    return out.reshape(shape)


def make_qkv(B, Hq, Hkv, L, D, Lq, seed, k_outliers=False, dtype="bf16"):
    """Q [B,Hq,Lq,D], K,V [B,Hkv,L,D] as bf16 (or fp16) bit patterns.

    One PCG64 stream per tensor: seed+0 -> Q, seed+1 -> K, seed+2 -> V,
    seed+3 -> key channel scales (log-uniform in [0.1, 10], one per
    (kv head, channel), constant over tokens).
    """
    Q = normal_bf16(np.random.Generator(np.random.PCG64(seed + 0)), (B, Hq, Lq, D), dtype=dtype)
    V = normal_bf16(np.random.Generator(np.random.PCG64(seed + 2)), (B, Hkv, L, D), dtype=dtype)
    rk = np.random.Generator(np.random.PCG64(seed + 1))
    rnd = f32_to_bf16_bits if dtype == "bf16" else f32_to_f16_bits
    if not k_outliers:
        K = normal_bf16(rk, (B, Hkv, L, D), dtype=dtype)
    else:
        rs = np.random.Generator(np.random.PCG64(seed + 3))
        scales = np.exp(rs.uniform(np.log(0.1), np.log(10.0), size=(Hkv, D))).astype(np.float32)
        K = np.empty((B, Hkv, L, D), dtype=np.uint16)
        for b in range(B):
            for h in range(Hkv):
                K[b, h] = rnd(rk.standard_normal((L, D), dtype=np.float32) * scales[h][None, :])
    return Q, K, V


def make_config(name, L=None, B=None):
    """Inputs of a named workload (optionally shortened to L tokens / B batch rows
    for parity cases the oracle can finish).  Decode configs get Lq = 1."""
    c = dict(CONFIGS[name])
    if L is not None:
        c["L"] = L
    if B is not None:
        c["B"] = B
    Lq = 1 if c["phase"] == "decode" else c["L"]
    Q, K, V = make_qkv(c["B"], c["Hq"], c["Hkv"], c["L"], c["D"], Lq, c["seed"], c["k_outliers"])
    if c["phase"] == "decode":
        Q = Q[:, :, 0, :].copy()
    return c, Q, K, V


def sample_rows(B, Hq, Lq, n, seed, extra=()):
    """n seeded (b, hq, i) query rows, plus any extra rows the caller wants covered."""
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = [(int(rng.integers(B)), int(rng.integers(Hq)), int(rng.integers(Lq))) for _ in range(n)]
    return rows + [tuple(r) for r in extra]
