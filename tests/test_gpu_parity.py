"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same
seeded inputs.  Packed values, metadata, pools and maps: bit-exact.  Attention
outputs: max|d| <= 1e-2 * max|ref| and mean|d| / mean|ref| <= 2e-3."""
import numpy as np
import pytest
import torch

from oracle import hs_layout as hl
from oracle import hs_oracle as orc
from paper_2604_16864_amd import binding as hb
from paper_2604_16864_amd import workloads as wl

pytestmark = pytest.mark.gpu

MAX_TOL, MEAN_TOL = 1e-2, 2e-3


def _dev(bits, dtype="bf16"):
    return hb.bits_to_bf16_tensor(bits, "cuda", torch.float16 if dtype == "fp16" else torch.bfloat16)


def _f32(t):
    return t.float().cpu().numpy().astype(np.float64)


def assert_close(out, ref, what):
    out = np.asarray(out, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.isfinite(out).all(), what
    err = np.abs(out - ref)
    mx, mean = err.max() / max(np.abs(ref).max(), 1e-30), err.mean() / max(np.abs(ref).mean(), 1e-30)
    print(f"[{what}] max rel {mx:.3e} mean rel {mean:.3e}", flush=True)
    assert mx <= MAX_TOL, (what, mx)
    assert mean <= MEAN_TOL, (what, mean)


def assert_lse_close(lse, ref, what):
    lse = np.asarray(lse, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    inf = np.isneginf(ref)
    assert (np.isneginf(lse) == inf).all(), what
    assert np.allclose(lse[~inf], ref[~inf], rtol=1e-4, atol=1e-4), (what, np.abs(lse[~inf] - ref[~inf]).max())


def compress_both(B, Hq, Hkv, L, K, V, dtype="bf16", **pol):
    sh = hb.make_shape(B, Hq, Hkv, L, dtype=hb.FP16 if dtype == "fp16" else hb.BF16)
    lib_pol = dict(pol)
    if "element_rule" in lib_pol:
        lib_pol["element_rule"] = {"magnitude": hb.RULE_MAGNITUDE, "nonzero": hb.RULE_NONZERO}[lib_pol["element_rule"]]
    policy = hb.make_policy(**lib_pol)
    kv = hb.compress_kv(sh, policy, _dev(K, dtype), _dev(V, dtype))
    torch.cuda.synchronize()
    hb.check_state_flag(policy)          # explicit states: nothing left out, every pair valid
    pk, pv, info = orc.compress_kv(K, V, Bt=64, dtype=dtype, **pol)
    return sh, kv, pk, pv, info


def lib_maps(k_map, v_map):
    """The library's map arrays as (signed index map of K, signed index map of V, encoding flag of V):
    a v_map entry of a bf16 cache may carry HS_MAP_F16 in its magnitude, which is not part of the
    paper's signed index map (Sec. III-B) and is compared on its own."""
    km = k_map.cpu().numpy()
    vm = v_map.cpu().numpy().astype(np.int64)
    mag = np.abs(vm)
    assert not ((np.abs(km.astype(np.int64)) & hb.MAP_F16) != 0).any()
    return km, (np.sign(vm) * (mag & ~hb.MAP_F16)).astype(np.int32), (mag & hb.MAP_F16) != 0


def assert_maps_equal(kv, pk, pv, sel=None, osel=None):
    """sel / osel: index into the library's / the oracle's [B, Hkv, T] arrays (default: everything)."""
    km, vm, flag = lib_maps(kv.k_map if sel is None else kv.k_map[sel], kv.v_map if sel is None else kv.v_map[sel])
    o = (lambda a: a) if osel is None else (lambda a: a[osel])
    assert (km == o(pk.map)).all() and (vm == o(pv.map)).all(), "signed index maps"
    assert (flag == o(pv.f16)).all(), "fp16-encoding predicate of the V tiles"


def check_packed_bit_exact(sh, kv, pk, pv):
    assert_maps_equal(kv, pk, pv)
    B, H = sh.B, sh.Hkv
    for name, p, dense, nnz, meta, cd, cs in (("k", pk, kv.k_dense, kv.k_nnz, kv.k_meta, kv.counts[1], kv.counts[2]),
                                               ("v", pv, kv.v_dense, kv.v_nnz, kv.v_meta, kv.counts[3], kv.counts[4])):
        ph = hl.physical_pools(p)
        for b in range(B):
            for h in range(H):
                nd, ns = int(ph["n_dense"][b, h]), int(ph["n_sparse"][b, h])
                assert nd <= cd and ns <= cs
                if nd:
                    got = dense.cpu().numpy().reshape(B, H, cd, 16384)[b, h, :nd]
                    assert (got == ph["dense"][b, h, :nd]).all(), (name, "dense", b, h)
                if ns:
                    got = nnz.cpu().numpy().reshape(B, H, cs, 8192)[b, h, :ns]
                    assert (got == ph["nnz"][b, h, :ns]).all(), (name, "nnz", b, h)
                    got = meta.cpu().numpy().reshape(B, H, cs, 1024)[b, h, :ns]
                    assert (got == ph["meta"][b, h, :ns]).all(), (name, "meta", b, h)
    Ku, Vu = hb.unpack_kv(sh, kv)
    torch.cuda.synchronize()
    assert (hb.bf16_tensor_to_bits(Ku) == orc.unpack_tensor(pk)).all()
    assert (hb.bf16_tensor_to_bits(Vu) == orc.unpack_tensor(pv)).all()


def _mixed_states(B, Hkv, T, seed, p_skip=0.2):
    rng = np.random.default_rng(seed)
    sk = rng.choice([1, 2], size=(B, Hkv, T)).astype(np.int8)
    sv = rng.choice([1, 2], size=(B, Hkv, T)).astype(np.int8)
    skip = rng.random((B, Hkv, T)) < p_skip
    sk[skip] = 0
    sv[skip] = 0
    return sk, sv


# ------------------------------------------------------------------ compress
def test_compress_cfg0_bit_exact():
    c, Q, K, V = wl.make_config("cfg0_decode_small")
    # plant ties, zeros, negative zeros and an all-zero group
    K[0, 0, 5, :8] = wl.f32_to_bf16_bits(np.array([1, 1, -1, 1, 0, -0.0, 0, 0], dtype=np.float32))
    V[0, 0, 8:12, 7] = wl.f32_to_bf16_bits(np.array([2, -2, 2, -2], dtype=np.float32))
    sh, kv, pk, pv, _ = compress_both(c["B"], c["Hq"], c["Hkv"], c["L"], K, V)
    check_packed_bit_exact(sh, kv, pk, pv)
    assert kv.nbytes == pk.nbytes() + pv.nbytes()


def test_compress_explicit_mixed_states_bit_exact():
    B, Hq, Hkv, L = 2, 8, 2, 64 * 11
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 64, seed=21)
    sk, sv = _mixed_states(B, Hkv, L // 64, seed=22)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, state_k=sk, state_v=sv)
    check_packed_bit_exact(sh, kv, pk, pv)


def test_compress_strided_input():
    """K, V as slices of a wider buffer (token stride 256 elements)."""
    B, Hq, Hkv, L = 1, 4, 2, 256
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 64, seed=23)
    sh = hb.make_shape(B, Hq, Hkv, L)
    wide_k = torch.zeros((B, Hkv, L, 256), dtype=torch.bfloat16, device="cuda")
    wide_v = torch.zeros_like(wide_k)
    wide_k[..., :128] = _dev(K)
    wide_v[..., :128] = _dev(V)
    kv = hb.compress_kv(sh, hb.make_policy(), wide_k[..., :128], wide_v[..., :128])
    pk, pv, _ = orc.compress_kv(K, V)
    check_packed_bit_exact(sh, kv, pk, pv)


@pytest.mark.parametrize("skip,sfk,sfv", [(0.25, 1.0, 1.0), (0.5, 1.0, 1.0), (0.75, 1.0, 1.0), (0.25, 0.5, 1.0),
                                          (0.0, 0.3, 0.7), (0.5, 0.0, 0.0)])
def test_compress_policy_ranking(skip, sfk, sfv):
    B, Hq, Hkv, L = 2, 8, 2, 64 * 40
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 64, seed=31)
    # an exact tie in energy and in loss: two identical tiles
    K[0, 0, 64 * 9:64 * 10] = K[0, 0, 64 * 3:64 * 4]
    V[0, 0, 64 * 9:64 * 10] = V[0, 0, 64 * 3:64 * 4]
    sh, kv, pk, pv, info = compress_both(B, Hq, Hkv, L, K, V, skip_frac=skip, sparse_frac_k=sfk, sparse_frac_v=sfv)
    # fp64 sums in a different order: scores agree to ~1e-15; the cut must not sit on a
    # near-tie other than the planted exact one for the maps to be unique
    for key in ("energy", "loss_k", "loss_v"):
        s = np.sort(info[key], axis=-1)
        gaps = np.diff(s, axis=-1) / s[..., 1:]
        assert ((gaps > 1e-12) | (gaps == 0)).all()
    check_packed_bit_exact(sh, kv, pk, pv)


@pytest.mark.parametrize("skip,sfk,sfv,first,last", [(0.0, 1.0, 1.0, 1, 2), (0.5, 1.0, 1.0, 1, 4), (0.25, 0.5, 0.3, 2, 3),
                                                     (0.0, 1.0, 0.0, 3, 0), (0.5, 1.0, 1.0, 30, 30)])
def test_compress_protected_end_tiles(skip, sfk, sfv, first, last):
    """Sink / local-window tiles stay dense (both the host-built map path and the ranked one);
    the all-zero end tiles would be the first skipped if they took part in the ranking."""
    B, Hq, Hkv, L = 2, 8, 2, 64 * 40
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=33)
    K[0, 0, :64] = 0
    V[0, 0, :64] = 0
    K[1, 1, -64:] = 0
    V[1, 1, -64:] = 0
    pol = dict(skip_frac=skip, sparse_frac_k=sfk, sparse_frac_v=sfv, dense_first_tiles=first, dense_last_tiles=last)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, **pol)
    assert (pk.map[:, :, :min(first, 40)] > 0).all() and (pv.map[:, :, 40 - min(last, 40 - min(first, 40)):] > 0).all()
    check_packed_bit_exact(sh, kv, pk, pv)
    q = Q[:, :, 0, :].copy()
    O, LSE = hb.decode_attn(sh, _dev(q), kv)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, pk, pv)
    assert_close(_f32(O), Or, f"decode protected tiles {pol}")
    assert_lse_close(LSE.cpu().numpy(), Lr, "decode protected tiles lse")


def test_compress_nonzero_rule_premasked_input():
    """Generic compressor (Sec. IV-B): K, V arrive with an arbitrary 2:4 element mask applied
    (zeros at pruned places); under the non-zero rule the packed form decodes to the input."""
    B, Hq, Hkv, L = 1, 4, 2, 64 * 6
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=35)
    rng = np.random.default_rng(36)
    K[K == 0] = 0x3F80
    V[V == 0] = 0x3F80
    pairs = np.array([[1, 1, 0, 0], [1, 0, 1, 0], [1, 0, 0, 1], [0, 1, 1, 0], [0, 1, 0, 1], [0, 0, 1, 1]], dtype=bool)
    mk = pairs[rng.integers(0, 6, size=(B, Hkv, L, 32))].reshape(B, Hkv, L, 128)
    mv = pairs[rng.integers(0, 6, size=(B, Hkv, L // 4, 128))].transpose(0, 1, 2, 4, 3).reshape(B, Hkv, L, 128)
    Km, Vm = np.where(mk, K, 0).astype(np.uint16), np.where(mv, V, 0).astype(np.uint16)
    Km[0, 0, 7, 0:8] = [0, 0x4000, 0, 0, 0, 0, 0, 0]        # one survivor; an empty group
    Vm[0, 1, 8:12, 5] = [0x8000, 0, 0xC000, 0x4000]         # a negative zero counts as pruned
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, Km, Vm, element_rule="nonzero", skip_frac=0.2, sparse_frac_k=0.75)
    check_packed_bit_exact(sh, kv, pk, pv)
    Ku, Vu = hb.unpack_kv(sh, kv)
    kept = np.repeat(pk.map != 0, 64, axis=-1)[..., None]
    Vw = Vm.copy()
    Vw[0, 1, 8, 5] = 0
    assert (hb.bf16_tensor_to_bits(Ku) == np.where(kept, Km, 0)).all()
    assert (hb.bf16_tensor_to_bits(Vu) == np.where(kept, Vw, 0)).all()


# ------------------------------------------------------------------ decode
def _decode_case(B, Hq, Hkv, L, seed, n_splits=0, k_outliers=False, **pol):
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=seed, k_outliers=k_outliers)
    q = Q[:, :, 0, :].copy()
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, **pol)
    O, LSE = hb.decode_attn(sh, _dev(q), kv, n_splits=n_splits)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, pk, pv)
    return _f32(O), LSE.cpu().numpy(), Or, Lr


def test_decode_cfg0_full():
    c, q, K, V = wl.make_config("cfg0_decode_small")
    sh, kv, pk, pv, _ = compress_both(c["B"], c["Hq"], c["Hkv"], c["L"], K, V)
    Or, Lr = orc.attention_decode(q, pk, pv)
    for ns in (0, 1, 2, 7, 32):
        O, LSE = hb.decode_attn(sh, _dev(q), kv, n_splits=ns)
        torch.cuda.synchronize()
        assert_close(_f32(O), Or, f"decode cfg0 splits={ns}")
        assert_lse_close(LSE.cpu().numpy(), Lr, f"decode cfg0 lse splits={ns}")


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_decode_gqa_groups(G):
    O, LSE, Or, Lr = _decode_case(2, 2 * G, 2, 64 * 13, seed=40 + G)
    assert_close(O, Or, f"decode G={G}")
    assert_lse_close(LSE, Lr, f"decode G={G} lse")


def test_decode_all_dense_is_plain_attention():
    B, Hq, Hkv, L = 1, 8, 2, 64 * 9
    O, LSE, Or, Lr = _decode_case(B, Hq, Hkv, L, seed=50, sparse_frac_k=0.0, sparse_frac_v=0.0)
    assert_close(O, Or, "decode dense")
    # and against the library routine directly
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=50)
    f = lambda x: torch.from_numpy(wl.bf16_bits_to_f32(x).astype(np.float64))
    ref = torch.nn.functional.scaled_dot_product_attention(
        f(Q), f(K).repeat_interleave(4, 1), f(V).repeat_interleave(4, 1))[:, :, 0].numpy()
    assert_close(O, ref, "decode dense vs sdpa")


@pytest.mark.parametrize("sfk,sfv", [(0.0, 1.0), (1.0, 0.0), (0.5, 1.0), (0.0, 0.4)])
def test_decode_and_prefill_per_tensor_kinds(sfk, sfv):
    """Keys dense / values 2:4 (the paper's quality-preserving setting) and the other combinations
    that select per-tensor specialised kernels."""
    O, LSE, Or, Lr = _decode_case(1, 8, 2, 64 * 12, seed=65, sparse_frac_k=sfk, sparse_frac_v=sfv)
    assert_close(O, Or, f"decode S_K={sfk} S_V={sfv}")
    assert_lse_close(LSE, Lr, f"decode S_K={sfk} S_V={sfv} lse")
    O, LSE, Or, Lr = _prefill_case(1, 8, 2, 64 * 6, 64 * 6, seed=66, sparse_frac_k=sfk, sparse_frac_v=sfv)
    assert_close(O, Or, f"prefill S_K={sfk} S_V={sfv}")
    assert_lse_close(LSE, Lr, f"prefill S_K={sfk} S_V={sfv} lse")


def test_decode_mixed_and_skip():
    B, Hq, Hkv, L = 2, 8, 2, 64 * 21
    sk, sv = _mixed_states(B, Hkv, L // 64, seed=61)
    sk[1, 1, :] = 0     # one row with every tile skipped: O = 0, LSE = -inf
    sv[1, 1, :] = 0
    O, LSE, Or, Lr = _decode_case(B, Hq, Hkv, L, seed=60, state_k=sk, state_v=sv, n_splits=3)
    assert (O[1, 4:8] == 0).all() and np.isneginf(LSE[1, 4:8]).all()
    assert_close(O, Or, "decode mixed")
    assert_lse_close(LSE, Lr, "decode mixed lse")


@pytest.mark.parametrize("skip", [0.25, 0.75])
def test_decode_skip_policy_outlier_keys(skip):
    O, LSE, Or, Lr = _decode_case(1, 32, 8, 64 * 64, seed=70, k_outliers=True, skip_frac=skip)
    assert_close(O, Or, f"decode skip={skip}")
    assert_lse_close(LSE, Lr, f"decode skip={skip} lse")


# Rows long enough for the library to hand the kept tiles out by count (from 128 tiles per split with all-2:4
# tensors, from 256 otherwise): every wave gets the same number of tiles whatever the skip pattern.  The results
# must not depend on it.
@pytest.mark.parametrize("n_splits", [1, 2, 3, 7])
@pytest.mark.parametrize("pol", [dict(skip_frac=0.5), dict(skip_frac=0.75, sparse_frac_k=0.5, sparse_frac_v=0.25),
                                 dict(skip_frac=0.3, sparse_frac_k=0.0, sparse_frac_v=1.0)])
def test_decode_tiles_handed_out_by_count(pol, n_splits):
    O, LSE, Or, Lr = _decode_case(2, 8, 2, 64 * 512, seed=75, n_splits=n_splits, k_outliers=True, **pol)
    assert_close(O, Or, f"decode by count {pol} splits={n_splits}")
    assert_lse_close(LSE, Lr, f"decode by count {pol} splits={n_splits} lse")


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_decode_by_count_explicit_states_with_empty_and_nearly_empty_rows(dtype):
    B, Hq, Hkv, L = 2, 8, 2, 64 * 520
    T = L // 64
    sk, sv = _mixed_states(B, Hkv, T, seed=76, p_skip=0.6)
    sk[0, 1, :] = 0                       # a row with nothing kept
    sv[0, 1, :] = 0
    sk[1, 0, :] = 0                       # a row with fewer kept tiles (1) than splits (2): one split gets none
    sv[1, 0, :] = 0
    sk[1, 0, 77] = 2
    sv[1, 0, 77] = 1
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=77, dtype=dtype)
    if dtype == "bf16":                   # both V encodings in one row: a few values fp16 cannot hold
        V = V.copy()
        V[:, :, 64 * 5 + 3, 9] = 0x0080   # 2^-126
        V[:, :, 64 * 350 + 1, 100] = 0x4780   # 65536
    q = Q[:, :, 0, :].copy()
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, dtype=dtype, state_k=sk, state_v=sv)
    Or, Lr = orc.attention_decode(q, pk, pv)
    for ns in (1, 2):
        O, LSE = hb.decode_attn(sh, _dev(q, dtype), kv, n_splits=ns)
        torch.cuda.synchronize()
        O, LSE = _f32(O), LSE.cpu().numpy()
        assert (O[0, 4:8] == 0).all() and np.isneginf(LSE[0, 4:8]).all()
        assert_close(O, Or, f"decode by count mixed {dtype} splits={ns}")
        assert_lse_close(LSE, Lr, f"decode by count mixed {dtype} splits={ns} lse")


@pytest.mark.parametrize("n_splits", [1, 3])
def test_decode_by_count_row_longer_than_one_scan_step_and_one_list(n_splits):
    """4608 tiles in a row: three scan steps of 2048 tiles; with one split its 3456 kept tiles fill the
    workgroup's list of 2048 twice."""
    B, Hq, Hkv, L = 1, 2, 1, 64 * 4608
    O, LSE, Or, Lr = _decode_case(B, Hq, Hkv, L, seed=78, n_splits=n_splits, skip_frac=0.25)
    assert_close(O, Or, f"decode long row splits={n_splits}")
    assert_lse_close(LSE, Lr, f"decode long row splits={n_splits} lse")


def test_decode_by_count_with_a_dense_tail():
    """The dense tail's partial sits behind the cache splits whichever way the tiles are handed out."""
    B, Hq, Hkv, L = 1, 8, 2, 64 * 300
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L + 64, 128, 1, seed=79)
    q = Q[:, :, 0, :].copy()
    Kc, Vc, Kt, Vt = K[:, :, :L].copy(), V[:, :, :L].copy(), K[:, :, L:].copy(), V[:, :, L:].copy()
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, Kc, Vc, skip_frac=0.6)
    for ns in (1, 2):      # 300 and 150 tiles per split: by count
        O, LSE = hb.decode_attn(sh, _dev(q), kv, n_splits=ns, tail_k=_dev(Kt), tail_v=_dev(Vt), tail_len=23)
        torch.cuda.synchronize()
        Or, Lr = orc.attention_decode(q, pk, pv, tail_k=Kt, tail_v=Vt, tail_len=23)
        assert_close(_f32(O), Or, f"decode by count with tail, splits {ns}")
        assert_lse_close(LSE.cpu().numpy(), Lr, "decode by count with tail lse")


def test_decode_cfg1_full_size():
    """The benchmark workload at full size, in the launch configuration the benchmark times."""
    c, q, K, V = wl.make_config("cfg1_decode_llama8b_32k")
    sh = hb.make_shape(c["B"], c["Hq"], c["Hkv"], c["L"])
    Kd, Vd = _dev(K), _dev(V)
    kv = hb.compress_kv(sh, hb.make_policy(), Kd, Vd)
    O, LSE = hb.decode_attn(sh, _dev(q), kv)
    kvd = hb.compress_kv(sh, hb.make_policy(sparse_frac_k=0.0, sparse_frac_v=0.0), Kd, Vd)
    Od, LSEd = hb.decode_attn(sh, _dev(q), kvd)
    torch.cuda.synchronize()
    pk, pv, _ = orc.compress_kv(K, V)
    Or, Lr = orc.attention_decode(q, pk, pv)
    assert_close(_f32(O), Or, "decode cfg1 2:4")
    assert_lse_close(LSE.cpu().numpy(), Lr, "decode cfg1 lse")
    st = np.full((c["B"], c["Hkv"], c["L"] // 64), 1, dtype=np.int8)
    pk, pv, _ = orc.compress_kv(K, V, state_k=st, state_v=st)
    Or, Lr = orc.attention_decode(q, pk, pv)
    assert_close(_f32(Od), Or, "decode cfg1 dense")


# ------------------------------------------------------------------ prefill
def _prefill_case(B, Hq, Hkv, L, Lq, seed, causal=True, rows=None, **pol):
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, Lq, seed=seed)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, **pol)
    O, LSE = hb.prefill_attn(sh, _dev(Q), kv, causal=causal)
    torch.cuda.synchronize()
    if rows is None:
        rows = [(b, h, i) for b in range(B) for h in range(Hq) for i in range(Lq)]
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=causal)
    idx = tuple(np.array(rows).T)
    return _f32(O)[idx], LSE.cpu().numpy()[idx], Or, Lr


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_prefill_causal_gqa_groups(G):
    O, LSE, Or, Lr = _prefill_case(1, 2 * G, 2, 64 * 5, 64 * 5, seed=80 + G)
    assert_close(O, Or, f"prefill G={G}")
    assert_lse_close(LSE, Lr, f"prefill G={G} lse")


def test_prefill_all_dense_and_noncausal():
    O, LSE, Or, Lr = _prefill_case(2, 4, 1, 64 * 4, 64 * 4, seed=90, sparse_frac_k=0.0, sparse_frac_v=0.0)
    assert_close(O, Or, "prefill dense causal")
    O, LSE, Or, Lr = _prefill_case(1, 4, 1, 64 * 4, 64 * 4, seed=91, causal=False)
    assert_close(O, Or, "prefill 2:4 non-causal")
    assert_lse_close(LSE, Lr, "prefill non-causal lse")


def test_prefill_mixed_skip_and_empty_rows():
    B, Hq, Hkv, L = 1, 8, 2, 64 * 9
    sk, sv = _mixed_states(B, Hkv, L // 64, seed=101, p_skip=0.3)
    sk[0, 0, 0] = sv[0, 0, 0] = 0      # first tile skipped: rows 0..63 of heads 0..3 see nothing
    sk[0, 0, 1] = sv[0, 0, 1] = 0
    sk[0, 1, 0] = 2
    sv[0, 1, 0] = 1
    O, LSE, Or, Lr = _prefill_case(B, Hq, Hkv, L, L, seed=100, state_k=sk, state_v=sv)
    assert_close(O, Or, "prefill mixed")
    assert_lse_close(LSE, Lr, "prefill mixed lse")
    assert np.isneginf(Lr).sum() >= 4 * 128


def test_prefill_chunk_lq_less_than_l():
    O, LSE, Or, Lr = _prefill_case(1, 8, 2, 64 * 8, 64 * 3, seed=110, skip_frac=0.25)
    assert_close(O, Or, "prefill Lq<L")
    assert_lse_close(LSE, Lr, "prefill Lq<L lse")


@pytest.mark.parametrize("q_start,Lq", [(0, 64 * 7), (64 * 5, 64 * 2), (64 * 3 + 17, 64 * 2), (64 * 12 - 64, 64)])
def test_prefill_queries_placed_inside_a_capacity_cache(q_start, Lq):
    """A cache allocated for 12 tiles that holds 7 so far (the rest SKIP): queries stand where the caller
    says (chunked prefill, growing caches), not at the end of the capacity.  Positions that are not a
    multiple of the tile, and queries beyond the filled part (they see everything filled), included."""
    B, Hq, Hkv, T_cap, T_now = 2, 8, 2, 12, 7
    L = 64 * T_cap
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, Lq, seed=250, k_outliers=True)
    sk, sv = _mixed_states(B, Hkv, T_cap, seed=251, p_skip=0.1)
    sk[:, :, T_now:], sv[:, :, T_now:] = 0, 0
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, state_k=sk, state_v=sv)
    O, LSE = hb.prefill_attn(sh, _dev(Q), kv, q_start=q_start)
    torch.cuda.synchronize()
    rows = [(b, h, i) for b in range(B) for h in range(Hq) for i in range(Lq)]
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True, q_offset=q_start)
    idx = tuple(np.array(rows).T)
    assert_close(_f32(O)[idx], Or, f"prefill at {q_start}")
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, f"prefill at {q_start} lse")
    if q_start == 0:
        for bad in (-1, L - Lq + 1):
            with pytest.raises(hb.HsError):
                hb.prefill_attn(sh, _dev(Q), kv, q_start=bad)


def test_decode_equals_last_prefill_row():
    B, Hq, Hkv, L = 1, 8, 2, 64 * 6
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=120)
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv = hb.compress_kv(sh, hb.make_policy(), _dev(K), _dev(V))
    O, _ = hb.prefill_attn(sh, _dev(Q), kv)
    Od, _ = hb.decode_attn(sh, _dev(Q[:, :, -1, :].copy()), kv)
    torch.cuda.synchronize()
    assert_close(_f32(Od), _f32(O)[:, :, -1, :], "decode vs last prefill row")


def test_prefill_cfg2_full_size_sampled_rows():
    c, Q, K, V = wl.make_config("cfg2_prefill_llama8b_16k")
    rows = wl.sample_rows(c["B"], c["Hq"], c["L"], 256, seed=c["seed"] + 4,
                          extra=[(0, 0, 0), (0, 31, c["L"] - 1), (0, 5, 63), (0, 5, 64)])
    sh = hb.make_shape(c["B"], c["Hq"], c["Hkv"], c["L"])
    kv = hb.compress_kv(sh, hb.make_policy(), _dev(K), _dev(V))
    O, LSE = hb.prefill_attn(sh, _dev(Q), kv)
    torch.cuda.synchronize()
    pk, pv, _ = orc.compress_kv(K, V)
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True)
    idx = tuple(np.array(rows).T)
    assert_close(_f32(O)[idx], Or, "prefill cfg2 sampled")
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, "prefill cfg2 lse")


@pytest.mark.parametrize("pol", [dict(), dict(sparse_frac_k=0.0, sparse_frac_v=1.0)])
def test_prefill_on_the_benchmark_workload_full_size_sampled_rows(pol):
    """Causal prefill on the inputs the benchmark's step times (L = 32768, keys with outlier channels, which
    drive the lazily renewed softmax reference through its redo path), all tiles 2:4 and keys dense /
    values 2:4: 160 seeded rows plus the first and last row and the rows around the first tile edge."""
    c = wl.CONFIGS["cfg1_decode_llama8b_32k"]
    B, Hq, Hkv, L = c["B"], c["Hq"], c["Hkv"], c["L"]
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, c["D"], L, c["seed"], c["k_outliers"])
    rows = wl.sample_rows(B, Hq, L, 160, seed=c["seed"] + 4,
                          extra=[(0, 0, 0), (0, Hq - 1, L - 1), (0, 7, 63), (0, 7, 64), (0, 13, L - 65)])
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv = hb.compress_kv(sh, hb.make_policy(**pol), _dev(K), _dev(V))
    O, LSE = hb.prefill_attn(sh, _dev(Q), kv)
    torch.cuda.synchronize()
    pk, pv, _ = orc.compress_kv(K, V, **pol)
    assert_maps_equal(kv, pk, pv)
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True)
    idx = tuple(np.array(rows).T)
    assert_close(_f32(O)[idx], Or, f"prefill benchmark workload {sorted(pol)}")
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, "prefill benchmark workload lse")


def test_decode_cfg3_shape_one_batch_row_skip75():
    """Hierarchical decode sweep workload (L = 131072, 32/8 heads) at its full context for one
    batch row, 75 % of the tiles skipped + 2:4 in the rest, default launch configuration."""
    c, q, K, V = wl.make_config("cfg3_decode_b8_128k", B=1)
    sh, kv, pk, pv, info = compress_both(c["B"], c["Hq"], c["Hkv"], c["L"], K, V, skip_frac=0.75)
    assert_maps_equal(kv, pk, pv)
    assert int((pk.map == 0).sum()) == 8 * 1536
    O, LSE = hb.decode_attn(sh, _dev(q), kv)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, pk, pv)
    assert_close(_f32(O), Or, "decode cfg3 B=1 skip 0.75")
    assert_lse_close(LSE.cpu().numpy(), Lr, "decode cfg3 lse")


@pytest.mark.parametrize("pol", [dict(skip_frac=0.25), dict(skip_frac=0.5), dict(skip_frac=0.75),
                                 dict(sparse_frac_k=0.0, sparse_frac_v=1.0)])
def test_decode_cfg3_full_batch_sampled_rows(pol):
    """The hierarchical decode workload at its full size (B = 8, L = 131072: 4.3 GB of K and V, pools past
    2^31 bytes), default launch configuration.  Inputs are drawn on the device (seeded); the oracle
    compresses and attends three sampled (batch, kv head) rows, each of which is ranked on its own."""
    B, Hq, Hkv, L = 8, 32, 8, 131072
    g = torch.Generator(device="cuda")
    g.manual_seed(300)
    K = torch.randn((B, Hkv, L, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    V = torch.randn((B, Hkv, L, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    q = torch.randn((B, Hq, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv = hb.compress_kv(sh, hb.make_policy(**pol), K, V)
    O, LSE = hb.decode_attn(sh, q, kv)
    torch.cuda.synchronize()
    G = Hq // Hkv
    for b, h in ((0, 0), (3, 5), (7, 7)):
        print(f"[cfg3 full batch {sorted(pol)}] row b={b} hkv={h}", flush=True)
        Kb, Vb = hb.bf16_tensor_to_bits(K[b:b + 1, h:h + 1]), hb.bf16_tensor_to_bits(V[b:b + 1, h:h + 1])
        pk, pv, _ = orc.compress_kv(Kb, Vb, Bt=64, **pol)
        assert_maps_equal(kv, pk, pv, sel=(b, h), osel=(0, 0))
        for p, dense, nnz, meta, cd, cs in ((pk, kv.k_dense, kv.k_nnz, kv.k_meta, kv.counts[1], kv.counts[2]),
                                            (pv, kv.v_dense, kv.v_nnz, kv.v_meta, kv.counts[3], kv.counts[4])):
            ph = hl.physical_pools(p)
            nd, ns = int(ph["n_dense"][0, 0]), int(ph["n_sparse"][0, 0])
            for slot in {0, nd // 2, nd - 1} - {-1}:           # first, middle and last used slot
                if nd:
                    assert (dense.view(B, Hkv, cd, 16384)[b, h, slot].cpu().numpy() == ph["dense"][0, 0, slot]).all()
            for slot in {0, ns // 2, ns - 1} - {-1}:
                if ns:
                    assert (nnz.view(B, Hkv, cs, 8192)[b, h, slot].cpu().numpy() == ph["nnz"][0, 0, slot]).all()
                    assert (meta.view(B, Hkv, cs, 1024)[b, h, slot].cpu().numpy() == ph["meta"][0, 0, slot]).all()
        qb = hb.bf16_tensor_to_bits(q[b:b + 1, G * h:G * (h + 1)])
        Or, Lr = orc.attention_decode(qb, pk, pv)
        assert_close(_f32(O[b:b + 1, G * h:G * (h + 1)]), Or, f"decode cfg3 full batch b{b} hkv{h}")
        assert_lse_close(LSE[b:b + 1, G * h:G * (h + 1)].cpu().numpy(), Lr, "decode cfg3 full batch lse")


def _check_sampled_heads(sh, kv, K, V, Q, O, LSE, q_dec, O_dec, LSE_dec, pol, heads, n_rows, seed, dtype="bf16", q_start=None):
    """Oracle check of device-generated full-size inputs on sampled (batch, kv head) rows: maps and a few pool
    slots bit for bit, prefill on n_rows sampled queries of one query head of the group, decode on the group."""
    B, Hq, Hkv, L = sh.B, sh.Hq, sh.Hkv, sh.L
    G = Hq // Hkv
    rng = np.random.default_rng(seed)
    for b, h in heads:
        print(f"[sampled heads] b={b} hkv={h} {sorted(pol)}", flush=True)
        Kb, Vb = hb.bf16_tensor_to_bits(K[b:b + 1, h:h + 1]), hb.bf16_tensor_to_bits(V[b:b + 1, h:h + 1])
        pk, pv, _ = orc.compress_kv(Kb, Vb, Bt=64, dtype=dtype, **pol)
        assert_maps_equal(kv, pk, pv, sel=(b, h), osel=(0, 0))
        if Q is not None:
            Lq = Q.shape[2]
            hq = G * h + int(rng.integers(G))
            qi = sorted(set([0, Lq - 1] + [int(x) for x in rng.integers(0, Lq, size=n_rows)]))
            Qb = hb.bf16_tensor_to_bits(Q[b:b + 1, hq:hq + 1])
            Or, Lr = orc.attention_rows(Qb, pk, pv, [(0, 0, i) for i in qi], causal=True, q_offset=q_start)
            assert_close(_f32(O[b, hq])[qi], Or, f"prefill sampled b{b} hq{hq}")
            assert_lse_close(LSE[b, hq].cpu().numpy()[qi], Lr, f"prefill sampled lse b{b} hq{hq}")
        if q_dec is not None:
            qb = hb.bf16_tensor_to_bits(q_dec[b:b + 1, G * h:G * (h + 1)])
            Or, Lr = orc.attention_decode(qb, pk, pv)
            assert_close(_f32(O_dec[b:b + 1, G * h:G * (h + 1)]), Or, f"decode sampled b{b} hkv{h}")
            assert_lse_close(LSE_dec[b:b + 1, G * h:G * (h + 1)].cpu().numpy(), Lr, f"decode sampled lse b{b} hkv{h}")


@pytest.mark.parametrize("pol", [dict(), dict(sparse_frac_k=0.0, sparse_frac_v=1.0)])
def test_paper_kernel_shape_b8_32k_sampled_heads(pol):
    """The shape of the paper's own kernel benchmarks (Sec. V-B: batch 8, 32K tokens, 32 / 8 heads) at full size,
    as the benchmark leg runs it: prefill and decode, all tiles 2:4 and keys dense / values 2:4, against the
    oracle on two sampled (batch, kv head) rows."""
    B, Hq, Hkv, L = 8, 32, 8, 32768
    g = torch.Generator(device="cuda")
    g.manual_seed(500)
    K = torch.randn((B, Hkv, L, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    V = torch.randn((B, Hkv, L, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    Q = torch.randn((B, Hq, L, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv = hb.compress_kv(sh, hb.make_policy(**pol), K, V)
    O, LSE = hb.prefill_attn(sh, Q, kv)
    q = Q[:, :, -1, :].contiguous()
    Od, LSEd = hb.decode_attn(sh, q, kv)
    torch.cuda.synchronize()
    _check_sampled_heads(sh, kv, K, V, Q, O, LSE, q, Od, LSEd, pol, [(0, 0), (6, 5)], 24, seed=501)


def test_fp16_benchmark_shape_sampled_heads():
    """fp16 (the paper's element type) at the benchmark workload's shape (L = 32768), as the fp16 leg runs it."""
    B, Hq, Hkv, L = 1, 32, 8, 32768
    g = torch.Generator(device="cuda")
    g.manual_seed(510)
    K = torch.randn((B, Hkv, L, 128), device="cuda", dtype=torch.float16, generator=g)
    V = torch.randn((B, Hkv, L, 128), device="cuda", dtype=torch.float16, generator=g)
    Q = torch.randn((B, Hq, L, 128), device="cuda", dtype=torch.float16, generator=g)
    sh = hb.make_shape(B, Hq, Hkv, L, dtype=hb.FP16)
    for pol in (dict(), dict(sparse_frac_k=0.0, sparse_frac_v=1.0)):
        kv = hb.compress_kv(sh, hb.make_policy(**pol), K, V)
        O, LSE = hb.prefill_attn(sh, Q, kv)
        q = Q[:, :, -1, :].contiguous()
        Od, LSEd = hb.decode_attn(sh, q, kv)
        torch.cuda.synchronize()
        _check_sampled_heads(sh, kv, K, V, Q, O, LSE, q, Od, LSEd, pol, [(0, 3)], 32, seed=511, dtype="fp16")


def test_chunked_prefill_128k_in_32k_chunks_sampled_head():
    """Chunked prefill as the benchmark leg runs it (a cache allocated for 128K tokens, 32K-token chunks, per
    chunk one append and one causal attention call at the chunk's position): the last chunk's outputs and the
    final cache against the oracle on one sampled kv head."""
    Hq, Hkv, Lc, chunk = 32, 8, 131072, 32768
    Tc, nct = Lc // 64, chunk // 64
    g = torch.Generator(device="cuda")
    g.manual_seed(520)
    K = torch.randn((1, Hkv, Lc, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    V = torch.randn((1, Hkv, Lc, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    Q = torch.randn((1, Hq, chunk, 128), device="cuda", dtype=torch.bfloat16, generator=g)
    sh = hb.make_shape(1, Hq, Hkv, Lc)
    kv = hb.PackedKV(sh, [0, Tc, 0, 0, Tc])                  # keys dense, values 2:4
    kv.uniform = 0
    kv.k_map.zero_()
    kv.v_map.zero_()
    ovf = torch.zeros(1, dtype=torch.int32, device="cuda")
    for c in range(Lc // chunk):
        hb.append_tile(sh, kv, nct * c, K[:, :, chunk * c:chunk * (c + 1)], V[:, :, chunk * c:chunk * (c + 1)],
                       state_k=hb.DENSE, state_v=hb.SPARSE24, overflow=ovf)
        O, LSE = hb.prefill_attn(sh, Q, kv, q_start=chunk * c)
    torch.cuda.synchronize()
    assert int(ovf.item()) == 0
    pol = dict(sparse_frac_k=0.0, sparse_frac_v=1.0)          # what the appended states amount to
    _check_sampled_heads(sh, kv, K, V, Q, O, LSE, None, None, None, pol, [(0, 6)], 12, seed=521, q_start=Lc - chunk)


def test_selection_on_a_row_longer_than_the_register_cache():
    """Tile selection with more than 8 tiles per thread (rows over 2048 tiles take the path that re-reads
    the scores instead of holding them in registers): maps against the oracle, with planted equal tiles
    so that ties on the cut are broken by tile index."""
    B, Hq, Hkv, T = 1, 1, 1, 2304
    L = 64 * T
    rng = np.random.default_rng(240)
    K = wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, L, 128)).astype(np.float32))
    V = wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, L, 128)).astype(np.float32))
    for t in (7, 900, 2200):                                 # the three quietest tiles are identical
        K[0, 0, 64 * t:64 * t + 64] = K[0, 0, 64 * 7:64 * 7 + 64] & 0x8000 | 0x3000
        V[0, 0, 64 * t:64 * t + 64] = V[0, 0, 64 * 7:64 * 7 + 64] & 0x8000 | 0x3000
    pol = dict(skip_frac=2 / (T - 4) + 1e-9, sparse_frac_k=0.5, sparse_frac_v=0.7, dense_first_tiles=1, dense_last_tiles=3)
    sh, kv, pk, pv, info = compress_both(B, Hq, Hkv, L, K, V, **pol)
    assert int((pk.map == 0).sum()) == 2 and pk.map[0, 0, 7] == 0 and pk.map[0, 0, 900] == 0 and pk.map[0, 0, 2200] != 0
    assert_maps_equal(kv, pk, pv)
    Ku, Vu = hb.unpack_kv(sh, kv)
    torch.cuda.synchronize()
    assert (hb.bf16_tensor_to_bits(Ku) == orc.unpack_tensor(pk)).all()
    assert (hb.bf16_tensor_to_bits(Vu) == orc.unpack_tensor(pv)).all()


def test_prefill_cfg4_full_size_skip75_sampled_rows():
    """Long causal prefill at the highest hierarchical sparsity (L = 65536, 75 % of the tiles
    skipped, 2:4 in the rest): seeded sampled rows plus rows that see no token at all."""
    c, Q, K, V = wl.make_config("cfg4_prefill_64k")
    sh, kv, pk, pv, info = compress_both(c["B"], c["Hq"], c["Hkv"], c["L"], K, V, skip_frac=0.75)
    assert_maps_equal(kv, pk, pv)
    # rows whose own and all earlier tiles are skipped (kv head 0 ... 7): O = 0, LSE = -inf
    extra = []
    for hkv in range(c["Hkv"]):
        first_kept = int(np.nonzero(pk.map[0, hkv] != 0)[0][0])
        if first_kept > 0:
            extra += [(0, 4 * hkv, 0), (0, 4 * hkv + 3, 64 * first_kept - 1)]
        extra += [(0, 4 * hkv + 1, 64 * first_kept), (0, 4 * hkv + 2, c["L"] - 1)]
    rows = wl.sample_rows(c["B"], c["Hq"], c["L"], 160, seed=c["seed"] + 4, extra=extra)
    O, LSE = hb.prefill_attn(sh, _dev(Q), kv)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True)
    idx = tuple(np.array(rows).T)
    got, lse = _f32(O)[idx], LSE.cpu().numpy()[idx]
    empty = np.isneginf(Lr)
    assert empty.sum() >= 1
    assert (got[empty] == 0).all()
    assert_close(got, Or, "prefill cfg4 skip 0.75 sampled")
    assert_lse_close(lse, Lr, "prefill cfg4 lse")


def test_decode_with_dense_tail():
    """Cache of whole tiles plus 0..64 recent tokens that are not compressed yet."""
    B, Hq, Hkv, L = 2, 8, 2, 64 * 7
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L + 64, 128, 1, seed=160)
    q = Q[:, :, 0, :].copy()
    Kc, Vc, Kt, Vt = K[:, :, :L].copy(), V[:, :, :L].copy(), K[:, :, L:].copy(), V[:, :, L:].copy()
    sk, sv = _mixed_states(B, Hkv, L // 64, seed=161, p_skip=0.3)
    for pol in (dict(), dict(state_k=sk, state_v=sv)):
        sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, Kc, Vc, **pol)
        for tail_len in (0, 1, 17, 64):
            for ns in (0, 3):
                O, LSE = hb.decode_attn(sh, _dev(q), kv, n_splits=ns, tail_k=_dev(Kt), tail_v=_dev(Vt), tail_len=tail_len)
                torch.cuda.synchronize()
                Or, Lr = orc.attention_decode(q, pk, pv, tail_k=Kt, tail_v=Vt, tail_len=tail_len)
                assert_close(_f32(O), Or, f"decode tail {tail_len} splits {ns} {sorted(pol)}")
                assert_lse_close(LSE.cpu().numpy(), Lr, f"decode tail {tail_len} lse")
    # every cached tile skipped: the tail alone answers
    z = np.zeros((B, Hkv, L // 64), dtype=np.int8)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, Kc, Vc, state_k=z, state_v=z)
    O, LSE = hb.decode_attn(sh, _dev(q), kv, tail_k=_dev(Kt), tail_v=_dev(Vt), tail_len=5)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, pk, pv, tail_k=Kt, tail_v=Vt, tail_len=5)
    assert_close(_f32(O), Or, "decode tail only")
    assert_lse_close(LSE.cpu().numpy(), Lr, "decode tail only lse")
    import ctypes as C
    kvs = kv.struct()
    qd = _dev(q)
    assert hb.lib().hs_decode_attn_tail(C.byref(sh), 0.0, 0, hb._ptr(qd), C.byref(kvs), None, None, 65, hb._ptr(qd), None,
                                        hb._ptr(qd), None) == -1
    assert hb.lib().hs_decode_attn_tail(C.byref(sh), 0.0, 0, hb._ptr(qd), C.byref(kvs), None, None, 3, hb._ptr(qd), None,
                                        hb._ptr(qd), None) == -1


def test_append_tiles_during_decode():
    """A cache allocated for 9 tiles, compressed with 4, then grown tile by tile (mixed tile kinds, the last
    one from a strided buffer); after every append decode equals the oracle's, and at the end pools and maps
    are those of compressing everything at once."""
    B, Hq, Hkv, L = 2, 8, 2, 64 * 9
    T = L // 64
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=170)
    q = Q[:, :, 0, :].copy()
    rng = np.random.default_rng(171)
    sk = rng.choice([1, 2], size=(T,)).astype(np.int8)
    sv = rng.choice([1, 2], size=(T,)).astype(np.int8)
    full_k, full_v = np.broadcast_to(sk, (B, Hkv, T)).copy(), np.broadcast_to(sv, (B, Hkv, T)).copy()
    pre_k, pre_v = full_k.copy(), full_v.copy()
    pre_k[:, :, 4:] = 0
    pre_v[:, :, 4:] = 0
    sh = hb.make_shape(B, Hq, Hkv, L)
    caps = [0, int((sk == 1).sum()), int((sk == 2).sum()), int((sv == 1).sum()), int((sv == 2).sum())]
    kv = hb.PackedKV(sh, caps)
    hb.compress_kv(sh, hb.make_policy(state_k=pre_k, state_v=pre_v), _dev(K), _dev(V), out=kv)
    pk, pv, _ = orc.compress_kv(K, V, state_k=pre_k, state_v=pre_v)
    ovf = torch.zeros(1, dtype=torch.int32, device="cuda")
    Kd, Vd = _dev(K), _dev(V)
    for t in range(4, T):
        kt, vt = Kd[:, :, 64 * t:64 * (t + 1)], Vd[:, :, 64 * t:64 * (t + 1)]      # strided views of the full tensors
        if t % 2 == 0:
            kt, vt = kt.contiguous(), vt.contiguous()
        hb.append_tile(sh, kv, t, kt, vt, state_k=int(sk[t]), state_v=int(sv[t]), overflow=ovf)
        orc.append_tile(pk, pv, t, K[:, :, 64 * t:64 * (t + 1)], V[:, :, 64 * t:64 * (t + 1)], int(sk[t]), int(sv[t]))
        O, LSE = hb.decode_attn(sh, _dev(q), kv)
        torch.cuda.synchronize()
        Or, Lr = orc.attention_decode(q, pk, pv)
        assert_close(_f32(O), Or, f"decode after append of tile {t}")
        assert_lse_close(LSE.cpu().numpy(), Lr, f"decode after append of tile {t} lse")
    assert int(ovf.item()) == 0
    pk1, pv1, _ = orc.compress_kv(K, V, state_k=full_k, state_v=full_v)
    check_packed_bit_exact(sh, kv, pk1, pv1)
    # a full pool: the tile stays skipped and the flag goes up
    kv2 = hb.PackedKV(sh, [0, 1, 4, 1, 4])
    z = np.zeros((B, Hkv, T), dtype=np.int8)
    z[:, :, :4] = 2
    hb.compress_kv(sh, hb.make_policy(state_k=z, state_v=z), Kd, Vd, out=kv2)
    hb.append_tile(sh, kv2, 4, Kd[:, :, 256:320].contiguous(), Vd[:, :, 256:320].contiguous(), overflow=ovf)
    torch.cuda.synchronize()
    assert int(ovf.item()) == 1
    assert (kv2.k_map[:, :, 4].cpu().numpy() == 0).all() and (kv2.v_map[:, :, 4].cpu().numpy() == 0).all()
    import ctypes as C
    kvs = kv2.struct()
    args = (hb._ptr(Kd), hb._ptr(Vd), None, C.byref(kvs), None, None)
    assert hb.lib().hs_append_tile(C.byref(sh), T, 2, 2, 0, *args) == -1          # tile out of range
    assert hb.lib().hs_append_tile(C.byref(sh), 5, 0, 2, 0, *args) == -1          # SKIP is not a state to append
    assert hb.lib().hs_append_tile(C.byref(sh), 5, 2, 2, 7, *args) == -1          # unknown element rule


def test_batch_rows_of_different_length_decode_and_append():
    """A batch whose sequences hold 3, 9 and 6 tiles and 17, 0 and 64 tail tokens: decode with one tail
    length per batch row; the row with the full tail (and only that one) appends it at its own position;
    decode again.  Against the oracle throughout, packed state bit for bit."""
    B, Hq, Hkv, T = 3, 8, 2, 10
    L = 64 * T
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=270, k_outliers=True)
    q = Q[:, :, 0, :].copy()
    held = [3, 9, 6]
    sk = np.full((B, Hkv, T), orc.DENSE, dtype=np.int8)
    sv = np.full((B, Hkv, T), orc.SPARSE24, dtype=np.int8)
    for b in range(B):
        sk[b, :, held[b]:] = 0
        sv[b, :, held[b]:] = 0
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv = hb.PackedKV(sh, [0, T, 0, 0, T])
    kv.uniform = 0
    hb.compress_kv(sh, hb.make_policy(state_k=sk, state_v=sv), _dev(K), _dev(V), out=kv)
    pk, pv, _ = orc.compress_kv(K, V, state_k=sk, state_v=sv)
    _, tk, tv = wl.make_qkv(B, Hq, Hkv, 64, 128, 1, seed=271)
    lens = np.array([17, 0, 64], dtype=np.int32)
    lens_d = torch.from_numpy(lens).cuda()
    O, LSE = hb.decode_attn(sh, _dev(q), kv, tail_k=_dev(tk), tail_v=_dev(tv), tail_len=lens_d, n_splits=2)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, pk, pv, tail_k=tk, tail_v=tv, tail_len=lens)
    for b in range(B):
        assert_close(_f32(O)[b], Or[b], f"decode ragged batch row {b}")
    assert_lse_close(LSE.cpu().numpy(), Lr, "decode ragged batch lse")
    where = np.array([-1, -1, held[2]], dtype=np.int32)
    ovf = torch.zeros(1, dtype=torch.int32, device="cuda")
    hb.append_tile(sh, kv, torch.from_numpy(where).cuda(), _dev(tk), _dev(tv), state_k=hb.DENSE, state_v=hb.SPARSE24, overflow=ovf)
    orc.append_tile(pk, pv, where, tk, tv, orc.DENSE, orc.SPARSE24)
    torch.cuda.synchronize()
    assert int(ovf.item()) == 0
    check_packed_bit_exact(sh, kv, pk, pv)
    lens2 = np.array([18, 1, 0], dtype=np.int32)            # one more token each; row 2 starts a new tail
    O, LSE = hb.decode_attn(sh, _dev(q), kv, tail_k=_dev(tk), tail_v=_dev(tv), tail_len=torch.from_numpy(lens2).cuda())
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, pk, pv, tail_k=tk, tail_v=tv, tail_len=lens2)
    for b in range(B):
        assert_close(_f32(O)[b], Or[b], f"decode ragged batch after append row {b}")
    assert_lse_close(LSE.cpu().numpy(), Lr, "decode ragged batch after append lse")


def test_serving_loop_two_sequences_of_different_length():
    """The calls in the order a serving loop issues them, for a batch of two sequences of different length:
    compress the whole tiles of each prompt (keys dense, values 2:4), prune the keys further for decode,
    then 70 decode steps in which every new token goes to the dense tail and a full tail moves into the
    cache of its own sequence.  Oracle state and outputs are checked along the way."""
    B, Hq, Hkv, T = 2, 8, 2, 8
    L = 64 * T
    prompt = [64 * 5 + 17, 64 * 3 + 40]
    steps = 70
    total = max(prompt) + steps
    rng = np.random.default_rng(280)
    Kall = wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, total, 128)).astype(np.float32))
    Vall = wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, total, 128)).astype(np.float32))
    Qall = wl.f32_to_bf16_bits(rng.standard_normal((B, Hq, steps, 128)).astype(np.float32))
    held = [p // 64 for p in prompt]
    tail_n = [p % 64 for p in prompt]
    K0, V0 = np.zeros((B, Hkv, L, 128), dtype=np.uint16), np.zeros((B, Hkv, L, 128), dtype=np.uint16)
    sk, sv = np.zeros((B, Hkv, T), dtype=np.int8), np.zeros((B, Hkv, T), dtype=np.int8)
    tk, tv = np.zeros((B, Hkv, 64, 128), dtype=np.uint16), np.zeros((B, Hkv, 64, 128), dtype=np.uint16)
    for b in range(B):
        n = 64 * held[b]
        K0[b, :, :n], V0[b, :, :n] = Kall[b, :, :n], Vall[b, :, :n]
        sk[b, :, :held[b]], sv[b, :, :held[b]] = orc.DENSE, orc.SPARSE24
        tk[b, :, :tail_n[b]], tv[b, :, :tail_n[b]] = Kall[b, :, n:prompt[b]], Vall[b, :, n:prompt[b]]
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv_prefill = hb.PackedKV(sh, [0, T, 0, 0, T])
    kv_prefill.uniform = 0
    hb.compress_kv(sh, hb.make_policy(state_k=sk, state_v=sv), _dev(K0), _dev(V0), out=kv_prefill)
    pk, pv, _ = orc.compress_kv(K0, V0, state_k=sk, state_v=sv)
    # decode policy: every key tile 2:4 as well
    kv = hb.recompress_kv(sh, kv_prefill, hb.make_policy(), counts=[0, 0, T, 0, T])
    pk, pv = orc.recompress_kv(pk, pv, np.where(sk == 0, 0, 2), np.where(sv == 0, 0, 2))
    torch.cuda.synchronize()
    check_packed_bit_exact(sh, kv, pk, pv)
    tk_d, tv_d = _dev(tk), _dev(tv)
    ovf = torch.zeros(1, dtype=torch.int32, device="cuda")
    pos = list(prompt)
    checked = 0
    for s_ in range(steps):
        for b in range(B):                                   # the new token's K, V join the tail of its sequence
            tk[b, :, tail_n[b]], tv[b, :, tail_n[b]] = Kall[b, :, pos[b]], Vall[b, :, pos[b]]
            tk_d[b, :, tail_n[b]] = _dev(Kall[b, :, pos[b]])
            tv_d[b, :, tail_n[b]] = _dev(Vall[b, :, pos[b]])
            tail_n[b] += 1
            pos[b] += 1
        q = Qall[:, :, s_, :].copy()
        lens = np.array(tail_n, dtype=np.int32)
        O, LSE = hb.decode_attn(sh, _dev(q), kv, tail_k=tk_d, tail_v=tv_d, tail_len=torch.from_numpy(lens).cuda(), n_splits=2)
        if s_ in (0, 23, 24, 46, 47, 48, steps - 1):
            torch.cuda.synchronize()
            Or, Lr = orc.attention_decode(q, pk, pv, tail_k=tk, tail_v=tv, tail_len=lens)
            for b in range(B):
                assert_close(_f32(O)[b], Or[b], f"serving step {s_} sequence {b}")
            assert_lse_close(LSE.cpu().numpy(), Lr, f"serving step {s_} lse")
            checked += 1
        where = np.array([held[b] if tail_n[b] == 64 else -1 for b in range(B)], dtype=np.int32)
        if (where >= 0).any():                               # a full tail becomes the next tile of its sequence
            hb.append_tile(sh, kv, torch.from_numpy(where).cuda(), tk_d, tv_d, state_k=hb.SPARSE24, state_v=hb.SPARSE24, overflow=ovf)
            orc.append_tile(pk, pv, where, tk, tv, orc.SPARSE24, orc.SPARSE24)
            for b in range(B):
                if where[b] >= 0:
                    held[b] += 1
                    tail_n[b] = 0
    torch.cuda.synchronize()
    assert checked == 7 and int(ovf.item()) == 0 and held == [6, 4] and tail_n == [23, 46]
    check_packed_bit_exact(sh, kv, pk, pv)


def test_chunked_prefill_appends_a_chunk_then_attends_from_its_position():
    """Chunked prefill (the paper's long-context runs use chunks): a cache allocated for the whole sequence
    starts empty; each chunk of 3 tiles is appended in one call (keys dense, values 2:4) and its queries attend
    from their position.  Outputs equal the oracle's causal attention over the one-shot cache; the final
    pools equal one-shot compression; a pool that runs out mid-chunk keeps the tiles that fit."""
    B, Hq, Hkv, T, n = 2, 8, 2, 12, 3
    L = 64 * T
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=260, k_outliers=True)
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv = hb.PackedKV(sh, [0, T, 0, 0, T])
    kv.uniform = 0
    kv.k_map.zero_()
    kv.v_map.zero_()
    sk = np.full((B, Hkv, T), orc.DENSE, dtype=np.int8)
    sv = np.full((B, Hkv, T), orc.SPARSE24, dtype=np.int8)
    pk, pv, _ = orc.compress_kv(K, V, state_k=sk, state_v=sv)
    Kd, Vd, Qd = _dev(K), _dev(V), _dev(Q)
    ovf = torch.zeros(1, dtype=torch.int32, device="cuda")
    for c in range(T // n):
        lo, hi = 64 * n * c, 64 * n * (c + 1)
        hb.append_tile(sh, kv, n * c, Kd[:, :, lo:hi], Vd[:, :, lo:hi], state_k=hb.DENSE, state_v=hb.SPARSE24, overflow=ovf)
        O, LSE = hb.prefill_attn(sh, Qd[:, :, lo:hi].contiguous(), kv, q_start=lo)
        torch.cuda.synchronize()
        rows = [(b, h, i) for b in range(B) for h in range(Hq) for i in range(lo, hi, 5)]
        Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True, q_offset=0)
        got = _f32(O)[:, :, ::5].reshape(-1, 128)
        assert_close(got, Or, f"chunk {c}")
        assert_lse_close(LSE.cpu().numpy()[:, :, ::5].reshape(-1), Lr, f"chunk {c} lse")
    assert int(ovf.item()) == 0
    check_packed_bit_exact(sh, kv, pk, pv)
    small = hb.PackedKV(sh, [0, 4, 0, 0, 5])                # room for 4 dense K tiles and 5 2:4 V tiles
    small.uniform = 0
    small.k_map.zero_()
    small.v_map.zero_()
    hb.append_tile(sh, small, 2, Kd[:, :, :64 * 6], Vd[:, :, :64 * 6], state_k=hb.DENSE, state_v=hb.SPARSE24, overflow=ovf)
    torch.cuda.synchronize()
    assert int(ovf.item()) == 1
    assert (small.k_map.cpu().numpy()[0, 0] == [0, 0, 1, 2, 3, 4, 0, 0, 0, 0, 0, 0]).all()
    assert ((np.abs(small.v_map.cpu().numpy()[1, 1]) & ~hb.MAP_F16) == [0, 0, 1, 2, 3, 4, 0, 0, 0, 0, 0, 0]).all()
    import ctypes as C
    kvs = small.struct()
    args = (hb._ptr(Kd), hb._ptr(Vd), None, C.byref(kvs), None, None)
    assert hb.lib().hs_append_tiles(C.byref(sh), 10, 3, 1, 2, 0, *args) == -1      # runs past the capacity
    assert hb.lib().hs_append_tiles(C.byref(sh), 0, 0, 1, 2, 0, *args) == -1


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_and_policies(seed):
    """Seeded sweep over shapes (batch, heads, GQA group, tiles, query chunk) and policies (fractions with
    ranking, protected end tiles, explicit states, non-zero rule); every stage against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.integers(1, 4))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 4, 8]))
    Hq = Hkv * G
    T = int(rng.integers(1, 14))
    L = 64 * T
    Tq = int(rng.integers(1, T + 1))
    Lq = 64 * Tq
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, Lq, seed=2000 + seed, k_outliers=bool(rng.integers(0, 2)))
    kind = int(rng.integers(0, 4))
    if kind == 0:
        pol = dict(skip_frac=float(rng.choice([0.0, 0.25, 0.5])), sparse_frac_k=float(rng.choice([0.0, 0.5, 1.0])),
                   sparse_frac_v=float(rng.choice([0.0, 0.3, 1.0])))
    elif kind == 1:
        pol = dict(skip_frac=float(rng.choice([0.0, 0.4])), dense_first_tiles=int(rng.integers(0, 3)),
                   dense_last_tiles=int(rng.integers(0, 5)))
    elif kind == 2:
        sk, sv = _mixed_states(B, Hkv, T, seed=3000 + seed, p_skip=float(rng.choice([0.0, 0.3])))
        pol = dict(state_k=sk, state_v=sv)
    else:
        pol = dict(element_rule="nonzero", sparse_frac_v=float(rng.choice([0.5, 1.0])))
    sh, kv, pk, pv, info = compress_both(B, Hq, Hkv, L, K, V, **pol)
    if "energy" in info:       # ranked: the cut must not sit on a rounding-level near-tie (see test_compress_policy_ranking)
        for key in ("energy", "loss_k", "loss_v"):
            sc = np.sort(info[key], axis=-1)
            gaps = np.diff(sc, axis=-1) / np.maximum(sc[..., 1:], 1e-300)
            assert ((gaps > 1e-12) | (gaps == 0)).all()
    check_packed_bit_exact(sh, kv, pk, pv)
    causal = bool(rng.integers(0, 4))          # mostly causal
    O, LSE = hb.prefill_attn(sh, _dev(Q), kv, causal=causal)
    n_rows = min(96, B * Hq * Lq)
    flat = rng.choice(B * Hq * Lq, size=n_rows, replace=False)
    rows = [(int(f // (Hq * Lq)), int((f // Lq) % Hq), int(f % Lq)) for f in flat]
    rows.append((B - 1, Hq - 1, Lq - 1))
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=causal)
    idx = tuple(np.array(rows).T)
    what = f"seed {seed}: B{B} Hq{Hq} Hkv{Hkv} L{L} Lq{Lq} causal={causal} {sorted(pol)}"
    torch.cuda.synchronize()
    assert_close(_f32(O)[idx], Or, "prefill " + what)
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, "prefill lse " + what)
    q = Q[:, :, -1, :].copy()
    ns = int(rng.choice([0, 1, 5, 40]))
    Od, LSEd = hb.decode_attn(sh, _dev(q), kv, n_splits=ns)
    torch.cuda.synchronize()
    Odr, Ldr = orc.attention_decode(q, pk, pv)
    assert_close(_f32(Od), Odr, f"decode splits {ns} " + what)
    assert_lse_close(LSEd.cpu().numpy(), Ldr, "decode lse " + what)


@pytest.mark.parametrize("seed", range(8))
def test_random_long_rows_decode(seed):
    """Seeded sweep over rows long enough for decode to hand its tiles out by count (and some just under the
    limits, which go by range): random skip patterns, kinds, protected end tiles, split counts, GQA groups."""
    rng = np.random.default_rng(5000 + seed)
    B = int(rng.integers(1, 3))
    Hkv = int(rng.integers(1, 3))
    G = int(rng.choice([1, 2, 4, 8]))
    Hq = Hkv * G
    T = int(rng.integers(120, 1100))
    L = 64 * T
    dtype = "fp16" if seed % 4 == 3 else "bf16"
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=6000 + seed, k_outliers=bool(rng.integers(0, 2)), dtype=dtype)
    kind = int(rng.integers(0, 3))
    if kind == 0:
        pol = dict(skip_frac=float(rng.choice([0.1, 0.5, 0.9])))
    elif kind == 1:
        pol = dict(skip_frac=float(rng.choice([0.0, 0.6])), sparse_frac_k=float(rng.choice([0.0, 0.5, 1.0])),
                   sparse_frac_v=float(rng.choice([0.3, 1.0])), dense_first_tiles=int(rng.integers(0, 3)),
                   dense_last_tiles=int(rng.integers(0, 5)))
    else:
        sk, sv = _mixed_states(B, Hkv, T, seed=7000 + seed, p_skip=float(rng.choice([0.2, 0.8])))
        pol = dict(state_k=sk, state_v=sv)
    q = Q[:, :, 0, :].copy()
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, dtype=dtype, **pol)
    Or, Lr = orc.attention_decode(q, pk, pv)
    for ns in (1, int(rng.integers(2, 9))):
        O, LSE = hb.decode_attn(sh, _dev(q, dtype), kv, n_splits=ns)
        torch.cuda.synchronize()
        what = f"seed {seed}: B{B} Hq{Hq} Hkv{Hkv} T{T} {dtype} splits {ns} {sorted(pol)}"
        assert_close(_f32(O), Or, "decode " + what)
        assert_lse_close(LSE.cpu().numpy(), Lr, "decode lse " + what)


def test_explicit_states_on_the_device_run_with_no_host_wait():
    """A pruner that leaves its block-level masks on the device (Sec. III-A: the compressor takes the
    masks M as an input): compress with those states, causal prefill and decode are issued back to
    back on one stream with no host synchronisation in between (the states are produced by device
    work queued just before), and match the oracle."""
    B, Hq, Hkv, T = 2, 8, 2, 13
    L = 64 * T
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=300, k_outliers=True)
    sk, sv = _mixed_states(B, Hkv, T, seed=301, p_skip=0.2)
    sh = hb.make_shape(B, Hq, Hkv, L)
    Kd, Vd, Qd = _dev(K), _dev(V), _dev(Q)
    qd = _dev(Q[:, :, -1, :].copy())
    kv = hb.PackedKV(sh, [0, T, T, T, T])
    kv.uniform = 0
    stream = torch.cuda.Stream()
    stage = torch.from_numpy(np.stack([sk, sv])).cuda()          # uploaded before the stream work starts
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        # the "pruner": device work that produces the states on the same stream
        sk_d = (stage[0] + 0).contiguous()
        sv_d = (stage[1] + 0).contiguous()
        pol = hb.make_policy(state_k=sk_d, state_v=sv_d)
        hb.compress_kv(sh, pol, Kd, Vd, out=kv)
        O, LSE = hb.prefill_attn(sh, Qd, kv)
        Od, LSEd = hb.decode_attn(sh, qd, kv, n_splits=3)
    stream.synchronize()
    hb.check_state_flag(pol)
    pk, pv, _ = orc.compress_kv(K, V, state_k=sk, state_v=sv)
    check_packed_bit_exact(sh, kv, pk, pv)
    rows = wl.sample_rows(B, Hq, L, 150, seed=302, extra=[(0, 0, 0), (B - 1, Hq - 1, L - 1)])
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True)
    idx = tuple(np.array(rows).T)
    assert_close(_f32(O)[idx], Or, "prefill after device-state compress")
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, "prefill after device-state compress lse")
    Odr, Ldr = orc.attention_decode(Q[:, :, -1, :].copy(), pk, pv)
    assert_close(_f32(Od), Odr, "decode after device-state compress")
    assert_lse_close(LSEd.cpu().numpy(), Ldr, "decode after device-state compress lse")


def test_explicit_states_into_pools_that_are_too_small():
    """Pools with fewer slots than the states ask for: the tiles that find no slot when their turn comes
    are left out of K and V, take no slot, and the flag goes up; the oracle walks the same counters."""
    B, Hq, Hkv, T = 2, 4, 2, 11
    L = 64 * T
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=310)
    sk, sv = _mixed_states(B, Hkv, T, seed=311, p_skip=0.1)
    caps = (2, 3, 3, 2)
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv = hb.PackedKV(sh, [0, *caps])
    kv.uniform = 0
    pol = hb.make_policy(state_k=sk, state_v=sv)
    hb.compress_kv(sh, pol, _dev(K), _dev(V), out=kv)
    torch.cuda.synchronize()
    with pytest.raises(hb.HsError, match="more slots"):
        hb.check_state_flag(pol)
    pk, pv, info = orc.compress_kv(K, V, state_k=sk, state_v=sv, caps=caps)
    assert info["dropped"]
    check_packed_bit_exact(sh, kv, pk, pv)
    q = Q[:, :, 0, :].copy()
    O, LSE = hb.decode_attn(sh, _dev(q), kv, n_splits=2)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, pk, pv)
    assert_close(_f32(O), Or, "decode over capacity-limited pools")


def test_recompress_into_small_pools_then_append():
    """Further pruning into pools that are too small, then an append: the dropped tiles took no slot, so
    the appended tile gets a slot that no live tile uses (slots stay 0 .. n-1 per pool)."""
    B, Hq, Hkv, T = 2, 4, 2, 10
    L = 64 * T
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=320)
    # source: keys dense, values mixed; the last two tiles not filled yet
    sk = np.full((B, Hkv, T), orc.DENSE, dtype=np.int8)
    _, sv = _mixed_states(B, Hkv, T, seed=321, p_skip=0.0)
    sk[:, :, 8:], sv[:, :, 8:] = 0, 0
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, state_k=sk, state_v=sv)
    tk = np.full((B, Hkv, T), orc.SPARSE24, dtype=np.int8)
    tv = np.full((B, Hkv, T), orc.SPARSE24, dtype=np.int8)
    caps = (0, 5, 0, 7)                                      # 5 key slots for 8 tiles
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    kv2 = hb.recompress_kv(sh, kv, hb.make_policy(state_k=tk, state_v=tv), counts=[0, *caps], overflow=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1
    rk, rv, dropped = orc.recompress_kv(pk, pv, tk, tv, caps=caps)
    assert dropped
    check_packed_bit_exact(sh, kv2, rk, rv)
    assert (np.abs(rv.map).max(axis=-1) == 5).all()          # V holds 5 tiles too: the dropped ones took no V slot
    # append tile 8 as dense K? no dense pool: 2:4 K is full -> stays skipped, flag; V-only room does not help
    flag.zero_()
    Kd, Vd = _dev(K), _dev(V)
    hb.append_tile(sh, kv2, 8, Kd[:, :, 512:576].contiguous(), Vd[:, :, 512:576].contiguous(), overflow=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1 and (kv2.k_map[:, :, 8].cpu().numpy() == 0).all()
    # with room for one more key tile the append takes slot 5 (the 6th) in K and in V
    kv3 = hb.recompress_kv(sh, kv, hb.make_policy(state_k=tk, state_v=tv), counts=[0, 0, 6, 0, 7])
    rk3, rv3, _ = orc.recompress_kv(pk, pv, tk, tv, caps=(0, 6, 0, 7))
    # drop two tiles by hand so that room appears: recompress again towards a target that skips tiles 0, 1
    tk2, tv2 = tk.copy(), tv.copy()
    tk2[:, :, :2], tv2[:, :, :2] = 0, 0
    kv4 = hb.recompress_kv(sh, kv3, hb.make_policy(state_k=tk2, state_v=tv2), counts=[0, 0, 6, 0, 7])
    rk4, rv4, _ = orc.recompress_kv(rk3, rv3, tk2, tv2, caps=(0, 6, 0, 7))
    hb.append_tile(sh, kv4, 8, Kd[:, :, 512:576].contiguous(), Vd[:, :, 512:576].contiguous(), overflow=flag)
    orc.append_tile(rk4, rv4, 8, K[:, :, 512:576], V[:, :, 512:576], orc.SPARSE24, orc.SPARSE24)
    torch.cuda.synchronize()
    check_packed_bit_exact(sh, kv4, rk4, rv4)
    live = rk4.map[0, 0][rk4.map[0, 0] != 0]
    assert sorted((-live).tolist()) == list(range(1, live.size + 1))       # every slot used once
    q = Q[:, :, 0, :].copy()
    O, LSE = hb.decode_attn(sh, _dev(q), kv4, n_splits=2)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, rk4, rv4)
    assert_close(_f32(O), Or, "decode after recompress into small pools + append")


# ------------------------------------------------------------------ fp16 (the paper's element type)
# fp16 output rounding alone is 8x finer than bf16's, so the same bars leave more room; the values checked
# are the same ones as for bf16.
@pytest.mark.parametrize("pol", [dict(), dict(sparse_frac_k=0.0, sparse_frac_v=0.0), dict(sparse_frac_k=0.0),
                                 dict(skip_frac=0.25, sparse_frac_k=0.5, sparse_frac_v=0.7)])
def test_fp16_all_stages(pol):
    B, Hq, Hkv, L = 2, 8, 2, 64 * 12
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=180, k_outliers=True, dtype="fp16")
    K[0, 0, 5, :8] = wl.f32_to_f16_bits(np.array([1, 1, -1, 1, 0, -0.0, 0, 0], dtype=np.float32))    # ties and zeros
    V[0, 1, 8:12, 7] = wl.f32_to_f16_bits(np.array([6e-8, -6e-8, 1e-7, 0], dtype=np.float32))        # subnormals
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, dtype="fp16", **pol)
    check_packed_bit_exact(sh, kv, pk, pv)
    O, LSE = hb.prefill_attn(sh, _dev(Q, "fp16"), kv)
    torch.cuda.synchronize()
    rows = wl.sample_rows(B, Hq, L, 160, seed=181, extra=[(0, 0, 0), (B - 1, Hq - 1, L - 1)])
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True)
    idx = tuple(np.array(rows).T)
    assert_close(_f32(O)[idx], Or, f"fp16 prefill {sorted(pol)}")
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, "fp16 prefill lse")
    assert np.abs(_f32(O)[idx] - Or).mean() / np.abs(Or).mean() < 4e-4        # one fp16 term of P is enough
    q = Q[:, :, -1, :].copy()
    for ns in (0, 5):
        Od, LSEd = hb.decode_attn(sh, _dev(q, "fp16"), kv, n_splits=ns)
        torch.cuda.synchronize()
        Odr, Ldr = orc.attention_decode(q, pk, pv)
        assert_close(_f32(Od), Odr, f"fp16 decode {sorted(pol)} splits {ns}")
        assert_lse_close(LSEd.cpu().numpy(), Ldr, "fp16 decode lse")
    Kt, Vt = K[:, :, :64].copy(), V[:, :, :64].copy()
    Od, LSEd = hb.decode_attn(sh, _dev(q, "fp16"), kv, tail_k=_dev(Kt, "fp16"), tail_v=_dev(Vt, "fp16"), tail_len=9)
    torch.cuda.synchronize()
    Odr, Ldr = orc.attention_decode(q, pk, pv, tail_k=Kt, tail_v=Vt, tail_len=9)
    assert_close(_f32(Od), Odr, "fp16 decode with tail")


def test_fp16_large_logits_and_long_flat_rows():
    """fp16 numerators: the reference has to be renewed before a numerator reaches 65504 (keys that grow
    along the sequence), and small numerators of a long, flat row must not be flushed away."""
    B, Hq, Hkv, L = 1, 4, 1, 64 * 24
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=190, dtype="fp16")
    Kf = wl.f16_bits_to_f32(K)
    ramp = np.linspace(0.05, 6.0, L, dtype=np.float32)[None, None, :, None]     # logits grow to the hundreds
    Kb = wl.f32_to_f16_bits(Kf * ramp)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, Kb, V, dtype="fp16")
    O, LSE = hb.prefill_attn(sh, _dev(Q, "fp16"), kv)
    Od, LSEd = hb.decode_attn(sh, _dev(Q[:, :, -1, :].copy(), "fp16"), kv)
    torch.cuda.synchronize()
    rows = [(0, h, i) for h in range(Hq) for i in range(0, L, 7)] + [(0, h, L - 1) for h in range(Hq)]
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True)
    idx = tuple(np.array(rows).T)
    assert_close(_f32(O)[idx], Or, "fp16 prefill growing logits")
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, "fp16 prefill growing logits lse")
    Odr, Ldr = orc.attention_decode(Q[:, :, -1, :].copy(), pk, pv)
    assert_close(_f32(Od), Odr, "fp16 decode growing logits")
    # flat row: one key far above 1500 equal ones; the many small numerators carry weight together
    Kz = np.zeros_like(K)
    Kz[0, 0, 100] = wl.f32_to_f16_bits(Q[0, 0, -1].view(np.float16).astype(np.float32) * 1.23)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, Kz, V, dtype="fp16", sparse_frac_k=0.0, sparse_frac_v=0.0)
    Od, LSEd = hb.decode_attn(sh, _dev(Q[:, :, -1, :].copy(), "fp16"), kv, n_splits=1)
    O, LSE = hb.prefill_attn(sh, _dev(Q, "fp16"), kv)
    torch.cuda.synchronize()
    Odr, Ldr = orc.attention_decode(Q[:, :, -1, :].copy(), pk, pv)
    assert_close(_f32(Od), Odr, "fp16 decode flat row")
    assert_lse_close(LSEd.cpu().numpy(), Ldr, "fp16 decode flat row lse")
    Or, Lr = orc.attention_rows(Q, pk, pv, [(0, 0, L - 1)], causal=True)
    assert_close(_f32(O)[0, 0, L - 1][None], Or, "fp16 prefill flat row")


# ------------------------------------------------------------------ edges and errors
@pytest.mark.parametrize("planted", ["tiny", "huge", "both"])
@pytest.mark.parametrize("pol", [dict(), dict(sparse_frac_k=0.0, sparse_frac_v=0.0), dict(sparse_frac_v=0.5),
                                 dict(skip_frac=0.25, sparse_frac_k=0.5, sparse_frac_v=0.7)])
def test_bf16_cache_with_both_v_tile_encodings(pol, planted):
    """V tiles of a bf16 cache whose stored values fp16 holds exactly carry the encoding bit and go
    through the fp16 matrix instructions; tiles with values under fp16's subnormal step or over its
    largest number stay bf16.  Both kinds in one row, in every kernel specialisation."""
    B, Hq, Hkv, L = 2, 8, 2, 64 * 14
    T = L // 64
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=190, k_outliers=True)
    Vf = wl.bf16_bits_to_f32(V)
    rng = np.random.default_rng(191)
    kind = rng.integers(0, 3, size=(B, Hkv, T))          # 0: as drawn, 1: tiny, 2: huge
    kind[0, 0, :] = 0                                       # one row with fp16 tiles only
    kind[1, 1, :] = 1 if planted != "huge" else 2           # one row with bf16 tiles only
    for b in range(B):
        for h in range(Hkv):
            for t in range(T):
                if kind[b, h, t] == 1 and planted in ("tiny", "both"):
                    Vf[b, h, 64 * t:64 * t + 64] *= 2.0 ** -20
                if kind[b, h, t] == 2 and planted in ("huge", "both"):
                    Vf[b, h, 64 * t:64 * t + 64] *= 2.0 ** 18
    V = wl.f32_to_bf16_bits(Vf)                             # exact: powers of two
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, **pol)
    flagged = pv.f16
    live = pv.map != 0
    assert (flagged & live).any() and (~flagged & live).any()
    check_packed_bit_exact(sh, kv, pk, pv)
    O, LSE = hb.prefill_attn(sh, _dev(Q), kv)
    torch.cuda.synchronize()
    rows = wl.sample_rows(B, Hq, L, 200, seed=192, extra=[(0, 0, 0), (B - 1, Hq - 1, L - 1)])
    Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True)
    idx = tuple(np.array(rows).T)
    got = _f32(O)[idx]
    if planted == "tiny":                                   # no huge tile hides the others' error
        assert_close(got, Or, f"prefill v encodings {sorted(pol)}")
    else:                                                   # per (b, h) row block: scales differ by 2^18
        for b in range(B):
            for h in range(Hq):
                sel = (idx[0] == b) & (idx[1] == h)
                if sel.any():
                    assert_close(got[sel], Or[sel], f"prefill v encodings {planted} b{b} h{h}")
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, "prefill v encodings lse")
    q = Q[:, :, -1, :].copy()
    Odr, Ldr = orc.attention_decode(q, pk, pv)
    for ns in (0, 3):
        Od, LSEd = hb.decode_attn(sh, _dev(q), kv, n_splits=ns)
        torch.cuda.synchronize()
        for b in range(B):
            for hk in range(Hkv):
                g = slice(hk * (Hq // Hkv), (hk + 1) * (Hq // Hkv))
                assert_close(_f32(Od)[b, g], Odr[b, g], f"decode v encodings {planted} splits {ns} b{b} hkv{hk}")
        assert_lse_close(LSEd.cpu().numpy(), Ldr, "decode v encodings lse")


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_recompress_explicit_states_bit_exact_and_attention(dtype):
    """Further pruning of a packed cache (dense -> 2:4, anything -> dropped, the rest carried over) against
    the oracle, bit for bit, then attention over the result."""
    B, Hq, Hkv, L = 2, 8, 2, 64 * 19
    T = L // 64
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=210, k_outliers=True, dtype=dtype)
    if dtype == "bf16":
        Vf = wl.bf16_bits_to_f32(V)
        Vf[:, :, 64 * 2:64 * 3:4] = 2.0 ** -40          # dense form not exact in fp16, 2:4 form exact
        Vf[:, :, 64 * 3:64 * 4] *= 2.0 ** -22           # never exact
        V = wl.f32_to_bf16_bits(Vf)
    sk, sv = _mixed_states(B, Hkv, T, seed=211, p_skip=0.15)
    sk[:, :, 2:4], sv[:, :, 2:4] = 1, 1
    tk, tv = _mixed_states(B, Hkv, T, seed=212, p_skip=0.15)
    tk[:, :, 2:4], tv[:, :, 2:4] = 2, 2
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, dtype=dtype, state_k=sk, state_v=sv)
    kv2 = hb.recompress_kv(sh, kv, hb.make_policy(state_k=tk, state_v=tv))
    torch.cuda.synchronize()
    rk, rv = orc.recompress_kv(pk, pv, tk, tv)
    check_packed_bit_exact(sh, kv2, rk, rv)
    check_packed_bit_exact(sh, kv, pk, pv)                  # the source is untouched
    O, LSE = hb.prefill_attn(sh, _dev(Q, dtype), kv2)
    torch.cuda.synchronize()
    rows = wl.sample_rows(B, Hq, L, 120, seed=213, extra=[(B - 1, Hq - 1, L - 1)])
    Or, Lr = orc.attention_rows(Q, rk, rv, rows, causal=True)
    idx = tuple(np.array(rows).T)
    assert_close(_f32(O)[idx], Or, f"prefill after recompress {dtype}")
    assert_lse_close(LSE.cpu().numpy()[idx], Lr, "prefill after recompress lse")
    q = Q[:, :, -1, :].copy()
    Od, LSEd = hb.decode_attn(sh, _dev(q, dtype), kv2, n_splits=3)
    torch.cuda.synchronize()
    Odr, Ldr = orc.attention_decode(q, rk, rv)
    assert_close(_f32(Od), Odr, f"decode after recompress {dtype}")
    assert_lse_close(LSEd.cpu().numpy(), Ldr, "decode after recompress lse")


@pytest.mark.parametrize("first,last", [(0, 0), (1, 3)])
def test_recompress_prefill_policy_to_decode_policy(first, last):
    """The paper's differentiated setting: prefill with keys dense and values 2:4, then every key tile
    pruned for decode (optionally sink / local-window tiles kept dense).  Equals compressing the
    original tensors with the decode policy, on the GPU and in the oracle."""
    B, Hq, Hkv, L = 1, 8, 2, 64 * 16
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=220, k_outliers=True)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, sparse_frac_k=0.0, sparse_frac_v=1.0)
    assert kv.uniform == 1
    tgt = dict(sparse_frac_k=1.0, sparse_frac_v=1.0, dense_first_tiles=first, dense_last_tiles=last)
    kv2 = hb.recompress_kv(sh, kv, hb.make_policy(**tgt))
    torch.cuda.synchronize()
    assert kv2.uniform == (1 if first + last == 0 else 0)
    sh2, kv_direct, ck, cv, info = compress_both(B, Hq, Hkv, L, K, V, **tgt)
    rk, rv = orc.recompress_kv(pk, pv, info["state_k"], info["state_v"])
    check_packed_bit_exact(sh, kv2, rk, rv)
    # V was 2:4 everywhere already: its protected tiles cannot go back to dense; K equals the direct result
    assert (rv.map < 0).all() and (rk.map == ck.map).all()
    Ku, _ = hb.unpack_kv(sh, kv2)
    Kd, _ = hb.unpack_kv(sh, kv_direct)
    torch.cuda.synchronize()
    assert torch.equal(Ku.view(torch.int16), Kd.view(torch.int16))
    q = Q[:, :, 0, :].copy()
    Od, LSEd = hb.decode_attn(sh, _dev(q), kv2)
    torch.cuda.synchronize()
    Odr, Ldr = orc.attention_decode(q, rk, rv)
    assert_close(_f32(Od), Odr, "decode after recompress to S_K=1")
    assert_lse_close(LSEd.cpu().numpy(), Ldr, "decode after recompress lse")


def test_recompress_ranked_targets_from_kept_tile_scores():
    """Decode-phase policy with fractions (skip the quietest quarter, half of the key tiles 2:4 by lowest
    pruning loss, sink and local-window tiles dense) applied to a prefill cache (keys dense, values 2:4): the
    ranking uses the tile scores taken from the original tensors (hs_score_tiles), which equal the oracle's,
    and the result equals the oracle's further pruning towards the states that policy gives the originals."""
    B, Hq, Hkv, T = 2, 8, 2, 24
    L = 64 * T
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=330, k_outliers=True)
    K[0, 0, 64 * 9:64 * 10] = K[0, 0, 64 * 3:64 * 4]           # an exact tie in energy and in loss
    V[0, 0, 64 * 9:64 * 10] = V[0, 0, 64 * 3:64 * 4]
    Kd, Vd = _dev(K), _dev(V)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, sparse_frac_k=0.0, sparse_frac_v=1.0)
    scores = hb.score_tiles(sh, Kd, Vd)
    tgt = dict(skip_frac=0.25, sparse_frac_k=0.5, sparse_frac_v=1.0, dense_first_tiles=1, dense_last_tiles=2)
    _, _, info = orc.compress_kv(K, V, **tgt)                    # states the policy gives the original tensors
    torch.cuda.synchronize()
    sc = scores.cpu().numpy()
    for plane, key in enumerate(("energy", "loss_k", "loss_v")):
        assert np.allclose(sc[plane], info[key], rtol=1e-12, atol=0.0), key
        srt = np.sort(info[key], axis=-1)
        gaps = np.diff(srt, axis=-1) / srt[..., 1:]
        assert ((gaps > 1e-12) | (gaps == 0)).all()              # no cut on a rounding-level near-tie
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    kv2 = hb.recompress_kv(sh, kv, hb.make_policy(tile_scores=scores, **tgt), overflow=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0 and kv2.uniform == 0
    rk, rv = orc.recompress_kv(pk, pv, info["state_k"], info["state_v"])
    check_packed_bit_exact(sh, kv2, rk, rv)
    assert int((rk.map == 0).sum()) == B * Hkv * 5 and (rv.map[:, :, 0] < 0).all()      # V was 2:4 already: stays
    q = Q[:, :, 0, :].copy()
    O, LSE = hb.decode_attn(sh, _dev(q), kv2, n_splits=3)
    torch.cuda.synchronize()
    Or, Lr = orc.attention_decode(q, rk, rv)
    assert_close(_f32(O), Or, "decode after ranked recompress")
    assert_lse_close(LSE.cpu().numpy(), Lr, "decode after ranked recompress lse")


def test_recompress_capacity_overflow_and_argument_errors():
    B, Hq, Hkv, L = 1, 4, 1, 64 * 8
    T = L // 64
    _, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=230)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V, sparse_frac_k=0.0, sparse_frac_v=0.0)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    # room for 5 of the 8 key tiles: the first 5 tiles survive, the rest is left out of K and V alike
    kv2 = hb.recompress_kv(sh, kv, hb.make_policy(), counts=[0, 0, 5, 0, T], overflow=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1
    assert kv2.k_map.cpu().numpy().reshape(-1).tolist() == [-1, -2, -3, -4, -5, 0, 0, 0]
    vm = kv2.v_map.cpu().numpy().reshape(-1)
    assert ((np.abs(vm) & ~hb.MAP_F16) == [1, 2, 3, 4, 5, 0, 0, 0]).all() and (vm <= 0).all()
    flag.zero_()
    hb.recompress_kv(sh, kv, hb.make_policy(), overflow=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    with pytest.raises(hb.HsError):                         # a ranked target needs the tile scores
        hb.recompress_kv(sh, kv, hb.make_policy(sparse_frac_k=0.5))
    with pytest.raises(hb.HsError):
        hb.recompress_kv(sh, kv, hb.make_policy(skip_frac=0.25))
    import ctypes as C
    a = kv.struct()
    ws = torch.empty(hb.workspace_bytes(sh, 3), dtype=torch.uint8, device="cuda")
    pol = hb.make_policy()
    assert hb.lib().hs_recompress_kv(C.byref(sh), C.byref(pol), C.byref(a), C.byref(a), ws.data_ptr(), None, None) == -1


def test_single_tile_and_odd_batch_shapes():
    """L = 64 (one tile, one split), B = 3, 3 KV heads: smallest grid dimensions on every kernel."""
    for (B, Hq, Hkv, L) in ((1, 1, 1, 64), (3, 6, 3, 64 * 3), (2, 16, 2, 64 * 2)):
        Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=130 + B)
        sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, K, V)
        check_packed_bit_exact(sh, kv, pk, pv)
        O, LSE = hb.prefill_attn(sh, _dev(Q), kv)
        q = Q[:, :, -1, :].copy()
        Od, LSEd = hb.decode_attn(sh, _dev(q), kv)
        torch.cuda.synchronize()
        rows = [(b, h, i) for b in range(B) for h in range(Hq) for i in range(L)]
        Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True)
        assert_close(_f32(O).reshape(-1, 128), Or, f"prefill B{B} Hq{Hq} Hkv{Hkv} L{L}")
        Odr, Ldr = orc.attention_decode(q, pk, pv)
        assert_close(_f32(Od), Odr, f"decode B{B} Hq{Hq} Hkv{Hkv} L{L}")
        assert_lse_close(LSEd.cpu().numpy(), Ldr, "decode lse")


def test_scale_argument_and_large_logits():
    """Explicit softmax scale, and keys scaled so that logits reach the hundreds (the lazily
    updated softmax reference must follow without overflow)."""
    B, Hq, Hkv, L = 1, 4, 1, 64 * 6
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=140)
    Kbig = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(K) * 24.0)
    # a late tile with much larger keys: the reference has to jump upwards mid-sequence
    Kbig[:, :, 64 * 4:64 * 5] = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(K[:, :, 64 * 4:64 * 5]) * 96.0)
    sh, kv, pk, pv, _ = compress_both(B, Hq, Hkv, L, Kbig, V)
    for scale in (0.0, 0.25):
        O, LSE = hb.prefill_attn(sh, _dev(Q), kv, scale=scale)
        Od, LSEd = hb.decode_attn(sh, _dev(Q[:, :, -1, :].copy()), kv, scale=scale)
        torch.cuda.synchronize()
        rows = [(0, h, i) for h in range(Hq) for i in range(L)]
        Or, Lr = orc.attention_rows(Q, pk, pv, rows, causal=True, scale=None if scale == 0.0 else scale)
        assert_close(_f32(O).reshape(-1, 128), Or, f"prefill large logits scale={scale}")
        assert_lse_close(LSE.cpu().numpy().reshape(-1), Lr, f"prefill large logits lse scale={scale}")
        Odr, Ldr = orc.attention_decode(Q[:, :, -1, :].copy(), pk, pv, scale=None if scale == 0.0 else scale)
        assert_close(_f32(Od), Odr, f"decode large logits scale={scale}")


def test_matrix_rate_probe_runs_and_counts_its_work():
    """The benchmark's register-resident matrix-instruction loop: runs, reports the flops of the launch
    (2 workgroups per compute unit x 4 waves x 8 instructions x iterations x 2*16*16*K) and the clocks spent."""
    import ctypes as C
    sink = torch.zeros(4, dtype=torch.int64, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for kind, k in ((0, 32), (1, 64)):
        flop = hb.probe_mfma_rate(kind, 500, sink)
        torch.cuda.synchronize()
        assert flop == 2 * cus * 4 * 8 * 500 * 2 * 16 * 16 * k
        clocks, ticks, _, never = sink.cpu().tolist()
        assert clocks > 500 * 8 * 8 and ticks > 0 and never == 0     # >= 8 clocks per matrix instruction
    f = C.c_double(0.0)
    assert hb.lib().hs_probe_mfma_rate(2, 10, sink.data_ptr(), C.byref(f), None) == -1
    assert hb.lib().hs_probe_mfma_rate(0, 0, sink.data_ptr(), C.byref(f), None) == -1


def test_stream_read_probe_runs():
    """The benchmark's load-only kernel (the decode kernel's access pattern): runs over a buffer of pool-shaped
    regions, with and without its epilogue, and rejects shapes it cannot split evenly."""
    n_tiles, n_wg = 512, 32
    buf = torch.ones(n_tiles * 18432, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16 + 512 * n_wg, dtype=torch.float32, device="cuda")
    hb.probe_stream_read(buf, n_tiles, n_wg, True, sink)
    torch.cuda.synchronize()
    # every byte is 1: each lane's xor over 4 x 18 tiles' words ends up 0 -> the combined partials are 0
    assert float(sink[16:].abs().max().item()) == 0.0
    hb.probe_stream_read(buf, n_tiles, n_wg, False, sink)
    torch.cuda.synchronize()
    with pytest.raises(hb.HsError):
        hb.probe_stream_read(buf, n_tiles, 24, True, sink)            # 512 tiles do not split over 24 workgroups of 4 waves


def test_argument_errors_on_device_calls():
    B, Hq, Hkv, L = 1, 4, 1, 256
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, L, seed=150)
    sh = hb.make_shape(B, Hq, Hkv, L)
    Kd, Vd = _dev(K), _dev(V)
    # pools sized for an all-2:4 policy cannot take a policy that needs dense tiles
    kv = hb.PackedKV(sh, hb.tile_counts(sh, hb.make_policy()))
    with pytest.raises(hb.HsError):
        hb.compress_kv(sh, hb.make_policy(sparse_frac_k=0.5), Kd, Vd, out=kv)
    # explicit states: a tile skipped in K only is inconsistent.  Host arrays are checked by the binding;
    # states that are already on the device are checked by the kernel that turns them into maps: the tile
    # is stored as SKIP and bit 1 of the policy's flag goes up
    sk = np.array([[[2, 0, 2, 2]]], dtype=np.int8)
    sv = np.array([[[2, 2, 2, 7]]], dtype=np.int8)
    with pytest.raises(hb.HsError):
        hb.make_policy(state_k=sk, state_v=sv)
    pol_dev = hb.make_policy(state_k=torch.from_numpy(sk).cuda(), state_v=torch.from_numpy(sv).cuda())
    kv.uniform = 0
    hb.compress_kv(sh, pol_dev, Kd, Vd, out=kv)
    torch.cuda.synchronize()
    assert kv.k_map.cpu().numpy().reshape(-1).tolist() == [-1, 0, -2, 0]
    assert (np.abs(kv.v_map.cpu().numpy().reshape(-1)) & ~hb.MAP_F16).tolist() == [1, 0, 2, 0]
    with pytest.raises(hb.HsError, match="not valid"):
        hb.check_state_flag(pol_dev)
    kv = hb.compress_kv(sh, hb.make_policy(), Kd, Vd)
    # Lq not a multiple of the tile, Lq > L
    import ctypes as C
    kvs = kv.struct()
    Qd = _dev(Q)
    O = torch.empty_like(Qd)
    assert hb.lib().hs_prefill_attn(C.byref(sh), 100, 0.0, 1, hb._ptr(Qd), C.byref(kvs), hb._ptr(O), None, None, None) == -2
    assert hb.lib().hs_prefill_attn(C.byref(sh), 512, 0.0, 1, hb._ptr(Qd), C.byref(kvs), hb._ptr(O), None, None, None) == -1
    # a pool of more than 4 GiB per (batch, kv head) row: prefill addresses tiles with 32-bit offsets
    kvs.cap_sparse_v = (1 << 32) // 8192 + 1
    assert hb.lib().hs_prefill_attn(C.byref(sh), 256, 0.0, 1, hb._ptr(Qd), C.byref(kvs), hb._ptr(O), None, None, None) == -2
    kvs = kv.struct()
    # a uniform promise that the capacities contradict
    kvs.cap_sparse_k = 2
    assert hb.lib().hs_decode_attn(C.byref(sh), 0.0, 0, hb._ptr(Qd), C.byref(kvs), hb._ptr(O), None, hb._ptr(O), None) == -1
    torch.cuda.synchronize()
