"""Pins for the CPU oracle against things other than itself: exhaustive
invariants, closed forms the paper prints (Sec. III-D), an independent library
attention routine, exact rational arithmetic and brute force in Python floats."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import hs_oracle as orc
from paper_2604_16864_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _bits(vals):
    return wl.f32_to_bf16_bits(np.asarray(vals, dtype=np.float32))


# ---------------------------------------------------------------- element mask
def test_top2_exhaustive_small_alphabet():
    """Every 4-tuple over an alphabet with ties, signed zeros and sign flips:
    exactly two kept; no dropped magnitude exceeds a kept one; among equal
    magnitudes the kept ones are the leftmost (Eq. 2a-b with a strict count)."""
    alphabet = _bits([0.0, -0.0, 0.5, -0.5, 1.0, -2.0, 3.0])
    groups = np.array(list(itertools.product(alphabet, repeat=4)), dtype=np.uint16)
    keep = orc._top2_of_4(groups)
    mag = np.abs(wl.bf16_bits_to_f32(groups))
    assert (keep.sum(axis=-1) == 2).all()
    for g in range(groups.shape[0]):
        k = keep[g]
        kept_min = mag[g][k].min()
        assert mag[g][~k].max() <= kept_min
        # ties at the boundary: every dropped element equal to the smallest kept
        # magnitude sits to the right of every kept element of that magnitude
        tied_drop = [i for i in range(4) if not k[i] and mag[g][i] == kept_min]
        tied_keep = [i for i in range(4) if k[i] and mag[g][i] == kept_min]
        if tied_drop:
            assert max(tied_keep) < min(tied_drop)


def test_top2_all_bit_patterns_pairs():
    """Magnitude order equals integer order of bits & 0x7fff for every finite bf16:
    check the mask on groups built from random finite patterns against float abs."""
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 1 << 16, size=(200000, 4), dtype=np.uint32).astype(np.uint16)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    bits = bits[finite.all(axis=-1)]
    keep = orc._top2_of_4(bits)
    mag = np.abs(wl.bf16_bits_to_f32(bits).astype(np.float64))
    assert (keep.sum(-1) == 2).all()
    kept_min = np.where(keep, mag, np.inf).min(-1)
    drop_max = np.where(~keep, mag, -np.inf).max(-1)
    assert (drop_max <= kept_min).all()


def test_mask_axes():
    """K groups run along channels, V groups along tokens (Table II, Trans-Both)."""
    K = _bits(np.arange(1, 1 + 8 * 8, dtype=np.float32).reshape(1, 1, 8, 8))
    mk = orc.element_mask_k(K)
    mv = orc.element_mask_v(K)
    # increasing values: the last two of each group survive
    assert (mk.reshape(8, 2, 4) == np.array([False, False, True, True])).all()
    assert (mv.reshape(2, 4, 8).transpose(0, 2, 1) == np.array([False, False, True, True])).all()


# ---------------------------------------------------------------- pack / unpack
def _rand_kv(seed, B=2, H=2, L=32, D=16):
    rng = np.random.default_rng(seed)
    K = wl.normal_bf16(rng, (B, H, L, D))
    V = wl.normal_bf16(rng, (B, H, L, D))
    return K, V


def test_roundtrip_bit_exact_and_nibbles():
    K, V = _rand_kv(1, L=64, D=32)
    # plant ties, zeros and negative zeros
    K[0, 0, 3, :8] = _bits([1, 1, 1, 1, 0, -0.0, 0, 0])
    V[0, 1, 4:8, 5] = _bits([-2, 2, 2, -2])
    pk, pv, info = orc.compress_kv(K, V, Bt=16)
    assert (orc.unpack_tensor(pk) == np.where(info["mask_k"], K, 0)).all()
    assert (orc.unpack_tensor(pv) == np.where(info["mask_v"], V, 0)).all()
    legal = {0x4, 0x8, 0xC, 0x9, 0xD, 0xE}
    for p in (pk, pv):
        nib = orc._words_to_nibbles(p.meta)
        assert set(np.unique(nib).tolist()) <= legal
    # ties keep the leftmost two, all-zero groups keep positions 0, 1
    assert (info["mask_k"][0, 0, 3, :8] == [True, True, False, False, True, True, False, False]).all()
    # the sign bit of a kept negative zero survives the round trip
    assert orc.unpack_tensor(pk)[0, 0, 3, 5] == 0x8000


def test_mixed_states_roundtrip_and_map():
    K, V = _rand_kv(2, B=1, H=2, L=16 * 9, D=16)
    S, Dn, Sp = orc.SKIP, orc.DENSE, orc.SPARSE24
    sk = np.array([[[Dn, Sp, S, Sp, Dn, Dn, S, Sp, Sp], [Sp, Sp, Sp, S, S, Dn, Dn, Dn, Sp]]], dtype=np.int8)
    sv = np.array([[[Sp, Sp, S, Dn, Dn, Sp, S, Dn, Sp], [Dn, Sp, Dn, S, S, Sp, Dn, Sp, Dn]]], dtype=np.int8)
    pk, pv, info = orc.compress_kv(K, V, Bt=16, state_k=sk, state_v=sv)
    for p, st, X, m in ((pk, sk, K, info["mask_k"]), (pv, sv, V, info["mask_v"])):
        for h in range(2):
            mp = p.map[0, h]
            assert ((mp == 0) == (st[0, h] == S)).all()
            # the paper's signed index map and nothing else: 1-based slots per pool in sequence order
            assert (mp[st[0, h] == Dn] == np.arange(1, 1 + (st[0, h] == Dn).sum())).all()
            assert (mp[st[0, h] == Sp] == -np.arange(1, 1 + (st[0, h] == Sp).sum())).all()
            assert p.kind == "v" or not p.f16.any()
        tile_state = np.repeat(st, 16, axis=-1)[..., None]
        want = np.where(tile_state == Dn, X, np.where(tile_state == Sp, np.where(m, X, 0), 0))
        assert (orc.unpack_tensor(p) == want).all()


# ---------------------------------------------------------------- byte accounting
def _golden_ratios():
    rows, fr = [], {}
    for line in open(os.path.join(GOLD, "paper_sec3d_ratios.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        if len(f) == 5:
            rows.append(tuple(float(x) for x in f))
        else:
            fr[f[0]] = float(f[1])
    return rows, fr


def test_sizes_match_paper_sec3d():
    rows, fr = _golden_ratios()
    K, V = _rand_kv(3, B=1, H=1, L=64 * 4, D=128)
    pk, pv, _ = orc.compress_kv(K, V, Bt=64)           # all tiles 2:4
    dense_bytes = K.nbytes
    assert pk.nnz.nbytes == fr["nnz"] * dense_bytes
    assert pk.meta.nbytes == fr["meta"] * dense_bytes
    assert pv.nnz.nbytes == fr["nnz"] * dense_bytes
    assert pv.meta.nbytes == fr["meta"] * dense_bytes
    assert pk.nnz[0, 0, 0].nbytes + pk.meta[0, 0, 0].nbytes == 9216
    for S_K, S_V, r, sp, sd in rows:
        assert round(orc.compression_ratio(S_K, S_V), 2) == r
        assert round(orc.ideal_prefill_speedup(S_K, S_V), 2) == sp
        assert round(orc.ideal_decode_speedup(S_K, S_V), 2) == sd
    # measured bytes equal the model with the index term (Sec. V-B: achieves theory exactly);
    # the map here is int32 per tile per tensor = 2 elements, the paper counts one
    T = 4
    total = pk.nbytes() + pv.nbytes()
    assert total == 2 * T * 9216 + 2 * T * 4
    model = 1.0 / (1.0 - 0.21875 * 2 + 2.0 / (64 * 128))
    assert abs((2 * dense_bytes) / total - model) < 1e-12
    # half the tiles sparse in K, all in V
    sk = np.array([[[1, 2, 1, 2]]], dtype=np.int8)
    sv = np.full((1, 1, 4), 2, dtype=np.int8)
    pk, pv, _ = orc.compress_kv(K, V, Bt=64, state_k=sk, state_v=sv)
    r = (2 * dense_bytes) / (pk.nbytes() + pv.nbytes() - 2 * T * 4)
    assert round(r, 2) == 1.49


# ---------------------------------------------------------------- tile selection
def test_skip_selection_exact_rational():
    """The skipped set is the n lowest-energy tiles, checked in exact arithmetic."""
    K, V = _rand_kv(4, B=1, H=2, L=16 * 12, D=16)
    # two tiles with identical content -> identical energy -> tie goes to the lower index
    K[0, 0, 16 * 7:16 * 8] = K[0, 0, 16 * 2:16 * 3]
    V[0, 0, 16 * 7:16 * 8] = V[0, 0, 16 * 2:16 * 3]
    for frac in (0.0, 0.25, 0.5, 0.75):
        pk, pv, info = orc.compress_kv(K, V, Bt=16, skip_frac=frac)
        n = int(math.floor(frac * 12))
        for h in range(2):
            e = []
            for t in range(12):
                acc = Fraction(0)
                for X in (K, V):
                    for x in wl.bf16_bits_to_f32(X[0, h, 16 * t:16 * (t + 1)]).ravel():
                        acc += Fraction(float(x)) ** 2
                e.append(acc)
            order = sorted(range(12), key=lambda t: (e[t], t))
            assert set(np.nonzero(pk.map[0, h] == 0)[0].tolist()) == set(order[:n])
            assert ((pk.map[0, h] == 0) == (pv.map[0, h] == 0)).all()
    # force the tie to straddle the cut: make tiles 2 and 7 the lowest-energy ones
    K[0, 0, 16 * 2:16 * 3] = 0
    K[0, 0, 16 * 7:16 * 8] = 0
    V[0, 0, 16 * 2:16 * 3] = 0
    V[0, 0, 16 * 7:16 * 8] = 0
    pk, _, _ = orc.compress_kv(K, V, Bt=16, skip_frac=1 / 12 + 1e-9)
    assert np.nonzero(pk.map[0, 0] == 0)[0].tolist() == [2]


def test_block_sparsity_by_pruning_loss_exact():
    """Eq. 2c-d: the S fraction of kept blocks with the lowest L1 pruning loss go sparse."""
    K, V = _rand_kv(6, B=1, H=1, L=16 * 8, D=16)
    pk, pv, info = orc.compress_kv(K, V, Bt=16, skip_frac=0.25, sparse_frac_k=0.5, sparse_frac_v=1.0)
    kept = np.nonzero(pk.map[0, 0] != 0)[0].tolist()
    assert len(kept) == 6
    loss = {}
    for t in kept:
        tile = wl.bf16_bits_to_f32(K[0, 0, 16 * t:16 * (t + 1)]).reshape(16, 4, 4)
        acc = Fraction(0)
        for row in tile.reshape(-1, 4):
            a = sorted((abs(float(x)) for x in row))
            acc += Fraction(a[0]) + Fraction(a[1])      # the two smallest magnitudes are removed
        loss[t] = acc
    want_sparse = set(sorted(kept, key=lambda t: (loss[t], t))[:3])
    assert set(np.nonzero(pk.map[0, 0] < 0)[0].tolist()) == want_sparse
    assert (pv.map[0, 0][kept] < 0).all()


def test_protected_end_tiles_stay_dense_and_outside_the_ranking():
    """Sink and local-window tiles (Sec. V-A): dense whatever their scores, and the fractions
    count over the tiles in between; the ranking of those is checked in exact arithmetic."""
    K, V = _rand_kv(8, B=1, H=2, L=16 * 12, D=16)
    # the protected tiles would otherwise be the first to be skipped: all zero
    for X in (K, V):
        X[0, :, :16 * 2] = 0
        X[0, :, 16 * 9:] = 0
    pk, pv, _ = orc.compress_kv(K, V, Bt=16, skip_frac=0.5, sparse_frac_k=1.0, sparse_frac_v=0.5,
                                dense_first_tiles=2, dense_last_tiles=3)
    for h in range(2):
        assert (pk.map[0, h, :2] > 0).all() and (pk.map[0, h, 9:] > 0).all()
        assert (pv.map[0, h, :2] > 0).all() and (pv.map[0, h, 9:] > 0).all()
        mid = list(range(2, 9))
        e, lv = {}, {}
        for t in mid:
            e[t] = sum(Fraction(float(x)) ** 2 for X in (K, V)
                       for x in wl.bf16_bits_to_f32(X[0, h, 16 * t:16 * (t + 1)]).ravel())
            tile = wl.bf16_bits_to_f32(V[0, h, 16 * t:16 * (t + 1)])        # [token, channel]
            acc = Fraction(0)
            for g in range(4):
                for c in range(16):
                    a = sorted(abs(float(x)) for x in tile[4 * g:4 * g + 4, c])
                    acc += Fraction(a[0]) + Fraction(a[1])
            lv[t] = acc
        skipped = set(sorted(mid, key=lambda t: (e[t], t))[:3])               # floor(0.5 * 7)
        assert set(np.nonzero(pk.map[0, h] == 0)[0].tolist()) == skipped
        kept = [t for t in mid if t not in skipped]
        assert (pk.map[0, h][kept] < 0).all()                                 # S_K = 1 over the 4 kept
        v_sparse = set(sorted(kept, key=lambda t: (lv[t], t))[:2])            # floor(0.5 * 4)
        assert set(np.nonzero(pv.map[0, h] < 0)[0].tolist()) == v_sparse
    # protection wider than the sequence: everything dense, nothing to rank
    pk, pv, _ = orc.compress_kv(K, V, Bt=16, skip_frac=0.5, dense_first_tiles=7, dense_last_tiles=9)
    assert (pk.map > 0).all() and (pv.map > 0).all()
    assert (orc.unpack_tensor(pk) == K).all() and (orc.unpack_tensor(pv) == V).all()


def test_nonzero_rule_keeps_a_given_element_mask():
    """Generic compressor of Sec. IV-B: input that already carries some 2:4 element mask (not the
    magnitude one) packs and unpacks to itself bit for bit; the magnitude rule would not."""
    rng = np.random.default_rng(9)
    K, V = _rand_kv(9, B=1, H=2, L=32, D=16)
    K[K == 0] = 0x3F80
    V[V == 0] = 0x3F80
    # random 2-of-4 masks along channels (K) and tokens (V), unrelated to magnitudes
    pairs = np.array([m for m in itertools.product([0, 1], repeat=4) if sum(m) == 2], dtype=bool)
    mk = pairs[rng.integers(0, 6, size=(1, 2, 32, 4))].reshape(1, 2, 32, 16)
    mv = pairs[rng.integers(0, 6, size=(1, 2, 8, 16))]                        # [.., group, channel, 4]
    mv = mv.transpose(0, 1, 2, 4, 3).reshape(1, 2, 32, 16)
    Km, Vm = np.where(mk, K, 0).astype(np.uint16), np.where(mv, V, 0).astype(np.uint16)
    # a group with a single survivor and an all-zero group, and a negative zero as "pruned"
    Km[0, 0, 3, 0:4] = [0, 0x4000, 0, 0]
    Km[0, 0, 3, 4:8] = 0
    Km[0, 0, 4, 0:4] = [0x8000, 0x4000, 0x3F80, 0]
    pk, pv, info = orc.compress_kv(Km, Vm, Bt=16, element_rule="nonzero")
    Ku, Vu = orc.unpack_tensor(pk), orc.unpack_tensor(pv)
    Kw = Km.copy()
    Kw[0, 0, 4, 0] = 0x8000 if info["mask_k"][0, 0, 4, 0] else 0              # -0 dropped -> stored as +0
    assert not info["mask_k"][0, 0, 4, 0]
    assert (Ku == Kw).all() and (Vu == Vm).all()
    assert (info["mask_k"] | ~mk)[0, 1].all() and (info["mask_v"] | ~mv).all()  # given survivors all kept
    assert info["mask_k"].reshape(-1, 4).sum(-1).tolist() == [2] * (info["mask_k"].size // 4)
    # single survivor: filled up with the leftmost zero; empty group: positions 0 and 1
    assert info["mask_k"][0, 0, 3, 0:8].tolist() == [True, True, False, False, True, True, False, False]
    # the magnitude rule on the unmasked data does not reproduce the given mask
    pk2, _, info2 = orc.compress_kv(K, V, Bt=16)
    assert (info2["mask_k"] != mk).any()


# ---------------------------------------------------------------- attention
def _sdpa(Qf, Kf, Vf, mask=None, causal=False):
    """Independent library routine: torch CPU scaled_dot_product_attention in fp64."""
    q = torch.from_numpy(Qf).double()
    k = torch.from_numpy(Kf).double()
    v = torch.from_numpy(Vf).double()
    G = q.shape[1] // k.shape[1]
    k = k.repeat_interleave(G, dim=1)
    v = v.repeat_interleave(G, dim=1)
    m = None if mask is None else torch.from_numpy(mask)
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=m, is_causal=causal and m is None).numpy()


def _f(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


@pytest.mark.parametrize("G", [1, 4])
def test_attention_all_dense_equals_library_sdpa(G):
    B, Hkv, L, D, Bt = 2, 2, 64, 32, 16
    Q, K, V = wl.make_qkv(B, Hkv * G, Hkv, L, D, L, seed=11)
    st = np.full((B, Hkv, L // Bt), orc.DENSE, dtype=np.int8)
    pk, pv, _ = orc.compress_kv(K, V, Bt=Bt, state_k=st, state_v=st)
    rows = [(b, h, i) for b in range(B) for h in range(Hkv * G) for i in range(L)]
    O, LSE = orc.attention_rows(Q, pk, pv, rows, causal=True)
    ref = _sdpa(_f(Q), _f(K), _f(V), causal=True)
    assert np.allclose(O.reshape(B, Hkv * G, L, D), ref, rtol=1e-10, atol=1e-12)
    O2, _ = orc.attention_rows(Q, pk, pv, rows, causal=False)
    ref2 = _sdpa(_f(Q), _f(K), _f(V), causal=False)
    assert np.allclose(O2.reshape(B, Hkv * G, L, D), ref2, rtol=1e-10, atol=1e-12)
    # LSE against a direct logsumexp of the score matrix
    s = np.einsum("bhid,bhjd->bhij", _f(Q), np.repeat(_f(K), G, axis=1)) / math.sqrt(D)
    lse_ref = torch.logsumexp(torch.from_numpy(s), dim=-1).numpy()
    _, LSE2 = orc.attention_rows(Q, pk, pv, rows, causal=False)
    assert np.allclose(LSE2.reshape(B, Hkv * G, L), lse_ref, rtol=1e-12)


def test_attention_sparse24_equals_sdpa_on_masked_kv():
    B, Hkv, G, L, D, Bt = 1, 2, 4, 64, 32, 16
    Q, K, V = wl.make_qkv(B, Hkv * G, Hkv, L, D, L, seed=12)
    pk, pv, info = orc.compress_kv(K, V, Bt=Bt)
    rows = [(b, h, i) for b in range(B) for h in range(Hkv * G) for i in range(L)]
    O, _ = orc.attention_rows(Q, pk, pv, rows, causal=True)
    ref = _sdpa(_f(Q), _f(K) * info["mask_k"], _f(V) * info["mask_v"], causal=True)
    assert np.allclose(O.reshape(B, Hkv * G, L, D), ref, rtol=1e-10, atol=1e-12)


def test_skipped_tiles_contribute_nothing():
    """Decode: deleting the skipped tiles' tokens from K, V gives the same output.
    Prefill: same with an additive -inf mask; rows that see nothing are zero."""
    B, Hkv, G, L, D, Bt = 1, 2, 2, 96, 32, 16
    Q, K, V = wl.make_qkv(B, Hkv * G, Hkv, L, D, L, seed=13)
    st = np.full((B, Hkv, L // Bt), orc.SPARSE24, dtype=np.int8)
    st[0, 0, [0, 3]] = orc.SKIP
    st[0, 1, [1, 2, 5]] = orc.SKIP
    pk, pv, info = orc.compress_kv(K, V, Bt=Bt, state_k=st, state_v=st)
    Km, Vm = _f(K) * info["mask_k"], _f(V) * info["mask_v"]
    q = Q[:, :, -1, :]
    Od, LSEd = orc.attention_decode(q, pk, pv)
    for h in range(Hkv):
        keep = np.repeat(st[0, h] != orc.SKIP, Bt)
        ref = _sdpa(_f(q)[:, h * G:(h + 1) * G, None, :], Km[:, h:h + 1][:, :, keep], Vm[:, h:h + 1][:, :, keep])
        assert np.allclose(Od[:, h * G:(h + 1) * G], ref[:, :, 0], rtol=1e-10, atol=1e-12)
    # prefill with boolean mask
    rows = [(0, h, i) for h in range(Hkv * G) for i in range(L)]
    O, LSE = orc.attention_rows(Q, pk, pv, rows, causal=True)
    O = O.reshape(Hkv * G, L, D)
    LSE = LSE.reshape(Hkv * G, L)
    for hq in range(Hkv * G):
        h = hq // G
        vis = np.repeat(st[0, h] != orc.SKIP, Bt)[None, :] & np.tril(np.ones((L, L), dtype=bool))
        empty = ~vis.any(axis=-1)
        ref = _sdpa(_f(Q)[:, hq:hq + 1], Km[:, h:h + 1], Vm[:, h:h + 1], mask=vis[None, None] | empty[None, None, :, None])
        assert np.allclose(O[hq][~empty], ref[0, 0][~empty], rtol=1e-10, atol=1e-12)
        assert (O[hq][empty] == 0).all() and np.isneginf(LSE[hq][empty]).all()
        if h == 0:
            assert empty[:Bt].all() and not empty[Bt:].any()


def test_decode_equals_last_causal_row():
    B, Hkv, G, L, D, Bt = 2, 1, 4, 64, 32, 16
    Q, K, V = wl.make_qkv(B, Hkv * G, Hkv, L, D, L, seed=14)
    pk, pv, _ = orc.compress_kv(K, V, Bt=Bt, skip_frac=0.25)
    rows = [(b, h, L - 1) for b in range(B) for h in range(Hkv * G)]
    O, LSE = orc.attention_rows(Q, pk, pv, rows, causal=True)
    Od, LSEd = orc.attention_decode(Q[:, :, -1, :], pk, pv)
    assert np.allclose(O.reshape(B, Hkv * G, D), Od, rtol=1e-12, atol=1e-14)
    assert np.allclose(LSE.reshape(B, Hkv * G), LSEd, rtol=1e-12)


def test_decode_with_dense_tail_equals_library_sdpa_on_concatenation():
    """Tail tokens join the softmax unpruned: equals the library attention over [masked cache ; tail]."""
    rng = np.random.default_rng(11)
    K, V = _rand_kv(11, B=2, H=2, L=48, D=16)
    q = wl.f32_to_bf16_bits(rng.standard_normal((2, 4, 16)).astype(np.float32))
    tk = wl.f32_to_bf16_bits(rng.standard_normal((2, 2, 16, 16)).astype(np.float32))
    tv = wl.f32_to_bf16_bits(rng.standard_normal((2, 2, 16, 16)).astype(np.float32))
    sk = np.array([[[2, 0, 1]] * 2] * 2, dtype=np.int8)
    pk, pv, info = orc.compress_kv(K, V, Bt=16, state_k=sk, state_v=sk)
    for tail_len in (1, 7, 16):
        O, LSE = orc.attention_decode(q, pk, pv, tail_k=tk, tail_v=tv, tail_len=tail_len)
        Km = np.where(info["mask_k"], K, 0).astype(np.uint16)
        Vm = np.where(info["mask_v"], V, 0).astype(np.uint16)
        Km[:, :, 32:] = K[:, :, 32:]                               # tile 2 dense
        Vm[:, :, 32:] = V[:, :, 32:]
        keep = np.r_[0:16, 32:48]                                  # tile 1 skipped
        Kc = np.concatenate([Km[:, :, keep], tk[:, :, :tail_len]], axis=2)
        Vc = np.concatenate([Vm[:, :, keep], tv[:, :, :tail_len]], axis=2)
        ref = _sdpa(_f(q)[:, :, None, :], np.repeat(_f(Kc), 2, axis=1), np.repeat(_f(Vc), 2, axis=1))
        assert np.allclose(O, ref[:, :, 0, :], rtol=1e-12, atol=1e-13)
    # an empty tail is the plain decode
    O0, L0 = orc.attention_decode(q, pk, pv)
    O1, L1 = orc.attention_decode(q, pk, pv, tail_k=tk, tail_v=tv, tail_len=0)
    assert (O0 == O1).all() and (L0 == L1).all()


def test_append_in_tile_order_rebuilds_the_one_shot_cache():
    """Compressing a prefix with the rest of the capacity SKIP and appending the remaining tiles one
    by one gives the pools and maps of compressing everything at once (slots follow tile order)."""
    K, V = _rand_kv(12, B=2, H=2, L=16 * 7, D=16)
    rng = np.random.default_rng(12)
    sk = rng.choice([1, 2], size=(7,)).astype(np.int8)
    sv = rng.choice([1, 2], size=(7,)).astype(np.int8)
    full_k = np.broadcast_to(sk, (2, 2, 7)).copy()
    full_v = np.broadcast_to(sv, (2, 2, 7)).copy()
    pk1, pv1, _ = orc.compress_kv(K, V, Bt=16, state_k=full_k, state_v=full_v)
    pre_k, pre_v = full_k.copy(), full_v.copy()
    pre_k[:, :, 3:] = 0
    pre_v[:, :, 3:] = 0
    pk2, pv2, _ = orc.compress_kv(K, V, Bt=16, state_k=pre_k, state_v=pre_v)
    q = wl.f32_to_bf16_bits(rng.standard_normal((2, 4, 16)).astype(np.float32))
    O_pre, _ = orc.attention_decode(q, pk2, pv2)
    O_ref, _ = orc.attention_rows(np.repeat(q[:, :, None, :], 16 * 7, axis=2), pk1, pv1,
                                  [(b, h, 16 * 3 - 1) for b in range(2) for h in range(4)], causal=True, q_offset=0)
    assert np.allclose(O_pre.reshape(-1, 16), O_ref, rtol=1e-12, atol=1e-13)   # unfilled capacity = causal prefix
    for t in range(3, 7):
        orc.append_tile(pk2, pv2, t, K[:, :, 16 * t:16 * (t + 1)], V[:, :, 16 * t:16 * (t + 1)], int(sk[t]), int(sv[t]))
    for a, b in ((pk1, pk2), (pv1, pv2)):
        assert (a.map == b.map).all() and (a.f16 == b.f16).all()
        nd, ns = a.dense.shape[2], a.nnz.shape[2]
        assert (a.dense == b.dense[:, :, :nd]).all() and (a.nnz == b.nnz[:, :, :ns]).all() and (a.meta == b.meta[:, :, :ns]).all()
    assert (orc.unpack_tensor(pk2) == orc.unpack_tensor(pk1)).all()


def _same_packed(a, b):
    assert (a.map == b.map).all() and (a.f16 == b.f16).all()
    for t in np.argwhere(a.map != 0):
        m = int(a.map[tuple(t)])
        slot = orc.map_slot(m)
        if m > 0:
            assert (a.dense[t[0], t[1], slot] == b.dense[t[0], t[1], slot]).all()
        else:
            assert (a.nnz[t[0], t[1], slot] == b.nnz[t[0], t[1], slot]).all()
            assert (a.meta[t[0], t[1], slot] == b.meta[t[0], t[1], slot]).all()


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_further_pruning_of_a_packed_cache_equals_compressing_with_the_sparser_states(dtype):
    """Pruning the packed cache again towards target states B gives, bit for bit, what compressing the
    original tensors with the tile-wise sparser of (A, B) gives: 2:4 tiles keep what they hold, dense
    tiles are pruned from the values they store (which are the original ones), dropped tiles vanish,
    slots are handed out again in sequence order.  By hand on one group as well."""
    rng = np.random.default_rng(14)
    B, H, T, Bt, D = 2, 2, 9, 16, 16
    to_bits = wl.f32_to_f16_bits if dtype == "fp16" else wl.f32_to_bf16_bits
    Kf = rng.standard_normal((B, H, T * Bt, D)).astype(np.float32)
    Vf = rng.standard_normal((B, H, T * Bt, D)).astype(np.float32)
    if dtype == "bf16":
        Vf = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(Vf))
        # tile 2: one value per group of 4 tokens far under fp16's range and small enough to be pruned:
        # the dense tile is not exact in fp16, its 2:4 form is
        Vf[:, :, 2 * Bt:3 * Bt:4] = 2.0 ** -40
        Vf[:, :, 3 * Bt:4 * Bt] *= 2.0 ** -22            # tile 3: stays bf16 in either form
    K, V = to_bits(Kf), to_bits(Vf)
    order = {orc.DENSE: 0, orc.SPARSE24: 1, orc.SKIP: 2}
    A_k = rng.choice([1, 2], size=(B, H, T)).astype(np.int8)
    A_v = rng.choice([1, 2], size=(B, H, T)).astype(np.int8)
    A_v[:, :, 2:4] = orc.DENSE
    skip_a = rng.random((B, H, T)) < 0.15
    skip_a[:, :, 2:4] = False
    A_k[skip_a] = 0
    A_v[skip_a] = 0
    B_k = rng.choice([1, 2], size=(B, H, T)).astype(np.int8)
    B_v = rng.choice([1, 2], size=(B, H, T)).astype(np.int8)
    B_v[:, :, 2:4] = orc.SPARSE24
    skip_b = rng.random((B, H, T)) < 0.15
    skip_b[:, :, 2:4] = False
    B_k[skip_b] = 0
    B_v[skip_b] = 0
    pk, pv, _ = orc.compress_kv(K, V, Bt=Bt, state_k=A_k, state_v=A_v, dtype=dtype)
    if dtype == "bf16":
        assert not pv.f16[0, 0, 2] and not pv.f16[0, 0, 3]
    keep = (pk.map.copy(), pk.dense.copy(), pk.nnz.copy())
    rk, rv = orc.recompress_kv(pk, pv, B_k, B_v)
    assert (keep[0] == pk.map).all() and (keep[1] == pk.dense).all() and (keep[2] == pk.nnz).all()   # source untouched
    merge = np.vectorize(lambda a, b: a if order[a] >= order[b] else b)
    C_k, C_v = merge(A_k, B_k).astype(np.int8), merge(A_v, B_v).astype(np.int8)
    assert (C_k[skip_a | skip_b] == 0).all() and (C_k[(A_k == 2) & ~skip_b] == 2).all()
    ck, cv, _ = orc.compress_kv(K, V, Bt=Bt, state_k=C_k, state_v=C_v, dtype=dtype)
    _same_packed(rk, ck)
    _same_packed(rv, cv)
    if dtype == "bf16":
        assert rv.f16[0, 0, 2] and not rv.f16[0, 0, 3]
    # no further pruning asked for: nothing changes
    nk, nv = orc.recompress_kv(pk, pv, np.where(A_k == 0, 0, 1), np.where(A_v == 0, 0, 1))
    _same_packed(nk, pk)
    _same_packed(nv, pv)
    # by hand: a dense K tile whose first group of token 0 is (1, -3, 2, 0.5) keeps -3 and 2
    Kh = np.zeros((1, 1, Bt, D), dtype=np.float32)
    Kh[0, 0, 0, :4] = [1.0, -3.0, 2.0, 0.5]
    Vh = np.zeros((1, 1, Bt, D), dtype=np.float32)
    Vh[0, 0, :4, 5] = [0.25, 4.0, -0.125, -8.0]           # tokens 0..3 of channel 5: keeps 4 and -8
    dense = np.ones((1, 1, 1), dtype=np.int8)
    hk, hv, _ = orc.compress_kv(to_bits(Kh), to_bits(Vh), Bt=Bt, state_k=dense, state_v=dense, dtype=dtype)
    hk2, hv2 = orc.recompress_kv(hk, hv, 2 * dense, 2 * dense)
    assert hk2.map[0, 0, 0] < 0 and hv2.map[0, 0, 0] < 0
    assert orc.to_f64(orc.unpack_tensor(hk2), dtype)[0, 0, 0, :4].tolist() == [0.0, -3.0, 2.0, 0.0]
    assert orc.to_f64(orc.unpack_tensor(hv2), dtype)[0, 0, :4, 5].tolist() == [0.0, 4.0, 0.0, -8.0]


def test_pools_of_a_given_size_keep_the_blocks_that_find_a_slot_in_sequence_order():
    """Sec. III-B counters with bounded pools, by hand: 2 dense-K, 2 sparse-K, 3 dense-V, 1 sparse-V slots.
    A block needs a slot in its K pool and in its V pool; one that finds either full is left out of both
    and takes no slot, so later blocks of the other kind still fit and the used slots have no holes."""
    D_, S_, X_ = orc.DENSE, orc.SPARSE24, orc.SKIP
    sk = np.array([[[D_, S_, D_, D_, S_, X_, S_, D_]]], dtype=np.int8)
    sv = np.array([[[D_, S_, D_, D_, S_, X_, D_, S_]]], dtype=np.int8)
    #   t0 K dense 1/2, V dense 1/3      kept
    #   t1 K sparse 1/2, V sparse 1/1    kept
    #   t2 K dense 2/2, V dense 2/3      kept
    #   t3 K dense: full                 dropped (its V dense slot is not taken)
    #   t4 V sparse: full                dropped (its K sparse slot is not taken)
    #   t5 skipped
    #   t6 K sparse 2/2, V dense 3/3     kept
    #   t7 K dense: full                 dropped
    nk, nv, dropped = orc.fit_states_to_capacity(sk, sv, (2, 2, 3, 1))
    assert dropped
    assert nk[0, 0].tolist() == [D_, S_, D_, X_, X_, X_, S_, X_]
    assert nv[0, 0].tolist() == [D_, S_, D_, X_, X_, X_, D_, X_]
    assert orc.build_map(nk)[0, 0].tolist() == [1, -1, 2, 0, 0, 0, -2, 0]
    assert orc.build_map(nv)[0, 0].tolist() == [1, -1, 2, 0, 0, 0, 3, 0]
    same_k, same_v, dropped = orc.fit_states_to_capacity(sk, sv, (4, 3, 4, 3))
    assert not dropped and (same_k == sk).all() and (same_v == sv).all()
    # through the whole compressor and through further pruning: same survivors, and an append goes on
    # from the used counts
    K, V = _rand_kv(21, B=1, H=1, L=16 * 8, D=16)
    pk, pv, info = orc.compress_kv(K, V, Bt=16, state_k=sk, state_v=sv, caps=(2, 2, 3, 1))
    assert info["dropped"] and pk.map[0, 0].tolist() == [1, -1, 2, 0, 0, 0, -2, 0]
    fk, fv, _ = orc.compress_kv(K, V, Bt=16, state_k=np.where(sk == X_, X_, D_), state_v=np.where(sv == X_, X_, D_))
    rk, rv, dropped = orc.recompress_kv(fk, fv, sk, sv, caps=(2, 2, 3, 1))
    assert dropped
    _same_packed(rk, pk)
    _same_packed(rv, pv)
    orc.append_tile(rk, rv, 5, K[:, :, 16 * 5:16 * 6], V[:, :, 16 * 5:16 * 6], S_, D_)
    assert rk.map[0, 0, 5] == -3 and rv.map[0, 0, 5] == 4                  # next free slots: no slot is handed out twice
    slots = sorted(abs(int(m)) for m in rk.map[0, 0] if m < 0)
    assert slots == [1, 2, 3]


def test_batch_rows_of_different_length_equal_separate_sequences():
    """Sequences of a batch differ in length: per-row tail lengths in decode and per-row append positions
    give, row by row, what each sequence gives on its own (the one-sequence forms are pinned above)."""
    rng = np.random.default_rng(15)
    B, H, Hq, Bt, D, T = 3, 2, 4, 16, 16, 6
    K, V = _rand_kv(15, B=B, H=H, L=Bt * T, D=D)
    held = [2, 5, 3]                                         # tiles each sequence holds so far
    sk = np.full((B, H, T), orc.SPARSE24, dtype=np.int8)
    sv = np.full((B, H, T), orc.DENSE, dtype=np.int8)
    for b in range(B):
        sk[b, :, held[b]:] = 0
        sv[b, :, held[b]:] = 0
    pk, pv, _ = orc.compress_kv(K, V, Bt=Bt, state_k=sk, state_v=sv)
    q = wl.f32_to_bf16_bits(rng.standard_normal((B, Hq, D)).astype(np.float32))
    tail_k = wl.f32_to_bf16_bits(rng.standard_normal((B, H, Bt, D)).astype(np.float32))
    tail_v = wl.f32_to_bf16_bits(rng.standard_normal((B, H, Bt, D)).astype(np.float32))
    lens = np.array([5, 0, 16])
    O, LSE = orc.attention_decode(q, pk, pv, tail_k=tail_k, tail_v=tail_v, tail_len=lens)
    for b in range(B):
        pkb, pvb, _ = orc.compress_kv(K[b:b + 1], V[b:b + 1], Bt=Bt, state_k=sk[b:b + 1], state_v=sv[b:b + 1])
        Ob, Lb = orc.attention_decode(q[b:b + 1], pkb, pvb, tail_k=tail_k[b:b + 1], tail_v=tail_v[b:b + 1], tail_len=int(lens[b]))
        assert np.array_equal(O[b], Ob[0]) and np.array_equal(LSE[b], Lb[0])
    # sequences 0 and 2 move their (full) tail into the cache at their own position, sequence 1 does not
    where = np.array([held[0], -1, held[2]])
    orc.append_tile(pk, pv, where, tail_k, tail_v, orc.SPARSE24, orc.DENSE)
    for b in range(B):
        Kb, Vb, skb, svb = K[b:b + 1].copy(), V[b:b + 1].copy(), sk[b:b + 1].copy(), sv[b:b + 1].copy()
        if where[b] >= 0:
            t = int(where[b])
            Kb[:, :, Bt * t:Bt * (t + 1)], Vb[:, :, Bt * t:Bt * (t + 1)] = tail_k[b:b + 1], tail_v[b:b + 1]
            skb[:, :, t], svb[:, :, t] = orc.SPARSE24, orc.DENSE
        pkb, pvb, _ = orc.compress_kv(Kb, Vb, Bt=Bt, state_k=skb, state_v=svb)
        assert (pk.map[b] == pkb.map[0]).all() and (pv.map[b] == pvb.map[0]).all()
        assert (orc.unpack_tensor(pk)[b] == orc.unpack_tensor(pkb)[0]).all()
        assert (orc.unpack_tensor(pv)[b] == orc.unpack_tensor(pvb)[0]).all()


def test_fp16_patterns_are_read_as_ieee_binary16():
    """The fp16 path differs from bf16 only in what the 16-bit patterns mean: same masks and packed bits,
    values per IEEE binary16 (checked on hand-written patterns and against struct's 'e' format), scores and
    attention computed on those values (library SDPA on the converted tensors)."""
    import struct
    pats = np.array([0x3C00, 0xC000, 0x0001, 0x0400, 0x7BFF, 0x3555, 0x8000], dtype=np.uint16)
    want = [1.0, -2.0, 2.0 ** -24, 2.0 ** -14, 65504.0, struct.unpack("<e", struct.pack("<H", 0x3555))[0], -0.0]
    assert orc.to_f64(pats, "fp16").tolist() == want
    assert orc.to_f64(np.array([0x3F80, 0xC000], dtype=np.uint16), "bf16").tolist() == [1.0, -2.0]
    rng = np.random.default_rng(13)
    K = wl.f32_to_f16_bits(rng.standard_normal((1, 2, 48, 16)).astype(np.float32))
    V = wl.f32_to_f16_bits(rng.standard_normal((1, 2, 48, 16)).astype(np.float32))
    q = wl.f32_to_f16_bits(rng.standard_normal((1, 4, 16)).astype(np.float32))
    pk, pv, info = orc.compress_kv(K, V, Bt=16, dtype="fp16", skip_frac=1 / 3, sparse_frac_k=0.5)
    pkb, pvb, infob = orc.compress_kv(K, V, Bt=16, dtype="bf16", state_k=info["state_k"], state_v=info["state_v"])
    assert (info["mask_k"] == infob["mask_k"]).all() and (pk.nnz == pkb.nnz).all() and (pv.meta == pvb.meta).all()
    f = lambda b: np.ascontiguousarray(b).view(np.float16).astype(np.float64)
    e = (f(K) ** 2).reshape(1, 2, 3, -1).sum(-1) + (f(V) ** 2).reshape(1, 2, 3, -1).sum(-1)
    assert np.allclose(info["energy"], e, rtol=1e-13)
    assert (np.argmin(e, axis=-1) == np.argmax(pk.map == 0, axis=-1)).all()          # one of three tiles skipped
    O, LSE = orc.attention_decode(q, pk, pv)
    Ku, Vu = f(orc.unpack_tensor(pk)), f(orc.unpack_tensor(pv))
    for h in range(4):
        vis = np.repeat(pk.map[0, h // 2] != 0, 16)
        ref = _sdpa(f(q)[0, h][None, None, None, :], Ku[0, h // 2][vis][None, None], Vu[0, h // 2][vis][None, None])
        assert np.allclose(O[0, h], ref[0, 0, 0], rtol=1e-12, atol=1e-13)


def test_v_tiles_in_fp16_encoding_hold_the_same_values():
    """A V tile of a bf16 cache is kept in fp16 encoding exactly when every stored value survives the
    round trip; the decision and the conversion are checked value by value with Python floats / struct."""
    import struct
    def bf(x):        # bf16 pattern of a float that bf16 holds exactly
        return struct.unpack("<I", struct.pack("<f", x))[0] >> 16
    def as_f16(bits):
        return struct.unpack("<e", struct.pack("<H", int(bits)))[0]
    def as_bf16(bits):
        return struct.unpack("<f", struct.pack("<I", int(bits) << 16))[0]
    ok = [1.0, -2.5, 0.0, -0.0, 65280.0, 2.0 ** -14, 2.0 ** -24, 3 * 2.0 ** -24, 255 * 2.0 ** -24, float("inf")]
    bad = [65536.0, 1e30, 2.0 ** -25, 129 * 2.0 ** -25, -3 * 2.0 ** -26, float("nan")]
    bits = np.array([bf(x) for x in ok + bad], dtype=np.uint16)
    assert orc.bf16_bits_exact_in_f16(bits).tolist() == [True] * len(ok) + [False] * len(bad)
    conv = orc.bf16_bits_to_f16_bits(bits[:len(ok)])
    for b, c in zip(bits[:len(ok)], conv):
        assert as_f16(c) == as_bf16(b) and (c >> 15) == (b >> 15)
    assert (orc.f16_bits_to_bf16_bits(conv) == bits[:len(ok)]).all()
    # tiles: 0 plain, 1 has one value fp16 cannot hold, 2 has such a value only where 2:4 pruning removes it
    K, V = _rand_kv(14, B=1, H=1, L=16 * 3, D=16)
    V[0, 0, 16 + 3, 5] = bf(1e30)
    V[0, 0, 32:36, 7] = [bf(1.0), bf(-2.0), bf(2.0 ** -30), bf(0.5)]
    pk, pv, info = orc.compress_kv(K, V, Bt=16)
    assert pv.f16[0, 0].tolist() == [True, False, True]
    assert not pk.f16.any()
    assert (pv.map[0, 0] == [-1, -2, -3]).all()                                      # the index map stays the paper's
    assert (orc.unpack_tensor(pv) == np.where(info["mask_v"], V, 0)).all()           # values unchanged either way
    assert (pv.nnz[0, 0, 1] == orc.pack_v_tile(V[0, 0, 16:32], info["mask_v"][0, 0, 16:32])[0]).all()   # tile 1: bf16 bits
    assert (pv.nnz[0, 0, 0] != orc.pack_v_tile(V[0, 0, :16], info["mask_v"][0, 0, :16])[0]).any()       # tile 0: other encoding
    pkd, pvd, _ = orc.compress_kv(K, V, Bt=16, sparse_frac_k=0.0, sparse_frac_v=0.0)
    assert pvd.f16[0, 0].tolist() == [True, False, False]                            # dense: every value is stored
    assert (orc.unpack_tensor(pvd) == V).all()
    pkh, pvh, _ = orc.compress_kv(K, V, Bt=16, dtype="fp16")
    assert not pvh.f16.any()                                                         # fp16 caches need no flag


def test_brute_force_python_floats_tiny():
    """Whole path (prune, skip, attention) redone with Python lists and math.exp."""
    B, Hkv, G, L, D, Bt = 1, 1, 2, 16, 8, 4
    Q, K, V = wl.make_qkv(B, Hkv * G, Hkv, L, D, L, seed=15)
    st = np.array([[[2, 0, 1, 2]]], dtype=np.int8)
    pk, pv, _ = orc.compress_kv(K, V, Bt=Bt, state_k=st, state_v=st)
    Kf = wl.bf16_bits_to_f32(K)[0, 0].tolist()
    Vf = wl.bf16_bits_to_f32(V)[0, 0].tolist()
    Qf = wl.bf16_bits_to_f32(Q)[0].tolist()

    def top2(vals):
        order = sorted(range(4), key=lambda i: (-abs(vals[i]), i))[:2]
        return [vals[i] if i in order else 0.0 for i in range(4)]

    Kp = [row[:] for row in Kf]
    Vp = [row[:] for row in Vf]
    for t in range(4):
        if st[0, 0, t] != 2:
            continue
        for tok in range(4 * t, 4 * t + 4):
            for g in range(D // 4):
                Kp[tok][4 * g:4 * g + 4] = top2(Kf[tok][4 * g:4 * g + 4])
        for c in range(D):
            col = top2([Vf[4 * t + j][c] for j in range(4)])
            for j in range(4):
                Vp[4 * t + j][c] = col[j]
    rows = [(0, h, i) for h in range(2) for i in range(L)]
    O, LSE = orc.attention_rows(Q, pk, pv, rows, causal=True)
    for n, (_, h, i) in enumerate(rows):
        toks = [j for j in range(i + 1) if st[0, 0, j // Bt] != 0]
        s = [sum(Qf[h][i][c] * Kp[j][c] for c in range(D)) / math.sqrt(D) for j in toks]
        m = max(s)
        p = [math.exp(x - m) for x in s]
        l = sum(p)
        o = [sum(p[a] * Vp[j][c] for a, j in enumerate(toks)) / l for c in range(D)]
        assert np.allclose(O[n], o, rtol=1e-12, atol=1e-14)
        assert abs(LSE[n] - (m + math.log(l))) < 1e-12
