"""Pins for oracle/hs_layout.py (the in-tile byte order of the packed pools) against something
other than itself: a numpy emulation of the gfx950 matrix instructions, written here from the
operand semantics of the two instruction forms, consumes the *physical* bytes the way the layout
contract says a wave consumes them (chunk c = 64 lanes x 16 B, lane l at byte 16 l; which chunk
and which index half feed which instruction) and must reproduce K~ Q^T and V~^T P^T of the
canonical tile as computed by a plain numpy matmul.  All values are small integers, so every
product and sum is exact and the comparison is equality.

Operand semantics emulated (CDNA4 ISA, 64-lane wave; a = l // 16, r = l % 16):
  v_mfma_f32_16x16x32    A[row r][k = 8a + e],  B[k = 8a + e][col r],  e = 0..7
                         D lane l, register i = D[row 4a + i][col r]
  v_smfmac_f32_16x16x64  A: lane l holds the 8 kept values of row r among k in [16a, 16a + 16):
                         kept value e sits in group e // 2 at position (idx >> 2e) & 3,
                         idx = the 16-bit half of the lane's index register that ABID selects
                         B[k = 32 (e // 8) + 8a + e % 8][col r], e = 0..15;  D as above.

A slip planted into the layout (chunk order, lane order, index half, nibble order, token order)
must turn these tests red; test_planted_slips_are_caught shows that on the CPU.
"""
import numpy as np
import pytest

from oracle import hs_layout as hl
from oracle import hs_oracle as orc
from paper_2604_16864_amd import workloads as wl

LANES = np.arange(64)
A_OF, R_OF = LANES // 16, LANES % 16


# ------------------------------------------------------------------ instruction emulators
def emu_mfma_16x16x32(A, B):
    """A, B: [64 lanes, 8] -> D [64 lanes, 4]."""
    Af = np.zeros((16, 32))
    Bf = np.zeros((32, 16))
    for l in range(64):
        for e in range(8):
            Af[l % 16, 8 * (l // 16) + e] = A[l, e]
            Bf[8 * (l // 16) + e, l % 16] = B[l, e]
    Df = Af @ Bf
    return np.array([[Df[4 * (l // 16) + i, l % 16] for i in range(4)] for l in range(64)])


def emu_smfmac_16x16x64(A, B, idx16):
    """A: [64, 8] kept values, B: [64, 16], idx16: [64] the 16 index bits of each lane -> D [64, 4]."""
    Af = np.zeros((16, 64))
    Bf = np.zeros((64, 16))
    for l in range(64):
        for e in range(8):
            pos = (int(idx16[l]) >> (2 * e)) & 3
            Af[l % 16, 16 * (l // 16) + 4 * (e // 2) + pos] = A[l, e]
        for e in range(16):
            Bf[32 * (e // 8) + 8 * (l // 16) + e % 8, l % 16] = B[l, e]
    Df = Af @ Bf
    return np.array([[Df[4 * (l // 16) + i, l % 16] for i in range(4)] for l in range(64)])


def d_to_matrix(D):
    """D registers [64, 4] -> the 16 x 16 result block."""
    M = np.zeros((16, 16))
    for l in range(64):
        for i in range(4):
            M[4 * (l // 16) + i, l % 16] = D[l, i]
    return M


# ------------------------------------------------------------------ how a wave reads a pool slot
def chunk_regs(slot_bytes, c):
    """Chunk c of a slot as the 8 16-bit register halves of each lane, as real numbers."""
    u16 = np.ascontiguousarray(slot_bytes[1024 * c:1024 * (c + 1)]).view(np.uint16).reshape(64, 8)
    return wl.bf16_bits_to_f32(u16).astype(np.float64)


def lane_index_words(meta_bytes):
    """The four 32-bit index words each lane holds (16 B per lane)."""
    return np.ascontiguousarray(meta_bytes).view(np.uint32).reshape(64, 4)


def gemm1_b_regs(Qblock, kb=None, s=None):
    """Q^T as the B operand.  Qblock: [16 queries, 128 channels].  Sparse form (kb): channel of
    element e = 64 kb + (B's k); dense form (s): channel = 32 s + 8a + e."""
    if kb is not None:
        return np.array([[Qblock[l % 16, 64 * kb + 32 * (e // 8) + 8 * (l // 16) + e % 8] for e in range(16)]
                         for l in range(64)])
    return np.array([[Qblock[l % 16, 32 * s + 8 * (l // 16) + e] for e in range(8)] for l in range(64)])


def gemm2_b_regs(Pblock):
    """GEMM1's accumulators handed to GEMM2 unmoved: lane l held, for row block m and register i,
    token 16m + 4a + i of its query column; those 16 numbers are B elements e = 4m + i.
    Pblock: [16 queries, 64 tokens] -> [64 lanes, 16]."""
    return np.array([[Pblock[l % 16, 16 * (e // 4) + 4 * (l // 16) + e % 4] for e in range(16)] for l in range(64)])


def k_times_q_sparse(nnz_bytes, meta_bytes, Q):
    """S^T [64 tokens, n queries] from the physical bytes of a 2:4 K tile."""
    words = lane_index_words(meta_bytes)
    S = np.zeros((64, Q.shape[0]))
    for qb in range(Q.shape[0] // 16):
        Qb = Q[16 * qb:16 * qb + 16]
        for m in range(4):
            D = np.zeros((64, 4))
            for kb in range(2):          # chunk 2m + kb; index half kb of the lane's word m
                D += emu_smfmac_16x16x64(chunk_regs(nnz_bytes, 2 * m + kb), gemm1_b_regs(Qb, kb=kb),
                                         (words[:, m] >> (16 * kb)) & 0xFFFF)
            S[16 * m:16 * m + 16, 16 * qb:16 * qb + 16] = d_to_matrix(D)
    return S


def k_times_q_dense(dense_bytes, Q):
    S = np.zeros((64, Q.shape[0]))
    for qb in range(Q.shape[0] // 16):
        Qb = Q[16 * qb:16 * qb + 16]
        for m in range(4):
            D = np.zeros((64, 4))
            for s in range(4):           # chunk 4m + s
                D += emu_mfma_16x16x32(chunk_regs(dense_bytes, 4 * m + s), gemm1_b_regs(Qb, s=s))
            S[16 * m:16 * m + 16, 16 * qb:16 * qb + 16] = d_to_matrix(D)
    return S


def vt_times_pt_sparse(nnz_bytes, meta_bytes, P):
    """O^T [128 channels, n queries] from the physical bytes of a 2:4 V tile.  P: [n queries, 64 tokens]."""
    words = lane_index_words(meta_bytes)
    O = np.zeros((128, P.shape[0]))
    for qb in range(P.shape[0] // 16):
        B = gemm2_b_regs(P[16 * qb:16 * qb + 16])
        for mb in range(8):              # chunk mb; index half mb % 2 of the lane's word mb // 2
            D = emu_smfmac_16x16x64(chunk_regs(nnz_bytes, mb), B, (words[:, mb // 2] >> (16 * (mb % 2))) & 0xFFFF)
            O[16 * mb:16 * mb + 16, 16 * qb:16 * qb + 16] = d_to_matrix(D)
    return O


def vt_times_pt_dense(dense_bytes, P):
    O = np.zeros((128, P.shape[0]))
    for qb in range(P.shape[0] // 16):
        B = gemm2_b_regs(P[16 * qb:16 * qb + 16])
        for mb in range(8):
            D = np.zeros((64, 4))
            for h in range(2):           # chunk 2mb + h takes B elements 8h .. 8h + 7
                D += emu_mfma_16x16x32(chunk_regs(dense_bytes, 2 * mb + h), B[:, 8 * h:8 * h + 8])
            O[16 * mb:16 * mb + 16, 16 * qb:16 * qb + 16] = d_to_matrix(D)
    return O


# ------------------------------------------------------------------ inputs
def _int_tile(seed):
    """A 64 x 128 tile of small non-zero integers (exact in bf16), all magnitudes in a group distinct."""
    rng = np.random.default_rng(seed)
    mags = np.stack([rng.permutation(np.arange(1, 9))[:4] for _ in range(64 * 32)]).reshape(64, 128)
    sign = rng.choice([-1.0, 1.0], size=(64, 128))
    return wl.f32_to_bf16_bits((mags * sign).astype(np.float32))


def _canonical_k(seed):
    tile = _int_tile(seed)
    mask = orc.element_mask_k(tile[None, None])[0, 0]
    nnz, meta = orc.pack_k_tile(tile, mask)
    return tile, mask, nnz, meta


def _canonical_v(seed):
    tile = _int_tile(seed).reshape(128, 64).T.copy()     # groups of distinct magnitudes run along tokens
    mask = orc.element_mask_v(tile[None, None])[0, 0]
    nnz, meta = orc.pack_v_tile(tile, mask)
    return tile, mask, nnz, meta


def _f(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


IDENT = np.eye(128)


# ------------------------------------------------------------------ the checks (take the layout functions as arguments)
def check_k_sparse(physical):
    tile, mask, nnz, meta = _canonical_k(1)
    pn, pm = physical(nnz, meta)
    assert pn.shape == (8192,) and pm.shape == (1024,) and pn.dtype == np.uint8 and pm.dtype == np.uint8
    Kt = _f(np.where(mask, tile, 0))
    # with Q = identity the product is the tile itself: the physical bytes decode to the canonical tile
    assert (k_times_q_sparse(pn, pm, IDENT) == Kt).all()
    Q = np.random.default_rng(2).integers(-4, 5, size=(32, 128)).astype(np.float64)
    assert (k_times_q_sparse(pn, pm, Q) == Kt @ Q.T).all()


def check_v_sparse(physical):
    tile, mask, nnz, meta = _canonical_v(3)
    pn, pm = physical(nnz, meta)
    assert pn.shape == (8192,) and pm.shape == (1024,)
    Vt = _f(np.where(mask, tile, 0))                     # [64 tokens, 128 channels]
    assert (vt_times_pt_sparse(pn, pm, np.eye(64)) == Vt.T).all()
    P = np.random.default_rng(4).integers(0, 6, size=(16, 64)).astype(np.float64)
    assert (vt_times_pt_sparse(pn, pm, P) == Vt.T @ P.T).all()


def check_k_dense(physical):
    tile = _int_tile(5)
    pd = physical(tile)
    assert pd.shape == (16384,)
    assert (k_times_q_dense(pd, IDENT) == _f(tile)).all()
    Q = np.random.default_rng(6).integers(-4, 5, size=(16, 128)).astype(np.float64)
    assert (k_times_q_dense(pd, Q) == _f(tile) @ Q.T).all()


def check_v_dense(physical):
    tile = _int_tile(7)
    pd = physical(tile)
    assert pd.shape == (16384,)
    assert (vt_times_pt_dense(pd, np.eye(64)) == _f(tile).T).all()
    P = np.random.default_rng(8).integers(0, 6, size=(16, 64)).astype(np.float64)
    assert (vt_times_pt_dense(pd, P) == _f(tile).T @ P.T).all()


def test_k_sparse_physical_feeds_gemm1():
    check_k_sparse(hl.k_sparse_physical)


def test_v_sparse_physical_feeds_gemm2():
    check_v_sparse(hl.v_sparse_physical)


def test_k_dense_physical_feeds_gemm1():
    check_k_dense(hl.k_dense_physical)


def test_v_dense_physical_feeds_gemm2():
    check_v_dense(hl.v_dense_physical)


# ------------------------------------------------------------------ permutations
def test_every_physical_order_is_a_permutation_of_the_canonical_elements():
    ids = np.arange(64 * 64, dtype=np.uint16).reshape(64, 64)
    zero_meta = np.zeros((64, 4), dtype=np.uint32)
    pn, _ = hl.k_sparse_physical(ids, zero_meta)
    assert sorted(pn.view(np.uint16).tolist()) == list(range(4096))
    pn, _ = hl.v_sparse_physical(ids.reshape(16, 2, 128), np.zeros((16, 16), dtype=np.uint32))
    assert sorted(pn.view(np.uint16).tolist()) == list(range(4096))
    ids = np.arange(64 * 128, dtype=np.uint16).reshape(64, 128)
    assert sorted(hl.k_dense_physical(ids).view(np.uint16).tolist()) == list(range(8192))
    assert sorted(hl.v_dense_physical(ids).view(np.uint16).tolist()) == list(range(8192))
    # metadata: every canonical nibble lands in exactly one physical nibble (one-hot, a seeded sample)
    rng = np.random.default_rng(9)
    seen_k, seen_v = set(), set()
    for _ in range(48):
        tok, g = int(rng.integers(64)), int(rng.integers(32))
        meta = np.zeros((64, 4), dtype=np.uint32)
        meta[tok, g // 8] = np.uint32(0xF) << np.uint32(4 * (g % 8))
        _, pm = hl.k_sparse_physical(np.zeros((64, 64), dtype=np.uint16), meta)
        nib = np.nonzero(orc._words_to_nibbles(pm.view(np.uint32)[None])[0])[0]
        assert nib.size == 1
        seen_k.add(int(nib[0]))
        grp, ch = int(rng.integers(16)), int(rng.integers(128))
        meta = np.zeros((16, 16), dtype=np.uint32)
        meta[grp, ch // 8] = np.uint32(0xF) << np.uint32(4 * (ch % 8))
        _, pm = hl.v_sparse_physical(np.zeros((16, 2, 128), dtype=np.uint16), meta)
        nib = np.nonzero(orc._words_to_nibbles(pm.view(np.uint32)[None])[0])[0]
        assert nib.size == 1
        seen_v.add(int(nib[0]))
    assert len(seen_k) >= 40 and len(seen_v) >= 40       # distinct inputs land in distinct places


def test_token_of_k_follows_from_the_accumulator_and_operand_lane_maps():
    """Contraction index k of GEMM2 means the token that GEMM1 left in the register which the B
    operand reads for k: D register i of row block m in lane group a is token 16m + 4a + i and is
    handed over as B element e = 4m + i, which the sparse form reads as k = 32 (e // 8) + 8a + e % 8."""
    tok = {}
    for a in range(4):
        for e in range(16):
            tok[32 * (e // 8) + 8 * a + e % 8] = 16 * (e // 4) + 4 * a + e % 4
    assert sorted(tok) == list(range(64))
    assert hl.TOKEN_OF_K.tolist() == [tok[k] for k in range(64)]
    # the same through the emulators: GEMM1 on a tile whose row t is t * ones puts "token index" into
    # the accumulators; reading them as the B operand of GEMM2 against A = one-hot rows gives k -> token
    K = np.repeat(np.arange(64, dtype=np.float64)[:, None], 32, axis=1)       # [64 tokens, 32 channels]
    ones_q = np.zeros((16, 32))
    ones_q[:, 0] = 1.0                                                         # every query picks channel 0
    acc = np.zeros((64, 16))
    for m in range(4):
        A = np.array([[K[16 * m + l % 16, 8 * (l // 16) + e] for e in range(8)] for l in range(64)])
        B = np.array([[ones_q[l % 16, 8 * (l // 16) + e] for e in range(8)] for l in range(64)])
        acc[:, 4 * m:4 * m + 4] = emu_mfma_16x16x32(A, B)
    for k in (0, 5, 13, 31, 32, 47, 63):
        A = np.zeros((64, 8))
        idx = np.zeros(64, dtype=np.int64)
        lane = 16 * (k // 16)                                                  # row 0, lane group holding k
        A[lane, 2 * ((k % 16) // 4)] = 1.0                                     # kept value 2g at position k % 4
        idx[lane] = (k % 4) << (4 * ((k % 16) // 4)) | (3 if k % 4 != 3 else 2) << (4 * ((k % 16) // 4) + 2)
        D = d_to_matrix(emu_smfmac_16x16x64(A, acc, idx))
        assert D[0, 0] == hl.TOKEN_OF_K[k], k


# ------------------------------------------------------------------ planted slips
def _perm_chunks(b, shape, axes):
    return np.ascontiguousarray(b.reshape(shape + (1024,)).transpose(axes + (len(shape),))).reshape(-1)


def test_planted_slips_are_caught():
    """Each plausible mistake in a layout function turns its check red."""
    def swap_lane_halves(b):          # lane l = 16a + r  ->  4r + a inside every chunk
        c = b.reshape(-1, 4, 16, 16)
        return np.ascontiguousarray(c.transpose(0, 2, 1, 3)).reshape(-1)

    def k_sparse_chunk_order(nnz, meta):      # chunk kb * 4 + m instead of m * 2 + kb
        pn, pm = hl.k_sparse_physical(nnz, meta)
        return _perm_chunks(pn, (4, 2), (1, 0)), pm

    def k_sparse_lanes(nnz, meta):
        pn, pm = hl.k_sparse_physical(nnz, meta)
        return swap_lane_halves(pn), pm

    def k_sparse_index_halves(nnz, meta):     # kb = 0 in the high half
        pn, pm = hl.k_sparse_physical(nnz, meta)
        w = pm.view(np.uint32)
        return pn, ((w >> np.uint32(16)) | (w << np.uint32(16))).view(np.uint8)

    def k_sparse_nibble_shift(nnz, meta):     # groups of a half in the opposite order
        pn, pm = hl.k_sparse_physical(nnz, meta)
        h = pm.view(np.uint16).astype(np.uint32)
        r = ((h & 0xF) << 12) | ((h & 0xF0) << 4) | ((h & 0xF00) >> 4) | ((h & 0xF000) >> 12)
        return pn, r.astype(np.uint16).view(np.uint8)

    def k_sparse_word_order(nnz, meta):       # word-major instead of lane-major index words
        pn, pm = hl.k_sparse_physical(nnz, meta)
        return pn, np.ascontiguousarray(pm.view(np.uint32).reshape(64, 4).T).reshape(-1).view(np.uint8)

    for bad in (k_sparse_chunk_order, k_sparse_lanes, k_sparse_index_halves, k_sparse_nibble_shift, k_sparse_word_order):
        with pytest.raises(AssertionError):
            check_k_sparse(bad)

    def v_sparse_natural_groups(nnz, meta):   # token groups 4a + q instead of the accumulator order
        real = hl.TOKEN_OF_K.copy()
        try:
            hl.TOKEN_OF_K = np.arange(64)
            return hl.v_sparse_physical(nnz, meta)
        finally:
            hl.TOKEN_OF_K = real

    def v_sparse_lanes(nnz, meta):
        pn, pm = hl.v_sparse_physical(nnz, meta)
        return swap_lane_halves(pn), pm

    def v_sparse_index_pairing(nnz, meta):    # half mb % 2 of word mb // 2  ->  half mb // 4 of word mb % 4
        pn, pm = hl.v_sparse_physical(nnz, meta)
        h = pm.view(np.uint16).reshape(64, 4, 2)
        return pn, np.ascontiguousarray(h.reshape(64, 2, 4).transpose(0, 2, 1)).reshape(-1).view(np.uint8)

    def v_sparse_pair_order(nnz, meta):       # higher position first
        pn, pm = hl.v_sparse_physical(nnz, meta)
        return np.ascontiguousarray(pn.view(np.uint16).reshape(-1, 2)[:, ::-1]).reshape(-1).view(np.uint8), pm

    for bad in (v_sparse_natural_groups, v_sparse_lanes, v_sparse_index_pairing, v_sparse_pair_order):
        with pytest.raises(AssertionError):
            check_v_sparse(bad)

    def k_dense_chunk_order(tile):            # chunk s * 4 + m
        return _perm_chunks(hl.k_dense_physical(tile), (4, 4), (1, 0))

    def k_dense_lanes(tile):
        return swap_lane_halves(hl.k_dense_physical(tile))

    for bad in (k_dense_chunk_order, k_dense_lanes):
        with pytest.raises(AssertionError):
            check_k_dense(bad)

    def v_dense_natural_tokens(tile):
        real = hl.TOKEN_OF_K.copy()
        try:
            hl.TOKEN_OF_K = np.arange(64)
            return hl.v_dense_physical(tile)
        finally:
            hl.TOKEN_OF_K = real

    def v_dense_chunk_order(tile):            # chunk h * 8 + mb
        return _perm_chunks(hl.v_dense_physical(tile), (8, 2), (1, 0))

    for bad in (v_dense_natural_tokens, v_dense_chunk_order):
        with pytest.raises(AssertionError):
            check_v_dense(bad)


def test_physical_pools_places_tiles_by_slot_and_keeps_stored_encodings():
    """physical_pools: slot s of the canonical pool goes to slot s of the physical pool, through the
    function of its kind; a V tile held in fp16 encoding is laid out from its stored (fp16) bits."""
    rng = np.random.default_rng(11)
    K = wl.normal_bf16(rng, (1, 2, 64 * 3, 128))
    V = wl.normal_bf16(rng, (1, 2, 64 * 3, 128))
    V[0, 0, 64:128] = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(V[0, 0, 64:128]) * np.float32(2.0 ** -22))   # stays bf16
    sk = np.array([[[2, 1, 2], [1, 0, 1]]], dtype=np.int8)
    sv = np.array([[[2, 2, 1], [2, 0, 2]]], dtype=np.int8)
    pk, pv, _ = orc.compress_kv(K, V, state_k=sk, state_v=sv)
    assert pv.f16[0, 0].tolist() == [True, False, True]
    for p, dense_fn, sparse_fn in ((pk, hl.k_dense_physical, hl.k_sparse_physical), (pv, hl.v_dense_physical, hl.v_sparse_physical)):
        ph = hl.physical_pools(p)
        for h in range(2):
            for t in range(3):
                m = int(p.map[0, h, t])
                if m > 0:
                    assert (ph["dense"][0, h, m - 1] == dense_fn(p.dense[0, h, m - 1])).all()
                elif m < 0:
                    n, e = sparse_fn(p.nnz[0, h, -m - 1], p.meta[0, h, -m - 1])
                    assert (ph["nnz"][0, h, -m - 1] == n).all() and (ph["meta"][0, h, -m - 1] == e).all()
        assert ph["n_dense"].tolist() == (p.map > 0).sum(-1).tolist() and ph["n_sparse"].tolist() == (p.map < 0).sum(-1).tolist()
    # the fp16-encoded 2:4 V tile decodes, through the emulated GEMM2 read as fp16, to the same values
    ph = hl.physical_pools(pv)
    n16 = np.ascontiguousarray(ph["nnz"][0, 0, 0]).view(np.float16).astype(np.float32)
    as_bf16_bytes = wl.f32_to_bf16_bits(n16).view(np.uint8)            # exact: these values fit both formats
    Vt = _f(np.where(orc.element_mask_v(V[:1, :1, :64])[0, 0], V[0, 0, :64], 0))
    assert (vt_times_pt_sparse(as_bf16_bytes, ph["meta"][0, 0, 0], np.eye(64)) == Vt.T).all()
