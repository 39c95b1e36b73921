"""Plain, slow, obviously-correct CPU oracle for HieraSparse (numpy, fp64).

TEST INFRASTRUCTURE ONLY -- the product path never imports this module, and this
module imports nothing from the HIP package.

What the method computes (paper Sec. III): the KV cache is cut into blocks of
``Bt`` tokens; each block is stored dense, or pruned 2:4 along the contraction
axis and stored as kept values + 2-bit positions (Sec. III-A, Eq. 2a-b;
Sec. III-B), or -- the extension this build's workloads add -- skipped
altogether.  A signed block index map locates each block in its pool
(Sec. III-B).  Attention over the packed cache (Algorithm 1) is, given the
pruned cache, exactly softmax(Q K~^T / sqrt(d)) V~ (Eq. 1) over the
decompressed, masked K~, V~.  So the oracle is that definition written out:
prune -> pack -> unpack -> plain attention, all in fp64 on the exact values of
the bf16 inputs.

Pins (tests/test_oracle_pins.py; tests/test_oracle_layout_pins.py for hs_layout): top-2-of-4 invariants over exhaustive small
alphabets; pack/unpack bit-exact round trip; pool byte counts and compression
ratios printed in Sec. III-D; attention special cases against an independent
library routine (all-dense, masked, token-deleted); decode == last causal row;
brute force in Python floats on tiny shapes; exact rational tile ranking.
No function here is "parity unpinned".

All tensors are numpy arrays.  bf16 tensors are carried as uint16 bit patterns.
Shapes: K, V [B, Hkv, L, D]; Q prefill [B, Hq, Lq, D]; q decode [B, Hq, D].
Tile states: 0 = SKIP, 1 = DENSE, 2 = SPARSE24.
"""
import numpy as np

SKIP, DENSE, SPARSE24 = 0, 1, 2

def map_slot(entry):
    """Pool slot (0-based) named by a non-zero entry of the signed block index map (Sec. III-B)."""
    return abs(int(entry)) - 1


# ----------------------------------------------------------------------------
# 16-bit patterns <-> real numbers
# ----------------------------------------------------------------------------
def bf16_to_f64(bits):
    """Exact value of bf16 bit patterns (uint16) as float64."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def bf16_bits_exact_in_f16(bits):
    """Elementwise: the bf16 value is a finite number (or an infinity) that IEEE fp16 holds exactly."""
    v = (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    with np.errstate(over="ignore"):
        h = v.astype(np.float16)
    return h.astype(np.float32) == v            # NaN compares unequal: stays bf16


def bf16_bits_to_f16_bits(bits):
    v = (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    with np.errstate(over="ignore"):
        return v.astype(np.float16).view(np.uint16)


def f16_bits_to_bf16_bits(bits):
    """Exact for every value that bf16_bits_exact_in_f16 let through."""
    v = np.ascontiguousarray(np.asarray(bits, dtype=np.uint16)).view(np.float16).astype(np.float32)
    return (v.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def to_f64(bits, dtype="bf16"):
    """Exact value of 16-bit patterns: "bf16", or "fp16" = IEEE binary16 (the paper's type)."""
    if dtype == "fp16":
        return np.ascontiguousarray(np.asarray(bits, dtype=np.uint16)).view(np.float16).astype(np.float64)
    assert dtype == "bf16"
    return bf16_to_f64(bits)


# ----------------------------------------------------------------------------
# element-level 2:4 mask (Sec. III-A, Eq. 2a-b; fused top-2 form of Sec. IV-B)
# ----------------------------------------------------------------------------
def _top2_of_4(bits_g, rule="magnitude"):
    """bits_g: uint16 [..., 4].  Boolean keep mask with exactly two True per group.

    Order is by magnitude, i.e. by the integer (bits & 0x7FFF), descending; equal
    magnitudes are resolved in favour of the lower position, so that exactly two
    survive (Eq. 2b would keep more than two on ties, which the 2:4 format cannot
    store).

    rule "nonzero" is the generic compressor of Sec. IV-B for input that already carries an
    element mask (pruned entries are zero): the key is "is non-zero", so the non-zero entries
    are kept and a group with fewer than two of them is filled up with its leftmost zeros.
    """
    key = (bits_g & np.uint16(0x7FFF)).astype(np.int32)
    if rule == "nonzero":
        key = (key != 0).astype(np.int32)
    else:
        assert rule == "magnitude"
    pos = np.arange(4, dtype=np.int32)
    # beats[..., i, j] = element j is ranked ahead of element i
    ki = key[..., :, None]
    kj = key[..., None, :]
    beats = (kj > ki) | ((kj == ki) & (pos[None, :] < pos[:, None]))
    rank = beats.sum(axis=-1)
    return rank < 2


def element_mask_k(K_bits, rule="magnitude"):
    """K is the sparse operand of S^T = K Q^T, contraction over channels: groups
    are 4 consecutive channels of one token (Sec. III-C, Table II)."""
    K_bits = np.asarray(K_bits, dtype=np.uint16)
    B, H, L, D = K_bits.shape
    assert D % 4 == 0
    m = _top2_of_4(K_bits.reshape(B, H, L, D // 4, 4), rule)
    return m.reshape(B, H, L, D)


def element_mask_v(V_bits, rule="magnitude"):
    """V^T is the sparse operand of O^T = V^T P^T, contraction over tokens: groups
    are 4 consecutive tokens of one channel (Sec. III-C, Table II)."""
    V_bits = np.asarray(V_bits, dtype=np.uint16)
    B, H, L, D = V_bits.shape
    assert L % 4 == 0
    g = V_bits.reshape(B, H, L // 4, 4, D).transpose(0, 1, 2, 4, 3)  # [..., L/4, D, 4]
    m = _top2_of_4(g, rule)
    return m.transpose(0, 1, 2, 4, 3).reshape(B, H, L, D)


# ----------------------------------------------------------------------------
# block-level decisions (Sec. III-A Eq. 2c-d; skip = workload extension)
# ----------------------------------------------------------------------------
def tile_energy(K_bits, V_bits, Bt, dtype="bf16"):
    """Skip score per tile: sum of squares of the tile's K and V entries (the
    squared joint L2 norm), accumulated in fp64.  [B, Hkv, T]."""
    K = to_f64(K_bits, dtype)
    V = to_f64(V_bits, dtype)
    B, H, L, D = K.shape
    T = L // Bt
    e = (K * K).reshape(B, H, T, Bt * D).sum(axis=-1) + (V * V).reshape(B, H, T, Bt * D).sum(axis=-1)
    return e


def tile_prune_loss(X_bits, mask, Bt, dtype="bf16"):
    """Eq. 2c: L1 norm of what the element mask removes, per block.  [B, Hkv, T]."""
    X = np.abs(to_f64(X_bits, dtype)) * (~mask)
    B, H, L, D = X.shape
    return X.reshape(B, H, L // Bt, Bt * D).sum(axis=-1)


def _lowest(scores_row, n, eligible):
    """Indices of the n eligible tiles with the lowest score; ties -> lower index."""
    idx = [t for t in range(len(scores_row)) if eligible[t]]
    idx.sort(key=lambda t: (scores_row[t], t))
    return idx[:n]


def select_states(energy, loss_k, loss_v, skip_frac, sparse_frac_k, sparse_frac_v, dense_first=0, dense_last=0):
    """Tile states for K and V, per (b, hkv) row.

    The first dense_first and the last dense_last tiles stay DENSE and take no part in any
    ranking (the sink / local-window tokens the paper's evaluation keeps dense, Sec. V-A).
    Of the T_mid tiles in between, n_skip = floor(skip_frac * T_mid) lowest-energy ones are
    SKIP for both tensors; of the remaining n_keep, floor(sparse_frac_x * n_keep) with the
    lowest pruning loss (Eq. 2c-d) become SPARSE24, the rest stay DENSE.
    Returns (state_k, state_v) int8 [B, Hkv, T].
    """
    B, H, T = energy.shape
    sk = np.full((B, H, T), DENSE, dtype=np.int8)
    sv = np.full((B, H, T), DENSE, dtype=np.int8)
    dense_first = min(dense_first, T)
    dense_last = min(dense_last, T - dense_first)
    mid = [dense_first <= t < T - dense_last for t in range(T)]
    n_mid = sum(mid)
    n_skip = int(np.floor(skip_frac * n_mid))
    for b in range(B):
        for h in range(H):
            skipped = _lowest(energy[b, h], n_skip, mid)
            kept = list(mid)
            for t in skipped:
                kept[t] = False
                sk[b, h, t] = SKIP
                sv[b, h, t] = SKIP
            n_keep = n_mid - n_skip
            for st, loss, frac in ((sk, loss_k, sparse_frac_k), (sv, loss_v, sparse_frac_v)):
                n_sp = int(np.floor(frac * n_keep))
                for t in _lowest(loss[b, h], n_sp, kept):
                    st[b, h, t] = SPARSE24
    return sk, sv


def build_map(state):
    """Signed block index map (Sec. III-B): walking the blocks in sequence order
    with one counter per pool, a dense block gets +(slot+1), a sparse block
    -(slot+1); 0 marks a skipped block.  int32 [B, Hkv, T]."""
    B, H, T = state.shape
    mp = np.zeros((B, H, T), dtype=np.int32)
    for b in range(B):
        for h in range(H):
            nd = ns = 0
            for t in range(T):
                if state[b, h, t] == DENSE:
                    nd += 1
                    mp[b, h, t] = nd
                elif state[b, h, t] == SPARSE24:
                    ns += 1
                    mp[b, h, t] = -ns
    return mp


# ----------------------------------------------------------------------------
# pack / unpack in the canonical logical layout (Sec. III-B, Sec. IV-B)
# ----------------------------------------------------------------------------
def _nibbles_to_words(nib):
    """nib: uint32 [..., n] -> uint32 [..., ceil(n/8)], nibble g in bits 4*(g%8) of
    word g//8 (a short last word is zero-filled)."""
    n = nib.shape[-1]
    if n % 8:
        pad = np.zeros(nib.shape[:-1] + (8 - n % 8,), dtype=nib.dtype)
        nib = np.concatenate([nib, pad], axis=-1)
        n = nib.shape[-1]
    w = nib.reshape(nib.shape[:-1] + (n // 8, 8)).astype(np.uint32)
    sh = (4 * np.arange(8, dtype=np.uint32))
    return (w << sh).sum(axis=-1).astype(np.uint32)


def _words_to_nibbles(words):
    sh = (4 * np.arange(8, dtype=np.uint32))
    nib = (words[..., None] >> sh) & np.uint32(0xF)
    return nib.reshape(words.shape[:-1] + (words.shape[-1] * 8,))


def _compress_groups(bits_g, mask_g):
    """bits_g, mask_g: [..., 4] with exactly two kept per group.
    Returns (vals [..., 2] uint16 in ascending position order, nibble [...] uint32
    = i0 | i1 << 2)."""
    pos = np.arange(4)
    # positions of the two kept entries, ascending
    order = np.argsort(np.where(mask_g, pos, pos + 4), axis=-1, kind="stable")
    i0 = order[..., 0]
    i1 = order[..., 1]
    v0 = np.take_along_axis(bits_g, i0[..., None], axis=-1)[..., 0]
    v1 = np.take_along_axis(bits_g, i1[..., None], axis=-1)[..., 0]
    vals = np.stack([v0, v1], axis=-1).astype(np.uint16)
    nib = (i0 | (i1 << 2)).astype(np.uint32)
    return vals, nib


def pack_k_tile(tile_bits, tile_mask):
    """One K tile [Bt, D] -> nnz [Bt, D/2] uint16, meta [Bt, ceil(D/32)] uint32."""
    Bt, D = tile_bits.shape
    vals, nib = _compress_groups(tile_bits.reshape(Bt, D // 4, 4), tile_mask.reshape(Bt, D // 4, 4))
    return vals.reshape(Bt, D // 2), _nibbles_to_words(nib)


def pack_v_tile(tile_bits, tile_mask):
    """One V tile [Bt, D] -> nnz [Bt/4, 2, D] uint16, meta [Bt/4, D/8] uint32
    (one nibble per (token group, channel))."""
    Bt, D = tile_bits.shape
    g = tile_bits.reshape(Bt // 4, 4, D).transpose(0, 2, 1)
    mg = tile_mask.reshape(Bt // 4, 4, D).transpose(0, 2, 1)
    vals, nib = _compress_groups(g, mg)          # [Bt/4, D, 2], [Bt/4, D]
    return vals.transpose(0, 2, 1).copy(), _nibbles_to_words(nib)


def unpack_k_tile(nnz, meta):
    Bt = nnz.shape[0]
    D = nnz.shape[1] * 2
    nib = _words_to_nibbles(meta)[:, : D // 4]
    out = np.zeros((Bt, D // 4, 4), dtype=np.uint16)
    v = nnz.reshape(Bt, D // 4, 2)
    i0 = (nib & 3).astype(np.int64)
    i1 = ((nib >> 2) & 3).astype(np.int64)
    np.put_along_axis(out, i0[..., None], v[..., 0:1], axis=-1)
    np.put_along_axis(out, i1[..., None], v[..., 1:2], axis=-1)
    return out.reshape(Bt, D)


def unpack_v_tile(nnz, meta):
    G, _, D = nnz.shape
    nib = _words_to_nibbles(meta)[:, :D]
    out = np.zeros((G, D, 4), dtype=np.uint16)
    i0 = (nib & 3).astype(np.int64)
    i1 = ((nib >> 2) & 3).astype(np.int64)
    np.put_along_axis(out, i0[..., None], nnz[:, 0, :, None], axis=-1)
    np.put_along_axis(out, i1[..., None], nnz[:, 1, :, None], axis=-1)
    return out.transpose(0, 2, 1).reshape(G * 4, D)


class PackedKV:
    """Canonical packed cache for one tensor (K or V): pools + signed block index map.

    map  int32 [B, Hkv, T]: the paper's map (Sec. III-B): +(slot+1) dense pool, -(slot+1) sparse
         pool, 0 skipped.  Nothing else is folded into it.
    f16  bool [B, Hkv, T]: a separate per-tile predicate, not part of the paper's format: the
         tile's stored values are held in the pool in fp16 encoding (see v_tile_f16).  Always
         False for K and for fp16 caches.
    """

    def __init__(self, kind, Bt, D, mp, dense, nnz, meta, dtype="bf16", f16=None):
        self.kind, self.Bt, self.D, self.dtype = kind, Bt, D, dtype
        self.map, self.dense, self.nnz, self.meta = mp, dense, nnz, meta
        self.f16 = np.zeros(mp.shape, dtype=bool) if f16 is None else f16

    def nbytes(self):
        """Bytes actually occupied (used slots only) + the map."""
        nd = int((self.map > 0).sum())
        ns = int((self.map < 0).sum())
        tile = self.Bt * self.D * 2
        return nd * tile + ns * (tile // 2 + tile // 16) + 4 * self.map.size


def v_tile_f16(stored_bits, v_f16):
    """The encoding predicate of one V tile, from its stored values (all of a dense tile, the kept
    ones of a 2:4 tile): True when the cache is bf16 (v_f16) and every stored value is exact in
    fp16.  Such a tile is kept in fp16 encoding -- the softmax numerators can then enter the
    second product as one fp16 term (11 significant bits) instead of two bf16 terms.  The values
    are the same either way; this is a storage choice of this build, outside the paper's format."""
    return bool(v_f16 and bf16_bits_exact_in_f16(stored_bits).all())


def _v_tile_store(stored_bits, v_f16):
    """(bits to store, encoding predicate) of one V tile."""
    if v_tile_f16(stored_bits, v_f16):
        return bf16_bits_to_f16_bits(stored_bits), True
    return stored_bits, False


def pack_tensor(kind, X_bits, mask, state, Bt, v_f16=False):
    """Walk the blocks in sequence order (Sec. III-B) and fill the pools.
    Pools are rectangular [B, Hkv, cap, ...] with cap = the largest per-row count;
    unused slots stay zero.  v_f16: V tensor of a bf16 cache (see _v_tile_store)."""
    X_bits = np.asarray(X_bits, dtype=np.uint16)
    B, H, L, D = X_bits.shape
    T = L // Bt
    mp = build_map(state)
    f16 = np.zeros(mp.shape, dtype=bool)
    cap_d = max(1, int((state == DENSE).sum(axis=-1).max()))
    cap_s = max(1, int((state == SPARSE24).sum(axis=-1).max()))
    dense = np.zeros((B, H, cap_d, Bt, D), dtype=np.uint16)
    if kind == "k":
        nnz = np.zeros((B, H, cap_s, Bt, D // 2), dtype=np.uint16)
        meta = np.zeros((B, H, cap_s, Bt, (D // 4 + 7) // 8), dtype=np.uint32)
    else:
        nnz = np.zeros((B, H, cap_s, Bt // 4, 2, D), dtype=np.uint16)
        meta = np.zeros((B, H, cap_s, Bt // 4, (D + 7) // 8), dtype=np.uint32)
    for b in range(B):
        for h in range(H):
            for t in range(T):
                m = mp[b, h, t]
                tile = X_bits[b, h, t * Bt:(t + 1) * Bt]
                if m > 0:
                    if kind == "v":
                        dense[b, h, m - 1], f16[b, h, t] = _v_tile_store(tile, v_f16)
                    else:
                        dense[b, h, m - 1] = tile
                elif m < 0:
                    tm = mask[b, h, t * Bt:(t + 1) * Bt]
                    if kind == "k":
                        nnz[b, h, -m - 1], meta[b, h, -m - 1] = pack_k_tile(tile, tm)
                    else:
                        vals, meta[b, h, -m - 1] = pack_v_tile(tile, tm)
                        nnz[b, h, -m - 1], f16[b, h, t] = _v_tile_store(vals, v_f16)
    return PackedKV(kind, Bt, D, mp, dense, nnz, meta, f16=f16)


def append_tile(pk, pv, tile, K_tile_bits, V_tile_bits, state_k, state_v, element_rule="magnitude"):
    """Fill tile `tile` of a cache whose pools grow during decode (Sec. III-B: blocks are handed
    to the dense or the sparse pool in sequence order, one counter per pool).  The tile must be
    SKIP (not filled yet) in every row; it takes the next slot of its pool, i.e. the number of
    tiles of the same kind the row already holds.  K_tile_bits, V_tile_bits: [B, Hkv, Bt, D];
    state_k, state_v: DENSE or SPARSE24, the same for every row.  Works in place.
    tile: one index, or one per batch row (sequences of a batch differ in length; a negative
    entry leaves that batch row as it is)."""
    K_tile_bits = np.asarray(K_tile_bits, dtype=np.uint16)
    V_tile_bits = np.asarray(V_tile_bits, dtype=np.uint16)
    B, H, Bt, D = K_tile_bits.shape
    assert Bt == pk.Bt and state_k in (DENSE, SPARSE24) and state_v in (DENSE, SPARSE24)
    masks = (element_mask_k(K_tile_bits, element_rule), element_mask_v(V_tile_bits, element_rule))
    tiles = np.broadcast_to(np.asarray(tile, dtype=np.int64), (B,))
    for p, X, mask, state in ((pk, K_tile_bits, masks[0], state_k), (pv, V_tile_bits, masks[1], state_v)):
        for b in range(B):
            t_b = int(tiles[b])
            if t_b < 0:
                continue
            assert (p.map[b, :, t_b] == 0).all()
            for h in range(H):
                v_f16 = p.kind == "v" and p.dtype == "bf16"
                if state == DENSE:
                    slot = int((p.map[b, h] > 0).sum())
                    if slot >= p.dense.shape[2]:
                        p.dense = np.concatenate([p.dense, np.zeros_like(p.dense[:, :, :1])], axis=2)
                    p.dense[b, h, slot], p.f16[b, h, t_b] = _v_tile_store(X[b, h], v_f16)
                    p.map[b, h, t_b] = slot + 1
                else:
                    slot = int((p.map[b, h] < 0).sum())
                    if slot >= p.nnz.shape[2]:
                        p.nnz = np.concatenate([p.nnz, np.zeros_like(p.nnz[:, :, :1])], axis=2)
                        p.meta = np.concatenate([p.meta, np.zeros_like(p.meta[:, :, :1])], axis=2)
                    pack = pack_k_tile if p.kind == "k" else pack_v_tile
                    vals, p.meta[b, h, slot] = pack(X[b, h], mask[b, h])
                    p.nnz[b, h, slot], p.f16[b, h, t_b] = _v_tile_store(vals, v_f16)
                    p.map[b, h, t_b] = -(slot + 1)


def _sparser(cur, target):
    """Tile state after further pruning: a tile only ever moves DENSE -> SPARSE24 -> SKIP."""
    order = {DENSE: 0, SPARSE24: 1, SKIP: 2}
    return cur if order[cur] >= order[target] else target


def recompress(p, target_state, element_rule="magnitude"):
    """Prune a packed tensor further (Sec. III, overview: after the prefill phase the dense pool
    can be pruned and compressed again, so that decode runs at another sparsity than prefill).
    target_state: [B, Hkv, T] of SKIP / DENSE / SPARSE24.  A tile ends in the sparser of its
    current and its target state: a tile that keeps its kind keeps its stored bits (and its
    encoding); a DENSE tile that becomes SPARSE24 is pruned from the values it stores; a tile that
    becomes SKIP is dropped.  Pools are refilled in sequence order (Sec. III-B).  Returns a new
    PackedKV; `p` is left as it is."""
    B, H, T = p.map.shape
    target_state = np.asarray(target_state)
    assert target_state.shape == (B, H, T)
    cur = np.where(p.map > 0, DENSE, np.where(p.map < 0, SPARSE24, SKIP)).astype(np.int8)
    new = np.array([[[_sparser(int(cur[b, h, t]), int(target_state[b, h, t])) for t in range(T)]
                     for h in range(H)] for b in range(B)], dtype=np.int8).reshape(B, H, T)
    mp = build_map(new)
    f16 = np.zeros(mp.shape, dtype=bool)
    cap_d = max(1, int((new == DENSE).sum(axis=-1).max()))
    cap_s = max(1, int((new == SPARSE24).sum(axis=-1).max()))
    dense = np.zeros((B, H, cap_d) + p.dense.shape[3:], dtype=np.uint16)
    nnz = np.zeros((B, H, cap_s) + p.nnz.shape[3:], dtype=np.uint16)
    meta = np.zeros((B, H, cap_s) + p.meta.shape[3:], dtype=np.uint32)
    v_f16 = p.kind == "v" and p.dtype == "bf16"
    for b in range(B):
        for h in range(H):
            for t in range(T):
                m_old, m = int(p.map[b, h, t]), int(mp[b, h, t])
                if m == 0:
                    continue
                old_slot, old_flag = map_slot(m_old), bool(p.f16[b, h, t])
                if m > 0:                                   # DENSE stays DENSE
                    dense[b, h, m - 1] = p.dense[b, h, old_slot]
                    f16[b, h, t] = old_flag
                elif m_old < 0:                             # SPARSE24 stays SPARSE24
                    nnz[b, h, -m - 1] = p.nnz[b, h, old_slot]
                    meta[b, h, -m - 1] = p.meta[b, h, old_slot]
                    f16[b, h, t] = old_flag
                else:                                       # DENSE -> SPARSE24: prune what is stored
                    tile = p.dense[b, h, old_slot]
                    if old_flag:
                        tile = f16_bits_to_bf16_bits(tile)
                    if p.kind == "k":
                        tm = element_mask_k(tile[None, None], element_rule)[0, 0]
                        nnz[b, h, -m - 1], meta[b, h, -m - 1] = pack_k_tile(tile, tm)
                    else:
                        tm = element_mask_v(tile[None, None], element_rule)[0, 0]
                        vals, meta[b, h, -m - 1] = pack_v_tile(tile, tm)
                        nnz[b, h, -m - 1], f16[b, h, t] = _v_tile_store(vals, v_f16)
    return PackedKV(p.kind, p.Bt, p.D, mp, dense, nnz, meta, dtype=p.dtype, f16=f16)


def fit_states_to_capacity(state_k, state_v, caps):
    """Walk the blocks of every row in sequence order with the pools' running counters
    (Sec. III-B): a block is stored only if the pool its K state names and the pool its V state
    names both still have a free slot; otherwise it is left out of K and V alike and takes no
    slot.  caps = (dense K, sparse K, dense V, sparse V) slots per row.  Returns the states that
    are actually stored and whether anything was left out."""
    sk, sv = np.array(state_k, dtype=np.int8), np.array(state_v, dtype=np.int8)
    B, H, T = sk.shape
    dropped = False
    for b in range(B):
        for h in range(H):
            n = {("k", DENSE): 0, ("k", SPARSE24): 0, ("v", DENSE): 0, ("v", SPARSE24): 0}
            cap = {("k", DENSE): caps[0], ("k", SPARSE24): caps[1], ("v", DENSE): caps[2], ("v", SPARSE24): caps[3]}
            for t in range(T):
                a, c = int(sk[b, h, t]), int(sv[b, h, t])
                if a == SKIP:
                    continue
                if n["k", a] < cap["k", a] and n["v", c] < cap["v", c]:
                    n["k", a] += 1
                    n["v", c] += 1
                else:
                    sk[b, h, t] = sv[b, h, t] = SKIP
                    dropped = True
    return sk, sv, dropped


def recompress_kv(pk, pv, target_k, target_v, element_rule="magnitude", caps=None):
    """recompress for K and V together; a tile is dropped from both or from neither.
    caps: optional pool capacities of the result (see fit_states_to_capacity); then the third
    return value says whether a tile was left out for lack of room."""
    target_k, target_v = np.asarray(target_k), np.asarray(target_v)
    assert ((target_k == SKIP) == (target_v == SKIP)).all()
    if caps is None:
        return recompress(pk, target_k, element_rule), recompress(pv, target_v, element_rule)
    cur_k = np.where(pk.map > 0, DENSE, np.where(pk.map < 0, SPARSE24, SKIP))
    cur_v = np.where(pv.map > 0, DENSE, np.where(pv.map < 0, SPARSE24, SKIP))
    merge = np.vectorize(_sparser)
    new_k, new_v, dropped = fit_states_to_capacity(merge(cur_k, target_k), merge(cur_v, target_v), caps)
    return recompress(pk, new_k, element_rule), recompress(pv, new_v, element_rule), dropped


def unpack_tensor(p):
    """Packed -> dense bf16 bits [B, Hkv, L, D] with zeros at pruned positions and
    in skipped tiles."""
    B, H, T = p.map.shape
    out = np.zeros((B, H, T * p.Bt, p.D), dtype=np.uint16)
    for b in range(B):
        for h in range(H):
            for t in range(T):
                m = p.map[b, h, t]
                if m == 0:
                    continue
                slot = map_slot(m)
                back = f16_bits_to_bf16_bits if p.f16[b, h, t] else (lambda x: x)
                if m > 0:
                    out[b, h, t * p.Bt:(t + 1) * p.Bt] = back(p.dense[b, h, slot])
                elif p.kind == "k":
                    out[b, h, t * p.Bt:(t + 1) * p.Bt] = unpack_k_tile(p.nnz[b, h, slot], p.meta[b, h, slot])
                else:
                    out[b, h, t * p.Bt:(t + 1) * p.Bt] = unpack_v_tile(back(p.nnz[b, h, slot]), p.meta[b, h, slot])
    return out


def compress_kv(K_bits, V_bits, Bt=64, skip_frac=0.0, sparse_frac_k=1.0, sparse_frac_v=1.0,
                state_k=None, state_v=None, dense_first_tiles=0, dense_last_tiles=0, element_rule="magnitude",
                dtype="bf16", caps=None):
    """Whole compress step: element masks, tile states (policy or explicit),
    maps, pools.  Returns (PackedKV for K, PackedKV for V, dict of intermediates).
    dtype names the 16-bit format of the patterns; it matters for the tile scores and for
    attention, not for the element masks (the magnitude order is the order of bits & 0x7fff in
    both formats) nor for the packing (bits are copied)."""
    K_bits = np.asarray(K_bits, dtype=np.uint16)
    V_bits = np.asarray(V_bits, dtype=np.uint16)
    mk = element_mask_k(K_bits, element_rule)
    mv = element_mask_v(V_bits, element_rule)
    info = {"mask_k": mk, "mask_v": mv}
    if state_k is None:
        energy = tile_energy(K_bits, V_bits, Bt, dtype)
        loss_k = tile_prune_loss(K_bits, mk, Bt, dtype)
        loss_v = tile_prune_loss(V_bits, mv, Bt, dtype)
        state_k, state_v = select_states(energy, loss_k, loss_v, skip_frac, sparse_frac_k, sparse_frac_v,
                                         dense_first_tiles, dense_last_tiles)
        info.update(energy=energy, loss_k=loss_k, loss_v=loss_v)
    state_k = np.asarray(state_k, dtype=np.int8)
    state_v = np.asarray(state_v, dtype=np.int8)
    assert ((state_k == SKIP) == (state_v == SKIP)).all(), "a skipped tile removes its tokens from K and V alike"
    if caps is not None:     # pools of a given size: blocks that find no free slot are left out (Sec. III-B counters)
        state_k, state_v, info["dropped"] = fit_states_to_capacity(state_k, state_v, caps)
    info.update(state_k=state_k, state_v=state_v)
    pk = pack_tensor("k", K_bits, mk, state_k, Bt)
    pv = pack_tensor("v", V_bits, mv, state_v, Bt, v_f16=(dtype == "bf16"))
    pk.dtype = pv.dtype = dtype
    return pk, pv, info


# ----------------------------------------------------------------------------
# attention (Eq. 1) over the decompressed cache
# ----------------------------------------------------------------------------
def _softmax_av(s, Vt):
    """s [n] fp64 scores of the visible tokens, Vt [n, D].  Returns (o [D], lse)."""
    if s.size == 0:
        return np.zeros(Vt.shape[1], dtype=np.float64), -np.inf
    m = s.max()
    p = np.exp(s - m)
    l = p.sum()
    return (p @ Vt) / l, m + np.log(l)


def attention_rows(Q_bits, pk, pv, rows, causal, scale=None, q_offset=None):
    """Attention for selected query rows.

    Q_bits [B, Hq, Lq, D]; rows = iterable of (b, hq, i).  Query i sees token j
    iff j's tile is not SKIP and (not causal or j <= i + q_offset), with
    q_offset = L - Lq by default.  Returns (O [n, D] fp64, LSE [n] fp64);
    a row that sees nothing has O = 0, LSE = -inf.
    """
    Q_bits = np.asarray(Q_bits, dtype=np.uint16)
    B, Hq, Lq, D = Q_bits.shape
    Hkv = pk.map.shape[1]
    G = Hq // Hkv
    L = pk.map.shape[2] * pk.Bt
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    if q_offset is None:
        q_offset = L - Lq
    Kd = to_f64(unpack_tensor(pk), pk.dtype)
    Vd = to_f64(unpack_tensor(pv), pk.dtype)
    tok_visible = np.repeat(pk.map != 0, pk.Bt, axis=-1)       # [B, Hkv, L]
    rows = list(rows)
    O = np.zeros((len(rows), D), dtype=np.float64)
    LSE = np.zeros(len(rows), dtype=np.float64)
    for n, (b, hq, i) in enumerate(rows):
        h = hq // G
        vis = tok_visible[b, h].copy()
        if causal:
            vis[i + q_offset + 1:] = False
        q = to_f64(Q_bits[b, hq, i], pk.dtype)
        s = (Kd[b, h][vis] @ q) * scale
        O[n], LSE[n] = _softmax_av(s, Vd[b, h][vis])
    return O, LSE


def attention_decode(q_bits, pk, pv, scale=None, tail_k=None, tail_v=None, tail_len=0):
    """One new query token per (b, hq) against the whole cache.  q_bits [B, Hq, D].
    Returns (O [B, Hq, D] fp64, LSE [B, Hq] fp64).

    tail_k, tail_v (bf16 bits [B, Hkv, >= tail_len, D]): recent tokens that are not in the
    packed cache yet; they are kept as they are (the local window stays dense, Sec. V-A)
    and the query sees the first tail_len of them after the cache.  tail_len: one number, or
    one per batch row (sequences of a batch differ in length).
    """
    q_bits = np.asarray(q_bits, dtype=np.uint16)
    B, Hq, D = q_bits.shape
    tail_lens = np.broadcast_to(np.asarray(tail_len, dtype=np.int64), (B,))
    if not tail_lens.any():
        rows = [(b, h, 0) for b in range(B) for h in range(Hq)]
        O, LSE = attention_rows(q_bits[:, :, None, :], pk, pv, rows, causal=False, scale=scale)
        return O.reshape(B, Hq, D), LSE.reshape(B, Hq)
    Hkv = pk.map.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    Kd = to_f64(unpack_tensor(pk), pk.dtype)
    Vd = to_f64(unpack_tensor(pv), pk.dtype)
    Kt = to_f64(np.asarray(tail_k, dtype=np.uint16), pk.dtype)
    Vt = to_f64(np.asarray(tail_v, dtype=np.uint16), pk.dtype)
    tok_visible = np.repeat(pk.map != 0, pk.Bt, axis=-1)
    O = np.zeros((B, Hq, D), dtype=np.float64)
    LSE = np.zeros((B, Hq), dtype=np.float64)
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            vis = tok_visible[b, h]
            n = int(tail_lens[b])
            Kall = np.concatenate([Kd[b, h][vis], Kt[b, h, :n]], axis=0)
            Vall = np.concatenate([Vd[b, h][vis], Vt[b, h, :n]], axis=0)
            s = (Kall @ to_f64(q_bits[b, hq], pk.dtype)) * scale
            O[b, hq], LSE[b, hq] = _softmax_av(s, Vall)
    return O, LSE


# ----------------------------------------------------------------------------
# analytical model (Sec. III-D)
# ----------------------------------------------------------------------------
def compression_ratio(S_K, S_V, Bt=None, D=None):
    """r_comp of Sec. III-D; the 1/(B*D) index term is included when Bt, D are given."""
    idx = 0.0 if Bt is None else 1.0 / (Bt * D)
    return 1.0 / (1.0 - 0.21875 * (S_K + S_V) + idx)


def ideal_prefill_speedup(S_K, S_V):
    return 4.0 / (4.0 - (S_K + S_V))


def ideal_decode_speedup(S_K, S_V):
    return compression_ratio(S_K, S_V)
