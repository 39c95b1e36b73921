"""Oracle-side statement of the in-tile byte order of the packed pools.

TEST INFRASTRUCTURE ONLY (see hs_oracle.py).  The canonical logical form (values
in position order + one nibble per group) is what hs_oracle.pack_* produces; the
library stores each tile in the order in which the lanes of the gfx950 matrix
instructions consume it.  This module derives that order from the instruction
semantics alone, independently of the library's index arithmetic:

  dense  16x16x32: A lane l = row l%16, k = 8*(l//16) + e   (e = 0..7)
                   B lane l = col l%16, k = 8*(l//16) + e
                   D lane l = col l%16, rows 4*(l//16) + i   (i = 0..3)
  sparse 16x16x64: A lane l = row l%16, the kept values of k in [16*(l//16), +16)
                   B lane l = col l%16, k = 32*(e//8) + 8*(l//16) + e%8  (e = 0..15)
                   index: 2 bits per kept value, value e at bits 2e of a 16-bit half;
                   a lane keeps the four 32-bit index words of a tile side by side (16 B)

GEMM1 (S^T = K Q^T) has tokens as rows: its D registers hold, for lane group a,
tokens 16m + 4a + i of row block m.  GEMM2 (O^T = V^T P^T) contracts over tokens
and takes those registers, unmoved, as its B operand, element 4m + i.  That
fixes which token each contraction index of GEMM2 means, hence V's token order.

Pins (tests/test_oracle_layout_pins.py, CPU only): an emulation of the two matrix
instructions, written in the test from the operand semantics above, reads the
physical bytes chunk by chunk and must reproduce K~ Q^T and V~^T P^T of the
canonical tile (exact integer data, equality); every order is shown to be a
permutation; TOKEN_OF_K is re-derived from the lane maps; planted slips (chunk
order, lane order, index halves, nibble order, token order) turn the checks red.
No function here is "parity unpinned".
"""
import numpy as np


def _gemm2_token_of_k():
    """token_of_k[k] for the 64 contraction indices of GEMM2 (sparse B layout)."""
    tok = np.full(64, -1, dtype=np.int64)
    for a in range(4):            # lane group
        for m in range(4):        # row block of GEMM1
            for i in range(4):    # D register
                e = 4 * m + i     # B element of GEMM2
                k = 32 * (e // 8) + 8 * a + e % 8
                tok[k] = 16 * m + 4 * a + i
    assert sorted(tok.tolist()) == list(range(64))
    return tok


TOKEN_OF_K = _gemm2_token_of_k()


def k_sparse_physical(nnz, meta):
    """Canonical K tile (nnz [64, 64] u16, meta [64, 4] u32) -> (nnz bytes [8192], meta bytes [1024])."""
    out = np.zeros((4, 2, 64, 8), dtype=np.uint16)
    om = np.zeros((64, 4), dtype=np.uint32)             # lane-major: lane l owns words m = 0..3
    halves = meta.view(np.uint16).reshape(64, 8)        # 16-bit half h covers groups 4h..4h+3
    for m in range(4):
        for l in range(64):
            a, r = l // 16, l % 16
            tok = 16 * m + r
            for kb in range(2):
                # uncompressed channels 64kb + 16a .. +15 -> kept elements 32kb + 8a .. +7
                out[m, kb, l] = nnz[tok, 32 * kb + 8 * a: 32 * kb + 8 * a + 8]
                om[l, m] |= np.uint32(halves[tok, 4 * kb + a]) << np.uint32(16 * kb)
    return out.reshape(-1).view(np.uint8), om.reshape(-1).view(np.uint8)


def v_sparse_physical(nnz, meta):
    """Canonical V tile (nnz [16, 2, 128] u16, meta [16, 16] u32) -> physical bytes."""
    out = np.zeros((8, 64, 8), dtype=np.uint16)
    om = np.zeros((64, 4), dtype=np.uint32)             # lane-major: lane l owns words mb//2 = 0..3
    nib = (meta[:, :, None] >> (4 * np.arange(8, dtype=np.uint32))) & np.uint32(0xF)
    nib = nib.reshape(16, 128)                          # [token group, channel]
    for mb in range(8):
        for l in range(64):
            a, r = l // 16, l % 16
            c = 16 * mb + r
            for q in range(4):
                g = TOKEN_OF_K[16 * a + 4 * q] // 4     # token group of contraction indices 16a+4q..+3
                assert (TOKEN_OF_K[16 * a + 4 * q: 16 * a + 4 * q + 4] == 4 * g + np.arange(4)).all()
                out[mb, l, 2 * q] = nnz[g, 0, c]
                out[mb, l, 2 * q + 1] = nnz[g, 1, c]
                om[l, mb // 2] |= np.uint32(nib[g, c]) << np.uint32(16 * (mb % 2) + 4 * q)
    return out.reshape(-1).view(np.uint8), om.reshape(-1).view(np.uint8)


def k_dense_physical(tile):
    """K tile [64, 128] u16 -> bytes [16384] in dense A-operand order."""
    out = np.zeros((4, 4, 64, 8), dtype=np.uint16)
    for m in range(4):
        for s in range(4):
            for l in range(64):
                a, r = l // 16, l % 16
                out[m, s, l] = tile[16 * m + r, 32 * s + 8 * a: 32 * s + 8 * a + 8]
    return out.reshape(-1).view(np.uint8)


def v_dense_physical(tile):
    """V tile [64, 128] u16 -> bytes [16384]: A operand of the dense GEMM2 steps h = 0, 1,
    contraction index k = 32h + 8a + e."""
    out = np.zeros((8, 2, 64, 8), dtype=np.uint16)
    for mb in range(8):
        for h in range(2):
            for l in range(64):
                a, r = l // 16, l % 16
                for e in range(8):
                    out[mb, h, l, e] = tile[TOKEN_OF_K[32 * h + 8 * a + e], 16 * mb + r]
    return out.reshape(-1).view(np.uint8)


def physical_pools(p):
    """PackedKV (canonical) -> dict of uint8 arrays shaped like the library's pools:
    dense [B, Hkv, cap_d, 16384], nnz [B, Hkv, cap_s, 8192], meta [B, Hkv, cap_s, 1024].
    Only used slots are filled (others zero); `used` gives the per-row counts."""
    B, H, T = p.map.shape
    nd = (p.map > 0).sum(-1)
    ns = (p.map < 0).sum(-1)
    dense = np.zeros((B, H, max(1, int(nd.max())), 16384), dtype=np.uint8)
    nnz = np.zeros((B, H, max(1, int(ns.max())), 8192), dtype=np.uint8)
    meta = np.zeros((B, H, max(1, int(ns.max())), 1024), dtype=np.uint8)
    for b in range(B):
        for h in range(H):
            for s in range(int(nd[b, h])):
                dense[b, h, s] = (k_dense_physical if p.kind == "k" else v_dense_physical)(p.dense[b, h, s])
            for s in range(int(ns[b, h])):
                f = k_sparse_physical if p.kind == "k" else v_sparse_physical
                nnz[b, h, s], meta[b, h, s] = f(p.nnz[b, h, s], p.meta[b, h, s])
    return dict(dense=dense, nnz=nnz, meta=meta, n_dense=nd, n_sparse=ns)
