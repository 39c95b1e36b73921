// Prefill attention: Algorithm 1 (Trans-Both: S^T = K Q^T, O^T = V^T P^T with K and V^T as
// the first, possibly 2:4-sparse, operand of the matrix instruction) with the mixed
// dense/sparse dispatch of Sec. III-C-2, online softmax, and tile skipping.
//
// Work decomposition: a "slab" is 16 NB consecutive query positions of one query head (NB = 2:
// 32 positions); a wave owns one slab, keeps Q^T (B operand of GEMM1), the running softmax
// state and O^T (128 x 16 NB fp32) in registers for the whole kernel.  The 4 waves of a
// workgroup take 4 consecutive slabs in (position-tile, head-in-group) order, so for a GQA
// group of 4 they are the 4 query heads of one position tile and share every KV tile, which is
// copied once per workgroup into an LDS ring by direct global->LDS loads issued up to 3 tiles
// ahead.  Pools are stored in operand order, so LDS reads are conflict-free 16-byte-per-lane
// reads and GEMM1's accumulators become GEMM2's B operand in place (no re-layout step).
#include <type_traits>

#include "hs_common.h"

// Wave priority per phase.  Two waves share a SIMD; letting the one that is in its vector-ALU
// (softmax) phase issue first measured ~5 % faster than equal priorities or the opposite choice.
#ifndef HS_PRIO_MFMA
#define HS_PRIO_MFMA 0
#define HS_PRIO_VALU 1
#endif


namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  bf2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}

// p0, p1 -> hi = packed bf16 pair (round to nearest even) and lo = packed bf16 pair of the
// remainders p - hi, so that hi + lo reproduces p to ~16 bits.  The remainder is taken with the
// packed dot product hi . (-1, 0) + p0 (resp. (0, -1) + p1): one instruction per element, and
// exact, because bf16 products are exact in fp32 and p - hi is representable.
// The two selector pairs (-1, 0) and (0, -1) are handed in as opaque register values: written
// as literals the compiler folds the first into the inline constant -1.0, which the
// instruction does not read as the bf16 pair (-1, 0).
struct SplitConsts { uint32_t neg_lo, neg_hi; };
__device__ __forceinline__ SplitConsts split_consts() {
  SplitConsts c;
  asm volatile("s_mov_b32 %0, 0x0000bf80\n\ts_mov_b32 %1, 0xbf800000" : "=s"(c.neg_lo), "=s"(c.neg_hi));
  return c;
}
__device__ __forceinline__ void split_hi_lo(float p0, float p1, const SplitConsts& sc, uint32_t& hi, uint32_t& lo) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  hi = pack_bf16(p0, p1);
  const bf2 h = __builtin_bit_cast(bf2, hi);
  const float r0 = __builtin_amdgcn_fdot2_f32_bf16(h, __builtin_bit_cast(bf2, sc.neg_lo), p0, false);
  const float r1 = __builtin_amdgcn_fdot2_f32_bf16(h, __builtin_bit_cast(bf2, sc.neg_hi), p1, false);
  lo = pack_bf16(r0, r1);
}

// LDS staging ring.  One stage holds one tile: a K region then a V region, each 9 KiB (8 KiB of
// values + 1 KiB of metadata) when every tile of that tensor is 2:4 and 16 KiB otherwise.  Two
// workgroups share a compute unit's 160 KiB, so a ring may take 80 KiB: 4 stages when both tensors
// are 2:4 (tiles are requested 3 iterations before use), 3 when one is, 2 otherwise.
template <int KM> constexpr int region_bytes() { return KM == 0 ? 9216 : 16384; }
template <int KM, int VM> constexpr int stage_bytes() { return region_bytes<KM>() + region_bytes<VM>(); }
#ifndef HS_MAX_STAGES
#define HS_MAX_STAGES 4  // at most 2 tiles in flight behind the next one (see stage_wait)
#endif
template <int KM, int VM> constexpr int n_stages() {
  constexpr int fit = 81920 / stage_bytes<KM, VM>();
  return fit < HS_MAX_STAGES ? fit : HS_MAX_STAGES;
}
// fewest direct-to-LDS loads any of the 4 waves issues for one tile (chunks / 4; the metadata
// chunks go to waves 0 and 1 on top of that)
template <int KM, int VM> constexpr int min_loads_per_tile() { return (KM == 1 ? 4 : 2) + (VM == 1 ? 4 : 2); }

typedef __attribute__((address_space(3))) void* lptr_t;

// One direct global->LDS load of 64 lanes x 16 B: lane l's bytes come from gbase + voff (voff = 16 l
// plus the tile's offset in its pool) and land at LDS address lds_addr + IMM + 16 l.  Written as
// inline assembly on purpose: the compiler treats the built-in form as a vector-memory write to LDS
// that any later LDS read may alias, and puts a full vmcnt(0) wait in front of the first such read,
// i.e. right after the prefetch is issued.  Completion is tracked by hand instead (stage_wait +
// workgroup barrier before a stage is read).  gbase and lds_addr are wave-uniform.
template <int IMM>
__device__ __forceinline__ void lds_dma16(uint32_t lds_addr, const uint8_t* gbase, uint32_t voff) {
  asm volatile("s_add_i32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
               :
               : "s"(lds_addr), "i"(IMM), "v"(voff), "s"((uint64_t)gbase)
               : "memory", "m0", "scc");
}

__device__ __forceinline__ const uint8_t* uniform_ptr(const uint8_t* p) {
  const uint64_t g = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)g);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(g >> 32));
  return (const uint8_t*)(((uint64_t)hi << 32) | lo);
}

// Where a wave's copies of a tile come from: the pools of the workgroup's (batch, kv head) row with the
// wave's share of the 1 KiB chunks folded in (value chunk c of a tile goes to wave c % 4), one
// pointer per chunk, so that a tile costs one shift-add for its offset in the pool and nothing
// else per copy.  The per-tile scalar work counts: it is issued by every wave for every tile.
struct TileSrc {
  const uint8_t *k_sp[2], *k_meta, *k_dn[4], *v_sp[2], *v_meta, *v_dn[4];
};
template <int KM, int VM>
__device__ __forceinline__ TileSrc tile_src(const hs_kv_dev& kv, int64_t row, int w) {
  TileSrc s = {};
  if (KM != 1) {
    const uint8_t* b = kv.k_nnz + row * kv.cap_sparse_k * (int64_t)HS_TILE_NNZ_BYTES + w * 1024;
    s.k_sp[0] = uniform_ptr(b);
    s.k_sp[1] = uniform_ptr(b + 4096);
    s.k_meta = uniform_ptr(kv.k_meta + row * kv.cap_sparse_k * (int64_t)HS_TILE_META_BYTES);
  }
  if (KM != 0) {
    const uint8_t* b = kv.k_dense + row * kv.cap_dense_k * (int64_t)HS_TILE_DENSE_BYTES + w * 1024;
#pragma unroll
    for (int i = 0; i < 4; i++) s.k_dn[i] = uniform_ptr(b + 4096 * i);
  }
  if (VM != 1) {
    const uint8_t* b = kv.v_nnz + row * kv.cap_sparse_v * (int64_t)HS_TILE_NNZ_BYTES + w * 1024;
    s.v_sp[0] = uniform_ptr(b);
    s.v_sp[1] = uniform_ptr(b + 4096);
    s.v_meta = uniform_ptr(kv.v_meta + row * kv.cap_sparse_v * (int64_t)HS_TILE_META_BYTES);
  }
  if (VM != 0) {
    const uint8_t* b = kv.v_dense + row * kv.cap_dense_v * (int64_t)HS_TILE_DENSE_BYTES + w * 1024;
#pragma unroll
    for (int i = 0; i < 4; i++) s.v_dn[i] = uniform_ptr(b + 4096 * i);
  }
  return s;
}

// Copy one tile (K and V operands) from its pool slots into an LDS stage: a chunk is 64 lanes x 16 B =
// 1 KiB, stored in the pools in the order the lanes consume it.  The 4 waves share the chunks
// round-robin.  2:4 tile: 8 value chunks + 1 metadata chunk per tensor (value chunks at 0..8 KiB,
// metadata at 8 KiB of the tensor's region); dense: 16 chunks.  stage_w = LDS address of the stage
// + 1024 w.  Offsets inside a row's pool are 32-bit (the launcher checks the pool sizes).
template <int KM, int VM>
__device__ __forceinline__ void stage_issue(uint32_t stage_w, const TileSrc& src, int mk, int mv, int w,
                                            uint32_t lane_off) {
  const bool k_sparse = KM == 0 || (KM == 2 && mk < 0);
  const bool v_sparse = VM == 0 || (VM == 2 && mv < 0);
  constexpr int voff = region_bytes<KM>();
  if (k_sparse) {
    const uint32_t slot = (uint32_t)~mk;  // -mk - 1
    const uint32_t off = lane_off + slot * (uint32_t)HS_TILE_NNZ_BYTES;
    lds_dma16<0>(stage_w, src.k_sp[0], off);
    lds_dma16<4096>(stage_w, src.k_sp[1], off);
    if (w == 0) lds_dma16<8192>(stage_w, src.k_meta, lane_off + slot * (uint32_t)HS_TILE_META_BYTES);
  } else {
    const uint32_t off = lane_off + (uint32_t)(mk - 1) * (uint32_t)HS_TILE_DENSE_BYTES;
    lds_dma16<0>(stage_w, src.k_dn[0], off);
    lds_dma16<4096>(stage_w, src.k_dn[1], off);
    lds_dma16<8192>(stage_w, src.k_dn[2], off);
    lds_dma16<12288>(stage_w, src.k_dn[3], off);
  }
  if (v_sparse) {
    const uint32_t slot = ((uint32_t)(-mv) & 0x3fffffffu) - 1u;  // -mv = slot + 1 (+ the encoding bit)
    const uint32_t off = lane_off + slot * (uint32_t)HS_TILE_NNZ_BYTES;
    lds_dma16<voff>(stage_w, src.v_sp[0], off);
    lds_dma16<voff + 4096>(stage_w, src.v_sp[1], off);
    // wave 1's metadata chunk lands at the region's 8 KiB: stage_w already carries its 1024
    if (w == 1) lds_dma16<voff + 8192 - 1024>(stage_w, src.v_meta, lane_off + slot * (uint32_t)HS_TILE_META_BYTES);
  } else {
    const uint32_t off = lane_off + ((uint32_t)hs_map_plain(mv) - 1u) * (uint32_t)HS_TILE_DENSE_BYTES;
    lds_dma16<voff>(stage_w, src.v_dn[0], off);
    lds_dma16<voff + 4096>(stage_w, src.v_dn[1], off);
    lds_dma16<voff + 8192>(stage_w, src.v_dn[2], off);
    lds_dma16<voff + 12288>(stage_w, src.v_dn[3], off);
  }
}

// Wait until all but the newest `tiles_in_flight` tiles' worth of this wave's direct-to-LDS loads
// have landed (loads complete in order).  PER = loads per tile that every wave issues at least.
// Immediate: vmcnt in bits 3..0 and 15..14, the other counters left at their maxima.
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }
template <int PER>
__device__ __forceinline__ void stage_wait(int tiles_in_flight) {
  static_assert(2 * PER <= 63, "vmcnt range");
  switch (tiles_in_flight) {
    case 0: __builtin_amdgcn_s_waitcnt(vmcnt_imm(0)); break;
    case 1: __builtin_amdgcn_s_waitcnt(vmcnt_imm(PER)); break;
    default: __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * PER)); break;
  }
}

// stage_wait with this wave's own load count per tile: waves 0 and 1 also fetch the metadata chunk of a
// 2:4 K resp. V tile.  (Waiting by the smallest count of any wave made those two wait for the first
// load of a tile requested only one iteration ago, and the workgroup with them at the barrier.)  Mixed
// tensors: the count varies per tile, the smallest is used.
template <int KM, int VM>
__device__ __forceinline__ void stage_wait_wave(int tiles_in_flight, int w) {
  constexpr int base = min_loads_per_tile<KM, VM>();
  if ((KM == 0 && w == 0) || (VM == 0 && w == 1)) stage_wait<base + 1>(tiles_in_flight);
  else stage_wait<base>(tiles_in_flight);
}

union B16 {  // one B operand of the 16x16x64 sparse instruction = two of the dense 16x16x32 one
  uint4 q[2];
  uint32_t u[8];
};

// KM / VM (per tensor): 0 = every tile 2:4 or skipped, 1 = every tile dense or skipped, 2 = any mix
// (the specialised all-dense / all-sparse kernels of Sec. IV-C-3, chosen per tensor so that the
// keys-dense / values-2:4 setting of Sec. V-A carries no dynamic dispatch).
// NB: column blocks (of 16 queries) per wave: a wave owns a slab of 16*NB query positions of one
// head.  NB = 2 fits 2 waves per SIMD (NB = 4, 1 wave per SIMD, measured 1.3-1.4x slower).
// F16: element type of the cache (hs_elem).  A V tile of a bf16 cache may be stored in fp16 encoding
// (HS_MAP_F16 in its map entry).  Against fp16 V the numerators have 11 significant bits and enter
// GEMM2 as one fp16 term; against bf16 V they enter as two bf16 terms.  The reference is kept
// kShift binades under the running maximum and renewed before a numerator can reach the fp16
// maximum (constants below).
template <int KM, int VM, int NB, bool F16>
__global__ __launch_bounds__(256, NB == 2 ? 2 : 1) void prefill_kernel(int Hq, int Hkv, int T, int Lq, int off,
                                                                      float scale_log2, int causal,
                                                                      const uint16_t* __restrict__ Q, hs_kv_dev kv,
                                                                      uint16_t* __restrict__ O,
                                                                      float* __restrict__ LSE) {
  typedef hs_elem<F16> E;
  typedef hs_elem<true> E16;
  // Reference = running maximum - kShift at the time it was last renewed; it is renewed when a lane's
  // partial row sum passes kRedo, i.e. before a numerator can pass 2^15 (fp16 holds 65504).  A new
  // score may thus exceed the maximum seen so far by 15 - kShift = 11 binades before the tile has
  // to be redone; with 8 / 2^14 (6 binades) keys with large channels redid 5 % of the work.
  // What fp16 flushes to zero lies 24 + kShift binades under the largest numerator: a context of
  // 2^17 tokens loses < 2^-11 of a row sum even if every other token sits just under that level.
  constexpr float kShift = 4.f;
  constexpr float kRedo = 0x1p15f;
  constexpr int QS = 16 * NB;  // query positions per slab
  constexpr int NS = n_stages<KM, VM>(), D = NS - 1;  // ring size, prefetch distance in tiles
  // MID: the per-tile barrier sits between softmax and GEMM2 instead of at the end of the
  // iteration, so that the next tile's K operands can be fetched from LDS while GEMM2 runs.  Needs
  // the next tile requested at least two iterations ahead (NS >= 3: at least one tensor all 2:4).
  // It is used where every V tile the workgroup meets takes one fp16 term of P (fp16 caches; rows
  // of a bf16 cache whose V tiles are all in fp16 encoding): with both GEMM2 forms in the loop,
  // or mixed V, no registers are left for the K prefetch.
  constexpr bool MID_OK = KM != 2 && VM != 2 && NS >= 3;
  constexpr int kStage = stage_bytes<KM, VM>();
  __shared__ __attribute__((aligned(16))) uint8_t lds[NS * kStage];
  const int tid = threadIdx.x, l = tid & 63, a = l >> 4, c = l & 15;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, scalar: branches on it stay scalar
  const int G = Hq / Hkv;
  // kv head = block index mod Hkv: workgroups go round-robin over the 8 XCDs, so with 8 kv heads (or a
  // divisor of 8) each XCD's L2 streams the tiles of its own heads only (measured 1-2.5 % faster)
  const int hkv = blockIdx.x % Hkv, b = blockIdx.z;
  const int n_slabs = (Lq / QS) * G;
  // heavy (late) query positions first: causal work grows with the position
  const int grp = (int)(gridDim.x / Hkv) - 1 - (int)(blockIdx.x / Hkv);
  const int slab = 4 * grp + w;
  const bool valid = slab < n_slabs;
  const int qpos = valid ? (slab / G) * QS : 0, hg = valid ? slab % G : 0;
  const int hq = hkv * G + hg;
  const int64_t row = (int64_t)b * Hkv + hkv;
  const int32_t* km = kv.k_map + row * T;
  const int32_t* vm = kv.v_map + row * T;
  const TileSrc src = tile_src<KM, VM>(kv, row, w);
  // query i (absolute position i + off) sees token j iff j <= i + off; last KV tile this wave /
  // the workgroup may look at, and first tile that needs masking inside
  const int jmax_w = causal ? (qpos + QS - 1 + off) / HS_BT : T - 1;
  const int last_slab = min(4 * grp + 3, n_slabs - 1);
  const int jmax_wg = causal ? min(T - 1, ((last_slab / G) * QS + QS - 1 + off) / HS_BT) : T - 1;

  // Q^T (B operand): column block nb, 64-channel block kb: query qpos+16nb+c, channels
  // 64kb + 32h + 8a + e for element 8h+e
  B16 qb[NB][2];
  {
    const uint16_t* qp = Q + (((int64_t)b * Hq + hq) * Lq + qpos + c) * HS_D + 8 * a;
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int h = 0; h < 2; h++)
          qb[nb][kb].q[h] = valid ? *reinterpret_cast<const uint4*>(qp + (int64_t)(16 * nb) * HS_D + 64 * kb + 32 * h)
                                  : make_uint4(0, 0, 0, 0);
  }

  f32x4_t o[8][NB];
#pragma unroll
  for (int mb = 0; mb < 8; mb++)
#pragma unroll
    for (int nb = 0; nb < NB; nb++) o[mb][nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run[NB], l_run[NB];
  const SplitConsts sc = split_consts();
#pragma unroll
  for (int nb = 0; nb < NB; nb++) { m_run[nb] = -INFINITY; l_run[nb] = 0.f; }

  // Map entries steer branches around matrix instructions, which ignore the EXEC mask: they are
  // forced into scalar registers so that those branches are scalar too.
  // tj[i]: the i-th visible tile from the current one on (-1: none), tk / tv: its map entries;
  // tile tj[i] sits in (or is on its way to) stage (st + i) % NS.
  int tj[NS], tk[NS], tv[NS];
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lptr_t)lds) + 1024 * w;
  const uint32_t lane_off = 16 * l;
  // The maps are read 64 tiles at a time, lane t of the window holding the entries of tile
  // wbase + t; entries are picked out with readlane and the next tile is found on a ballot.
  // This keeps map reads (vector loads, which complete in order with the tile loads and would
  // otherwise have to wait for them) off the per-tile path.
  // Order of the tiles: up to three groups, one after the other over the whole range, ascending
  // inside a group: V tile in fp16 encoding and 2:4 (or of the tensor's only kind); in fp16 encoding
  // and dense (mixed V tensors); V tile in bf16 encoding (bf16 caches: tiles with a value that fp16
  // does not hold, e.g. ~5 % of dense N(0,1) tiles, which contain a number under 2^-17).  Softmax
  // does not care about the order and the causal mask goes by the tile's index.  The loop below
  // exists once per GEMM2 form; with this order a workgroup changes form at most twice.  (A change
  // is not cheap: the loops hold the accumulators in different registers, and the spill reloads
  // the compiler puts on the way wait for the tile loads in flight as well.)
  int wbase = 0, wgroup = 0;
  int32_t wk = 0, wv = 0;
  uint64_t wrem = 0;  // tiles of the window still to hand out
  auto window_load = [&](int base) {
    const int t = base + l;
    wk = t <= jmax_wg ? km[t] : 0;
    wv = t <= jmax_wg ? vm[t] : 0;
    const bool g2 = !F16 && !hs_map_f16(wv);
    const bool g1 = !g2 && VM == 2 && wv > 0;
    const int grp = g2 ? 2 : (g1 ? 1 : 0);
    wrem = __ballot(wk != 0 && grp == wgroup);
    wbase = base;
  };
  auto next_tile = [&]() -> int {  // next tile (<= jmax_wg, not skipped) in the order above, or -1
    for (;;) {
      if (wrem != 0) {
        const int t = __builtin_ctzll(wrem);
        wrem &= wrem - 1;
        return wbase + t;
      }
      if (wbase + 64 <= jmax_wg) {
        window_load(wbase + 64);
        continue;
      }
      do wgroup++;
      while ((wgroup == 1 && VM != 2) || (wgroup == 2 && F16));  // groups this kernel cannot meet
      if (wgroup > 2) return -1;
      window_load(0);
    }
  };
  int st = 0;
  window_load(0);
#pragma unroll
  for (int i = 0; i < D; i++) {
    tj[i] = i == 0 || tj[i - 1] >= 0 ? next_tile() : -1;
    tk[i] = tv[i] = 0;
    if (tj[i] >= 0) {
      tk[i] = __builtin_amdgcn_readlane(wk, tj[i] - wbase); tv[i] = __builtin_amdgcn_readlane(wv, tj[i] - wbase);
      stage_issue<KM, VM>(lds_wave + i * kStage, src, tk[i], tv[i], w, lane_off);
    }
  }
  stage_wait<1>(0);
  __syncthreads();
  // 2:4 operands of the sparse instruction are fetched from LDS a phase ahead of their use:
  // V of the current tile before the softmax, K of the next tile before GEMM2 (MID mode).
  uint4 ak[8], kix, av[8], vix;
  auto k_fetch = [&](int stage) {
    const uint4* kl = reinterpret_cast<const uint4*>(lds + stage * kStage);
#pragma unroll
    for (int i = 0; i < 8; i++) ak[i] = kl[i * 64 + l];  // a 2:4 tile in full; the first two row blocks of a dense one
    if (KM != 1) kix = kl[512 + l];
  };
  auto request = [&]() {  // look up the tile D ahead and start its copy into the stage D ahead
    tj[D] = tj[D - 1] >= 0 ? next_tile() : -1;
    tk[D] = tv[D] = 0;
    if (tj[D] >= 0) {
      tk[D] = __builtin_amdgcn_readlane(wk, tj[D] - wbase); tv[D] = __builtin_amdgcn_readlane(wv, tj[D] - wbase);
      int sd = st + D;
      if (sd >= NS) sd -= NS;
      stage_issue<KM, VM>(lds_wave + sd * kStage, src, tk[D], tv[D], w, lane_off);
    }
  };
  // mid_tag: MID mode; only16_tag: every V tile ahead is known to be in fp16 encoding
  auto main_loop = [&](auto mid_tag, auto only16_tag) {
    constexpr bool MID = decltype(mid_tag)::value, ONLY16 = F16 || decltype(only16_tag)::value;
    // 2:4 V operands are fetched from LDS before the softmax, unless the K prefetch of MID mode
    // already holds the registers (both together spill; measured no gain there)
    constexpr bool V_EARLY = F16 && VM == 0 && !MID;
    // One iteration = one tile.  The loop exists once per GEMM2 form (V tile dense or 2:4, one fp16
    // term of P or two bf16 terms), so that each copy is straight-line code around its matrix
    // instructions and keeps the accumulators where they are (a per-tile branch around GEMM2 made
    // the compiler move all 64 accumulator registers in and out of the branch).  The form is
    // scalar: map entries come through v_readlane.
    // enc: 0 = V tile in bf16 encoding, 1 = in fp16 encoding; vkind: 0 = V tile 2:4, 1 = dense,
    // 2 = look at the tile (the tensor has one kind, or the rare bf16-encoded tiles of a mixed one)
    auto iteration = [&](auto enc, auto vkind) {
      constexpr int kEnc = decltype(enc)::value;
      const int j = tj[0], mk = tk[0], mv = tv[0];
      // END mode: request the tile D ahead now; its stage held the tile of the previous iteration,
      // which every wave has left behind (barrier at the end of that iteration)
      if (!MID) request();
      const bool ok = valid && j <= jmax_w;
      const bool k_sparse = KM == 0 || (KM == 2 && mk < 0);
      constexpr int kVK = decltype(vkind)::value;
      const bool v_sparse = kVK == 2 ? (VM == 0 || (VM == 2 && mv < 0)) : kVK == 0;
      constexpr bool v_f16 = kEnc == 1;
      const uint4* kl = reinterpret_cast<const uint4*>(lds + st * kStage);
      const uint4* vl = reinterpret_cast<const uint4*>(lds + st * kStage + region_bytes<KM>());
      B16 ph[NB], pl[NB];
      if (ok) {
        // ---------------- GEMM1: S^T[64 tokens x 16 NB queries] ----------------
        __builtin_amdgcn_s_setprio(HS_PRIO_MFMA);
        f32x4_t s[4][NB];
#pragma unroll
        for (int m = 0; m < 4; m++)
#pragma unroll
          for (int nb = 0; nb < NB; nb++) s[m][nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (k_sparse) {
          if (!MID) k_fetch(st);
          const int kidx[4] = {(int)kix.x, (int)kix.y, (int)kix.z, (int)kix.w};
          // 4 NB independent accumulators between the two instructions that share one
#pragma unroll
          for (int nb = 0; nb < NB; nb++)
#pragma unroll
            for (int m = 0; m < 4; m++)
              s[m][nb] = E::template smma<0>(ak[2 * m], qb[nb][0].q[0], qb[nb][0].q[1], s[m][nb], kidx[m]);
#pragma unroll
          for (int nb = 0; nb < NB; nb++)
#pragma unroll
            for (int m = 0; m < 4; m++)
              s[m][nb] = E::template smma<1>(ak[2 * m + 1], qb[nb][1].q[0], qb[nb][1].q[1], s[m][nb], kidx[m]);
        } else {
#pragma unroll
          for (int m = 0; m < 4; m++) {
            uint4 a4[4];
#pragma unroll
            for (int st = 0; st < 4; st++) a4[st] = MID && m < 2 ? ak[4 * m + st] : kl[(4 * m + st) * 64 + l];
#pragma unroll
            for (int st = 0; st < 4; st++)
#pragma unroll
              for (int nb = 0; nb < NB; nb++)
                s[m][nb] = E::mma(a4[st], qb[nb][st >> 1].q[st & 1], s[m][nb]);
          }
        }
        if (V_EARLY) {  // V operands: on their way while the softmax runs
#pragma unroll
          for (int i = 0; i < 8; i++) av[i] = vl[i * 64 + l];
          vix = vl[512 + l];
          __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(HS_PRIO_VALU);
        // causal mask inside a tile that reaches past the slab's first query
        if (causal && HS_BT * j + HS_BT - 1 > qpos + off) {
          const int lim = qpos + off - HS_BT * j + c;  // query 16nb+c sees in-tile tokens <= lim + 16nb
#pragma unroll
          for (int nb = 0; nb < NB; nb++)
#pragma unroll
            for (int m = 0; m < 4; m++)
#pragma unroll
              for (int i = 0; i < 4; i++)
                if (16 * m + 4 * a + i > lim + 16 * nb) s[m][nb][i] = -INFINITY;
        }
        // ---------------- P = exp2(S*scale - m_run), reference m_run updated lazily ----------------
        // P is first computed against the current reference of each query column, with no look at
        // the tile's maximum.  Only if a partial row sum comes out huge (or the column has no
        // reference yet) is the exact running maximum taken, O and l rescaled, and P recomputed.
        // With a stale reference P merely holds larger numbers (harmless in fp32 / bf16); the final
        // O / l and LSE = m_run + log2(l) do not depend on which reference was used.
        // P goes through the matrix unit as two bf16 terms (hi + remainder): a single bf16 P alone
        // costs ~1.3e-3 mean relative error on the output, on top of the bf16 rounding of O itself.
        float psum[NB];
        auto softmax_as = [&](auto enc) {  // enc: std::true_type = fp16 numerators, one term
          constexpr bool kF16 = decltype(enc)::value;
#pragma unroll
          for (int nb = 0; nb < NB; nb++) {
            float acc = 0.f;
            const float mref = m_run[nb] > -INFINITY ? m_run[nb] : 0.f;
#pragma unroll
            for (int m = 0; m < 4; m++) {
              float p[4];
#pragma unroll
              for (int i = 0; i < 4; i++) {
                p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[m][nb][i], scale_log2, -mref));
                acc += p[i];
              }
              if (kF16) {
                ph[nb].u[2 * m] = E16::pack2(p[0], p[1]);
                ph[nb].u[2 * m + 1] = E16::pack2(p[2], p[3]);
              } else {
                split_hi_lo(p[0], p[1], sc, ph[nb].u[2 * m], pl[nb].u[2 * m]);
                split_hi_lo(p[2], p[3], sc, ph[nb].u[2 * m + 1], pl[nb].u[2 * m + 1]);
              }
            }
            psum[nb] = acc;
          }
        };
        auto softmax_tile = [&]() { softmax_as(std::integral_constant<bool, v_f16>{}); };
        softmax_tile();
        bool redo = false;
#pragma unroll
        for (int nb = 0; nb < NB; nb++) redo = redo || !(psum[nb] <= kRedo) || !(m_run[nb] > -INFINITY);
        if (__any(redo)) {
#pragma unroll
          for (int nb = 0; nb < NB; nb++) {
            float mx = s[0][nb][0];
#pragma unroll
            for (int m = 0; m < 4; m++)
#pragma unroll
              for (int i = 0; i < 4; i++) mx = fmaxf(mx, s[m][nb][i]);
            mx = mx * scale_log2 - kShift;
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // a column with nothing visible in this tile keeps its reference
            const float m_new = fmaxf(m_run[nb], mx);
            const float alpha = m_new > -INFINITY ? __builtin_amdgcn_exp2f(m_run[nb] - m_new) : 1.0f;
            m_run[nb] = m_new;
            l_run[nb] *= alpha;
#pragma unroll
            for (int mb = 0; mb < 8; mb++) o[mb][nb] *= alpha;
          }
          softmax_tile();
        }
#pragma unroll
        for (int nb = 0; nb < NB; nb++) l_run[nb] += psum[nb];
      }
      if (MID) {
        // The next tile must have landed in full (own loads, then everybody's: barrier) before its K
        // operands are fetched; tiles requested after it may still be in flight.  The stage of the
        // previous tile is free from here on (all of its reads precede this barrier).
        int later = 0;
#pragma unroll
        for (int i = 2; i < D; i++) later += tj[i] >= 0;
        stage_wait_wave<KM, VM>(later, w);
        __syncthreads();
        request();
        if (valid && tj[1] >= 0) {
          k_fetch(st + 1 == NS ? 0 : st + 1);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (ok) {
        __builtin_amdgcn_s_setprio(HS_PRIO_MFMA);
        if (v_sparse) {
          if (!V_EARLY) {
#pragma unroll
            for (int i = 0; i < 8; i++) av[i] = vl[i * 64 + l];
            vix = vl[512 + l];
          }
          const int vidx[4] = {(int)vix.x, (int)vix.y, (int)vix.z, (int)vix.w};
          if (v_f16) {  // one fp16 term
#pragma unroll
            for (int nb = 0; nb < NB; nb++)
#pragma unroll
              for (int mb = 0; mb < 8; mb++) {
                if (mb & 1)
                  o[mb][nb] = E16::template smma<1>(av[mb], ph[nb].q[0], ph[nb].q[1], o[mb][nb], vidx[mb >> 1]);
                else
                  o[mb][nb] = E16::template smma<0>(av[mb], ph[nb].q[0], ph[nb].q[1], o[mb][nb], vidx[mb >> 1]);
              }
          } else {
#pragma unroll
            for (int t2 = 0; t2 < 2; t2++)  // first the upper-half term of every block, then the remainder
#pragma unroll
              for (int nb = 0; nb < NB; nb++)
#pragma unroll
                for (int mb = 0; mb < 8; mb++) {
                  const B16& bp = t2 == 0 ? ph[nb] : pl[nb];
                  if (mb & 1)
                    o[mb][nb] = E::template smma<1>(av[mb], bp.q[0], bp.q[1], o[mb][nb], vidx[mb >> 1]);
                  else
                    o[mb][nb] = E::template smma<0>(av[mb], bp.q[0], bp.q[1], o[mb][nb], vidx[mb >> 1]);
                }
          }
        } else {
#pragma unroll
          for (int mb = 0; mb < 8; mb++) {
            const uint4 a0 = vl[(2 * mb) * 64 + l], a1 = vl[(2 * mb + 1) * 64 + l];
            if (v_f16) {
#pragma unroll
              for (int h = 0; h < 2; h++)
#pragma unroll
                for (int nb = 0; nb < NB; nb++) o[mb][nb] = E16::mma(h == 0 ? a0 : a1, ph[nb].q[h], o[mb][nb]);
            } else {
#pragma unroll
              for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
                for (int h = 0; h < 2; h++)
#pragma unroll
                  for (int nb = 0; nb < NB; nb++)
                    o[mb][nb] = E::mma(h == 0 ? a0 : a1, t2 == 0 ? ph[nb].q[h] : pl[nb].q[h], o[mb][nb]);
            }
          }
        }
      }
      __builtin_amdgcn_s_setprio(HS_PRIO_VALU);
      if (!MID) {
        // the next tile must have landed; the ones requested after it may still be in flight
        int later = 0;
#pragma unroll
        for (int i = 2; i <= D; i++) later += tj[i] >= 0;
        stage_wait_wave<KM, VM>(later, w);
        __syncthreads();
      }
#pragma unroll
      for (int i = 0; i < D; i++) { tj[i] = tj[i + 1]; tk[i] = tk[i + 1]; tv[i] = tv[i + 1]; }
      st = st + 1 == NS ? 0 : st + 1;
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    typedef std::integral_constant<int, 2> I2;
    if (MID && valid && tj[0] >= 0) k_fetch(0);
    while (tj[0] >= 0) {
      // one loop per GEMM2 form, each run over consecutive tiles of its form (a branch around GEMM2
      // inside one loop makes the compiler move all 64 accumulators per tile; going from one loop
      // to another costs that move once per change, which the tile order keeps rare)
      if (!ONLY16 && !hs_map_f16(tv[0])) {  // V tile in bf16 encoding: two terms of P; kind looked at per tile
        do iteration(I0{}, I2{});
        while (tj[0] >= 0 && !hs_map_f16(tv[0]));
      } else if (VM == 2 && tv[0] > 0) {
        do iteration(I1{}, I1{});
        while (tj[0] >= 0 && tv[0] > 0 && (ONLY16 || hs_map_f16(tv[0])));
      } else if (VM == 2) {
        do iteration(I1{}, I0{});
        while (tj[0] >= 0 && tv[0] < 0 && (ONLY16 || hs_map_f16(tv[0])));
      } else {
        do iteration(I1{}, I2{});
        while (tj[0] >= 0 && (ONLY16 || hs_map_f16(tv[0])));
      }
    }
  };
  if constexpr (F16) {
    main_loop(std::integral_constant<bool, MID_OK>{}, std::true_type{});
  } else if constexpr (MID_OK) {
    // bf16 cache: are all V tiles this workgroup can meet in fp16 encoding?  (every wave scans the
    // same entries, so the workgroup agrees; the answer is scalar)
    bool all16 = true;
    for (int base = 0; base <= jmax_wg; base += 64) {
      const int t = base + l;
      const int32_t m = t <= jmax_wg ? vm[t] : 0;
      all16 = all16 && !__any(m != 0 && !hs_map_f16(m));
    }
    if (all16) main_loop(std::integral_constant<bool, MID_OK>{}, std::true_type{});
    else main_loop(std::false_type{}, std::false_type{});
  } else {
    main_loop(std::false_type{}, std::false_type{});
  }

  // ---------------- epilogue: O = O^T / l, LSE ----------------
  if (!valid) return;
#pragma unroll
  for (int nb = 0; nb < NB; nb++) {
    float lt = l_run[nb];
    lt += __shfl_xor(lt, 16);
    lt += __shfl_xor(lt, 32);
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const int64_t qrow = ((int64_t)b * Hq + hq) * Lq + qpos + 16 * nb + c;
    uint16_t* op = O + qrow * HS_D + 4 * a;
#pragma unroll
    for (int mb = 0; mb < 8; mb++) {
      const uint2 v = make_uint2(E::pack2(o[mb][nb][0] * inv, o[mb][nb][1] * inv),
                                 E::pack2(o[mb][nb][2] * inv, o[mb][nb][3] * inv));
      *reinterpret_cast<uint2*>(op + 16 * mb) = v;
    }
    if (LSE != nullptr && a == 0)
      LSE[qrow] = lt > 0.f ? (m_run[nb] + __builtin_amdgcn_logf(lt)) * kLn2 : -INFINITY;
  }
}

}  // namespace

template <int KM, int VM, int NB>
static hipError_t launch_prefill(int B, int Hq, int Hkv, int T, int Lq, int q_start, float sl2, int causal, const uint16_t* Q,
                                 const hs_kv_dev& kv, uint16_t* O, float* LSE, hipStream_t st, bool f16) {
  const int G = Hq / Hkv;
  const int n_groups = ((Lq / (16 * NB)) * G + 3) / 4;
  if (f16)
    hipLaunchKernelGGL((prefill_kernel<KM, VM, NB, true>), dim3(n_groups * Hkv, 1, B), dim3(256), 0, st, Hq, Hkv, T, Lq,
                       q_start, sl2, causal, Q, kv, O, LSE);
  else
    hipLaunchKernelGGL((prefill_kernel<KM, VM, NB, false>), dim3(n_groups * Hkv, 1, B), dim3(256), 0, st, Hq, Hkv, T, Lq,
                       q_start, sl2, causal, Q, kv, O, LSE);
  return hipGetLastError();
}

hipError_t hs_launch_prefill(int B, int Hq, int Hkv, int T, int Tq, int q_start, float scale, int causal, const uint16_t* Q,
                             hs_kv_dev kv, uint16_t* O, float* LSE, hipStream_t st, int dtype) {
  const bool f16 = dtype == HS_FP16;
  const float sl2 = scale * kLog2e;
  const int Lq = Tq * HS_BT;
  const int km = kv.cap_dense_k == 0 ? 0 : (kv.cap_sparse_k == 0 ? 1 : 2);
  const int vm = kv.cap_dense_v == 0 ? 0 : (kv.cap_sparse_v == 0 ? 1 : 2);
#define HS_GO(KM_, VM_) return launch_prefill<KM_, VM_, 2>(B, Hq, Hkv, T, Lq, q_start, sl2, causal, Q, kv, O, LSE, st, f16)
  switch (km * 3 + vm) {
    case 0: HS_GO(0, 0);
    case 1: HS_GO(0, 1);
    case 2: HS_GO(0, 2);
    case 3: HS_GO(1, 0);
    case 4: HS_GO(1, 1);
    case 5: HS_GO(2, 2);  // dense K beside mixed V: the instantiation that looks at each K tile's kind measured faster than <1, 2>
    case 6: HS_GO(2, 0);
    case 7: HS_GO(2, 1);
    default: HS_GO(2, 2);
  }
#undef HS_GO
}
