// Decode attention: split-KV kernel + merge kernel (Sec. IV-C: each workgroup handles a
// subset of the KV blocks and emits a partial output with its log-sum-exp; a light
// post-processing kernel combines them; the query heads that share a KV head are folded
// into the N dimension of the matrix instruction).
//
// The kernel is HBM-bound: every byte of the packed cache is read exactly once, straight
// from global memory into matrix-core operand registers (the pools are stored in operand
// order), so there is no LDS staging and no cross-lane shuffle in the main loop.  The
// sparse matrix instruction is used as the decompressor: it consumes the 2-bit metadata
// natively, so no vector-ALU work is spent on selecting operands.
#include <mutex>
#include <type_traits>

#include "hs_common.h"

#ifndef HS_DEC_DEPTH
#define HS_DEC_DEPTH 2
#endif
#ifndef HS_DEC_BYCOUNT_MIN_PER
#define HS_DEC_BYCOUNT_MIN_PER 128  /* tiles per split from which the kept tiles are handed out by count */
#endif
#ifndef HS_DEC_EARLY
#define HS_DEC_EARLY 1  /* uniform caches: the first round of a wave guesses its tiles' form and loads them at once */
#endif
#ifndef HS_DEC_OCC
#define HS_DEC_OCC ((KM == 0 && VM == 0) || KM == 2 || VM == 2 ? 2 : 1)  /* a dense tensor at depth 2 needs > 256 registers */
#endif

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;


// streaming (non-temporal) 16-byte load: the packed cache is read once per call
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p)));
}



// Operand registers of one tile (K and V), filled by tile_load and consumed by tile_compute.
// KM / VM: kind of the K / V tile, 0 = 2:4, 1 = dense (the kernel sorts its tiles by kind first).
template <int KM, int VM>
struct TileRegs {
  static_assert((KM == 0 || KM == 1) && (VM == 0 || VM == 1), "one kind per operand");
  static constexpr int kNK = KM == 0 ? 8 : 16;  // 16-byte chunks per lane: 2:4 tile 8, dense tile 16
  static constexpr int kNV = VM == 0 ? 8 : 16;
  uint4 k[kNK];
  uint4 v[kNV];
  uint4 km, vm;  // the lane's four 32-bit index words of the K / V tile
};

template <int KM, int VM>
__device__ __forceinline__ void tile_load(TileRegs<KM, VM>& r, const hs_kv_dev& kv, int64_t row, int mk, int mv, int l) {  // mk, mv: wave-uniform
  mv = hs_map_plain(mv);
  r.km = make_uint4(0, 0, 0, 0);  // only 2:4 tiles carry index words
  r.vm = make_uint4(0, 0, 0, 0);
  constexpr bool k_sparse = KM == 0, v_sparse = VM == 0;
  if (k_sparse) {
    const int64_t slot = row * kv.cap_sparse_k + (-mk - 1);
    const uint4* p = reinterpret_cast<const uint4*>(kv.k_nnz + slot * (int64_t)HS_TILE_NNZ_BYTES) + l;
#pragma unroll
    for (int i = 0; i < 8; i++) r.k[i] = ld_stream(p + 64 * i);
    r.km = ld_stream(reinterpret_cast<const uint4*>(kv.k_meta + slot * (int64_t)HS_TILE_META_BYTES) + l);
  } else {
    const int64_t slot = row * kv.cap_dense_k + (mk - 1);
    const uint4* p = reinterpret_cast<const uint4*>(kv.k_dense + slot * (int64_t)HS_TILE_DENSE_BYTES) + l;
#pragma unroll
    for (int i = 0; i < 16; i++) r.k[i % TileRegs<KM, VM>::kNK] = ld_stream(p + 64 * i);
  }
  if (v_sparse) {
    const int64_t slot = row * kv.cap_sparse_v + (-mv - 1);
    const uint4* p = reinterpret_cast<const uint4*>(kv.v_nnz + slot * (int64_t)HS_TILE_NNZ_BYTES) + l;
#pragma unroll
    for (int i = 0; i < 8; i++) r.v[i] = ld_stream(p + 64 * i);
    r.vm = ld_stream(reinterpret_cast<const uint4*>(kv.v_meta + slot * (int64_t)HS_TILE_META_BYTES) + l);
  } else {
    const int64_t slot = row * kv.cap_dense_v + (mv - 1);
    const uint4* p = reinterpret_cast<const uint4*>(kv.v_dense + slot * (int64_t)HS_TILE_DENSE_BYTES) + l;
#pragma unroll
    for (int i = 0; i < 16; i++) r.v[i % TileRegs<KM, VM>::kNV] = ld_stream(p + 64 * i);
  }
}

// One tile: GEMM1 (S^T = K Q^T), online softmax, GEMM2 (O^T += V^T P^T).
// F16: element type of the cache (hs_elem).  A V tile of a bf16 cache may be stored in fp16
// encoding (HS_MAP_F16 in its map entry); the numerators then go into GEMM2 as fp16 too.  The
// running reference sits kShift = 8 binades under the running maximum, so that numerators reach
// 2^8 and what fp16 flushes to zero is below 2^-32 of the largest one (a context of 2^17 tokens
// then loses < 2^-15 of the sum).
// ENC: 0 = V tile in bf16, 1 = in fp16 (encoding bit, or an fp16 cache).
template <int KM, int VM, bool F16, int ENC>
__device__ __forceinline__ void tile_compute(const TileRegs<KM, VM>& r, const uint4 (&qb)[4], float scale_log2, int c,
                                             f32x4_t (&o)[8], float& m_run, float& l_run) {
  constexpr bool k_sparse = KM == 0, v_sparse = VM == 0;
  constexpr int kNK = TileRegs<KM, VM>::kNK, kNV = TileRegs<KM, VM>::kNV;
  typedef hs_elem<F16> E;
  typedef hs_elem<true> E16;
  constexpr float kShift = 8.f;
  constexpr bool v_f16 = ENC == 1;
  f32x4_t s[4];
  const int kidx[4] = {(int)r.km.x, (int)r.km.y, (int)r.km.z, (int)r.km.w};
  const int vidx[4] = {(int)r.vm.x, (int)r.vm.y, (int)r.vm.z, (int)r.vm.w};
#pragma unroll
  for (int m = 0; m < 4; m++) s[m] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  if (k_sparse) {  // the 4 row blocks are independent chains
#pragma unroll
    for (int m = 0; m < 4; m++)
      s[m] = E::template smma<0>(r.k[2 * m], qb[0], qb[1], s[m], kidx[m]);
#pragma unroll
    for (int m = 0; m < 4; m++)
      s[m] = E::template smma<1>(r.k[2 * m + 1], qb[2], qb[3], s[m], kidx[m]);
  }
#pragma unroll
  for (int m = 0; m < 4; m++) {
    if (!k_sparse) {
#pragma unroll
      for (int st = 0; st < 4; st++)
        s[m] = E::mma(r.k[(4 * m + st) % kNK], qb[st], s[m]);
    }
  }
  // online softmax for column c (log2 domain)
  float mx = -INFINITY;
#pragma unroll
  for (int m = 0; m < 4; m++)
#pragma unroll
    for (int i = 0; i < 4; i++) mx = fmaxf(mx, s[m][i]);
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m_run, mx * scale_log2 - kShift);
  const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on the first tile
  m_run = m_new;
  float psum = 0.f;
  // P^T as the B operand: element 8h+4u+i of lane group a <- token 16(2h+u)+4a+i.
  // Columns < 8 carry bf16(p), columns >= 8 carry bf16(p - bf16(p)), so that the sum of
  // the two accumulator columns sees p to ~16 bits although the operand type is bf16.
  float p[4][4];
#pragma unroll
  for (int m = 0; m < 4; m++)
#pragma unroll
    for (int i = 0; i < 4; i++) {
      p[m][i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[m][i], scale_log2, -m_new));
      psum += p[m][i];
    }
  uint32_t pb[8];
  auto pack_as = [&](auto enc) {
    typedef hs_elem<decltype(enc)::value> EP;
#pragma unroll
    for (int m = 0; m < 4; m++) {
      const uint32_t hi0 = EP::pack2(p[m][0], p[m][1]), hi1 = EP::pack2(p[m][2], p[m][3]);
      const uint32_t lo0 = EP::pack2(p[m][0] - EP::lo_f32(hi0), p[m][1] - EP::hi_f32(hi0));
      const uint32_t lo1 = EP::pack2(p[m][2] - EP::lo_f32(hi1), p[m][3] - EP::hi_f32(hi1));
      pb[2 * m] = c < 8 ? hi0 : lo0;
      pb[2 * m + 1] = c < 8 ? hi1 : lo1;
    }
  };
  if (v_f16) pack_as(std::true_type{});
  else pack_as(std::false_type{});
  l_run = l_run * alpha + psum;
#pragma unroll
  for (int i = 0; i < 8; i++) o[i] *= alpha;
  const uint4 pb_lo = make_uint4(pb[0], pb[1], pb[2], pb[3]);  // dense step h = 0
  const uint4 pb_hi = make_uint4(pb[4], pb[5], pb[6], pb[7]);  // dense step h = 1
  if (v_f16) {
#pragma unroll
    for (int mb = 0; mb < 8; mb++) {
      if (v_sparse) {
        if (mb & 1) o[mb] = E16::template smma<1>(r.v[mb], pb_lo, pb_hi, o[mb], vidx[mb >> 1]);
        else o[mb] = E16::template smma<0>(r.v[mb], pb_lo, pb_hi, o[mb], vidx[mb >> 1]);
      } else {
        o[mb] = E16::mma(r.v[(2 * mb) % kNV], pb_lo, o[mb]);
        o[mb] = E16::mma(r.v[(2 * mb + 1) % kNV], pb_hi, o[mb]);
      }
    }
  } else {
#pragma unroll
    for (int mb = 0; mb < 8; mb++) {
      if (v_sparse) {
        if (mb & 1) o[mb] = E::template smma<1>(r.v[mb], pb_lo, pb_hi, o[mb], vidx[mb >> 1]);
        else o[mb] = E::template smma<0>(r.v[mb], pb_lo, pb_hi, o[mb], vidx[mb >> 1]);
      } else {
        o[mb] = E::mma(r.v[(2 * mb) % kNV], pb_lo, o[mb]);
        o[mb] = E::mma(r.v[(2 * mb + 1) % kNV], pb_hi, o[mb]);
      }
    }
  }
}

// Which tile forms (bit 0 K dense, bit 1 V dense, bit 2 V in bf16 encoding) a kernel instantiation can meet:
// KM / VM 0 = every tile 2:4, 1 = every tile dense, 2 = any mix; an fp16 cache has no bf16-encoded tiles.
template <int KM, int VM, bool F16>
__host__ __device__ constexpr bool form_allowed(int f) {
  return ((f & 1) ? KM != 0 : KM != 1) && ((f & 2) ? VM != 0 : VM != 1) && ((f & 4) ? !F16 : true);
}
// fn(std::integral_constant<int, f>) for every allowed form f except SKIP_FORM, in ascending order
template <int KM, int VM, bool F16, int SKIP_FORM, int F = 0, typename Fn>
__device__ __forceinline__ void static_for_forms(Fn&& fn) {
  if constexpr (F < 8) {
    if constexpr (F != SKIP_FORM && form_allowed<KM, VM, F16>(F)) fn(std::integral_constant<int, F>{});
    static_for_forms<KM, VM, F16, SKIP_FORM, F + 1>(fn);
  }
}

// Split-KV kernel.  grid = (n_splits, Hkv, B); workgroup = 4 waves; split s owns tiles
// [s*per, (s+1)*per); wave w takes every 4th tile of them.  Each wave preloads the map
// entries of its tiles with one vector load, drops the skipped ones, and streams the rest
// with a two-deep register pipeline (the loads of tile i+1 are in flight while tile i is
// being multiplied).
// Each workgroup emits a normalised partial output and its log-sum-exp per query head.
//
// MODE (how the tiles of a row are handed out):
//   kByRange    split s owns tiles [s*per, (s+1)*per), wave w every 4th of them; skipped tiles are dropped
//               as they are met, so a split or a wave may end up with fewer tiles than its neighbours.
//   kUniform    as kByRange, for a cache the caller promises to be uniform (no tile skipped, one kind per
//               tensor, slot == tile): the K map is not read at all.
//   kByCount    the kept (not skipped) tiles of the row are numbered in tile order, split s owns the numbers
//               [n*s/S, n*(s+1)/S) and wave w every 4th of them: every wave of the grid gets the same number
//               of tiles to within one, whatever the skip pattern.  Costs two passes over the row's maps
//               at kernel start (count, then list through LDS), so the host picks it for long rows only.
enum { kByRange = 0, kUniform = 1, kByCount = 2 };
constexpr int kListCap = 2048;  // tiles listed in LDS at a time (kByCount); longer shares take several passes
constexpr int kScanBatch = 2048;  // tiles of the row looked at per scan step: 8 per thread

template <int KM, int VM, int MODE, bool F16>
__global__ __launch_bounds__(256, HS_DEC_OCC) void decode_split_kernel(int Hq, int Hkv, int T, float scale_log2,
                                                                             int n_splits, int per,
                                                                             const uint16_t* __restrict__ Q,
                                                                             hs_kv_dev kv, float* __restrict__ ws_o,
                                                                             float* __restrict__ ws_l) {
  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, l = tid & 63, a = l >> 4, c = l & 15;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, scalar: branches on it stay scalar
  const int G = Hq / Hkv;
  const int64_t row = (int64_t)b * Hkv + hkv;
  const int t_begin = split * per, t_end = min(T, t_begin + per);

  // Q^T as the B operand: columns 0..G-1 and 8..8+G-1 both hold head (hkv*G + column%8);
  // the second copy carries the low-order half of P in GEMM2.
  uint4 qb[4];  // dense k-steps s = 0..3 (channels 32s + 8a + e); sparse kb uses steps 2kb, 2kb+1
  {
    const int head = c & 7;
    const bool valid = head < G;
    const uint16_t* q = Q + ((int64_t)b * Hq + hkv * G + (valid ? head : 0)) * HS_D + 8 * a;
#pragma unroll
    for (int s = 0; s < 4; s++) qb[s] = valid ? *reinterpret_cast<const uint4*>(q + 32 * s) : make_uint4(0, 0, 0, 0);
  }

  f32x4_t o[8];
#pragma unroll
  for (int i = 0; i < 8; i++) o[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  // A tile's form: bit 0 = K tile dense, bit 1 = V tile dense, bit 2 = V tile stored in bf16 encoding (bf16
  // caches only; a V tile of a bf16 cache is normally stored in fp16 encoding, HS_MAP_F16).  The tiles are
  // worked through one form at a time ("sweeps"): the loads and matrix instructions of a sweep are all of one
  // type, no branch sits between them, and each sweep keeps as many tiles in flight as its operands leave
  // registers for.  The softmax recurrence does not care in which order tiles arrive.
  auto form_of = [](int mk, int mv) -> int { return (mk > 0 ? 1 : 0) | (mv > 0 ? 2 : 0) | ((!F16 && !hs_map_f16(mv)) ? 4 : 0); };
  constexpr bool kMixed = KM == 2 || VM == 2;
  constexpr int kFirstForm = (KM == 1 ? 1 : 0) | (VM == 1 ? 2 : 0);  // swept first: it also notes which other forms occur
  // One sweep.  The tiles come as a sequence of map entry pairs numbered [first, last): `entry(i, mk, mv)` yields
  // pair i; wave w takes every 4th pair starting at first + w.  Returns (COLLECT) the set of forms among them.
  // SPEC (uniform caches, first sweep): where the wave's first tiles sit is known without the maps (slot ==
  // tile), only their form is not (the encoding bit of the V map of a bf16 cache), so the first round is a
  // straight-line copy of its own that issues their loads at once, behind the map read instead of after it
  // and with no ballot or branch in front of them (4-6 % of the kernel at the 32K-context shape, fp16 caches,
  // which have no map to wait for, included).  If one of the tiles turns out to be of another form (a V tile
  // that fp16 cannot hold) the sweep returns kGuessFailed before it has touched the accumulators, and is run
  // again without guessing.
  constexpr unsigned kGuessFailed = 1u << 31;
  auto sweep = [&](auto form_c, auto collect_c, auto spec_c, int first, int last, auto entry) -> unsigned {
    constexpr int kForm = decltype(form_c)::value;
    constexpr bool COLLECT = decltype(collect_c)::value;
    constexpr bool SPEC = decltype(spec_c)::value;
    constexpr int KK = kForm & 1, VK = (kForm >> 1) & 1, kEnc = (kForm & 4) ? 0 : 1;
    // Tiles in flight per wave.  Measured on the 32K-context shape: depth 1, 2, 3 and 4 (the deeper ones at
    // 1 wave per SIMD) all land within run-to-run noise, and even a variant with the arithmetic removed is only
    // ~10 % faster: the kernel is bound by the load stream.  A kernel for mixed tensors runs at 2 waves per
    // SIMD, where only two 2:4 tiles (or one tile with a dense operand) fit.
    constexpr int DEPTH = kMixed ? ((KK == 0 && VK == 0) ? 2 : 1) : HS_DEC_DEPTH;
    TileRegs<KK, VK> ring[DEPTH];
    unsigned seen = 0;
// what the two copies of a round below share: the form ballots, and the loop that consumes the tiles in
// flight and refills their ring slots from `act`
#define HS_ROUND_BALLOTS                                                                                              \
  const int form_v = form_of(mk_v, mv_v);                                                                             \
  unsigned long long act = __ballot(mk_v != 0 && form_v == kForm);                                                    \
  if (COLLECT) {                                                                                                      \
    _Pragma("unroll") for (int f = 0; f < 8; f++)                                                                     \
      if (f != kForm && form_allowed<KM, VM, F16>(f)) seen |= (__ballot(mk_v != 0 && form_v == f) != 0ull ? 1u : 0u) << f; \
  }
#define HS_ROUND_CONSUME                                                                                              \
  bool go = have[0];                                                                                                  \
  while (go) {                                                                                                        \
    _Pragma("unroll") for (int d = 0; d < DEPTH; d++) {                                                               \
      if (go && have[d]) { /* tiles are consumed in issue order: the first empty slot ends the round */               \
        tile_compute<KK, VK, F16, kEnc>(ring[d], qb, scale_log2, c, o, m_run, l_run);                                 \
        have[d] = act != 0ull;                                                                                        \
        if (have[d]) {                                                                                                \
          const int i = __builtin_ctzll(act);                                                                         \
          act &= act - 1;                                                                                             \
          tile_load<KK, VK>(ring[d], kv, row, __builtin_amdgcn_readlane(mk_v, i), __builtin_amdgcn_readlane(mv_v, i), l); \
        }                                                                                                             \
      } else {                                                                                                        \
        go = false;                                                                                                   \
      }                                                                                                               \
    }                                                                                                                 \
  }
    int base = first + w;
    if constexpr (SPEC) {
      if (base < last) {  // first round, tiles guessed
        const int i_mine = base + 4 * l;
        int mk_v = 0, mv_v = 0;
        if (i_mine < last) entry(i_mine, mk_v, mv_v);
        bool have[DEPTH];
        unsigned long long guessed = 0ull;
#pragma unroll
        for (int d = 0; d < DEPTH; d++) {
          const int t = base + 4 * d;
          have[d] = t < last;
          if (have[d]) {
            guessed |= 1ull << d;
            tile_load<KK, VK>(ring[d], kv, row, KK == 0 ? -(t + 1) : t + 1, VK == 0 ? -(t + 1) : t + 1, l);
          }
        }
        HS_ROUND_BALLOTS
        if constexpr (!F16)  // an fp16 cache has one encoding: nothing to guess wrong
          if ((act & ((1ull << DEPTH) - 1ull)) != guessed) return kGuessFailed;
        act &= ~guessed;
        HS_ROUND_CONSUME
        base += 256;
      }
    }
    for (; base < last; base += 256) {  // up to 64 tiles of this wave per round
      const int i_mine = base + 4 * l;
      int mk_v = 0, mv_v = 0;
      if (i_mine < last) entry(i_mine, mk_v, mv_v);
      // Tile kinds must reach the branches below as scalar (wave-uniform) values: matrix
      // instructions ignore the EXEC mask, so a branch the compiler treats as divergent would run
      // both the dense and the 2:4 instruction on every tile.  Lane values are therefore read
      // with v_readlane, never with a lane shuffle.
      HS_ROUND_BALLOTS
      bool have[DEPTH];
#pragma unroll
      for (int d = 0; d < DEPTH; d++) {
        have[d] = act != 0ull;
        if (have[d]) {
          const int i = __builtin_ctzll(act);
          act &= act - 1;
          tile_load<KK, VK>(ring[d], kv, row, __builtin_amdgcn_readlane(mk_v, i), __builtin_amdgcn_readlane(mv_v, i), l);
        }
      }
      HS_ROUND_CONSUME
    }
#undef HS_ROUND_BALLOTS
#undef HS_ROUND_CONSUME
    return seen;
  };
  auto all_sweeps = [&](int first, int last, auto entry) {
    constexpr bool kGuess = HS_DEC_EARLY && MODE == kUniform;
    unsigned seen = sweep(std::integral_constant<int, kFirstForm>{}, std::true_type{}, std::integral_constant<bool, kGuess>{},
                          first, last, entry);
    if (kGuess && !F16 && seen == kGuessFailed)
      seen = sweep(std::integral_constant<int, kFirstForm>{}, std::true_type{}, std::false_type{}, first, last, entry);
    static_for_forms<KM, VM, F16, kFirstForm>([&](auto form_c) {
      if ((seen >> decltype(form_c)::value) & 1u) sweep(form_c, std::false_type{}, std::false_type{}, first, last, entry);
    });
  };
  auto from_map = [&](int t, int& mk, int& mv) {
    if (MODE == kUniform) {  // promised by the caller: no tile skipped, one kind per tensor, slot == tile
      mk = KM == 0 ? -(t + 1) : t + 1;
      mv = F16 ? (VM == 0 ? -(t + 1) : t + 1) : kv.v_map[row * T + t];  // bf16: encoding bit
    } else {
      mk = kv.k_map[row * T + t];
      mv = kv.v_map[row * T + t];
    }
  };
  if constexpr (MODE != kByCount) {
    all_sweeps(t_begin, t_end, from_map);
  } else {
    __shared__ int2 sm_list[kListCap];  // (k_map, v_map) entries of this workgroup's tiles, in tile order
    __shared__ int sm_cnt[36];          // [0..3] kept tiles per wave (count pass); [4 + 4 j + w] per scan segment
    const int* kmap = kv.k_map + row * T;
    const int* vmap = kv.v_map + row * T;
    const unsigned long long lanes_below = (1ull << l) - 1ull;
    // pass 1: kept tiles of the row
    int mine_cnt = 0;
    for (int b0 = 0; b0 < T; b0 += kScanBatch) {
#pragma unroll
      for (int j = 0; j < 8; j++) {
        const int t = b0 + 256 * j + tid;
        const int mk = t < T ? kmap[t] : 0;
        const int mv = t < T ? vmap[t] : 0;  // not needed yet: fetched so that pass 2 finds both maps in the L2
        asm volatile("" ::"v"(mv));
        mine_cnt += __builtin_popcountll(__ballot(mk != 0));
      }
    }
    if (l == 0) sm_cnt[w] = mine_cnt;
    __syncthreads();
    const int n_kept = sm_cnt[0] + sm_cnt[1] + sm_cnt[2] + sm_cnt[3];
    const int n_work = gridDim.x;
    const int lo = (int)((int64_t)n_kept * split / n_work), hi = (int)((int64_t)n_kept * (split + 1) / n_work);
    if (n_kept == T) {  // nothing skipped: a tile's number is its index, no list needed
      all_sweeps(lo, hi, from_map);
    } else
    for (int r0 = lo; r0 < hi; r0 += kListCap) {  // workgroup-uniform bounds: every thread takes the same trips
      const int r1 = min(hi, r0 + kListCap);
      // pass 2: list the tiles numbered [r0, r1)
      int carried = 0;  // kept tiles before the scan step
      for (int b0 = 0; b0 < T && carried < r1; b0 += kScanBatch) {
        int mk8[8], mv8[8];  // read again in every pass (from L2 by now) rather than held across the tile loop
#pragma unroll
        for (int j = 0; j < 8; j++) {
          const int t = b0 + 256 * j + tid;
          mk8[j] = t < T ? kmap[t] : 0;
          mv8[j] = t < T ? vmap[t] : 0;
        }
        unsigned long long kept[8];
#pragma unroll
        for (int j = 0; j < 8; j++) {
          kept[j] = __ballot(mk8[j] != 0);
          if (l == 0) sm_cnt[4 + 4 * j + w] = __builtin_popcountll(kept[j]);
        }
        __syncthreads();
        int run = carried;  // tile t = b0 + 256 j + 64 w + l: segments in (j, w) order are in tile order
#pragma unroll
        for (int j = 0; j < 8; j++) {
          int before = run;
#pragma unroll
          for (int ww = 0; ww < 4; ww++) {
            const int c_seg = sm_cnt[4 + 4 * j + ww];
            if (ww < w) before += c_seg;
            run += c_seg;
          }
          const int number = before + __builtin_popcountll(kept[j] & lanes_below);
          if (mk8[j] != 0 && number >= r0 && number < r1) sm_list[number - r0] = make_int2(mk8[j], mv8[j]);
        }
        carried = run;
        __syncthreads();  // the counts are rewritten by the next scan step
      }
      const int n_list = r1 - r0;
      // the same sweeps, over the list: pair i goes to wave i % 4
      auto from_list = [&](int i, int& mk, int& mv) {
        const int2 e = sm_list[i];
        mk = e.x;
        mv = e.y;
      };
      all_sweeps(0, n_list, from_list);
      __syncthreads();  // the list is rewritten by the next pass
    }
  }

  // ---------------- combine: lane groups, hi/lo columns, then the 4 waves ----------------
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) {  // column c + column c^8 (rotate by 8 inside the 16-lane row)
      const int other = __builtin_amdgcn_mov_dpp(__float_as_int(o[i][j]), 0x128, 0xf, 0xf, true);
      o[i][j] += __int_as_float(other);
    }

  __shared__ float sm_m[4][8], sm_l[4][8];
  __shared__ __attribute__((aligned(16))) float sm_o[4][8][HS_D];
  if (c < 8) {
    if (a == 0) { sm_m[w][c] = m_run; sm_l[w][c] = l_run; }
#pragma unroll
    for (int mb = 0; mb < 8; mb++)
      *reinterpret_cast<float4*>(&sm_o[w][c][16 * mb + 4 * a]) = make_float4(o[mb][0], o[mb][1], o[mb][2], o[mb][3]);
  }
  __syncthreads();
  // thread -> (head g = tid / 32, 4 channels)
  const int g = tid >> 5, ch = (tid & 31) * 4;
  const int64_t hq = (int64_t)b * Hq + hkv * G + (g < G ? g : 0);
  if (g < G) {
    float mstar = fmaxf(fmaxf(sm_m[0][g], sm_m[1][g]), fmaxf(sm_m[2][g], sm_m[3][g]));
    float lsum = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (mstar > -INFINITY) {
#pragma unroll
      for (int ww = 0; ww < 4; ww++) {
        const float f = __builtin_amdgcn_exp2f(sm_m[ww][g] - mstar);
        lsum += f * sm_l[ww][g];
#pragma unroll
        for (int i = 0; i < 4; i++) acc[i] += f * sm_o[ww][g][ch + i];
      }
    }
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
    float* po = ws_o + (hq * n_splits + split) * HS_D + ch;
    *reinterpret_cast<float4*>(po) = make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
    if ((tid & 31) == 0)
      ws_l[hq * n_splits + split] = lsum > 0.f ? (mstar + __builtin_amdgcn_logf(lsum)) * kLn2 : -INFINITY;
  }
}

// Merge of the split partials (Sec. IV-C "lightweight post-processing kernel"):
// O = sum_s e^{LSE_s - M} O_s / sum_s e^{LSE_s - M}, M = max_s LSE_s, done in one pass with a
// running reference per thread.  One workgroup of 256 threads per (b, query head):
// thread = (split lane tid/32 of 8, 4 channels); the 8 split lanes are combined in LDS.
// A separate launch on purpose: folding it into the split kernel ("last workgroup to arrive
// merges") needs device-scope visibility between workgroups on different XCDs, and both ways
// of getting it (a device-wide fence per workgroup, or write-through stores and L2-bypassing
// loads) measured slower than this launch.
template <bool F16>
__global__ __launch_bounds__(256) void decode_merge_kernel(int n_splits, const float* __restrict__ ws_o,
                                                           const float* __restrict__ ws_l, uint16_t* __restrict__ O,
                                                           float* __restrict__ LSE) {
  __shared__ float sm_acc[8][HS_D];
  __shared__ float sm_ml[8][2];
  const int hq = blockIdx.x, tid = threadIdx.x, sl = tid >> 5, ch = (tid & 31) * 4;
  const float* po = ws_o + (int64_t)hq * n_splits * HS_D + ch;
  const float* pl = ws_l + (int64_t)hq * n_splits;
  float M = -INFINITY, den = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int s = sl; s < n_splits; s += 8) {
    const float lse = pl[s];
    const float4 v = *reinterpret_cast<const float4*>(po + (int64_t)s * HS_D);
    if (lse > -INFINITY) {
      const float Mn = fmaxf(M, lse);
      const float fo = __expf(M - Mn), fn = __expf(lse - Mn);  // fo = 0 while M is still -inf
      den = den * fo + fn;
      acc[0] = acc[0] * fo + fn * v.x; acc[1] = acc[1] * fo + fn * v.y;
      acc[2] = acc[2] * fo + fn * v.z; acc[3] = acc[3] * fo + fn * v.w;
      M = Mn;
    }
  }
  if ((tid & 31) == 0) { sm_ml[sl][0] = M; sm_ml[sl][1] = den; }
#pragma unroll
  for (int i = 0; i < 4; i++) sm_acc[sl][ch + i] = acc[i];
  __syncthreads();
  if (tid < HS_D) {
    float Mt = -INFINITY;
#pragma unroll
    for (int k = 0; k < 8; k++) Mt = fmaxf(Mt, sm_ml[k][0]);
    float num = 0.f, d = 0.f;
    if (Mt > -INFINITY) {
#pragma unroll
      for (int k = 0; k < 8; k++) {
        const float f = __expf(sm_ml[k][0] - Mt);  // 0 for a split lane that saw nothing
        num += f * sm_acc[k][tid];
        d += f * sm_ml[k][1];
      }
    }
    const float out = d > 0.f ? num / d : 0.f;
    O[(int64_t)hq * HS_D + tid] = (uint16_t)(hs_elem<F16>::pack2(out, 0.f) & 0xffffu);
    if (LSE != nullptr && tid == 0) LSE[hq] = d > 0.f ? Mt + __logf(d) : -INFINITY;
  }
}


// Partial for the dense tail (at most one tile of not yet compressed tokens): plain fp32
// attention of the G query heads of one kv head over tail_len tokens, written as split `slot`.
// One workgroup per (kv head, b); thread t: phase 1 token t%64 for heads t/64 and t/64 + 4,
// phase 3 channel t%128 for heads t/128, t/128 + 2, ...
template <bool F16>
__global__ __launch_bounds__(256) void decode_tail_kernel(int Hq, int Hkv, float scale_log2, int n_slots, int slot,
                                                          int tail_len, const int32_t* __restrict__ tail_lens,
                                                          const uint16_t* __restrict__ Q,
                                                          const uint16_t* __restrict__ TK,
                                                          const uint16_t* __restrict__ TV, float* __restrict__ ws_o,
                                                          float* __restrict__ ws_l) {
  __shared__ float sq[8][HS_D];
  __shared__ float sp[8][HS_BT];
  __shared__ float sl_[8];
  const int tid = threadIdx.x, hkv = blockIdx.x, b = blockIdx.y;
  const int G = Hq / Hkv;
  if (tail_lens != nullptr) tail_len = min(max(tail_lens[b], 0), HS_BT);  // one per batch row, kept inside the tail buffer
  const int64_t hq0 = (int64_t)b * Hq + (int64_t)hkv * G;
  const uint16_t* tk = TK + ((int64_t)b * Hkv + hkv) * HS_BT * HS_D;
  const uint16_t* tv = TV + ((int64_t)b * Hkv + hkv) * HS_BT * HS_D;
  for (int i = tid; i < G * HS_D; i += 256) sq[i / HS_D][i % HS_D] = hs_elem<F16>::to_f32(Q[hq0 * HS_D + i]);
  __syncthreads();
  {  // scores (log2 units) and softmax numerators: wave w serves heads w and w + 4, lane = token
    const int tok = tid & 63, w = tid >> 6;
    for (int g = w; g < G; g += 4) {
      float sc = -INFINITY;
      if (tok < tail_len) {
        float acc = 0.f;
        for (int c = 0; c < HS_D; c += 8) {
          const uint4 kk = *reinterpret_cast<const uint4*>(tk + (int64_t)tok * HS_D + c);
          const uint32_t wds[4] = {kk.x, kk.y, kk.z, kk.w};
#pragma unroll
          for (int e = 0; e < 4; e++) {
            acc = fmaf(hs_elem<F16>::lo_f32(wds[e]), sq[g][c + 2 * e], acc);
            acc = fmaf(hs_elem<F16>::hi_f32(wds[e]), sq[g][c + 2 * e + 1], acc);
          }
        }
        sc = acc * scale_log2;
      }
      float mx = sc;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
      const float p = tok < tail_len ? __builtin_amdgcn_exp2f(sc - mx) : 0.f;
      float l = p;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
      sp[g][tok] = p;
      if (tok == 0) {
        sl_[g] = l;
        ws_l[(hq0 + g) * n_slots + slot] = l > 0.f ? (mx + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
      }
    }
  }
  __syncthreads();
  {
    const int ch = tid & 127;
    for (int g = tid >> 7; g < G; g += 2) {
      float acc = 0.f;
      for (int t = 0; t < tail_len; t++) acc = fmaf(sp[g][t], hs_elem<F16>::to_f32(tv[(int64_t)t * HS_D + ch]), acc);
      const float l = sl_[g];
      ws_o[((hq0 + g) * n_slots + slot) * HS_D + ch] = l > 0.f ? acc / l : 0.f;
    }
  }
}

}  // namespace

// Split partials of hs_decode_attn_static: a fixed array in device memory, one copy per GPU the
// library is loaded on, held until the process ends.  In host code the name `scratch` is only a
// handle for hipGetSymbolAddress; the address kernels and copies use is the one looked up below.
static __device__ __align__(256) unsigned char scratch[HS_STATIC_SCRATCH_BYTES];

hipError_t hs_static_scratch(void** ptr, size_t* bytes) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* per_device[kMaxDevices] = {};  // each GPU has its own copy of the array at its own address
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (per_device[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // for the current device
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    per_device[dev] = p;
  }
  *ptr = per_device[dev];
  *bytes = HS_STATIC_SCRATCH_BYTES;
  return hipSuccess;
}

// Workspace: [partial O (normalised) [B*Hq][n_splits][128] fp32][partial LSE [B*Hq][n_splits] fp32].
template <int KM, int VM, int MODE>
static hipError_t launch_split(dim3 grid, hipStream_t st, int Hq, int Hkv, int T, float sl2, int n_splits, int per,
                               const uint16_t* Q, const hs_kv_dev& kv, float* wo, float* wl, bool f16) {
  if (f16)
    hipLaunchKernelGGL((decode_split_kernel<KM, VM, MODE, true>), grid, dim3(256), 0, st, Hq, Hkv, T, sl2, n_splits,
                       per, Q, kv, wo, wl);
  else
    hipLaunchKernelGGL((decode_split_kernel<KM, VM, MODE, false>), grid, dim3(256), 0, st, Hq, Hkv, T, sl2, n_splits,
                       per, Q, kv, wo, wl);
  return hipGetLastError();
}

hipError_t hs_launch_decode(int B, int Hq, int Hkv, int T, float scale, int n_work, const uint16_t* Q, hs_kv_dev kv,
                            const uint16_t* tail_k, const uint16_t* tail_v, int tail_len, const int32_t* tail_lens,
                            uint16_t* O, float* LSE, float* ws, hipStream_t st, int phases, int dtype) {
  const dim3 grid(n_work, Hkv, B);
  const bool f16 = dtype == HS_FP16;
  const float sl2 = scale * kLog2e;
  const int per = (T + n_work - 1) / n_work;
  // partial slots per query head: the n_work cache splits, then one for the dense tail if there is
  // one (the kernels take the slot count as their stride)
  const int n_splits = n_work + (tail_len >= 0 ? 1 : 0);
  float* wo = ws;
  float* wl = wo + (size_t)B * Hq * n_splits * HS_D;
  const int km = kv.cap_dense_k == 0 ? 0 : (kv.cap_sparse_k == 0 ? 1 : 2);
  const int vm = kv.cap_dense_v == 0 ? 0 : (kv.cap_sparse_v == 0 ? 1 : 2);
  hipError_t e = hipSuccess;
  if (phases & 1) {
  // tiles by count on long splits only: the two passes over the maps at kernel start cost about 3 us, which
  // the even shares win back (3-7 % of the kernel when tiles are skipped) from 128 tiles per split for
  // all-2:4 tensors and from 256 for the other kernels (measured)
  const bool by_count = per >= (km == 0 && vm == 0 ? HS_DEC_BYCOUNT_MIN_PER : 2 * HS_DEC_BYCOUNT_MIN_PER);
#define HS_GO_DYN(KM_, VM_)                                                                                            \
  e = by_count ? launch_split<KM_, VM_, kByCount>(grid, st, Hq, Hkv, T, sl2, n_splits, per, Q, kv, wo, wl, f16)       \
               : launch_split<KM_, VM_, kByRange>(grid, st, Hq, Hkv, T, sl2, n_splits, per, Q, kv, wo, wl, f16);      \
  break
#define HS_GO(KM_, VM_)                                                                                       \
  if (kv.uniform) {                                                                                           \
    e = launch_split<KM_, VM_, kUniform>(grid, st, Hq, Hkv, T, sl2, n_splits, per, Q, kv, wo, wl, f16);       \
    break;                                                                                                    \
  }                                                                                                           \
  HS_GO_DYN(KM_, VM_)
  switch (km * 3 + vm) {
    case 0: HS_GO(0, 0);
    case 1: HS_GO(0, 1);
    case 2: HS_GO_DYN(0, 2);
    case 3: HS_GO(1, 0);
    case 4: HS_GO(1, 1);
    case 5: HS_GO_DYN(1, 2);
    case 6: HS_GO_DYN(2, 0);
    case 7: HS_GO_DYN(2, 1);
    default: HS_GO_DYN(2, 2);
  }
#undef HS_GO
#undef HS_GO_DYN
  }
  if (e == hipSuccess && (phases & 1) && tail_len >= 0) {
    if (f16)
      hipLaunchKernelGGL(decode_tail_kernel<true>, dim3(Hkv, B), dim3(256), 0, st, Hq, Hkv, sl2, n_splits, n_work,
                         tail_len, tail_lens, Q, tail_k, tail_v, wo, wl);
    else
      hipLaunchKernelGGL(decode_tail_kernel<false>, dim3(Hkv, B), dim3(256), 0, st, Hq, Hkv, sl2, n_splits, n_work,
                         tail_len, tail_lens, Q, tail_k, tail_v, wo, wl);
    e = hipGetLastError();
  }
  if (e != hipSuccess || !(phases & 2)) return e;
  if (f16)
    hipLaunchKernelGGL(decode_merge_kernel<true>, dim3(B * Hq), dim3(256), 0, st, n_splits, wo, wl, O, LSE);
  else
    hipLaunchKernelGGL(decode_merge_kernel<false>, dim3(B * Hq), dim3(256), 0, st, n_splits, wo, wl, O, LSE);
  return hipGetLastError();
}
