// Compress path: tile scoring, tile selection, fused 2:4 prune + pack, and unpack.
// Paper: hierarchical pruner Sec. III-A (Eq. 2a-d), cache compressor Sec. III-B,
// fused magnitude compressor Sec. IV-B.
#include "hs_common.h"

namespace {

constexpr int kVStride = 132;  // LDS row stride (elements) of a staged V tile: 8-byte aligned rows, shifted banks

// 16-byte global accesses of the compressor.  Every input byte is read once and every output byte
// written once per call, so the pool bytes of 2:4 tiles are written with non-temporal stores, and
// their inputs read non-temporally when the tensors are large (pack_kernel); for tiles that stay
// dense, where as many bytes are written as read, the plain forms measured faster and are kept.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ uint4 ld16(const void* p) {
  if (NT) return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p)));
  return *reinterpret_cast<const uint4*>(p);
}
template <bool NT>
__device__ __forceinline__ void st16(void* p, uint4 v) {
  if (NT) __builtin_nontemporal_store(__builtin_bit_cast(u32x4_t, v), reinterpret_cast<u32x4_t*>(p));
  else *reinterpret_cast<uint4*>(p) = v;
}

// Top-2-of-4 by magnitude (Eq. 2a-b with an exact count of two): x0..x3 are bf16 bit
// patterns; element j outranks element i if |x_j| > |x_i|, or |x_j| == |x_i| and j < i.
// Returns the 4-bit keep mask (exactly two bits set).
// rule != 0 (input already masked): the key is "non-zero" instead of the magnitude, so the
// non-zero entries win and ties (zeros) go to the lower position.
__device__ __forceinline__ uint32_t top2_mask(uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3, int rule) {
  uint32_t k0 = x0 & 0x7fffu, k1 = x1 & 0x7fffu, k2 = x2 & 0x7fffu, k3 = x3 & 0x7fffu;
  if (rule != 0) { k0 = k0 != 0; k1 = k1 != 0; k2 = k2 != 0; k3 = k3 != 0; }
  const uint32_t g01 = k0 >= k1, g02 = k0 >= k2, g03 = k0 >= k3, g12 = k1 >= k2, g13 = k1 >= k3, g23 = k2 >= k3;
  const uint32_t c0 = 3u - g01 - g02 - g03;        // how many outrank element 0
  const uint32_t c1 = g01 + 2u - g12 - g13;
  const uint32_t c2 = g02 + g12 + 1u - g23;
  const uint32_t c3 = g03 + g13 + g23;
  return (c0 < 2u) | ((c1 < 2u) << 1) | ((c2 < 2u) << 2) | ((c3 < 2u) << 3);
}

// From the keep mask: the two kept values packed (lower position in the low half) and
// the metadata nibble i0 | i1 << 2 (Sec. IV-B: 2-bit position of each kept element).
__device__ __forceinline__ void top2_emit(uint32_t mask, uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3,
                                          uint32_t& vals, uint32_t& nib) {
  const uint32_t i0 = (uint32_t)__builtin_ctz(mask);
  const uint32_t i1 = 31u - (uint32_t)__builtin_clz(mask);
  const uint32_t v0 = (mask & 1u) ? x0 : ((mask & 2u) ? x1 : x2);
  const uint32_t v1 = (mask & 8u) ? x3 : ((mask & 4u) ? x2 : x1);
  vals = (v0 & 0xffffu) | (v1 << 16);
  nib = i0 | (i1 << 2);
}

template <bool F16> __device__ __forceinline__ double elem_val(uint32_t bits) { return (double)hs_elem<F16>::to_f32(bits); }

// ----------------------------------------------------------------------------------
// Staging of one V tile [64 tokens][128 ch] into LDS with coalesced 16-byte loads.
// ----------------------------------------------------------------------------------
template <bool NT = false>
__device__ __forceinline__ void stage_v_tile(const uint16_t* vt, int64_t tok_stride, uint16_t* lds) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int q = tid + 256 * i;
    const int tok = q >> 4, c8 = q & 15;
    const uint4 d = ld16<NT>(vt + tok * tok_stride + 8 * c8);
    uint2* dst = reinterpret_cast<uint2*>(lds + tok * kVStride + 8 * c8);
    dst[0] = make_uint2(d.x, d.y);
    dst[1] = make_uint2(d.z, d.w);
  }
}

// ----------------------------------------------------------------------------------
// Tile scores: energy = sum K^2 + sum V^2 (skip ranking), loss_x = L1 norm of what the
// 2:4 mask removes (Eq. 2c).  fp64 (every term exact), fixed reduction order.
// scores = [3][rows][T].  WHAT: bit 0 = the policy ranks by energy, bit 1 = by the losses; a
// plane that is not asked for is written as zeros (the selection then falls back to tile order
// there, which is all it needs when a count is 0 or everything).
// ----------------------------------------------------------------------------------
template <bool F16> __device__ __forceinline__ double sum_sq8(uint4 d) {  // sum of squares of 8 elements
  const uint32_t w[4] = {d.x, d.y, d.z, d.w};
  double e = 0.0;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const double f0 = elem_val<F16>(w[i] & 0xffffu), f1 = elem_val<F16>(w[i] >> 16);
    e += f0 * f0 + f1 * f1;
  }
  return e;
}

// sum of the magnitudes of the two elements of a group that the 2:4 mask drops
template <bool F16>
__device__ __forceinline__ double dropped_l1(uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3, int rule) {
  const uint32_t drop = ~top2_mask(x0, x1, x2, x3, rule) & 15u;
  uint32_t pair, nib;
  top2_emit(drop, x0, x1, x2, x3, pair, nib);
  return fabs(elem_val<F16>(pair & 0xffffu)) + fabs(elem_val<F16>(pair >> 16));
}

// NT: non-temporal reads in the energy-only form.  They pay when K and V exceed the last-level
// cache (B 8 x L 131072: 1.32 -> 1.26 ms for score + select + pack) and cost when they fit, because
// the pack kernel's second read of the kept tiles then no longer hits that cache (L 32768: 56 -> 60 us).
template <bool F16, int WHAT, bool NT>
__global__ __launch_bounds__(256) void score_kernel(const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                                                    int64_t sb, int64_t sh, int64_t st, int Hkv, int T, int rule,
                                                    double* __restrict__ scores) {
  constexpr bool ENERGY = (WHAT & 1) != 0, LOSS = (WHAT & 2) != 0;
  __shared__ uint16_t vl[LOSS ? HS_BT * kVStride : 8];
  __shared__ double red[3][4];
  const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, a = l >> 4, r = l & 15;
  const uint16_t* kt = K + b * sb + h * sh + (int64_t)t * HS_BT * st;
  const uint16_t* vt = V + b * sb + h * sh + (int64_t)t * HS_BT * st;
  double e = 0.0, lk = 0.0, lv = 0.0;
  if (!LOSS) {
    // energy alone does not care which thread sees which element: coalesced 16-byte reads
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int q = tid + 256 * i, tok = q >> 4, c8 = q & 15;
      e += sum_sq8<F16>(ld16<NT>(kt + tok * st + 8 * c8));
      e += sum_sq8<F16>(ld16<NT>(vt + tok * st + 8 * c8));
    }
  } else {
    stage_v_tile(vt, st, vl);
    {  // K: this thread owns token 16w+r, channels 64kb+16a .. +15
      const uint16_t* row = kt + (int64_t)(16 * w + r) * st;
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
        const uint4 d0 = *reinterpret_cast<const uint4*>(row + 64 * kb + 16 * a);
        const uint4 d1 = *reinterpret_cast<const uint4*>(row + 64 * kb + 16 * a + 8);
        if (ENERGY) e += sum_sq8<F16>(d0) + sum_sq8<F16>(d1);
        const uint32_t wds[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
#pragma unroll
        for (int q = 0; q < 4; q++)
          lk += dropped_l1<F16>(wds[2 * q] & 0xffffu, wds[2 * q] >> 16, wds[2 * q + 1] & 0xffffu, wds[2 * q + 1] >> 16, rule);
      }
    }
    __syncthreads();
    {  // V: channel 16mb+r for mb = 2w, 2w+1; token groups of lane group a
#pragma unroll
      for (int j = 0; j < 2; j++) {
        const int c = 16 * (2 * w + j) + r;
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const int g = hs_v_group(a, q);
          const uint32_t x0 = vl[(4 * g + 0) * kVStride + c], x1 = vl[(4 * g + 1) * kVStride + c];
          const uint32_t x2 = vl[(4 * g + 2) * kVStride + c], x3 = vl[(4 * g + 3) * kVStride + c];
          if (ENERGY) {
            const double f0 = elem_val<F16>(x0), f1 = elem_val<F16>(x1), f2 = elem_val<F16>(x2), f3 = elem_val<F16>(x3);
            e += f0 * f0 + f1 * f1 + f2 * f2 + f3 * f3;
          }
          lv += dropped_l1<F16>(x0, x1, x2, x3, rule);
        }
      }
    }
  }
  // wave reduction (fixed butterfly), then 4 partials in LDS
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    e += __shfl_xor(e, off);
    if (LOSS) {
      lk += __shfl_xor(lk, off);
      lv += __shfl_xor(lv, off);
    }
  }
  if (l == 0) { red[0][w] = e; red[1][w] = lk; red[2][w] = lv; }
  __syncthreads();
  if (tid < 3) {
    const int64_t rows = (int64_t)gridDim.z * Hkv;
    const int64_t row = (int64_t)b * Hkv + h;
    scores[(tid * rows + row) * T + t] = (red[tid][0] + red[tid][1]) + (red[tid][2] + red[tid][3]);
  }
}

// ----------------------------------------------------------------------------------
// Tile selection per (b, kv head) row (Eq. 2d + the skip extension) and slot assignment (the two
// sequential counters of Sec. III-B, done as an exclusive prefix count), one workgroup per row.
// "The n tiles with the lowest (score, tile index)" is found by radix selection instead of by
// ranking every tile: scores are non-negative doubles, whose bit patterns order like unsigned
// integers; eight rounds of a 256-bin histogram over one byte each, from the top, pin down the
// key of the n-th smallest eligible tile (thr) and how many tiles with exactly that key belong
// to the set (take, by ascending tile index; see mark_lowest).  Every thread owns a contiguous run of tiles, so
// "ascending tile index" is thread order, and a thread only re-reads map entries it wrote itself.
// ----------------------------------------------------------------------------------
struct SelectShared {
  int hist[256];
  int wsum[4];
  int bin, want;
};

__device__ __forceinline__ int block_exclusive_scan(int v, int* wsum, int tid) {  // 256 threads; contains barriers
  const int l = tid & 63, w = tid >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int n = __shfl_up(incl, off);
    if (l >= off) incl += n;
  }
  __syncthreads();  // wsum may still be read from the previous call
  if (l == 63) wsum[w] = incl;
  __syncthreads();
  int base = 0;
  for (int i = 0; i < w; i++) base += wsum[i];
  return base + incl - v;
}

// The keys of this thread's tiles [t0, t1) that take part (eligible), held in registers when the
// run is short (kCache tiles: rows up to 2048 tiles), else re-read from memory on every pass.
constexpr int kCache = 8;
struct TileKeys {
  const double* keys;
  int t0, t1;
  bool cached;
  unsigned long long k[kCache];
  unsigned elig;  // bit i: tile t0 + i takes part (cached form)
};

template <class Eligible>
__device__ __forceinline__ TileKeys load_keys(const double* __restrict__ keys, int t0, int t1, int per, Eligible eligible) {
  TileKeys tk;
  tk.keys = keys; tk.t0 = t0; tk.t1 = t1; tk.cached = per <= kCache; tk.elig = 0;
#pragma unroll
  for (int i = 0; i < kCache; i++) {
    const int t = t0 + i;
    const bool e = tk.cached && t < t1 && eligible(t);
    tk.k[i] = e ? (unsigned long long)__double_as_longlong(keys[t]) : 0ull;
    tk.elig |= (unsigned)e << i;
  }
  return tk;
}

// f(t, key) for every eligible tile of the thread, ascending t
template <class Eligible, class F>
__device__ __forceinline__ void for_each_key(const TileKeys& tk, Eligible eligible, F f) {
  if (tk.cached) {
#pragma unroll
    for (int i = 0; i < kCache; i++)
      if ((tk.elig >> i) & 1u) f(tk.t0 + i, tk.k[i]);
  } else {
    for (int t = tk.t0; t < tk.t1; t++)
      if (eligible(t)) f(t, (unsigned long long)__double_as_longlong(tk.keys[t]));
  }
}

// Marks the n eligible tiles with the lowest (key, tile index): key < thr, or key == thr and among
// the first `take` such tiles.  `per` = tiles per thread (uniform).
template <class Eligible, class Mark>
__device__ __forceinline__ void mark_lowest(const double* __restrict__ keys, int t0, int t1, int per, Eligible eligible,
                                            int n, SelectShared& sm, int tid, Mark mark) {
  if (n <= 0) return;  // uniform: nobody is in the set
  const TileKeys tk = load_keys(keys, t0, t1, per, eligible);
  unsigned long long prefix = 0;
  int want = n;
  for (int d = 7; d >= 0; d--) {
    sm.hist[tid] = 0;
    __syncthreads();
    for_each_key(tk, eligible, [&](int, unsigned long long k) {
      if (d == 7 || (k >> (8 * (d + 1))) == (prefix >> (8 * (d + 1)))) atomicAdd(&sm.hist[(k >> (8 * d)) & 255], 1);
    });
    __syncthreads();
    const int h = sm.hist[tid];
    const int excl = block_exclusive_scan(h, sm.wsum, tid);
    if (excl < want && want <= excl + h) { sm.bin = tid; sm.want = want - excl; }
    __syncthreads();
    prefix |= (unsigned long long)sm.bin << (8 * d);
    want = sm.want;
  }
  const unsigned long long thr = prefix;
  const int take = want;
  int ties = 0;
  for_each_key(tk, eligible, [&](int, unsigned long long k) { ties += k == thr; });
  int tie_rank = block_exclusive_scan(ties, sm.wsum, tid);
  for_each_key(tk, eligible, [&](int t, unsigned long long k) {
    if (k < thr || (k == thr && tie_rank++ < take)) mark(t);
  });
}

// Tiles t < n_first or t >= T - n_last are protected: always kept dense, outside both rankings.
// Tile states live in registers while the selection runs (2 bits per tile) when a thread's run is
// short, else in the map arrays themselves; the maps are written once, at the end.
__global__ __launch_bounds__(256) void select_kernel(const double* __restrict__ scores, int rows, int T, int n_skip,
                                                     int n_sparse_k, int n_sparse_v, int n_first, int n_last,
                                                     int32_t* __restrict__ k_map, int32_t* __restrict__ v_map) {
  __shared__ SelectShared sm;
  const int row = blockIdx.x, tid = threadIdx.x;
  const double* en = scores + (int64_t)row * T;                // plane 0 = energy
  const double* lk = scores + ((int64_t)1 * rows + row) * T;   // planes 1, 2 = pruning losses
  const double* lv = scores + ((int64_t)2 * rows + row) * T;
  int32_t* km = k_map + (int64_t)row * T;
  int32_t* vm = v_map + (int64_t)row * T;
  const int per = (T + 255) / 256;
  const int t0 = min(tid * per, T), t1 = min(t0 + per, T);
  const bool in_regs = per <= kCache;
  unsigned rk = 0x5555u, rv = 0x5555u;  // HS_DENSE everywhere
  static_assert(HS_DENSE == 1 && 2 * kCache <= 32, "packed tile states");
  auto state_k = [&](int t) -> int { return in_regs ? (rk >> (2 * (t - t0))) & 3u : km[t]; };
  auto state_v = [&](int t) -> int { return in_regs ? (rv >> (2 * (t - t0))) & 3u : vm[t]; };
  auto set_k = [&](int t, int v) {
    if (in_regs) rk = (rk & ~(3u << (2 * (t - t0)))) | ((unsigned)v << (2 * (t - t0)));
    else km[t] = v;
  };
  auto set_v = [&](int t, int v) {
    if (in_regs) rv = (rv & ~(3u << (2 * (t - t0)))) | ((unsigned)v << (2 * (t - t0)));
    else vm[t] = v;
  };
  auto is_protected = [&](int t) { return t < n_first || t >= T - n_last; };
  if (!in_regs)
    for (int t = t0; t < t1; t++) km[t] = vm[t] = HS_DENSE;
  // the n_skip lowest-energy tiles are skipped
  mark_lowest(en, t0, t1, per, [&](int t) { return !is_protected(t); }, n_skip, sm, tid,
              [&](int t) { set_k(t, HS_SKIP); set_v(t, HS_SKIP); });
  // of the kept ones, the n_sparse_x with the lowest pruning loss are 2:4 (all of them: no ranking)
  auto kept = [&](int t) { return !is_protected(t) && state_k(t) != HS_SKIP; };
  const int n_keep = T - n_first - n_last - n_skip;
  if (n_sparse_k >= n_keep) {
    for (int t = t0; t < t1; t++) if (kept(t)) set_k(t, HS_SPARSE24);
  } else {
    mark_lowest(lk, t0, t1, per, kept, n_sparse_k, sm, tid, [&](int t) { set_k(t, HS_SPARSE24); });
  }
  if (n_sparse_v >= n_keep) {
    for (int t = t0; t < t1; t++) if (kept(t)) set_v(t, HS_SPARSE24);
  } else {
    mark_lowest(lv, t0, t1, per, kept, n_sparse_v, sm, tid, [&](int t) { set_v(t, HS_SPARSE24); });
  }
  // slots in ascending tile order
  int n[4] = {0, 0, 0, 0};  // dense K, 2:4 K, dense V, 2:4 V
  for (int t = t0; t < t1; t++) {
    const int sk = state_k(t), sv = state_v(t);
    n[0] += sk == HS_DENSE; n[1] += sk == HS_SPARSE24; n[2] += sv == HS_DENSE; n[3] += sv == HS_SPARSE24;
  }
#pragma unroll
  for (int i = 0; i < 4; i++) n[i] = block_exclusive_scan(n[i], sm.wsum, tid);
  for (int t = t0; t < t1; t++) {
    const int sk = state_k(t), sv = state_v(t);
    km[t] = sk == HS_DENSE ? ++n[0] : (sk == HS_SPARSE24 ? -(++n[1]) : 0);
    vm[t] = sv == HS_DENSE ? ++n[2] : (sv == HS_SPARSE24 ? -(++n[3]) : 0);
  }
}

// ----------------------------------------------------------------------------------
// Slot assignment for one row from known tile states (the two sequential counters per tensor of
// Sec. III-B): tile t in state (sk, sv) = state(t) takes the next slot of the pool each state names.
// A tile is stored only if both of its pools still have a free slot when its turn comes; otherwise
// it is left out of K and V alike, takes no slot in either pool (so the used slots of a pool are
// always 0 .. count-1 with no holes, which is what appending relies on), and bit 0 of *flag is set.
// state(t) must return a consistent pair (both SKIP or neither).  emit(t, mk, mv) receives the map
// entries +-(slot + 1) or 0.  One workgroup of 256 threads per row; each thread owns a contiguous
// run of tiles.  When everything fits (the totals say so) the slots are prefix counts; a row that
// overflows is walked again by one thread, in order, so that which tiles survive is exactly what a
// sequential walk gives.
// ----------------------------------------------------------------------------------
struct SlotShared {
  int wsum[4];
  int total[4];
};

template <class State, class Emit>
__device__ __forceinline__ void assign_slots_row(int T, int tid, int cap_dk, int cap_sk, int cap_dv, int cap_sv,
                                                 SlotShared& sm, int32_t* flag, State state, Emit emit) {
  const int per = (T + 255) / 256;
  const int t0 = min(tid * per, T), t1 = min(t0 + per, T);
  int n[4] = {0, 0, 0, 0};  // dense K, 2:4 K, dense V, 2:4 V
  for (int t = t0; t < t1; t++) {
    int sk, sv;
    state(t, sk, sv);
    n[0] += sk == HS_DENSE; n[1] += sk == HS_SPARSE24; n[2] += sv == HS_DENSE; n[3] += sv == HS_SPARSE24;
  }
  int base[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    base[i] = block_exclusive_scan(n[i], sm.wsum, tid);
    if (tid == 255) sm.total[i] = base[i] + n[i];
  }
  __syncthreads();
  const bool all_fit = sm.total[0] <= cap_dk && sm.total[1] <= cap_sk && sm.total[2] <= cap_dv && sm.total[3] <= cap_sv;
  if (all_fit) {
    for (int t = t0; t < t1; t++) {
      int sk, sv;
      state(t, sk, sv);
      const int mk = sk == HS_DENSE ? ++base[0] : (sk == HS_SPARSE24 ? -(++base[1]) : 0);
      const int mv = sv == HS_DENSE ? ++base[2] : (sv == HS_SPARSE24 ? -(++base[3]) : 0);
      emit(t, mk, mv);
    }
  } else if (tid == 0) {
    int c[4] = {0, 0, 0, 0};
    bool dropped = false;
    for (int t = 0; t < T; t++) {
      int sk, sv;
      state(t, sk, sv);
      int mk = 0, mv = 0;
      if (sk != HS_SKIP) {
        const bool room_k = sk == HS_DENSE ? c[0] < cap_dk : c[1] < cap_sk;
        const bool room_v = sv == HS_DENSE ? c[2] < cap_dv : c[3] < cap_sv;
        if (room_k && room_v) {
          mk = sk == HS_DENSE ? ++c[0] : -(++c[1]);
          mv = sv == HS_DENSE ? ++c[2] : -(++c[3]);
        } else {
          dropped = true;
        }
      }
      emit(t, mk, mv);
    }
    if (dropped && flag != nullptr) atomicOr(flag, 1);
  }
}

// Explicit per-tile states (device int8 [rows, T], the block-level masks a pruner hands over:
// Sec. III-A, "agnostic to the pruning algorithms") -> signed index maps (Sec. III-B).  A pair of
// states that is not valid (a value outside SKIP / DENSE / SPARSE24, or a tile skipped in only one
// of K and V) is stored as SKIP in both tensors and sets bit 1 of *flag.
__global__ __launch_bounds__(256) void states_to_maps_kernel(const int8_t* __restrict__ state_k,
                                                             const int8_t* __restrict__ state_v, int T, int cap_dk,
                                                             int cap_sk, int cap_dv, int cap_sv,
                                                             int32_t* __restrict__ k_map, int32_t* __restrict__ v_map,
                                                             int32_t* flag) {
  __shared__ SlotShared sm;
  const int row = blockIdx.x, tid = threadIdx.x;
  const int8_t* sk_row = state_k + (int64_t)row * T;
  const int8_t* sv_row = state_v + (int64_t)row * T;
  int32_t* km = k_map + (int64_t)row * T;
  int32_t* vm = v_map + (int64_t)row * T;
  bool invalid = false;
  assign_slots_row(
      T, tid, cap_dk, cap_sk, cap_dv, cap_sv, sm, flag,
      [&](int t, int& sk, int& sv) {
        sk = sk_row[t];
        sv = sv_row[t];
        if (sk < 0 || sk > 2 || sv < 0 || sv > 2 || (sk == HS_SKIP) != (sv == HS_SKIP)) {
          invalid = true;
          sk = sv = HS_SKIP;
        }
      },
      [&](int t, int mk, int mv) { km[t] = mk; vm[t] = mv; });
  if (invalid && flag != nullptr) atomicOr(flag, 2);
}

// Appending (Sec. III-B counters): map entries of tiles [tile, tile + n_tiles) of every row = the
// next slots of the pool their state names, counted from how many tiles of that kind the row
// holds; tiles for which a pool has no slot left stay skipped and raise *overflow.  One workgroup
// per row.
// tile_rows (or NULL): one tile index per batch row instead of `tile` (then n_tiles = 1); a batch
// row whose entry is not a tile index is left as it is.
__global__ __launch_bounds__(256) void append_slots_kernel(int Hkv, int T, int tile, int n_tiles,
                                                           const int32_t* __restrict__ tile_rows, int state_k,
                                                           int state_v, hs_kv_dev kv, int32_t* overflow) {
  __shared__ int part[4][4];
  const int row = blockIdx.x, tid = threadIdx.x;
  if (tile_rows != nullptr) {
    tile = tile_rows[row / Hkv];
    if (tile < 0 || tile >= T) return;  // the whole workgroup
  }
  int32_t* km = const_cast<int32_t*>(kv.k_map) + (int64_t)row * T;
  int32_t* vm = const_cast<int32_t*>(kv.v_map) + (int64_t)row * T;
  int n[4] = {0, 0, 0, 0};  // dense K, 2:4 K, dense V, 2:4 V
  for (int t = tid; t < T; t += 256) {
    if (t >= tile && t < tile + n_tiles) continue;
    const int a = km[t], c = vm[t];
    n[0] += a > 0; n[1] += a < 0; n[2] += c > 0; n[3] += c < 0;
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) n[i] += __shfl_xor(n[i], off);
    if ((tid & 63) == 0) part[i][tid >> 6] = n[i];
  }
  __syncthreads();
  int c[4];
#pragma unroll
  for (int i = 0; i < 4; i++) c[i] = part[i][0] + part[i][1] + part[i][2] + part[i][3];
  const int ck = state_k == HS_DENSE ? c[0] : c[1], cv = state_v == HS_DENSE ? c[2] : c[3];
  const int room_k = (state_k == HS_DENSE ? kv.cap_dense_k : kv.cap_sparse_k) - ck;
  const int room_v = (state_v == HS_DENSE ? kv.cap_dense_v : kv.cap_sparse_v) - cv;
  for (int i = tid; i < n_tiles; i += 256) {  // the i-th appended tile takes the i-th free slot of each pool
    const bool fits = i < room_k && i < room_v;
    km[tile + i] = !fits ? 0 : (state_k == HS_DENSE ? ck + i + 1 : -(ck + i + 1));
    vm[tile + i] = !fits ? 0 : (state_v == HS_DENSE ? cv + i + 1 : -(cv + i + 1));
    if (!fits && overflow != nullptr) *overflow = 1;
  }
}

// V tiles of a bf16 cache in fp16 encoding.  A bf16 pair is converted (round to nearest) and read
// back: equal values mean the pair survives the round trip (NaN never does, infinities do).
__device__ __forceinline__ bool pair_to_f16(uint32_t bf_pair, uint32_t& f16_pair) {
  const float f0 = hs_elem<false>::lo_f32(bf_pair), f1 = hs_elem<false>::hi_f32(bf_pair);
  f16_pair = hs_elem<true>::pack2(f0, f1);
  return hs_elem<true>::lo_f32(f16_pair) == f0 && hs_elem<true>::hi_f32(f16_pair) == f1;
}
__device__ __forceinline__ uint32_t pair_to_bf16(uint32_t f16_pair) {  // exact for what pair_to_f16 accepted
  const uint32_t lo = __float_as_uint(hs_elem<true>::lo_f32(f16_pair)), hi = __float_as_uint(hs_elem<true>::hi_f32(f16_pair));
  return (lo >> 16) | (hi & 0xffff0000u);
}

// ----------------------------------------------------------------------------------
// Tile writers shared by the compress, append and re-compress kernels.  Workgroup of 4 waves;
// wave w, lane l = 16a + r.
// ----------------------------------------------------------------------------------
// 2:4 K tile.  Lane (w, a, r) prunes token 16w + r, channels 64kb + 16a .. +16 for kb = 0, 1;
// load(kb, half) returns the 8 channels 64kb + 16a + 8 half .. +8 of that token.
template <class Load>
__device__ __forceinline__ void k_sparse_store(uint8_t* nnz, uint8_t* meta, int w, int l, int rule, Load load) {
  uint32_t idx = 0;
#pragma unroll
  for (int kb = 0; kb < 2; kb++) {
    const uint4 d0 = load(kb, 0);
    const uint4 d1 = load(kb, 1);
    const uint32_t wds[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
    uint32_t out[4];
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const uint32_t x0 = wds[2 * q] & 0xffffu, x1 = wds[2 * q] >> 16, x2 = wds[2 * q + 1] & 0xffffu, x3 = wds[2 * q + 1] >> 16;
      uint32_t nib;
      top2_emit(top2_mask(x0, x1, x2, x3, rule), x0, x1, x2, x3, out[q], nib);
      idx |= nib << (16 * kb + 4 * q);
    }
    st16<true>(nnz + ((w * 2 + kb) * 64 + l) * 16, make_uint4(out[0], out[1], out[2], out[3]));
  }
  *reinterpret_cast<uint32_t*>(meta + (l * 4 + w) * 4) = idx;
}

// V tile (dense if mv > 0, 2:4 if mv < 0; mv = +-(slot + 1), workgroup-uniform, != 0) from the
// tile staged in LDS as vl[token][channel] (row stride kVStride); the caller has synchronised.
// The words to store are built first.  v_f16 (bf16 cache): if every value the tile stores is
// exact in fp16 (workgroup vote), the tile is written in fp16 encoding and *map_entry, which the
// caller has set to mv, gets HS_MAP_F16, so that the attention kernels can feed the softmax
// numerators as one fp16 term.  Every thread of the workgroup must call this.
__device__ __forceinline__ void v_tile_store(const uint16_t* vl, int mv, int32_t* map_entry, const hs_kv_dev& kv,
                                             int64_t row, int rule, int v_f16, int tid) {
  const int w = tid >> 6, l = tid & 63, a = l >> 4, r = l & 15;
  uint32_t words[4][4];
  const int n_chunks = mv > 0 ? 4 : 2;  // 16-byte chunks this lane stores
  uint32_t idx = 0;
  if (mv > 0) {
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int ch = 4 * w + j, mb = ch >> 1, hh = ch & 1;
      const int c = 16 * mb + r;
#pragma unroll
      for (int p = 0; p < 4; p++) {
        const int e0 = 2 * p, e1 = 2 * p + 1;
        const int tok0 = 16 * (2 * hh + (e0 >> 2)) + 4 * a + (e0 & 3);
        const int tok1 = 16 * (2 * hh + (e1 >> 2)) + 4 * a + (e1 & 3);
        words[j][p] = (uint32_t)vl[tok0 * kVStride + c] | ((uint32_t)vl[tok1 * kVStride + c] << 16);
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int mb = 2 * w + j, c = 16 * mb + r;
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int g = hs_v_group(a, q);
        const uint32_t x0 = vl[(4 * g + 0) * kVStride + c], x1 = vl[(4 * g + 1) * kVStride + c];
        const uint32_t x2 = vl[(4 * g + 2) * kVStride + c], x3 = vl[(4 * g + 3) * kVStride + c];
        uint32_t nib;
        top2_emit(top2_mask(x0, x1, x2, x3, rule), x0, x1, x2, x3, words[j][q], nib);
        idx |= nib << (16 * j + 4 * q);
      }
    }
  }
  if (v_f16) {  // workgroup-uniform
    uint32_t conv[4][4];
    int bad = 0;
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int p = 0; p < 4; p++)
        if (j < n_chunks) bad |= !pair_to_f16(words[j][p], conv[j][p]);
    if (!__syncthreads_or(bad)) {
#pragma unroll
      for (int j = 0; j < 4; j++)
#pragma unroll
        for (int p = 0; p < 4; p++)
          if (j < n_chunks) words[j][p] = conv[j][p];
      if (tid == 0) *map_entry = mv > 0 ? (mv | HS_MAP_F16) : -(-mv | HS_MAP_F16);
    }
  }
  if (mv > 0) {
    uint8_t* dst = const_cast<uint8_t*>(kv.v_dense) + (row * kv.cap_dense_v + (mv - 1)) * (int64_t)HS_TILE_DENSE_BYTES;
#pragma unroll
    for (int j = 0; j < 4; j++)
      st16<false>(dst + ((4 * w + j) * 64 + l) * 16, make_uint4(words[j][0], words[j][1], words[j][2], words[j][3]));
  } else {
    const int64_t slot = row * kv.cap_sparse_v + (-mv - 1);
    uint8_t* nnz = const_cast<uint8_t*>(kv.v_nnz) + slot * (int64_t)HS_TILE_NNZ_BYTES;
    uint8_t* meta = const_cast<uint8_t*>(kv.v_meta) + slot * (int64_t)HS_TILE_META_BYTES;
#pragma unroll
    for (int j = 0; j < 2; j++)
      st16<true>(nnz + ((2 * w + j) * 64 + l) * 16, make_uint4(words[j][0], words[j][1], words[j][2], words[j][3]));
    *reinterpret_cast<uint32_t*>(meta + (l * 4 + w) * 4) = idx;
  }
}

// Dense V tile in pool order -> vl[token][channel], as bf16 patterns when the tile is held in fp16
// encoding (is_f16); the caller synchronises afterwards.
__device__ __forceinline__ void v_dense_to_lds(const uint8_t* src, bool is_f16, uint16_t* vl, int tid) {
  const int w = tid >> 6, l = tid & 63, a = l >> 4, r = l & 15;
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const int ch = 4 * w + j, mb = ch >> 1, hh = ch & 1, c = 16 * mb + r;
    const uint4 d = *reinterpret_cast<const uint4*>(src + (ch * 64 + l) * 16);
    uint32_t vals[4] = {d.x, d.y, d.z, d.w};
    if (is_f16) {
#pragma unroll
      for (int i = 0; i < 4; i++) vals[i] = pair_to_bf16(vals[i]);
    }
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const int tok = 16 * (2 * hh + (e >> 2)) + 4 * a + (e & 3);
      vl[tok * kVStride + c] = (uint16_t)((vals[e >> 1] >> (16 * (e & 1))) & 0xffffu);
    }
  }
}

// ----------------------------------------------------------------------------------
// Fused prune + pack (Sec. IV-B): one workgroup per tile, K then V.
// ----------------------------------------------------------------------------------
// uni_k / uni_v: 0 = read the tile's map entries (written by an earlier launch); HS_DENSE or
// HS_SPARSE24 = every tile of that tensor is of this kind, the entry is +-(tile+1) and this
// kernel writes it (saves the separate map-fill launch of the unranked policies).
// NTL: the inputs of tiles that become 2:4 are read non-temporally.  That pays when K and V exceed the
// last-level cache (B 8 x L 131072: 1.20 -> 1.08 ms) and costs a little when they fit (L 32768: 38.7 -> 40.3 us;
// the two 16-byte reads a lane makes of one K line then both go to L2), so the launcher decides by size.
template <bool NTL>
__global__ __launch_bounds__(256) void pack_kernel(const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                                                   int64_t sb, int64_t sh, int64_t st, int Hkv, int T, hs_kv_dev kv,
                                                   int uni_k, int uni_v, int rule, int t0, int v_f16,
                                                   const int32_t* __restrict__ t0_rows) {
  __shared__ uint16_t vl[HS_BT * kVStride];
  // source tile blockIdx.x of K, V goes to tile t of the cache (t0 = 0 except when appending;
  // t0_rows: one t0 per batch row, entries that are not a tile index leave the row out)
  const int ts = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (t0_rows != nullptr) {
    t0 = t0_rows[b];
    if (t0 < 0 || t0 >= T) return;  // the whole workgroup
  }
  const int t = ts + t0;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, a = l >> 4, r = l & 15;
  const int64_t row = (int64_t)b * Hkv + h;
  int mk, mv;
  if (uni_k != 0) {
    mk = uni_k == HS_DENSE ? t + 1 : -(t + 1);
    mv = uni_v == HS_DENSE ? t + 1 : -(t + 1);
    if (tid == 0) {
      const_cast<int32_t*>(kv.k_map)[row * T + t] = mk;
      const_cast<int32_t*>(kv.v_map)[row * T + t] = mv;
    }
  } else {
    mk = kv.k_map[row * T + t];
    mv = kv.v_map[row * T + t];
  }
  const uint16_t* kt = K + b * sb + h * sh + (int64_t)ts * HS_BT * st;
  const uint16_t* vt = V + b * sb + h * sh + (int64_t)ts * HS_BT * st;
  if (mv < 0) stage_v_tile<NTL>(vt, st, vl);
  else if (mv > 0) stage_v_tile<false>(vt, st, vl);

  // ---- K ----
  if (mk > 0) {  // dense: permuted copy into operand order
    uint8_t* dst = const_cast<uint8_t*>(kv.k_dense) + (row * kv.cap_dense_k + (mk - 1)) * (int64_t)HS_TILE_DENSE_BYTES;
    const uint16_t* src = kt + (int64_t)(16 * w + r) * st + 8 * a;
#pragma unroll
    for (int s = 0; s < 4; s++) {
      st16<false>(dst + ((w * 4 + s) * 64 + l) * 16, ld16<false>(src + 32 * s));
    }
  } else if (mk < 0) {
    const int64_t slot = row * kv.cap_sparse_k + (-mk - 1);
    const uint16_t* src = kt + (int64_t)(16 * w + r) * st + 16 * a;
    k_sparse_store(const_cast<uint8_t*>(kv.k_nnz) + slot * (int64_t)HS_TILE_NNZ_BYTES,
                   const_cast<uint8_t*>(kv.k_meta) + slot * (int64_t)HS_TILE_META_BYTES, w, l, rule,
                   [&](int kb, int half) { return ld16<NTL>(src + 64 * kb + 8 * half); });
  }

  // ---- V ----
  if (mv == 0) return;
  __syncthreads();
  v_tile_store(vl, mv, const_cast<int32_t*>(kv.v_map) + row * T + t, kv, row, rule, v_f16, tid);
}

// ----------------------------------------------------------------------------------
// Further pruning of a packed cache (Sec. III, overview: after the prefill phase the dense pool
// can be pruned and compressed again, so that decode runs at another sparsity than prefill).
// ----------------------------------------------------------------------------------
// New state of a tile = the sparser of its current state and its target (DENSE < 2:4 < SKIP).
__device__ __forceinline__ int sparser_state(int map_entry, int target) {
  const int cur = map_entry > 0 ? HS_DENSE : (map_entry < 0 ? HS_SPARSE24 : HS_SKIP);
  const int rc = cur == HS_SKIP ? 2 : cur - 1, rt = target == HS_SKIP ? 2 : target - 1;
  const int rn = rc > rt ? rc : rt;
  return rn == 2 ? HS_SKIP : rn + 1;
}

// Maps of the re-compressed cache: slots in ascending tile order with one counter per pool
// (Sec. III-B); a tile that keeps its kind keeps its encoding bit.  A tile for which a pool of dst
// has no slot left is left out of both tensors, takes no slot, and bit 0 of *overflow is raised
// (assign_slots_row).  Target of tile t: tgt_k / tgt_v (device int8 [rows, T]) when given -- a
// pair that is not valid leaves the tile as it is and raises bit 1 --; else the sign of
// tgt_map_k / tgt_map_v (maps the selection kernel wrote for a ranked target: > 0 dense, < 0 2:4,
// 0 skipped) when given; else DENSE for the n_first first and n_last last tiles of the row and
// frac_state_k / frac_state_v in between.  One workgroup per row.
__global__ __launch_bounds__(256) void restate_kernel(int T, hs_kv_dev src, const int8_t* __restrict__ tgt_k,
                                                      const int8_t* __restrict__ tgt_v,
                                                      const int32_t* __restrict__ tgt_map_k,
                                                      const int32_t* __restrict__ tgt_map_v, int frac_state_k,
                                                      int frac_state_v, int n_first, int n_last, hs_kv_dev dst,
                                                      int32_t* overflow) {
  __shared__ SlotShared sm;
  const int row = blockIdx.x, tid = threadIdx.x;
  const int32_t* skm = src.k_map + (int64_t)row * T;
  const int32_t* svm = src.v_map + (int64_t)row * T;
  int32_t* km = const_cast<int32_t*>(dst.k_map) + (int64_t)row * T;
  int32_t* vm = const_cast<int32_t*>(dst.v_map) + (int64_t)row * T;
  bool invalid = false;
  assign_slots_row(
      T, tid, dst.cap_dense_k, dst.cap_sparse_k, dst.cap_dense_v, dst.cap_sparse_v, sm, overflow,
      [&](int t, int& sk, int& sv) {
        int tk, tv;
        if (tgt_k != nullptr) {
          tk = tgt_k[(int64_t)row * T + t];
          tv = tgt_v[(int64_t)row * T + t];
          if (tk < 0 || tk > 2 || tv < 0 || tv > 2 || (tk == HS_SKIP) != (tv == HS_SKIP)) {
            invalid = true;
            tk = tv = HS_DENSE;  // no further pruning of this tile
          }
        } else if (tgt_map_k != nullptr) {
          const int a = tgt_map_k[(int64_t)row * T + t], c = tgt_map_v[(int64_t)row * T + t];
          tk = a > 0 ? HS_DENSE : (a < 0 ? HS_SPARSE24 : HS_SKIP);
          tv = c > 0 ? HS_DENSE : (c < 0 ? HS_SPARSE24 : HS_SKIP);
        } else {
          const bool prot = t < n_first || t >= T - n_last;
          tk = prot ? HS_DENSE : frac_state_k;
          tv = prot ? HS_DENSE : frac_state_v;
        }
        sk = sparser_state(skm[t], tk);
        sv = sparser_state(svm[t], tv);
        if (sk == HS_SKIP || sv == HS_SKIP) sk = sv = HS_SKIP;  // a tile leaves K and V together
      },
      [&](int t, int mk, int mv) {
        const int mv_old = svm[t];
        if (mv != 0 && (mv > 0) == (mv_old > 0) && hs_map_f16(mv_old)) mv = mv > 0 ? (mv | HS_MAP_F16) : -(-mv | HS_MAP_F16);
        km[t] = mk;
        vm[t] = mv;
      });
  if (invalid && overflow != nullptr) atomicOr(overflow, 2);
}

// One workgroup per tile: tiles that keep their kind are copied slot to slot; a dense tile that
// became 2:4 is read from its dense slot (pool order) and pruned with the writers above.
__global__ __launch_bounds__(256) void repack_kernel(int Hkv, int T, hs_kv_dev src, hs_kv_dev dst, int rule, int v_f16) {
  __shared__ uint16_t vl[HS_BT * kVStride];
  const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, a = l >> 4, r = l & 15;
  const int64_t row = (int64_t)b * Hkv + h;
  const int mk_old = src.k_map[row * T + t], mv_old_raw = src.v_map[row * T + t];
  const int mk = dst.k_map[row * T + t], mv_raw = dst.v_map[row * T + t];
  if (mk == 0 || mv_raw == 0) return;  // dropped (both tensors together)
  const int mv_old = hs_map_plain(mv_old_raw), mv = hs_map_plain(mv_raw);
  // ---- K ----
  if (mk > 0) {
    const uint4* s4 = reinterpret_cast<const uint4*>(src.k_dense + (row * src.cap_dense_k + (mk_old - 1)) * (int64_t)HS_TILE_DENSE_BYTES);
    uint4* d4 = reinterpret_cast<uint4*>(const_cast<uint8_t*>(dst.k_dense) + (row * dst.cap_dense_k + (mk - 1)) * (int64_t)HS_TILE_DENSE_BYTES);
#pragma unroll
    for (int i = 0; i < 4; i++) d4[i * 256 + tid] = s4[i * 256 + tid];
  } else {
    const int64_t slot = row * dst.cap_sparse_k + (-mk - 1);
    uint8_t* nnz = const_cast<uint8_t*>(dst.k_nnz) + slot * (int64_t)HS_TILE_NNZ_BYTES;
    uint8_t* meta = const_cast<uint8_t*>(dst.k_meta) + slot * (int64_t)HS_TILE_META_BYTES;
    if (mk_old < 0) {
      const int64_t so = row * src.cap_sparse_k + (-mk_old - 1);
      const uint4* s4 = reinterpret_cast<const uint4*>(src.k_nnz + so * (int64_t)HS_TILE_NNZ_BYTES);
      uint4* d4 = reinterpret_cast<uint4*>(nnz);
#pragma unroll
      for (int i = 0; i < 2; i++) d4[i * 256 + tid] = s4[i * 256 + tid];
      if (tid < 64)
        reinterpret_cast<uint4*>(meta)[tid] = reinterpret_cast<const uint4*>(src.k_meta + so * (int64_t)HS_TILE_META_BYTES)[tid];
    } else {
      // dense pool order: chunk 4w + s of lane (a', r) = token 16w + r, channels 32s + 8a' .. +8
      const uint8_t* sd = src.k_dense + (row * src.cap_dense_k + (mk_old - 1)) * (int64_t)HS_TILE_DENSE_BYTES;
      k_sparse_store(nnz, meta, w, l, rule, [&](int kb, int half) {
        const int s = 2 * kb + (a >> 1), a2 = 2 * (a & 1) + half;
        return *reinterpret_cast<const uint4*>(sd + ((w * 4 + s) * 64 + 16 * a2 + r) * 16);
      });
    }
  }
  // ---- V ---- (branches are workgroup-uniform)
  if (mv > 0) {
    const uint4* s4 = reinterpret_cast<const uint4*>(src.v_dense + (row * src.cap_dense_v + (mv_old - 1)) * (int64_t)HS_TILE_DENSE_BYTES);
    uint4* d4 = reinterpret_cast<uint4*>(const_cast<uint8_t*>(dst.v_dense) + (row * dst.cap_dense_v + (mv - 1)) * (int64_t)HS_TILE_DENSE_BYTES);
#pragma unroll
    for (int i = 0; i < 4; i++) d4[i * 256 + tid] = s4[i * 256 + tid];
  } else if (mv_old < 0) {
    const int64_t so = row * src.cap_sparse_v + (-mv_old - 1), sn = row * dst.cap_sparse_v + (-mv - 1);
    const uint4* s4 = reinterpret_cast<const uint4*>(src.v_nnz + so * (int64_t)HS_TILE_NNZ_BYTES);
    uint4* d4 = reinterpret_cast<uint4*>(const_cast<uint8_t*>(dst.v_nnz) + sn * (int64_t)HS_TILE_NNZ_BYTES);
#pragma unroll
    for (int i = 0; i < 2; i++) d4[i * 256 + tid] = s4[i * 256 + tid];
    if (tid < 64)
      reinterpret_cast<uint4*>(const_cast<uint8_t*>(dst.v_meta) + sn * (int64_t)HS_TILE_META_BYTES)[tid] =
          reinterpret_cast<const uint4*>(src.v_meta + so * (int64_t)HS_TILE_META_BYTES)[tid];
  } else {
    v_dense_to_lds(src.v_dense + (row * src.cap_dense_v + (mv_old - 1)) * (int64_t)HS_TILE_DENSE_BYTES,
                   hs_map_f16(mv_old_raw), vl, tid);
    __syncthreads();
    v_tile_store(vl, mv, const_cast<int32_t*>(dst.v_map) + row * T + t, dst, row, rule, v_f16, tid);
  }
}

// ----------------------------------------------------------------------------------
// Unpack (tests / debugging): packed -> dense bf16 [B, Hkv, L, D], zeros where pruned
// or skipped.
// ----------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void unpack_kernel(int Hkv, int T, hs_kv_dev kv, uint16_t* __restrict__ K_out,
                                                     uint16_t* __restrict__ V_out) {
  __shared__ uint16_t vl[HS_BT * kVStride];
  const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, a = l >> 4, r = l & 15;
  const int64_t row = (int64_t)b * Hkv + h;
  const int mk = kv.k_map[row * T + t], mv_raw = kv.v_map[row * T + t];
  const bool v_is_f16 = hs_map_f16(mv_raw);
  const int mv = hs_map_plain(mv_raw);  // +-(slot + 1)
  uint16_t* ko = K_out + (row * T + t) * (int64_t)(HS_BT * HS_D);
  uint16_t* vo = V_out + (row * T + t) * (int64_t)(HS_BT * HS_D);
  {  // K: token 16w+r
    uint16_t* dst = ko + (16 * w + r) * HS_D;
    if (mk > 0) {
      const uint8_t* src = kv.k_dense + (row * kv.cap_dense_k + (mk - 1)) * (int64_t)HS_TILE_DENSE_BYTES;
#pragma unroll
      for (int s = 0; s < 4; s++)
        *reinterpret_cast<uint4*>(dst + 32 * s + 8 * a) = *reinterpret_cast<const uint4*>(src + ((w * 4 + s) * 64 + l) * 16);
    } else if (mk < 0) {
      const int64_t slot = row * kv.cap_sparse_k + (-mk - 1);
      const uint8_t* nnz = kv.k_nnz + slot * (int64_t)HS_TILE_NNZ_BYTES;
      const uint32_t idx = *reinterpret_cast<const uint32_t*>(kv.k_meta + slot * (int64_t)HS_TILE_META_BYTES + (l * 4 + w) * 4);
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
        const uint4 d = *reinterpret_cast<const uint4*>(nnz + ((w * 2 + kb) * 64 + l) * 16);
        const uint32_t vals[4] = {d.x, d.y, d.z, d.w};
        uint16_t o[16];
#pragma unroll
        for (int i = 0; i < 16; i++) o[i] = 0;
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const uint32_t nib = (idx >> (16 * kb + 4 * q)) & 0xfu;
          const uint32_t i0 = nib & 3u, i1 = nib >> 2;
#pragma unroll
          for (int p = 0; p < 4; p++) {
            if (i0 == (uint32_t)p) o[4 * q + p] = (uint16_t)(vals[q] & 0xffffu);
            if (i1 == (uint32_t)p) o[4 * q + p] = (uint16_t)(vals[q] >> 16);
          }
        }
        uint32_t pk[8];
#pragma unroll
        for (int i = 0; i < 8; i++) pk[i] = (uint32_t)o[2 * i] | ((uint32_t)o[2 * i + 1] << 16);
        uint4* d4 = reinterpret_cast<uint4*>(dst + 64 * kb + 16 * a);
        d4[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        d4[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
      }
    } else {
#pragma unroll
      for (int s = 0; s < 4; s++) *reinterpret_cast<uint4*>(dst + 32 * s + 8 * a) = make_uint4(0, 0, 0, 0);
    }
  }
  // V: rebuild the tile in LDS in [token][channel] order, then store it coalesced
  if (mv > 0) {
    v_dense_to_lds(kv.v_dense + (row * kv.cap_dense_v + (mv - 1)) * (int64_t)HS_TILE_DENSE_BYTES, v_is_f16, vl, tid);
  } else if (mv < 0) {
    const int64_t slot = row * kv.cap_sparse_v + (-mv - 1);
    const uint8_t* nnz = kv.v_nnz + slot * (int64_t)HS_TILE_NNZ_BYTES;
    const uint32_t idx = *reinterpret_cast<const uint32_t*>(kv.v_meta + slot * (int64_t)HS_TILE_META_BYTES + (l * 4 + w) * 4);
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int mb = 2 * w + j, c = 16 * mb + r;
      const uint4 d = *reinterpret_cast<const uint4*>(nnz + (mb * 64 + l) * 16);
      uint32_t vals[4] = {d.x, d.y, d.z, d.w};
      if (v_is_f16) {
#pragma unroll
        for (int i = 0; i < 4; i++) vals[i] = pair_to_bf16(vals[i]);
      }
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int g = hs_v_group(a, q);
        const uint32_t nib = (idx >> (16 * j + 4 * q)) & 0xfu;
        const uint32_t i0 = nib & 3u, i1 = nib >> 2;
#pragma unroll
        for (int p = 0; p < 4; p++) {
          uint16_t v = 0;
          if (i0 == (uint32_t)p) v = (uint16_t)(vals[q] & 0xffffu);
          if (i1 == (uint32_t)p) v = (uint16_t)(vals[q] >> 16);
          vl[(4 * g + p) * kVStride + c] = v;
        }
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int q = tid + 256 * i, tok = q >> 4, c8 = q & 15;
    uint4 d = make_uint4(0, 0, 0, 0);
    if (mv != 0) {
      const uint2* s2 = reinterpret_cast<const uint2*>(vl + tok * kVStride + 8 * c8);
      const uint2 lo = s2[0], hi = s2[1];
      d = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
    *reinterpret_cast<uint4*>(vo + tok * HS_D + 8 * c8) = d;
  }
}

}  // namespace

hipError_t hs_launch_score(const uint16_t* K, const uint16_t* V, int64_t sb, int64_t sh, int64_t st_, int B, int Hkv,
                           int T, int rule, int dtype, int what, double* scores, hipStream_t st) {
  const dim3 grid(T, Hkv, B), block(256);
  // non-temporal reads once K and V together are larger than the 256 MB last-level cache
  const bool nt = what == 1 && 2.0 * B * Hkv * T * HS_BT * HS_D * 2.0 > 256e6;
#define HS_SCORE(F16_, WHAT_)                                                                                              \
  do {                                                                                                                     \
    if (nt) hipLaunchKernelGGL((score_kernel<F16_, WHAT_, true>), grid, block, 0, st, K, V, sb, sh, st_, Hkv, T, rule, scores); \
    else hipLaunchKernelGGL((score_kernel<F16_, WHAT_, false>), grid, block, 0, st, K, V, sb, sh, st_, Hkv, T, rule, scores);   \
  } while (0)
  if (dtype == HS_FP16) {
    if (what == 1) HS_SCORE(true, 1); else if (what == 2) HS_SCORE(true, 2); else HS_SCORE(true, 3);
  } else {
    if (what == 1) HS_SCORE(false, 1); else if (what == 2) HS_SCORE(false, 2); else HS_SCORE(false, 3);
  }
#undef HS_SCORE
  return hipGetLastError();
}

hipError_t hs_launch_select(const double* scores, int rows, int T, int n_skip, int n_sparse_k, int n_sparse_v,
                            int n_first, int n_last, int32_t* k_map, int32_t* v_map, hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(rows), dim3(256), 0, st, scores, rows, T, n_skip, n_sparse_k, n_sparse_v, n_first,
                     n_last, k_map, v_map);
  return hipGetLastError();
}

hipError_t hs_launch_pack(const uint16_t* K, const uint16_t* V, int64_t sb, int64_t sh, int64_t st_, int B, int Hkv,
                          int T, hs_kv_dev kv, int uni_k, int uni_v, int rule, int v_f16, hipStream_t st) {
  if (2.0 * B * Hkv * T * HS_BT * HS_D * 2.0 > 256e6)  // K and V together beyond the 256 MB last-level cache
    hipLaunchKernelGGL(pack_kernel<true>, dim3(T, Hkv, B), dim3(256), 0, st, K, V, sb, sh, st_, Hkv, T, kv, uni_k, uni_v, rule, 0,
                       v_f16, (const int32_t*)nullptr);
  else
    hipLaunchKernelGGL(pack_kernel<false>, dim3(T, Hkv, B), dim3(256), 0, st, K, V, sb, sh, st_, Hkv, T, kv, uni_k, uni_v, rule, 0,
                       v_f16, (const int32_t*)nullptr);
  return hipGetLastError();
}

hipError_t hs_launch_append(const uint16_t* K, const uint16_t* V, int64_t sb, int64_t sh, int64_t st_, int B, int Hkv,
                            int T, int tile, int n_tiles, const int32_t* tile_rows, int state_k, int state_v,
                            hs_kv_dev kv, int rule, int v_f16, int32_t* overflow, hipStream_t st) {
  hipLaunchKernelGGL(append_slots_kernel, dim3(B * Hkv), dim3(256), 0, st, Hkv, T, tile, n_tiles, tile_rows, state_k, state_v,
                     kv, overflow);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (2.0 * B * Hkv * n_tiles * HS_BT * HS_D * 2.0 > 256e6)
    hipLaunchKernelGGL(pack_kernel<true>, dim3(n_tiles, Hkv, B), dim3(256), 0, st, K, V, sb, sh, st_, Hkv, T, kv, 0, 0, rule, tile,
                       v_f16, tile_rows);
  else
    hipLaunchKernelGGL(pack_kernel<false>, dim3(n_tiles, Hkv, B), dim3(256), 0, st, K, V, sb, sh, st_, Hkv, T, kv, 0, 0, rule, tile,
                       v_f16, tile_rows);
  return hipGetLastError();
}

hipError_t hs_launch_states_to_maps(const int8_t* state_k, const int8_t* state_v, int rows, int T, hs_kv_dev kv,
                                    int32_t* flag, hipStream_t st) {
  hipLaunchKernelGGL(states_to_maps_kernel, dim3(rows), dim3(256), 0, st, state_k, state_v, T, kv.cap_dense_k,
                     kv.cap_sparse_k, kv.cap_dense_v, kv.cap_sparse_v, const_cast<int32_t*>(kv.k_map),
                     const_cast<int32_t*>(kv.v_map), flag);
  return hipGetLastError();
}

hipError_t hs_launch_recompress(int B, int Hkv, int T, hs_kv_dev src, const int8_t* tgt_k, const int8_t* tgt_v,
                                const int32_t* tgt_map_k, const int32_t* tgt_map_v, int frac_state_k, int frac_state_v,
                                int n_first, int n_last, hs_kv_dev dst, int rule, int v_f16, int32_t* overflow,
                                hipStream_t st) {
  hipLaunchKernelGGL(restate_kernel, dim3(B * Hkv), dim3(256), 0, st, T, src, tgt_k, tgt_v, tgt_map_k, tgt_map_v,
                     frac_state_k, frac_state_v, n_first, n_last, dst, overflow);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(repack_kernel, dim3(T, Hkv, B), dim3(256), 0, st, Hkv, T, src, dst, rule, v_f16);
  return hipGetLastError();
}

hipError_t hs_launch_unpack(int B, int Hkv, int T, hs_kv_dev kv, uint16_t* K_out, uint16_t* V_out, hipStream_t st) {
  hipLaunchKernelGGL(unpack_kernel, dim3(T, Hkv, B), dim3(256), 0, st, Hkv, T, kv, K_out, V_out);
  return hipGetLastError();
}
