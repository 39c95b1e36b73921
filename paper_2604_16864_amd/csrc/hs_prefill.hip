// Prefill attention: Algorithm 1 (Trans-Both: S^T = K Q^T, O^T = V^T P^T with K and V^T as
// the first, possibly 2:4-sparse, operand of the matrix instruction) with the mixed
// dense/sparse dispatch of Sec. III-C-2, online softmax, and tile skipping.
//
// Work decomposition: a "slab" is 64 consecutive query positions of one query head; a wave
// owns one slab (4 column blocks of 16 queries), keeps Q^T (B operand of GEMM1), the
// running softmax state and O^T (128 x 64 fp32) in registers for the whole kernel.  The 4
// waves of a workgroup take 4 consecutive slabs in (position-tile, head-in-group) order, so
// for a GQA group of 4 they are the 4 query heads of one 64-position tile and share every
// KV tile, which is staged once per workgroup in LDS (double buffered, prefetched through
// registers one tile ahead).  Pools are stored in operand order, so LDS reads are
// conflict-free 16-byte-per-lane reads and GEMM1's accumulators become GEMM2's B operand
// in place (no re-layout step).
#include <stdlib.h>

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

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }
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

constexpr int kBufBytes = 32768;  // one stage: K region 16 KiB + V region 16 KiB

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Copy one tile (K and V operands) from its pool slots into an LDS stage with direct
// global->LDS loads (no staging registers): a chunk is 64 lanes x 16 B = 1 KiB, lane l's
// 16 bytes land at chunk base + 16 l, which is the order the pools are stored in.  The 4
// waves share the chunks round-robin.  2:4 tile: 8 value chunks + 1 metadata chunk per
// tensor (value chunks at 0..8 KiB, metadata at 8 KiB of the tensor's region); dense: 16.
template <int KM, int VM>
__device__ __forceinline__ void stage_issue(uint8_t* buf, const hs_kv_dev& kv, int64_t row, int mk, int mv, int w,
                                            int l) {
  const bool k_sparse = KM == 0 || (KM == 2 && mk < 0);
  const bool v_sparse = VM == 0 || (VM == 2 && mv < 0);
  const uint8_t *kd, *km = nullptr, *vd, *vm = nullptr;
  int nk, nv;
  if (k_sparse) {
    const int64_t slot = row * kv.cap_sparse_k + (-mk - 1);
    kd = kv.k_nnz + slot * (int64_t)HS_TILE_NNZ_BYTES;
    km = kv.k_meta + slot * (int64_t)HS_TILE_META_BYTES;
    nk = 8;
  } else {
    kd = kv.k_dense + (row * kv.cap_dense_k + (mk - 1)) * (int64_t)HS_TILE_DENSE_BYTES;
    nk = 16;
  }
  if (v_sparse) {
    const int64_t slot = row * kv.cap_sparse_v + (-mv - 1);
    vd = kv.v_nnz + slot * (int64_t)HS_TILE_NNZ_BYTES;
    vm = kv.v_meta + slot * (int64_t)HS_TILE_META_BYTES;
    nv = 8;
  } else {
    vd = kv.v_dense + (row * kv.cap_dense_v + (mv - 1)) * (int64_t)HS_TILE_DENSE_BYTES;
    nv = 16;
  }
  for (int ch = w; ch < nk; ch += 4)
    __builtin_amdgcn_global_load_lds((gptr_t)(kd + ch * 1024 + l * 16), (lptr_t)(buf + ch * 1024), 16, 0, 0);
  for (int ch = w; ch < nv; ch += 4)
    __builtin_amdgcn_global_load_lds((gptr_t)(vd + ch * 1024 + l * 16), (lptr_t)(buf + 16384 + ch * 1024), 16, 0, 0);
  if (k_sparse && w == 0)
    __builtin_amdgcn_global_load_lds((gptr_t)(km + l * 16), (lptr_t)(buf + 8192), 16, 0, 0);
  if (v_sparse && w == 1)
    __builtin_amdgcn_global_load_lds((gptr_t)(vm + l * 16), (lptr_t)(buf + 16384 + 8192), 16, 0, 0);
}

// all of this wave's direct-to-LDS loads have landed (vmcnt = 0; other counters untouched)
__device__ __forceinline__ void stage_wait() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// next tile index > j (and <= jmax) whose map entry is not 0, or -1
__device__ __forceinline__ int next_active(const int32_t* km, int j, int jmax) {
  for (int t = j + 1; t <= jmax; t++)
    if (km[t] != 0) return t;
  return -1;
}

union B16 {  // one B operand of the 16x16x64 sparse instruction = two of the dense 16x16x32 one
  bf16x16_t v;
  uint4 q[2];
  uint32_t u[8];
};

// KM / VM (per tensor): 0 = every tile 2:4 or skipped, 1 = every tile dense or skipped, 2 = any mix
// (the specialised all-dense / all-sparse kernels of Sec. IV-C-3, chosen per tensor so that the
// keys-dense / values-2:4 setting of Sec. V-A carries no dynamic dispatch).
// NB: column blocks (of 16 queries) per wave: a wave owns a slab of 16*NB query positions of one
// head.  NB = 4 keeps 1 wave per SIMD (O^T alone is 128 registers); NB = 2 fits 2 waves per SIMD.
template <int KM, int VM, int NB>
__global__ __launch_bounds__(256, NB == 2 ? 2 : 1) void prefill_kernel(int Hq, int Hkv, int T, int Lq, int off,
                                                                      float scale_log2, int causal,
                                                                      const uint16_t* __restrict__ Q, hs_kv_dev kv,
                                                                      uint16_t* __restrict__ O,
                                                                      float* __restrict__ LSE) {
  constexpr int QS = 16 * NB;  // query positions per slab
  __shared__ __attribute__((aligned(16))) uint8_t lds[2 * kBufBytes];
  const int tid = threadIdx.x, l = tid & 63, a = l >> 4, c = l & 15;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, scalar: branches on it stay scalar
  const int G = Hq / Hkv;
  const int hkv = blockIdx.y, b = blockIdx.z;
  const int n_slabs = (Lq / QS) * G;
  // heavy (late) query positions first: causal work grows with the position
  const int grp = (int)gridDim.x - 1 - (int)blockIdx.x;
  const int slab = 4 * grp + w;
  const bool valid = slab < n_slabs;
  const int qpos = valid ? (slab / G) * QS : 0, hg = valid ? slab % G : 0;
  const int hq = hkv * G + hg;
  const int64_t row = (int64_t)b * Hkv + hkv;
  const int32_t* km = kv.k_map + row * T;
  const int32_t* vm = kv.v_map + row * T;
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
  int j = next_active(km, -1, jmax_wg);
  int mk = 0, mv = 0;
  if (j >= 0) {
    mk = __builtin_amdgcn_readfirstlane(km[j]); mv = __builtin_amdgcn_readfirstlane(vm[j]);
    stage_issue<KM, VM>(lds, kv, row, mk, mv, w, l);
  }
  stage_wait();
  __syncthreads();
  int buf = 0;
  while (j >= 0) {
    // prefetch the next visible tile into the other stage; it is waited for at the end of
    // this iteration, after the arithmetic on the current one
    const int jn = next_active(km, j, jmax_wg);
    int mkn = 0, mvn = 0;
    if (jn >= 0) {
      mkn = __builtin_amdgcn_readfirstlane(km[jn]); mvn = __builtin_amdgcn_readfirstlane(vm[jn]);
      stage_issue<KM, VM>(lds + (buf ^ 1) * kBufBytes, kv, row, mkn, mvn, w, l);
    }
    if (valid && j <= jmax_w) {
      const bool k_sparse = KM == 0 || (KM == 2 && mk < 0);
      const bool v_sparse = VM == 0 || (VM == 2 && mv < 0);
      const uint4* kl = reinterpret_cast<const uint4*>(lds + buf * kBufBytes);
      const uint4* vl = reinterpret_cast<const uint4*>(lds + buf * kBufBytes + 16384);
      // ---------------- GEMM1: S^T[64 tokens x 16 NB queries] ----------------
      __builtin_amdgcn_s_setprio(HS_PRIO_MFMA);
      f32x4_t s[4][NB];
#pragma unroll
      for (int m = 0; m < 4; m++)
#pragma unroll
        for (int nb = 0; nb < NB; nb++) s[m][nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      if (k_sparse) {
        uint4 ak[8];
#pragma unroll
        for (int i = 0; i < 8; i++) ak[i] = kl[i * 64 + l];
        const uint4 kix = kl[512 + l];
        const int kidx[4] = {(int)kix.x, (int)kix.y, (int)kix.z, (int)kix.w};
        // 4 NB independent accumulators between the two instructions that share one
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
          for (int m = 0; m < 4; m++)
            s[m][nb] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(ak[2 * m]), qb[nb][0].v, s[m][nb], kidx[m], 0, 0);
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
          for (int m = 0; m < 4; m++)
            s[m][nb] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(ak[2 * m + 1]), qb[nb][1].v, s[m][nb], kidx[m], 0, 1);
      } else {
#pragma unroll
        for (int m = 0; m < 4; m++) {
          uint4 ak[4];
#pragma unroll
          for (int st = 0; st < 4; st++) ak[st] = kl[(4 * m + st) * 64 + l];
#pragma unroll
          for (int st = 0; st < 4; st++)
#pragma unroll
            for (int nb = 0; nb < NB; nb++)
              s[m][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ak[st]), as_bf16x8(qb[nb][st >> 1].q[st & 1]), s[m][nb], 0, 0, 0);
        }
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
      B16 ph[NB], pl[NB];
      float psum[NB];
      auto softmax_tile = [&]() {
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
            split_hi_lo(p[0], p[1], sc, ph[nb].u[2 * m], pl[nb].u[2 * m]);
            split_hi_lo(p[2], p[3], sc, ph[nb].u[2 * m + 1], pl[nb].u[2 * m + 1]);
          }
          psum[nb] = acc;
        }
      };
      softmax_tile();
      bool redo = false;
#pragma unroll
      for (int nb = 0; nb < NB; nb++) redo = redo || !(psum[nb] <= 0x1p40f) || !(m_run[nb] > -INFINITY);
      if (__any(redo)) {
#pragma unroll
        for (int nb = 0; nb < NB; nb++) {
          float mx = s[0][nb][0];
#pragma unroll
          for (int m = 0; m < 4; m++)
#pragma unroll
            for (int i = 0; i < 4; i++) mx = fmaxf(mx, s[m][nb][i]);
          mx *= scale_log2;
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
      __builtin_amdgcn_s_setprio(HS_PRIO_MFMA);
      if (v_sparse) {
        uint4 av[8];
#pragma unroll
        for (int i = 0; i < 8; i++) av[i] = vl[i * 64 + l];
        const uint4 vix = vl[512 + l];
        const int vidx[4] = {(int)vix.x, (int)vix.y, (int)vix.z, (int)vix.w};
#pragma unroll
        for (int t2 = 0; t2 < 2; t2++)  // first the upper-half term of every block, then the remainder
#pragma unroll
          for (int nb = 0; nb < NB; nb++)
#pragma unroll
            for (int mb = 0; mb < 8; mb++) {
              const bf16x16_t bp = t2 == 0 ? ph[nb].v : pl[nb].v;
              if (mb & 1)
                o[mb][nb] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(av[mb]), bp, o[mb][nb], vidx[mb >> 1], 0, 1);
              else
                o[mb][nb] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(av[mb]), bp, o[mb][nb], vidx[mb >> 1], 0, 0);
            }
      } else {
#pragma unroll
        for (int mb = 0; mb < 8; mb++) {
          const uint4 a0 = vl[(2 * mb) * 64 + l], a1 = vl[(2 * mb + 1) * 64 + l];
#pragma unroll
          for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
            for (int h = 0; h < 2; h++)
#pragma unroll
              for (int nb = 0; nb < NB; nb++)
                o[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(h == 0 ? a0 : a1),
                                                                   as_bf16x8(t2 == 0 ? ph[nb].q[h] : pl[nb].q[h]),
                                                                   o[mb][nb], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_s_setprio(HS_PRIO_VALU);
    stage_wait();
    __syncthreads();
    j = jn; mk = mkn; mv = mvn;
    buf ^= 1;
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
      const uint2 v = make_uint2(pack_bf16(o[mb][nb][0] * inv, o[mb][nb][1] * inv),
                                 pack_bf16(o[mb][nb][2] * inv, o[mb][nb][3] * inv));
      *reinterpret_cast<uint2*>(op + 16 * mb) = v;
    }
    if (LSE != nullptr && a == 0)
      LSE[qrow] = lt > 0.f ? (m_run[nb] + __builtin_amdgcn_logf(lt)) * kLn2 : -INFINITY;
  }
}

}  // namespace

template <int KM, int VM, int NB>
static hipError_t launch_prefill(int B, int Hq, int Hkv, int T, int Lq, float sl2, int causal, const uint16_t* Q,
                                 const hs_kv_dev& kv, uint16_t* O, float* LSE, hipStream_t st) {
  const int G = Hq / Hkv;
  const int n_groups = ((Lq / (16 * NB)) * G + 3) / 4;
  hipLaunchKernelGGL((prefill_kernel<KM, VM, NB>), dim3(n_groups, Hkv, B), dim3(256), 0, st, Hq, Hkv, T, Lq,
                     T * HS_BT - Lq, sl2, causal, Q, kv, O, LSE);
  return hipGetLastError();
}

hipError_t hs_launch_prefill(int B, int Hq, int Hkv, int T, int Tq, float scale, int causal, const uint16_t* Q,
                             hs_kv_dev kv, uint16_t* O, float* LSE, hipStream_t st) {
  const float sl2 = scale * kLog2e;
  const int Lq = Tq * HS_BT;
  const int km = kv.cap_dense_k == 0 ? 0 : (kv.cap_sparse_k == 0 ? 1 : 2);
  const int vm = kv.cap_dense_v == 0 ? 0 : (kv.cap_sparse_v == 0 ? 1 : 2);
  // HS_PREFILL_NB=4 selects 64-query slabs at 1 wave per SIMD for the two uniform settings
  // (kept for comparison; 32-query slabs at 2 waves per SIMD measured 1.3-1.4x faster)
  static const int nb_env = [] { const char* e = getenv("HS_PREFILL_NB"); return e ? atoi(e) : 0; }();
#define HS_GO(KM_, VM_) return launch_prefill<KM_, VM_, 2>(B, Hq, Hkv, T, Lq, sl2, causal, Q, kv, O, LSE, st)
  if (nb_env == 4 && km == 0 && vm == 0) return launch_prefill<0, 0, 4>(B, Hq, Hkv, T, Lq, sl2, causal, Q, kv, O, LSE, st);
  if (nb_env == 4 && km == 1 && vm == 1) return launch_prefill<1, 1, 4>(B, Hq, Hkv, T, Lq, sl2, causal, Q, kv, O, LSE, st);
  switch (km * 3 + vm) {
    case 0: HS_GO(0, 0);
    case 1: HS_GO(0, 1);
    case 2: HS_GO(0, 2);
    case 3: HS_GO(1, 0);
    case 4: HS_GO(1, 1);
    case 5: HS_GO(1, 2);
    case 6: HS_GO(2, 0);
    case 7: HS_GO(2, 1);
    default: HS_GO(2, 2);
  }
#undef HS_GO
}
