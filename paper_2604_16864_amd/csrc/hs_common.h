// Internal definitions shared by the HIP translation units of libhs (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "hs.h"

// ---------------------------------------------------------------------------------
// Matrix-core operand layouts on gfx950 (measured with one-hot operands):
//
//  v_mfma_f32_16x16x32_bf16   A: lane l holds row l%16,  k = 8*(l/16) + e, e = 0..7
//                             B: lane l holds col l%16,  k = 8*(l/16) + e
//                             D: lane l holds col l%16,  rows 4*(l/16) + i, i = 0..3
//  v_smfmac_f32_16x16x64_bf16 A: lane l holds row l%16 and the 8 kept values of the
//                                16 uncompressed k = 16*(l/16) .. +15 (4 groups of 4,
//                                2 kept each, ascending position)
//                             B: lane l holds col l%16,  k = 32*(e/8) + 8*(l/16) + e%8,
//                                e = 0..15  (= the B operands of two consecutive dense
//                                16x16x32 steps, so dense and sparse tiles share Q/P
//                                registers; cf. the shared P^T fragment of Sec. IV-A)
//                             idx: 2 bits per kept value (its position in the group),
//                                value e at bits 2e..2e+1 of the 16-bit half selected
//                                by ABID bit 0 (CBSZ = 0)
//                             D: as the dense instruction.
//
// Physical order inside a tile slot = the order the lanes consume it ("chunks" of
// 64 lanes x 16 B, lane l at byte 16*l of its chunk; a = l/16, r = l%16):
//
//  K 2:4  nnz : chunk m*2+kb (m = 0..3, kb = 0..1): token 16m+r, kept values of channel
//               groups 16kb+4a+q, q = 0..3 (channels 4*group .. +3), lower position first.
//         meta: lane l owns 16 bytes = words m = 0..3 (u32, word 4l+m of the slot): bits 0..15
//               idx for kb = 0, bits 16..31 for kb = 1; nibble q (bits 4q..4q+3 of the half)
//               = i0 | i1<<2 of group 16kb+4a+q.
//  V 2:4  nnz : chunk mb (0..7): channel 16mb+r, kept values of token groups
//               g(a,q) = 4*(2*(a/2) + q%2) + 2*(a%2) + q/2, q = 0..3 (tokens 4g..4g+3).
//         meta: lane l owns words w = 0..3 (word 4l+w): low half mb = 2w, high half mb = 2w+1;
//               nibble q as above.
//  K dense    : chunk m*4+s (s = 0..3): token 16m+r, channels 32s+8a+e, e = 0..7.
//  V dense    : chunk mb*2+h (h = 0..1): channel 16mb+r, tokens 16*(2h+e/4)+4a+e%4.
//
// The token order of V is the one in which GEMM1's accumulator registers (lane holds
// tokens 16m+4a+i of its query column) line up, after conversion to bf16, as GEMM2's B
// operand with no cross-lane movement (the problem Sec. IV-C-2 solves with movmatrix).
// ---------------------------------------------------------------------------------

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x16_t __attribute__((ext_vector_type(16)));

#define HS_D 128
#define HS_BT 64

// Element type dependent pieces (hs_shape.dtype): conversions and the matrix instructions.  The
// 16-bit operand layouts of the bf16 and f16 forms of an instruction are the same, so everything
// about tiles, pools and lanes is type independent.  Device code only.
struct hs_u4x2 { uint4 lo, hi; };
template <bool F16> struct hs_elem;
template <> struct hs_elem<false> {
  static __device__ __forceinline__ float to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
  static __device__ __forceinline__ float lo_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
  static __device__ __forceinline__ float hi_f32(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {  // round to nearest even
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    bf2 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
  }
  static __device__ __forceinline__ f32x4_t mma(uint4 a, uint4 b, f32x4_t c) {  // dense 16x16x32
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
  template <int ABID>
  static __device__ __forceinline__ f32x4_t smma(uint4 a, uint4 b0, uint4 b1, f32x4_t c, int idx) {  // 2:4 16x16x64
    const hs_u4x2 b{b0, b1};
    return __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x16_t, b), c, idx, 0, ABID);
  }
};
template <> struct hs_elem<true> {
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  static __device__ __forceinline__ float to_f32(uint32_t bits16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
  }
  static __device__ __forceinline__ float lo_f32(uint32_t pair) { return (float)__builtin_bit_cast(h2, pair)[0]; }
  static __device__ __forceinline__ float hi_f32(uint32_t pair) { return (float)__builtin_bit_cast(h2, pair)[1]; }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {  // round to nearest even
    h2 v;
    v[0] = (_Float16)a;
    v[1] = (_Float16)b;
    return __builtin_bit_cast(uint32_t, v);
  }
  static __device__ __forceinline__ f32x4_t mma(uint4 a, uint4 b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
  template <int ABID>
  static __device__ __forceinline__ f32x4_t smma(uint4 a, uint4 b0, uint4 b1, f32x4_t c, int idx) {
    const hs_u4x2 b{b0, b1};
    return __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x16_t, b), c, idx, 0, ABID);
  }
};

struct hs_kv_dev {  // device-side view of hs_kv (passed by value to kernels)
  const uint8_t* k_dense; const uint8_t* k_nnz; const uint8_t* k_meta; const int32_t* k_map;
  const uint8_t* v_dense; const uint8_t* v_nnz; const uint8_t* v_meta; const int32_t* v_map;
  int32_t cap_dense_k, cap_sparse_k, cap_dense_v, cap_sparse_v;
  int32_t uniform;
};

static inline hs_kv_dev hs_make_kv_dev(const hs_kv* kv) {
  hs_kv_dev d;
  d.k_dense = (const uint8_t*)kv->k_dense; d.k_nnz = (const uint8_t*)kv->k_nnz;
  d.k_meta = (const uint8_t*)kv->k_meta;   d.k_map = kv->k_map;
  d.v_dense = (const uint8_t*)kv->v_dense; d.v_nnz = (const uint8_t*)kv->v_nnz;
  d.v_meta = (const uint8_t*)kv->v_meta;   d.v_map = kv->v_map;
  d.cap_dense_k = kv->cap_dense_k; d.cap_sparse_k = kv->cap_sparse_k;
  d.cap_dense_v = kv->cap_dense_v; d.cap_sparse_v = kv->cap_sparse_v;
  d.uniform = kv->uniform;
  return d;
}

// v_map entries: sign = pool (dense > 0, 2:4 < 0), magnitude = slot + 1, plus HS_MAP_F16 when the tile
// is stored in fp16 encoding
__host__ __device__ static inline bool hs_map_f16(int m) { return ((m < 0 ? -m : m) & HS_MAP_F16) != 0; }
__host__ __device__ static inline int hs_map_plain(int m) { return m < 0 ? -(-m & ~HS_MAP_F16) : (m & ~HS_MAP_F16); }

// token group of V held at pair q of lane group a (see layout note above)
__host__ __device__ static inline int hs_v_group(int a, int q) {
  return 4 * (2 * (a >> 1) + (q & 1)) + 2 * (a & 1) + (q >> 1);
}

// launchers implemented in the kernel translation units; all return a hipError_t
// what: 1 = tile energies only, 2 = pruning losses only, 3 = both (the other planes are zero)
hipError_t hs_launch_score(const uint16_t* K, const uint16_t* V, int64_t sb, int64_t sh, int64_t st_,
                           int B, int Hkv, int T, int rule, int dtype, int what, double* scores, hipStream_t st);
hipError_t hs_launch_select(const double* scores, int rows, int T, int n_skip, int n_sparse_k, int n_sparse_v,
                            int n_first, int n_last, int32_t* k_map, int32_t* v_map, hipStream_t st);
hipError_t hs_launch_pack(const uint16_t* K, const uint16_t* V, int64_t sb, int64_t sh, int64_t st_,
                          int B, int Hkv, int T, hs_kv_dev kv, int uni_k, int uni_v, int rule, int v_f16, hipStream_t st);
// n_tiles tiles [B, Hkv, 64 n_tiles, D] into tile indices tile .. of a cache of T tiles per row
hipError_t hs_launch_append(const uint16_t* K, const uint16_t* V, int64_t sb, int64_t sh, int64_t st_,
                            int B, int Hkv, int T, int tile, int n_tiles, const int32_t* tile_rows, int state_k, int state_v, hs_kv_dev kv, int rule,
                            int v_f16, int32_t* overflow, hipStream_t st);
// explicit tile states (device int8 [rows, T]) -> the maps of kv; flag (device, may be NULL): bit 0 = a pool
// capacity of kv was exceeded, bit 1 = a state pair was not valid (such tiles are stored as SKIP)
hipError_t hs_launch_states_to_maps(const int8_t* state_k, const int8_t* state_v, int rows, int T, hs_kv_dev kv,
                                    int32_t* flag, hipStream_t st);
// packed cache -> packed cache, each tile in the sparser of its state and its target: tgt_k / tgt_v (device
// int8 [rows, T]), or the signs of tgt_map_k / tgt_map_v (device int32 [rows, T]), or, when all are NULL,
// frac_state_k / frac_state_v for every tile but the n_first first and n_last last of a row, which stay as
// they are
hipError_t hs_launch_recompress(int B, int Hkv, int T, hs_kv_dev src, const int8_t* tgt_k, const int8_t* tgt_v,
                                const int32_t* tgt_map_k, const int32_t* tgt_map_v, int frac_state_k, int frac_state_v,
                                int n_first, int n_last, hs_kv_dev dst, int rule, int v_f16, int32_t* overflow,
                                hipStream_t st);
hipError_t hs_launch_unpack(int B, int Hkv, int T, hs_kv_dev kv, uint16_t* K_out, uint16_t* V_out, hipStream_t st);
// tail_len < 0: no tail slot; tail_len >= 0: one extra partial per query head, computed from the
// dense tail tokens (tail_k / tail_v, bf16 [B, Hkv, 64, D]); tail_lens (device, [B]) replaces
// tail_len per batch row when not NULL
hipError_t hs_launch_decode(int B, int Hq, int Hkv, int T, float scale, int n_splits, const uint16_t* Q,
                            hs_kv_dev kv, const uint16_t* tail_k, const uint16_t* tail_v, int tail_len, const int32_t* tail_lens,
                            uint16_t* O, float* LSE, float* ws, hipStream_t st, int phases, int dtype);
// address (on the current device) and size of the library's static device array that hs_decode_attn_static
// uses for its split partials; looked up once per device, never allocated
hipError_t hs_static_scratch(void** ptr, size_t* bytes);
// register-resident matrix-instruction loop (kind 0 dense 16x16x32, 1 sparse 16x16x64), 8 * iters instructions per wave
hipError_t hs_launch_mfma_rate(int kind, int iters, int n_workgroups, long long* sink, hipStream_t st);
// load-only kernel with the decode kernel's access pattern over n_tiles tiles laid out as four pool regions in buf
hipError_t hs_launch_stream_read(const uint8_t* buf, int n_tiles, int n_workgroups, int with_epilogue, float* sink,
                                 hipStream_t st);
// q_start: position in the cache of the first query (query i sees tokens <= q_start + i when causal)
hipError_t hs_launch_prefill(int B, int Hq, int Hkv, int T, int Tq, int q_start, float scale, int causal, const uint16_t* Q,
                             hs_kv_dev kv, uint16_t* O, float* LSE, hipStream_t st, int dtype);
