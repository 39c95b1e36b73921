/*
 * hs.h -- C ABI of the HieraSparse hot path for AMD MI355X (gfx950).
 *
 * The library implements attention over a hierarchically pruned KV cache
 * (paper Sec. III): the cache is cut into blocks ("tiles") of 64 tokens; a tile
 * is stored dense, or pruned 2:4 along the contraction axis and stored as kept
 * values + 2-bit positions (Sec. III-A/B), or -- an extension the benchmark
 * workloads add on top of the paper -- skipped.  A signed block index map
 * (Sec. III-B) locates every tile in its pool.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers unless marked [host].
 *   - Q, K, V, O are 16-bit floating point, raw bit patterns: bf16 (the benchmark workloads) or
 *     IEEE fp16 (the paper's type), chosen by hs_shape.dtype for all four; "bf16" in the
 *     descriptions below stands for that type.  D (head dim) is contiguous.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL =
 *     the default stream): no call waits for the device, copies from host memory or
 *     synchronises the stream.  The library allocates nothing, frees nothing and
 *     keeps no pointer after a call returns; the caller owns every buffer.
 *   - There is no context object: every call is a function of its arguments alone (the
 *     device is the one `stream` belongs to, which must be the current device), so there is
 *     nothing to create or destroy.
 *   - Return value: HS_OK (0) or a negative hs_status.  Arguments are checked
 *     on the host before anything is launched; nothing is launched when an
 *     error is returned.  Faults inside a kernel are not recoverable.
 *   - A process may call from several threads as long as two calls do not share
 *     an output or workspace buffer.
 */
#ifndef HS_H_
#define HS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef HS_BUILD
#define HS_API __attribute__((visibility("default")))
#else
#define HS_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HS_OK = 0,
  HS_EINVAL = -1,       /* null pointer, bad fraction, inconsistent states, capacity too small */
  HS_EUNSUPPORTED = -2, /* D != 128, tile != 64, L % 64 != 0, Hq % Hkv != 0, group size > 8 ... */
  HS_EHIP = -3,         /* a HIP runtime call failed; hs_last_hip_error() has the text */
  HS_ENOSPACE = -4      /* hs_decode_attn_static: the split partials would not fit the static array */
} hs_status;

/* Tile states (Sec. III-A block-level mask M, plus SKIP). */
enum { HS_SKIP = 0, HS_DENSE = 1, HS_SPARSE24 = 2 };

/* Sizes in bytes of one 64 x 128 bf16 tile in each pool (Sec. III-D: nnz = 1/2,
 * metadata = 1/16 of the dense tile). */
enum { HS_TILE_DENSE_BYTES = 16384, HS_TILE_NNZ_BYTES = 8192, HS_TILE_META_BYTES = 1024 };

/* Geometry.  Supported: D == 128, tile == 64, L % 64 == 0, Hq % Hkv == 0,
 * Hq / Hkv <= 8. */
typedef struct {
  int32_t B;    /* batch */
  int32_t Hq;   /* query heads */
  int32_t Hkv;  /* KV heads */
  int32_t L;    /* tokens in the cache */
  int32_t D;    /* head dim */
  int32_t tile; /* tokens per tile */
  int32_t dtype; /* HS_BF16 or HS_FP16: element type of Q, K, V, O and of the pools */
} hs_shape;

/* Bit 30 of the magnitude of a v_map entry (bf16 caches only): the tile's stored values (all of a
 * dense tile, the kept ones of a 2:4 tile) are every one exact in IEEE fp16 and are held in
 * the pool in fp16 encoding -- same values, other bit patterns; hs_unpack_kv gives the bf16
 * patterns back.  hs_compress_kv and hs_append_tile decide this per tile.  It lets attention
 * multiply such a tile by softmax numerators in one fp16 term instead of two bf16 terms.
 * Slot of an entry m != 0: (|m| & ~HS_MAP_F16) - 1; pool: dense if m > 0, 2:4 if m < 0. */
enum { HS_MAP_F16 = 1 << 30 };

/* Element types.  Pruning compares magnitudes through the bit patterns (bits & 0x7fff), which
 * orders both formats; packed values are copied bit for bit.  With fp16 the softmax
 * numerators enter the second product as one fp16 term (11 significant bits); with bf16 as
 * two bf16 terms. */
enum { HS_BF16 = 0, HS_FP16 = 1 };

/* Policy of the built-in magnitude pruner (Sec. III-A, Eq. 2a-d).
 *   skip_frac      floor(skip_frac * T) tiles per (b, kv head) with the lowest
 *                  energy  sum(K^2) + sum(V^2)  are dropped for K and V alike.
 *   sparse_frac_x  the paper's block sparsity S_K / S_V: of the tiles that are
 *                  kept, floor(S * n_kept) with the lowest pruning loss
 *                  || X * (1 - m) ||_1  (Eq. 2c) are stored 2:4, the rest dense.
 *   state_k/_v     optional explicit per-tile states (the block-level masks of an external
 *                  pruner, Sec. III-A), DEVICE int8 [B, Hkv, T], values HS_SKIP / HS_DENSE /
 *                  HS_SPARSE24; when non-NULL (both or neither) they replace the fractions.
 *                  A tile must be SKIP in both or in neither.  They are read by a kernel on
 *                  `stream` and turned into maps there, so a pruner that runs on the device
 *                  hands them over without a round trip through the host.
 *   state_flag     optional DEVICE int32 (set to 0 by the caller), written only with explicit
 *                  states, which the host cannot check: bit 0 = some row needed more slots than
 *                  a pool of `out` has (the tiles that no longer fit are stored as SKIP in K
 *                  and V and take no slot), bit 1 = a state pair was not valid (value outside
 *                  0..2, or SKIP in only one tensor; the tile is stored as SKIP).
 *   tile_scores    optional DEVICE double [3, B, Hkv, T] written by hs_score_tiles: what
 *                  hs_recompress_kv ranks by when its target has fractions (a packed cache no
 *                  longer holds the original values of its 2:4 tiles).  hs_compress_kv does not
 *                  read it: it scores the tensors it is given.
 *   dense_first_tiles, dense_last_tiles
 *                  the first / last so many tiles of every row stay DENSE in K and V and
 *                  take no part in either ranking (the "sink" and "local window" tokens
 *                  the paper's evaluation keeps dense, Sec. V-A: 64 and 256 tokens = 1 and
 *                  4 tiles); the fractions then apply to the T - first - last tiles in
 *                  between.  Ignored with explicit states.
 *   element_rule   HS_RULE_MAGNITUDE: keep the 2 largest magnitudes of every group of 4
 *                  (the fused magnitude compressor, Sec. IV-B).  HS_RULE_NONZERO: the input
 *                  already carries an element mask (pruned entries are zero): keep the
 *                  non-zero entries, and if a group has fewer than 2, fill up with its
 *                  lowest-position zeros (the generic compressor of Sec. IV-B).
 * Ties in either ranking go to the lower tile index. */
enum { HS_RULE_MAGNITUDE = 0, HS_RULE_NONZERO = 1 };
typedef struct {
  double skip_frac;
  double sparse_frac_k;
  double sparse_frac_v;
  const int8_t* state_k;
  const int8_t* state_v;
  int32_t* state_flag;
  const double* tile_scores;
  int32_t dense_first_tiles;
  int32_t dense_last_tiles;
  int32_t element_rule;
} hs_policy;

/* Packed cache: caller-owned device buffers, rectangular per (b, kv head).
 *   x_dense  [B, Hkv, cap_dense_x,  16384 B]   dense pool
 *   x_nnz    [B, Hkv, cap_sparse_x,  8192 B]   kept values of 2:4 tiles
 *   x_meta   [B, Hkv, cap_sparse_x,  1024 B]   2-bit positions
 *   x_map    [B, Hkv, T] int32: +(slot+1) dense, -(slot+1) sparse, 0 skipped;
 *            slots are handed out in ascending tile order per pool (the two
 *            running counters of Sec. III-B).
 * Inside a tile slot the bytes are in the order in which the lanes of the gfx950
 * matrix instructions consume them (64 lanes x 16 B per chunk; the exact index
 * formulas are in csrc/hs_common.h); hs_unpack_kv returns the logical content.
 * The pools of a capacity-0 kind may be NULL.  All pool pointers must be 16-byte
 * aligned. */
typedef struct {
  void* k_dense; void* k_nnz; void* k_meta; int32_t* k_map;
  void* v_dense; void* v_nnz; void* v_meta; int32_t* v_map;
  int32_t cap_dense_k, cap_sparse_k, cap_dense_v, cap_sparse_v;
  int32_t uniform; /* nonzero = the caller promises that no tile is skipped and that each
                      tensor's tiles are all of one kind, i.e. slot == tile index (what
                      skip_frac 0 with sparse fractions in {0, 1} produces); attention
                      kernels then skip the map lookup.  Needs the used capacities >= T. */
} hs_kv;

/* Library version (major * 100 + minor). [host, pure] */
HS_API int hs_version(void);

/* Text for a status code. [host, pure] */
HS_API const char* hs_strerror(int status);

/* Text of the last HIP error this thread saw inside the library. [host] */
HS_API const char* hs_last_hip_error(void);

/* Tile counts a fraction policy yields per (b, kv head): counts[0..4] = n_skip,
 * n_dense_k, n_sparse_k, n_dense_v, n_sparse_v.  These are the pool capacities to allocate.
 * With explicit states (device memory) the host cannot count: HS_EUNSUPPORTED; the caller sizes
 * each pool for the largest per-row count it may produce (L / 64 is always enough).
 * [host, pure] */
HS_API int hs_tile_counts(const hs_shape* shape, const hs_policy* policy, int32_t counts[5]);

/* Bytes of the packed cache for given capacities, whole batch:
 * bytes[0..7] = k_dense, k_nnz, k_meta, k_map, v_dense, v_nnz, v_meta, v_map.
 * (Sec. III-D byte accounting.) [host, pure] */
HS_API int hs_kv_bytes(const hs_shape* shape, const int32_t counts[5], size_t bytes[8]);

/* Workspace bytes needed by each call.  [host, pure]
 *   op = 0 compress, 1 prefill (Lq = arg), 2 decode (n_splits = arg, 0 = auto), 3 re-compress
 *   (op 1 needs none; op 3 only when the target ranks tiles: then 8 bytes per tile) */
HS_API int hs_workspace_bytes(const hs_shape* shape, int op, int32_t arg, size_t* bytes);

/* Number of KV splits hs_decode_attn uses when n_splits == 0. [host, pure] */
HS_API int hs_decode_auto_splits(const hs_shape* shape);

/* Compress (Sec. III-A + III-B; fused top-2-of-4 compressor of Sec. IV-B).
 * K, V: bf16 [B, Hkv, L, D]; kv_strides = element strides of the b, head and
 * token axes (NULL = contiguous).  Element mask: K keeps the 2 largest
 * magnitudes of every 4 consecutive channels of a token, V of every 4
 * consecutive tokens of a channel (magnitude = bits & 0x7fff, ties to the lower
 * position; with HS_RULE_NONZERO the key is magnitude != 0 instead).  Writes maps and pools of `out`; slots beyond the used count are
 * left untouched.  workspace: hs_workspace_bytes(op 0), 8-byte aligned (tile scores; only read
 * and written when the policy ranks tiles).  Capacities of `out` that a fraction policy would
 * exceed are HS_EINVAL; with explicit states see hs_policy.state_flag. */
HS_API int hs_compress_kv(const hs_shape* shape, const hs_policy* policy,
                   const void* K, const void* V, const int64_t kv_strides[3],
                   const hs_kv* out, void* workspace, void* stream);

/* Tile scores of K, V (same arguments as hs_compress_kv): scores = DEVICE double [3, B, Hkv, T],
 * plane 0 the tile energy sum(K^2) + sum(V^2), planes 1 and 2 the pruning losses of K and V
 * (Eq. 2c: L1 norm of what the 2:4 mask of `element_rule` removes), fp64, fixed summation order:
 * the numbers hs_compress_kv ranks by.  For hs_recompress_kv with ranked targets. */
HS_API int hs_score_tiles(const hs_shape* shape, const void* K, const void* V, const int64_t kv_strides[3],
                   int32_t element_rule, double* scores, void* stream);

/* Fill one tile of a cache that grows during decode.  The pools hand out slots in sequence
 * order with one counter per pool (Sec. III-B), so a cache can be allocated for a capacity of
 * shape->L tokens, compressed with the tiles beyond the current length SKIP (explicit states;
 * attention ignores SKIP tiles), and extended tile by tile: tile `tile` (0 <= tile < L/64), SKIP
 * in every (b, kv head) row on entry, becomes state_k / state_v (HS_DENSE or HS_SPARSE24, the
 * same for every row; 2:4 by `element_rule`) and takes the next slot of its pool = the number of
 * tiles of that kind the row already holds (appending in tile order keeps slots in tile order,
 * i.e. the result equals one hs_compress_kv over everything).
 * K_tile, V_tile: device bf16 [B, Hkv, 64, D], element strides tile_strides[3] = {batch, head,
 * token} (innermost contiguous; NULL = contiguous), 16-byte aligned.  kv->uniform must be 0.
 * A row whose pool has no free slot (capacity cap_* of `kv`) keeps the tile SKIP; if `overflow`
 * (device int32, set to 0 by the caller) is not NULL it is then set to 1.  No workspace. */
HS_API int hs_append_tile(const hs_shape* shape, int32_t tile, int32_t state_k, int32_t state_v,
                   int32_t element_rule, const void* K_tile, const void* V_tile,
                   const int64_t tile_strides[3], const hs_kv* kv, int32_t* overflow, void* stream);

/* The same for n_tiles consecutive tiles tile .. tile + n_tiles - 1 in one call (a prefill chunk,
 * Sec. V-B: 32K-token chunks): K_tile, V_tile are [B, Hkv, 64 n_tiles, D]; all of them take
 * state_k / state_v and consecutive slots.  Tiles that no longer fit a pool stay SKIP (overflow
 * as above).  1 <= n_tiles <= 65535, tile + n_tiles <= L / 64. */
HS_API int hs_append_tiles(const hs_shape* shape, int32_t tile, int32_t n_tiles, int32_t state_k, int32_t state_v,
                    int32_t element_rule, const void* K_tile, const void* V_tile,
                    const int64_t tile_strides[3], const hs_kv* kv, int32_t* overflow, void* stream);

/* hs_append_tile for a batch whose sequences differ in length: tiles = device int32 [B], the tile
 * index that batch row b fills (in all of its kv heads), or any value outside 0 .. L/64 - 1 to
 * leave that batch row as it is (its part of K_tile, V_tile is not read). */
HS_API int hs_append_tile_rows(const hs_shape* shape, const int32_t* tiles, int32_t state_k, int32_t state_v,
                        int32_t element_rule, const void* K_tile, const void* V_tile,
                        const int64_t tile_strides[3], const hs_kv* kv, int32_t* overflow, void* stream);

/* Prune a packed cache further (Sec. III, overview of the workflow: after the prefill phase the
 * dense pool can be pruned and compressed again, so that decode runs at another sparsity than
 * prefill; Sec. V evaluates prefill at S_K = 0, S_V = 1 followed by decode at S_K = S_V = 1).
 * Every tile of `dst` is in the sparser of its state in `src` and its target state (DENSE, then
 * 2:4, then SKIP): a tile that keeps its kind is copied bit for bit, a DENSE tile that becomes
 * 2:4 is pruned from the values it stores (element rule of `target`), a tile that becomes SKIP is
 * dropped; slots of `dst` are handed out again in tile order, one counter per pool (Sec. III-B).
 * The result equals hs_compress_kv of the original tensors with those states, bit for bit.
 * target: explicit states (device arrays, as for hs_compress_kv; target->state_flag is not used),
 * or fractions.  Whole-tensor fractions -- skip_frac == 0 and sparse_frac_k, sparse_frac_v each 0
 * or 1, with dense_first_tiles / dense_last_tiles kept DENSE -- need nothing else.  Any other
 * fractions rank the tiles exactly as hs_compress_kv would rank the original tensors (Eq. 2c-d;
 * lowest energy skipped), from the scores the caller kept: target->tile_scores (hs_score_tiles,
 * taken while the original K, V existed) and `workspace` of hs_workspace_bytes(op 3) bytes,
 * 4-byte aligned; without tile_scores such a target is HS_EUNSUPPORTED.  The target state of a
 * tile is the one that policy gives it; its new state is the sparser of that and its current one.
 * src, dst: distinct caches of the same shape (no overlap); dst's capacities are the caller's
 * choice: a tile for which one of its pools has no slot left when its turn comes (tile order) is
 * left SKIP in K and V, takes no slot in either pool -- the used slots of a pool stay 0 .. n-1, so
 * hs_append_tile can go on from there -- and bit 0 of `overflow` (device int32, set to 0 by the
 * caller; may be NULL) is set.  Bit 1 is set if an explicit target pair was not valid (such a tile
 * keeps its state).  dst->uniform is not read.  workspace: only for ranked targets, else may be NULL. */
HS_API int hs_recompress_kv(const hs_shape* shape, const hs_policy* target, const hs_kv* src, const hs_kv* dst,
                     void* workspace, int32_t* overflow, void* stream);

/* Inverse of the packing, for tests and debugging: dense bf16 [B, Hkv, L, D]
 * (contiguous) with zeros at pruned positions and in skipped tiles. */
HS_API int hs_unpack_kv(const hs_shape* shape, const hs_kv* kv, void* K_out, void* V_out, void* stream);

/* Prefill attention (Algorithm 1 with the mixed dense/sparse dispatch of
 * Sec. III-C-2).  Q: bf16 [B, Hq, Lq, D] contiguous, Lq % 64 == 0, Lq <= L.
 * Query i sees token j iff tile(j) is not skipped and (!causal or
 * j <= i + L - Lq).  scale == 0 selects 1/sqrt(D) (Eq. 1).
 * O: bf16 [B, Hq, Lq, D]; LSE: fp32 [B, Hq, Lq] or NULL.  A query that sees no
 * token gets O = 0, LSE = -inf.  A pool of more than 4 GiB per (batch, kv head) row
 * (capacity x tile bytes) is HS_EUNSUPPORTED. */
HS_API int hs_prefill_attn(const hs_shape* shape, int32_t Lq, float scale, int causal,
                    const void* Q, const hs_kv* kv, void* O, float* LSE,
                    void* workspace, void* stream);

/* The same with the queries anywhere in the cache: query i stands at token position q_start + i
 * (0 <= q_start <= L - Lq, any value) and, when causal, sees token j iff tile(j) is not skipped
 * and j <= q_start + i.  hs_prefill_attn is the case q_start = L - Lq.  For caches allocated
 * for a capacity (shape->L) beyond the tokens held so far -- the tiles not filled yet are SKIP --
 * and for chunked prefill (Sec. V-B runs 32K-token chunks), where each chunk's queries sit at the
 * end of what has been compressed so far, not at the end of the capacity. */
HS_API int hs_prefill_attn_at(const hs_shape* shape, int32_t Lq, int32_t q_start, float scale, int causal,
                       const void* Q, const hs_kv* kv, void* O, float* LSE,
                       void* workspace, void* stream);

/* Decode attention (split-KV kernel + merge, Sec. IV-C): one query token per
 * (b, query head) against all L cached tokens.  Q, O: bf16 [B, Hq, D];
 * LSE: fp32 [B, Hq] or NULL.  n_splits == 0 picks hs_decode_auto_splits.
 * workspace: hs_workspace_bytes(op 2, n_splits), 16-byte aligned (split partials;
 * no initial content needed).  Two calls in flight at once must not share one. */
HS_API int hs_decode_attn(const hs_shape* shape, float scale, int32_t n_splits,
                   const void* Q, const hs_kv* kv, void* O, float* LSE,
                   void* workspace, void* stream);

/* hs_decode_attn for callers that cannot allocate device memory or be handed a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as hs_decode_attn, without the workspace: the split partials go to a fixed array of
 * HS_STATIC_SCRATCH_BYTES (4 MiB) that the library holds in device memory on every GPU it is
 * loaded on, for the life of the process.  The call allocates and frees nothing (no hipMalloc,
 * hipFree or allocating library routine); the first call on a device looks the array's address up
 * once (hipGetSymbolAddress), so make that first call outside a graph capture.
 * If hs_workspace_bytes(op 2, n_splits) exceeds HS_STATIC_SCRATCH_BYTES: HS_ENOSPACE, nothing
 * launched (B * Hq * n_splits * 516 bytes; the benchmark shapes need 0.5 MiB).
 * All calls on one GPU share the one array: two calls that overlap in time on different streams of
 * the same GPU race on it; calls on one stream are ordered and safe.  The array keeps the last
 * call's partials; every entry a call reads it has written itself, so nothing needs clearing. */
enum { HS_STATIC_SCRATCH_BYTES = 4 << 20 };
HS_API int hs_decode_attn_static(const hs_shape* shape, float scale, int32_t n_splits,
                          const void* Q, const hs_kv* kv, void* O, float* LSE, void* stream);

/* Decode attention over the packed cache plus a dense tail: the tokens generated since the
 * last full tile was compressed are not in the pools yet; they are attended to as they are
 * (recent tokens stay dense, Sec. V-A; the cache itself only ever holds whole tiles, Sec.
 * III-B).  tail_k, tail_v: device, bf16 [B, Hkv, HS_TILE, D] contiguous, rows 0..tail_len-1
 * valid, 0 <= tail_len <= HS_TILE (tail_len == 0: pointers may be NULL and the call equals
 * hs_decode_attn).  The query sees every cached token of a non-skipped tile and the tail_len
 * tail tokens.  The tail is one more split: workspace must hold
 * hs_workspace_bytes(op 2, n + 1) bytes, n = n_splits or, for n_splits == 0,
 * hs_decode_auto_splits.  Everything else as hs_decode_attn. */
HS_API int hs_decode_attn_tail(const hs_shape* shape, float scale, int32_t n_splits,
                        const void* Q, const hs_kv* kv, const void* tail_k, const void* tail_v,
                        int32_t tail_len, void* O, float* LSE, void* workspace, void* stream);

/* The same for a batch whose sequences differ in length: tail_lens = device int32 [B], the number
 * of valid tail tokens of batch row b (values outside 0 .. HS_TILE are clamped into that range).
 * Rows that hold fewer tiles than others have the rest SKIP in their maps.  tail_k, tail_v,
 * tail_lens must not be NULL. */
HS_API int hs_decode_attn_tail_rows(const hs_shape* shape, float scale, int32_t n_splits,
                             const void* Q, const hs_kv* kv, const void* tail_k, const void* tail_v,
                             const int32_t* tail_lens, void* O, float* LSE, void* workspace, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HS_H_ */
