// C ABI of libhs: host-side validation, capacity arithmetic and kernel dispatch.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "hs_common.h"
#include "hs_bench.h"

namespace {

thread_local char g_hip_err[256] = "";

int hip_fail(hipError_t e) {
  snprintf(g_hip_err, sizeof(g_hip_err), "%s", hipGetErrorString(e));
  return HS_EHIP;
}

int check_shape(const hs_shape* s) {
  if (s == nullptr) return HS_EINVAL;
  if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->L <= 0) return HS_EINVAL;
  if (s->D != HS_D || s->tile != HS_BT) return HS_EUNSUPPORTED;
  if (s->L % HS_BT != 0 || s->Hq % s->Hkv != 0) return HS_EUNSUPPORTED;
  if (s->dtype != HS_BF16 && s->dtype != HS_FP16) return HS_EUNSUPPORTED;
  if (s->Hq / s->Hkv > 8) return HS_EUNSUPPORTED;
  if (s->B > 65535 || s->Hkv > 65535 || (int64_t)s->B * s->Hkv > 65535) return HS_EUNSUPPORTED;
  return HS_OK;
}

bool frac_ok(double f) { return f >= 0.0 && f <= 1.0; }

// Tile counts of a fraction policy (same for every row).
// Protected (always dense) tiles at both ends, clipped so that they never overlap.
void protected_tiles(int T, const hs_policy* p, int* n_first, int* n_last) {
  int f = p->dense_first_tiles < T ? p->dense_first_tiles : T;
  int l = p->dense_last_tiles < T - f ? p->dense_last_tiles : T - f;
  *n_first = f;
  *n_last = l;
}

void policy_counts(int T, const hs_policy* p, int32_t c[5]) {
  int n_first, n_last;
  protected_tiles(T, p, &n_first, &n_last);
  const int n_prot = n_first + n_last, n_mid = T - n_prot;
  const int n_skip = (int)floor(p->skip_frac * n_mid);
  const int n_keep = n_mid - n_skip;
  const int nsk = (int)floor(p->sparse_frac_k * n_keep);
  const int nsv = (int)floor(p->sparse_frac_v * n_keep);
  c[0] = n_skip; c[1] = n_prot + n_keep - nsk; c[2] = nsk; c[3] = n_prot + n_keep - nsv; c[4] = nsv;
}

int check_policy(const hs_policy* p) {
  if (p == nullptr) return HS_EINVAL;
  if ((p->state_k == nullptr) != (p->state_v == nullptr)) return HS_EINVAL;
  if (p->state_k == nullptr) {
    if (!(p->skip_frac >= 0.0 && p->skip_frac < 1.0)) return HS_EINVAL;
    if (!frac_ok(p->sparse_frac_k) || !frac_ok(p->sparse_frac_v)) return HS_EINVAL;
    if (p->dense_first_tiles < 0 || p->dense_last_tiles < 0) return HS_EINVAL;
  }
  if (p->element_rule != HS_RULE_MAGNITUDE && p->element_rule != HS_RULE_NONZERO) return HS_EINVAL;
  return HS_OK;
}

int check_kv(const hs_shape* s, const hs_kv* kv) {
  if (kv == nullptr || kv->k_map == nullptr || kv->v_map == nullptr) return HS_EINVAL;
  if (kv->cap_dense_k < 0 || kv->cap_sparse_k < 0 || kv->cap_dense_v < 0 || kv->cap_sparse_v < 0) return HS_EINVAL;
  if (kv->cap_dense_k > 0 && kv->k_dense == nullptr) return HS_EINVAL;
  if (kv->cap_sparse_k > 0 && (kv->k_nnz == nullptr || kv->k_meta == nullptr)) return HS_EINVAL;
  if (kv->cap_dense_v > 0 && kv->v_dense == nullptr) return HS_EINVAL;
  if (kv->cap_sparse_v > 0 && (kv->v_nnz == nullptr || kv->v_meta == nullptr)) return HS_EINVAL;
  const uintptr_t align = (uintptr_t)kv->k_dense | (uintptr_t)kv->k_nnz | (uintptr_t)kv->k_meta |
                          (uintptr_t)kv->v_dense | (uintptr_t)kv->v_nnz | (uintptr_t)kv->v_meta;
  if (align & 15u) return HS_EINVAL;
  (void)s;
  return HS_OK;
}

int append_common(const hs_shape* shape, int32_t tile, int32_t n_tiles, const int32_t* tile_rows, int32_t state_k,
                  int32_t state_v, int32_t element_rule, const void* K_tile, const void* V_tile,
                  const int64_t tile_strides[3], const hs_kv* kv, int32_t* overflow, void* stream);

constexpr int kSelectMaxTiles = 65536;  // one workgroup per row walks its tiles: 4M tokens per row

// shared body of the decode entry points; tail_len < 0: no dense tail
int decode_common(const hs_shape* shape, float scale, int32_t n_splits, const void* Q, const hs_kv* kv,
                  const void* tail_k, const void* tail_v, int tail_len, const int32_t* tail_lens, void* O, float* LSE,
                  void* workspace, void* stream, int phases) {
  if (phases < 1 || phases > 3) return HS_EINVAL;
  int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  rc = check_kv(shape, kv);
  if (rc != HS_OK) return rc;
  if (Q == nullptr || O == nullptr || workspace == nullptr) return HS_EINVAL;
  if (((uintptr_t)Q | (uintptr_t)workspace) & 15u) return HS_EINVAL;
  if (n_splits < 0 || n_splits > 65535) return HS_EINVAL;
  if (!(scale >= 0.f)) return HS_EINVAL;
  if (scale == 0.f) scale = 1.0f / sqrtf((float)HS_D);
  if (n_splits == 0) n_splits = hs_decode_auto_splits(shape);
  if (kv->uniform) {
    const int T = shape->L / HS_BT;
    const bool k_ok = (kv->cap_dense_k == 0 && kv->cap_sparse_k >= T) || (kv->cap_sparse_k == 0 && kv->cap_dense_k >= T);
    const bool v_ok = (kv->cap_dense_v == 0 && kv->cap_sparse_v >= T) || (kv->cap_sparse_v == 0 && kv->cap_dense_v >= T);
    if (!k_ok || !v_ok) return HS_EINVAL;
  }
  const hipError_t e = hs_launch_decode(shape->B, shape->Hq, shape->Hkv, shape->L / HS_BT, scale, n_splits,
                                        (const uint16_t*)Q, hs_make_kv_dev(kv), (const uint16_t*)tail_k,
                                        (const uint16_t*)tail_v, tail_len, tail_lens, (uint16_t*)O, LSE, (float*)workspace,
                                        (hipStream_t)stream, phases, shape->dtype);
  if (e != hipSuccess) return hip_fail(e);
  return HS_OK;
}

}  // namespace

extern "C" {

int hs_version(void) { return 100; }

const char* hs_strerror(int status) {
  switch (status) {
    case HS_OK: return "ok";
    case HS_EINVAL: return "invalid argument";
    case HS_EUNSUPPORTED: return "unsupported shape or option";
    case HS_EHIP: return "HIP runtime error";
    case HS_ENOSPACE: return "the call needs more scratch memory than the library's static array holds";
    default: return "unknown status";
  }
}

const char* hs_last_hip_error(void) { return g_hip_err; }

int hs_tile_counts(const hs_shape* shape, const hs_policy* policy, int32_t counts[5]) {
  int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  rc = check_policy(policy);
  if (rc != HS_OK) return rc;
  if (counts == nullptr) return HS_EINVAL;
  // explicit states live on the device: their counts are the caller's to know (at most T per pool)
  if (policy->state_k != nullptr) return HS_EUNSUPPORTED;
  policy_counts(shape->L / HS_BT, policy, counts);
  return HS_OK;
}

int hs_kv_bytes(const hs_shape* shape, const int32_t counts[5], size_t bytes[8]) {
  const int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  if (counts == nullptr || bytes == nullptr) return HS_EINVAL;
  const size_t rows = (size_t)shape->B * shape->Hkv;
  const size_t T = (size_t)(shape->L / HS_BT);
  bytes[0] = rows * (size_t)counts[1] * HS_TILE_DENSE_BYTES;
  bytes[1] = rows * (size_t)counts[2] * HS_TILE_NNZ_BYTES;
  bytes[2] = rows * (size_t)counts[2] * HS_TILE_META_BYTES;
  bytes[3] = rows * T * sizeof(int32_t);
  bytes[4] = rows * (size_t)counts[3] * HS_TILE_DENSE_BYTES;
  bytes[5] = rows * (size_t)counts[4] * HS_TILE_NNZ_BYTES;
  bytes[6] = rows * (size_t)counts[4] * HS_TILE_META_BYTES;
  bytes[7] = rows * T * sizeof(int32_t);
  return HS_OK;
}

int hs_decode_auto_splits(const hs_shape* shape) {
  if (check_shape(shape) != HS_OK) return 0;
  const int T = shape->L / HS_BT;
  const int rows = shape->B * shape->Hkv;
  // about 1024 waves (one workgroup per compute unit, measured best on the 32K-context
  // shape); every wave of a split gets the same number of tiles: per = 4 * ceil(tiles / 1024)
  const int64_t total = (int64_t)rows * T;
  const int per_wave = (int)((total + 1023) / 1024);
  const int per = 4 * (per_wave < 1 ? 1 : per_wave);
  int n = (T + per - 1) / per;
  if (n < 1) n = 1;
  return n;
}

int hs_workspace_bytes(const hs_shape* shape, int op, int32_t arg, size_t* bytes) {
  const int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  if (bytes == nullptr) return HS_EINVAL;
  const size_t rows = (size_t)shape->B * shape->Hkv;
  const size_t T = (size_t)(shape->L / HS_BT);
  switch (op) {
    case 0: *bytes = 3 * rows * T * sizeof(double); return HS_OK;
    case 1: *bytes = 0; return HS_OK;
    case 2: {
      int n = arg == 0 ? hs_decode_auto_splits(shape) : arg;
      if (n < 1) return HS_EINVAL;
      *bytes = (size_t)shape->B * shape->Hq * (size_t)n * (HS_D + 1) * sizeof(float);
      return HS_OK;
    }
    case 3: *bytes = 2 * rows * T * sizeof(int32_t); return HS_OK;
    default: return HS_EINVAL;
  }
}

int hs_compress_kv(const hs_shape* shape, const hs_policy* policy, const void* K, const void* V,
                   const int64_t kv_strides[3], const hs_kv* out, void* workspace, void* stream) {
  int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  rc = check_policy(policy);
  if (rc != HS_OK) return rc;
  rc = check_kv(shape, out);
  if (rc != HS_OK) return rc;
  if (K == nullptr || V == nullptr) return HS_EINVAL;
  if (((uintptr_t)K | (uintptr_t)V) & 15u) return HS_EINVAL;
  const int T = shape->L / HS_BT;
  const int rows = shape->B * shape->Hkv;
  int64_t sb = (int64_t)shape->Hkv * shape->L * HS_D, sh = (int64_t)shape->L * HS_D, st = HS_D;
  if (kv_strides != nullptr) { sb = kv_strides[0]; sh = kv_strides[1]; st = kv_strides[2]; }
  if (st < HS_D || sb < 0 || sh < 0 || (sb | sh | st) % 8 != 0) return HS_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  int32_t c[5];
  hipError_t e;
  int uni_k = 0, uni_v = 0;
  if (policy->state_k != nullptr) {
    // states -> maps on the device (prefix counts = the sequential counters of Sec. III-B); what the host
    // cannot see (a state pair that is not valid, a row that needs more slots than a pool has) is reported
    // through policy->state_flag and such tiles are stored as SKIP
    if (T > kSelectMaxTiles) return HS_EUNSUPPORTED;
    e = hs_launch_states_to_maps(policy->state_k, policy->state_v, rows, T, hs_make_kv_dev(out), policy->state_flag, s);
    if (e != hipSuccess) return hip_fail(e);
  } else {
    policy_counts(T, policy, c);
    if (c[1] > out->cap_dense_k || c[2] > out->cap_sparse_k || c[3] > out->cap_dense_v || c[4] > out->cap_sparse_v)
      return HS_EINVAL;
    int n_first, n_last;
    protected_tiles(T, policy, &n_first, &n_last);
    const int n_keep = T - n_first - n_last - c[0];
    const bool uniform_k = c[1] == 0 || c[2] == 0, uniform_v = c[3] == 0 || c[4] == 0;
    if (c[0] == 0 && uniform_k && uniform_v) {
      // no ranking needed: every tile in one state; the pack kernel writes the maps itself
      uni_k = c[2] ? HS_SPARSE24 : HS_DENSE;
      uni_v = c[4] ? HS_SPARSE24 : HS_DENSE;
    } else if (c[0] == 0 && (c[2] == 0 || c[2] == n_keep) && (c[4] == 0 || c[4] == n_keep)) {
      // no ranking needed either: protected end tiles dense, every tile in between in one state;
      // the selection kernel never looks at the scores then
      if (T > kSelectMaxTiles) return HS_EUNSUPPORTED;
      e = hs_launch_select(nullptr, rows, T, 0, c[2], c[4], n_first, n_last, out->k_map, out->v_map, s);
      if (e != hipSuccess) return hip_fail(e);
    } else {
      if (workspace == nullptr || ((uintptr_t)workspace & 7u)) return HS_EINVAL;
      if (T > kSelectMaxTiles) return HS_EUNSUPPORTED;
      // energies rank the skipped tiles; losses split the kept ones unless they all end up alike
      const int what = (c[0] > 0 ? 1 : 0) | ((c[2] != 0 && c[2] != n_keep) || (c[4] != 0 && c[4] != n_keep) ? 2 : 0);
      e = hs_launch_score((const uint16_t*)K, (const uint16_t*)V, sb, sh, st, shape->B, shape->Hkv, T,
                          policy->element_rule, shape->dtype, what, (double*)workspace, s);
      if (e != hipSuccess) return hip_fail(e);
      e = hs_launch_select((const double*)workspace, rows, T, c[0], c[2], c[4], n_first, n_last, out->k_map,
                           out->v_map, s);
      if (e != hipSuccess) return hip_fail(e);
    }
  }
  e = hs_launch_pack((const uint16_t*)K, (const uint16_t*)V, sb, sh, st, shape->B, shape->Hkv, T,
                     hs_make_kv_dev(out), uni_k, uni_v, policy->element_rule, shape->dtype == HS_BF16, s);
  if (e != hipSuccess) return hip_fail(e);
  return HS_OK;
}

int hs_append_tile(const hs_shape* shape, int32_t tile, int32_t state_k, int32_t state_v, int32_t element_rule,
                   const void* K_tile, const void* V_tile, const int64_t tile_strides[3], const hs_kv* kv,
                   int32_t* overflow, void* stream) {
  return hs_append_tiles(shape, tile, 1, state_k, state_v, element_rule, K_tile, V_tile, tile_strides, kv, overflow,
                         stream);
}

int hs_append_tiles(const hs_shape* shape, int32_t tile, int32_t n_tiles, int32_t state_k, int32_t state_v,
                    int32_t element_rule, const void* K_tile, const void* V_tile, const int64_t tile_strides[3],
                    const hs_kv* kv, int32_t* overflow, void* stream) {
  return append_common(shape, tile, n_tiles, nullptr, state_k, state_v, element_rule, K_tile, V_tile, tile_strides, kv,
                       overflow, stream);
}

int hs_append_tile_rows(const hs_shape* shape, const int32_t* tiles, int32_t state_k, int32_t state_v,
                        int32_t element_rule, const void* K_tile, const void* V_tile, const int64_t tile_strides[3],
                        const hs_kv* kv, int32_t* overflow, void* stream) {
  if (tiles == nullptr) return HS_EINVAL;
  return append_common(shape, 0, 1, tiles, state_k, state_v, element_rule, K_tile, V_tile, tile_strides, kv, overflow,
                       stream);
}

}  // extern "C"

namespace {
int append_common(const hs_shape* shape, int32_t tile, int32_t n_tiles, const int32_t* tile_rows, int32_t state_k,
                  int32_t state_v, int32_t element_rule, const void* K_tile, const void* V_tile,
                  const int64_t tile_strides[3], const hs_kv* kv, int32_t* overflow, void* stream) {
  int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  rc = check_kv(shape, kv);
  if (rc != HS_OK) return rc;
  const int T = shape->L / HS_BT;
  if (tile < 0 || n_tiles < 1 || n_tiles > 65535 || tile > T - n_tiles || kv->uniform) return HS_EINVAL;
  if ((state_k != HS_DENSE && state_k != HS_SPARSE24) || (state_v != HS_DENSE && state_v != HS_SPARSE24)) return HS_EINVAL;
  if (element_rule != HS_RULE_MAGNITUDE && element_rule != HS_RULE_NONZERO) return HS_EINVAL;
  if (K_tile == nullptr || V_tile == nullptr || (((uintptr_t)K_tile | (uintptr_t)V_tile) & 15u)) return HS_EINVAL;
  // a pool this call may write to has to exist
  if ((state_k == HS_DENSE ? kv->cap_dense_k : kv->cap_sparse_k) < 1) return HS_EINVAL;
  if ((state_v == HS_DENSE ? kv->cap_dense_v : kv->cap_sparse_v) < 1) return HS_EINVAL;
  int64_t sb = (int64_t)shape->Hkv * n_tiles * HS_BT * HS_D, sh = (int64_t)n_tiles * HS_BT * HS_D, st = HS_D;
  if (tile_strides != nullptr) {
    sb = tile_strides[0]; sh = tile_strides[1]; st = tile_strides[2];
    if (st < HS_D || sh < 0 || sb < 0 || ((sb | sh | st) & 7)) return HS_EINVAL;
  }
  const hipError_t e = hs_launch_append((const uint16_t*)K_tile, (const uint16_t*)V_tile, sb, sh, st, shape->B,
                                        shape->Hkv, T, tile, n_tiles, tile_rows, state_k, state_v, hs_make_kv_dev(kv),
                                        element_rule, shape->dtype == HS_BF16, overflow, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return HS_OK;
}
}  // namespace

extern "C" {

int hs_recompress_kv(const hs_shape* shape, const hs_policy* target, const hs_kv* src, const hs_kv* dst,
                     void* workspace, int32_t* overflow, void* stream) {
  int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  rc = check_policy(target);
  if (rc != HS_OK) return rc;
  rc = check_kv(shape, src);
  if (rc != HS_OK) return rc;
  rc = check_kv(shape, dst);
  if (rc != HS_OK) return rc;
  (void)workspace;
  if (src->k_map == dst->k_map || src->v_map == dst->v_map) return HS_EINVAL;  // not in place: slots move
  const int T = shape->L / HS_BT;
  if (T > kSelectMaxTiles) return HS_EUNSUPPORTED;
  int n_first = 0, n_last = 0, fk = HS_DENSE, fv = HS_DENSE;
  const int32_t* tgt_map_k = nullptr;
  const int32_t* tgt_map_v = nullptr;
  hipStream_t s = (hipStream_t)stream;
  if (target->state_k == nullptr) {
    protected_tiles(T, target, &n_first, &n_last);
    const bool whole = target->skip_frac == 0.0 && (target->sparse_frac_k == 0.0 || target->sparse_frac_k == 1.0) &&
                       (target->sparse_frac_v == 0.0 || target->sparse_frac_v == 1.0);
    if (whole) {
      fk = target->sparse_frac_k == 0.0 ? HS_DENSE : HS_SPARSE24;
      fv = target->sparse_frac_v == 0.0 ? HS_DENSE : HS_SPARSE24;
    } else {
      // ranked target: the states hs_compress_kv would give the original tensors, from the scores the
      // caller kept; the selection kernel writes them as maps into the workspace (only their signs are used)
      if (target->tile_scores == nullptr) return HS_EUNSUPPORTED;
      if (workspace == nullptr || ((uintptr_t)workspace & 3u) || ((uintptr_t)target->tile_scores & 7u)) return HS_EINVAL;
      int32_t c[5];
      policy_counts(T, target, c);
      int32_t* tk = (int32_t*)workspace;
      int32_t* tv = tk + (int64_t)shape->B * shape->Hkv * T;
      const hipError_t e0 = hs_launch_select(target->tile_scores, shape->B * shape->Hkv, T, c[0], c[2], c[4], n_first, n_last,
                                             tk, tv, s);
      if (e0 != hipSuccess) return hip_fail(e0);
      tgt_map_k = tk;
      tgt_map_v = tv;
    }
  }
  const hipError_t e = hs_launch_recompress(shape->B, shape->Hkv, T, hs_make_kv_dev(src), target->state_k, target->state_v,
                                            tgt_map_k, tgt_map_v, fk, fv, n_first, n_last, hs_make_kv_dev(dst),
                                            target->element_rule, shape->dtype == HS_BF16, overflow, s);
  if (e != hipSuccess) return hip_fail(e);
  return HS_OK;
}

int hs_score_tiles(const hs_shape* shape, const void* K, const void* V, const int64_t kv_strides[3], int32_t element_rule,
                   double* scores, void* stream) {
  const int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  if (K == nullptr || V == nullptr || scores == nullptr) return HS_EINVAL;
  if ((((uintptr_t)K | (uintptr_t)V) & 15u) || ((uintptr_t)scores & 7u)) return HS_EINVAL;
  if (element_rule != HS_RULE_MAGNITUDE && element_rule != HS_RULE_NONZERO) return HS_EINVAL;
  int64_t sb = (int64_t)shape->Hkv * shape->L * HS_D, sh = (int64_t)shape->L * HS_D, st = HS_D;
  if (kv_strides != nullptr) { sb = kv_strides[0]; sh = kv_strides[1]; st = kv_strides[2]; }
  if (st < HS_D || sb < 0 || sh < 0 || (sb | sh | st) % 8 != 0) return HS_EINVAL;
  const hipError_t e = hs_launch_score((const uint16_t*)K, (const uint16_t*)V, sb, sh, st, shape->B, shape->Hkv,
                                       shape->L / HS_BT, element_rule, shape->dtype, 3, scores, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return HS_OK;
}

int hs_unpack_kv(const hs_shape* shape, const hs_kv* kv, void* K_out, void* V_out, void* stream) {
  int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  rc = check_kv(shape, kv);
  if (rc != HS_OK) return rc;
  if (K_out == nullptr || V_out == nullptr || (((uintptr_t)K_out | (uintptr_t)V_out) & 15u)) return HS_EINVAL;
  const hipError_t e = hs_launch_unpack(shape->B, shape->Hkv, shape->L / HS_BT, hs_make_kv_dev(kv),
                                        (uint16_t*)K_out, (uint16_t*)V_out, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return HS_OK;
}

int hs_prefill_attn(const hs_shape* shape, int32_t Lq, float scale, int causal, const void* Q, const hs_kv* kv,
                    void* O, float* LSE, void* workspace, void* stream) {
  if (shape == nullptr) return HS_EINVAL;
  return hs_prefill_attn_at(shape, Lq, shape->L - Lq, scale, causal, Q, kv, O, LSE, workspace, stream);
}

int hs_prefill_attn_at(const hs_shape* shape, int32_t Lq, int32_t q_start, float scale, int causal, const void* Q,
                       const hs_kv* kv, void* O, float* LSE, void* workspace, void* stream) {
  (void)workspace;
  int rc = check_shape(shape);
  if (rc != HS_OK) return rc;
  rc = check_kv(shape, kv);
  if (rc != HS_OK) return rc;
  if (Q == nullptr || O == nullptr || (((uintptr_t)Q | (uintptr_t)O) & 15u)) return HS_EINVAL;
  if (Lq <= 0 || Lq > shape->L) return HS_EINVAL;
  if (q_start < 0 || q_start > shape->L - Lq) return HS_EINVAL;
  if (Lq % HS_BT != 0) return HS_EUNSUPPORTED;
  // the prefill kernel addresses a tile inside its row's pool with a 32-bit byte offset
  if ((int64_t)kv->cap_dense_k * HS_TILE_DENSE_BYTES > (int64_t)1 << 32 ||
      (int64_t)kv->cap_dense_v * HS_TILE_DENSE_BYTES > (int64_t)1 << 32 ||
      (int64_t)kv->cap_sparse_k * HS_TILE_NNZ_BYTES > (int64_t)1 << 32 ||
      (int64_t)kv->cap_sparse_v * HS_TILE_NNZ_BYTES > (int64_t)1 << 32)
    return HS_EUNSUPPORTED;
  if (!(scale >= 0.f)) return HS_EINVAL;
  if (scale == 0.f) scale = 1.0f / sqrtf((float)HS_D);
  const hipError_t e = hs_launch_prefill(shape->B, shape->Hq, shape->Hkv, shape->L / HS_BT, Lq / HS_BT, q_start, scale,
                                         causal != 0, (const uint16_t*)Q, hs_make_kv_dev(kv), (uint16_t*)O, LSE,
                                         (hipStream_t)stream, shape->dtype);
  if (e != hipSuccess) return hip_fail(e);
  return HS_OK;
}

int hs_decode_attn(const hs_shape* shape, float scale, int32_t n_splits, const void* Q, const hs_kv* kv, void* O,
                   float* LSE, void* workspace, void* stream) {
  return hs_decode_attn_phases(shape, scale, n_splits, Q, kv, O, LSE, workspace, stream, 3);
}

int hs_decode_attn_static(const hs_shape* shape, float scale, int32_t n_splits, const void* Q, const hs_kv* kv, void* O,
                          float* LSE, void* stream) {
  size_t need = 0;
  if (n_splits < 0) return HS_EINVAL;
  const int rc = hs_workspace_bytes(shape, 2, n_splits, &need);
  if (rc != HS_OK) return rc;
  if (need > HS_STATIC_SCRATCH_BYTES) return HS_ENOSPACE;
  void* ws = nullptr;
  size_t have = 0;
  const hipError_t e = hs_static_scratch(&ws, &have);  // a symbol lookup on the first call per device, no allocation
  if (e != hipSuccess) return hip_fail(e);
  if (need > have) return HS_ENOSPACE;
  // every partial the merge kernel reads is written by the split kernel of the same call: what an
  // earlier call left in the array does not matter and nothing has to be cleared
  return decode_common(shape, scale, n_splits, Q, kv, nullptr, nullptr, -1, nullptr, O, LSE, ws, stream, 3);
}

int hs_decode_attn_phases(const hs_shape* shape, float scale, int32_t n_splits, const void* Q, const hs_kv* kv, void* O,
                          float* LSE, void* workspace, void* stream, int phases) {
  return decode_common(shape, scale, n_splits, Q, kv, nullptr, nullptr, -1, nullptr, O, LSE, workspace, stream, phases);
}

int hs_decode_attn_tail(const hs_shape* shape, float scale, int32_t n_splits, const void* Q, const hs_kv* kv,
                        const void* tail_k, const void* tail_v, int32_t tail_len, void* O, float* LSE, void* workspace,
                        void* stream) {
  if (tail_len < 0 || tail_len > HS_BT) return HS_EINVAL;
  if (tail_len > 0 && (tail_k == nullptr || tail_v == nullptr)) return HS_EINVAL;
  if (((uintptr_t)tail_k | (uintptr_t)tail_v) & 15u) return HS_EINVAL;
  return decode_common(shape, scale, n_splits, Q, kv, tail_k, tail_v, tail_len, nullptr, O, LSE, workspace, stream, 3);
}

int hs_probe_mfma_rate(int kind, int32_t iters, void* sink, double* flop, void* stream) {
  if ((kind != 0 && kind != 1) || iters < 1 || sink == nullptr || ((uintptr_t)sink & 7u) || flop == nullptr) return HS_EINVAL;
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return hip_fail(e);
  const int n_wg = 2 * cus;  // 4 waves each: 2 waves per SIMD
  e = hs_launch_mfma_rate(kind, iters, n_wg, (long long*)sink, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  // dense-equivalent flops of the launch: 8 instructions per iteration and wave, 2*16*16*K each
  *flop = (double)n_wg * 4.0 * 8.0 * (double)iters * 2.0 * 16.0 * 16.0 * (kind == 0 ? 32.0 : 64.0);
  return HS_OK;
}

int hs_probe_stream_read(const void* buf, int32_t n_tiles, int32_t n_workgroups, int with_epilogue, void* sink,
                         void* stream) {
  if (buf == nullptr || sink == nullptr || (((uintptr_t)buf | (uintptr_t)sink) & 15u)) return HS_EINVAL;
  if (n_tiles < 1 || n_workgroups < 1 || n_workgroups > 65535 || n_tiles % (4 * n_workgroups) != 0) return HS_EINVAL;
  const hipError_t e = hs_launch_stream_read((const uint8_t*)buf, n_tiles, n_workgroups, with_epilogue != 0, (float*)sink,
                                             (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return HS_OK;
}

int hs_decode_attn_tail_rows(const hs_shape* shape, float scale, int32_t n_splits, const void* Q, const hs_kv* kv,
                             const void* tail_k, const void* tail_v, const int32_t* tail_lens, void* O, float* LSE,
                             void* workspace, void* stream) {
  if (tail_k == nullptr || tail_v == nullptr || tail_lens == nullptr) return HS_EINVAL;
  if (((uintptr_t)tail_k | (uintptr_t)tail_v) & 15u) return HS_EINVAL;
  return decode_common(shape, scale, n_splits, Q, kv, tail_k, tail_v, 0, tail_lens, O, LSE, workspace, stream, 3);
}

}  // extern "C"
