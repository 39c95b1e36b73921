"""ctypes binding over libhs.so: argument marshalling only.

Every step of the hot path runs in the library's HIP kernels; PyTorch supplies
device memory and the stream.  There is no fallback: if the library has not
been built, `lib()` raises.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhs.so")
_lib = None

SKIP, DENSE, SPARSE24 = 0, 1, 2
TILE = 64
HEAD_DIM = 128
TILE_DENSE_BYTES, TILE_NNZ_BYTES, TILE_META_BYTES = 16384, 8192, 1024


class HsShape(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("L", C.c_int32), ("D", C.c_int32),
                ("tile", C.c_int32), ("dtype", C.c_int32)]


class HsPolicy(C.Structure):
    _fields_ = [("skip_frac", C.c_double), ("sparse_frac_k", C.c_double), ("sparse_frac_v", C.c_double),
                ("state_k", C.c_void_p), ("state_v", C.c_void_p), ("state_flag", C.c_void_p),
                ("tile_scores", C.c_void_p), ("dense_first_tiles", C.c_int32), ("dense_last_tiles", C.c_int32), ("element_rule", C.c_int32)]


class HsKV(C.Structure):
    _fields_ = [("k_dense", C.c_void_p), ("k_nnz", C.c_void_p), ("k_meta", C.c_void_p), ("k_map", C.c_void_p),
                ("v_dense", C.c_void_p), ("v_nnz", C.c_void_p), ("v_meta", C.c_void_p), ("v_map", C.c_void_p),
                ("cap_dense_k", C.c_int32), ("cap_sparse_k", C.c_int32), ("cap_dense_v", C.c_int32),
                ("cap_sparse_v", C.c_int32), ("uniform", C.c_int32)]


EXPORTS = {
    "hs_version": (C.c_int, []),
    "hs_strerror": (C.c_char_p, [C.c_int]),
    "hs_last_hip_error": (C.c_char_p, []),
    "hs_tile_counts": (C.c_int, [C.POINTER(HsShape), C.POINTER(HsPolicy), C.POINTER(C.c_int32)]),
    "hs_kv_bytes": (C.c_int, [C.POINTER(HsShape), C.POINTER(C.c_int32), C.POINTER(C.c_size_t)]),
    "hs_workspace_bytes": (C.c_int, [C.POINTER(HsShape), C.c_int, C.c_int32, C.POINTER(C.c_size_t)]),
    "hs_decode_auto_splits": (C.c_int, [C.POINTER(HsShape)]),
    "hs_compress_kv": (C.c_int, [C.POINTER(HsShape), C.POINTER(HsPolicy), C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_int64), C.POINTER(HsKV), C.c_void_p, C.c_void_p]),
    "hs_append_tiles": (C.c_int, [C.POINTER(HsShape), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                  C.c_void_p, C.POINTER(C.c_int64), C.POINTER(HsKV), C.c_void_p, C.c_void_p]),
    "hs_append_tile_rows": (C.c_int, [C.POINTER(HsShape), C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_void_p, C.POINTER(C.c_int64), C.POINTER(HsKV), C.c_void_p, C.c_void_p]),
    "hs_decode_attn_tail_rows": (C.c_int, [C.POINTER(HsShape), C.c_float, C.c_int32, C.c_void_p, C.POINTER(HsKV), C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hs_score_tiles": (C.c_int, [C.POINTER(HsShape), C.c_void_p, C.c_void_p, C.POINTER(C.c_int64), C.c_int32, C.c_void_p,
                                 C.c_void_p]),
    "hs_unpack_kv": (C.c_int, [C.POINTER(HsShape), C.POINTER(HsKV), C.c_void_p, C.c_void_p, C.c_void_p]),
    "hs_probe_mfma_rate": (C.c_int, [C.c_int, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]),
    "hs_probe_stream_read": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int, C.c_void_p, C.c_void_p]),
    "hs_recompress_kv": (C.c_int, [C.POINTER(HsShape), C.POINTER(HsPolicy), C.POINTER(HsKV), C.POINTER(HsKV), C.c_void_p,
                                   C.c_void_p, C.c_void_p]),
    "hs_prefill_attn": (C.c_int, [C.POINTER(HsShape), C.c_int32, C.c_float, C.c_int, C.c_void_p, C.POINTER(HsKV),
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hs_prefill_attn_at": (C.c_int, [C.POINTER(HsShape), C.c_int32, C.c_int32, C.c_float, C.c_int, C.c_void_p,
                                     C.POINTER(HsKV), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hs_decode_attn": (C.c_int, [C.POINTER(HsShape), C.c_float, C.c_int32, C.c_void_p, C.POINTER(HsKV), C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_void_p]),
    "hs_decode_attn_static": (C.c_int, [C.POINTER(HsShape), C.c_float, C.c_int32, C.c_void_p, C.POINTER(HsKV), C.c_void_p,
                                        C.c_void_p, C.c_void_p]),
    "hs_append_tile": (C.c_int, [C.POINTER(HsShape), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_int64), C.POINTER(HsKV), C.c_void_p, C.c_void_p]),
    "hs_decode_attn_tail": (C.c_int, [C.POINTER(HsShape), C.c_float, C.c_int32, C.c_void_p, C.POINTER(HsKV), C.c_void_p,
                                      C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hs_decode_attn_phases": (C.c_int, [C.POINTER(HsShape), C.c_float, C.c_int32, C.c_void_p, C.POINTER(HsKV),
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]),
}


def lib():
    """The loaded C-ABI library.  Raises if libhs.so is missing (no CPU fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is not built: run `python -m paper_2604_16864_amd.build` "
                               "(or __graft_entry__.build()) first")
        L = C.CDLL(_LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


class HsError(RuntimeError):
    pass


def _check(rc):
    if rc != 0:
        L = lib()
        msg = L.hs_strerror(rc).decode()
        if rc == -3:
            msg += ": " + L.hs_last_hip_error().decode()
        raise HsError(f"libhs error {rc}: {msg}")


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


BF16, FP16 = 0, 1
MAP_F16 = 1 << 30   # in |v_map entry| of a bf16 cache: the tile's stored values are in fp16 encoding


def make_shape(B, Hq, Hkv, L, D=HEAD_DIM, tile=TILE, dtype=BF16):
    """dtype: BF16 or FP16 (or the torch dtype) = element type of Q, K, V, O."""
    if dtype is torch.bfloat16:
        dtype = BF16
    elif dtype is torch.float16:
        dtype = FP16
    return HsShape(B, Hq, Hkv, L, D, tile, int(dtype))


def torch_dtype(shape):
    return torch.float16 if shape.dtype == FP16 else torch.bfloat16


RULE_MAGNITUDE, RULE_NONZERO = 0, 1


def make_policy(skip_frac=0.0, sparse_frac_k=1.0, sparse_frac_v=1.0, state_k=None, state_v=None,
                dense_first_tiles=0, dense_last_tiles=0, element_rule=RULE_MAGNITUDE, device="cuda", tile_scores=None):
    """state_k/state_v: optional explicit tile states [B, Hkv, T]: int8 device tensors (handed to the
    library as they are), or host arrays -- a convenience of this binding: they are checked here (the
    library cannot read them on the host), copied to the device, and their per-row counts are kept
    for tile_counts.  The returned object keeps the device tensors alive and owns the library's
    device-side flag for explicit states (`state_flag`, see check_state_flag).
    tile_scores: float64 device tensor [3, B, Hkv, T] from score_tiles, for ranked recompress_kv targets."""
    p = HsPolicy(float(skip_frac), float(sparse_frac_k), float(sparse_frac_v), None, None, None, None,
                 int(dense_first_tiles), int(dense_last_tiles), int(element_rule))
    if tile_scores is not None:
        assert tile_scores.dtype == torch.float64 and tile_scores.is_cuda and tile_scores.is_contiguous()
        p.tile_scores = tile_scores.data_ptr()
        p._scores = tile_scores
    if state_k is not None:
        if torch.is_tensor(state_k):
            sk, sv = state_k, state_v
            assert sk.dtype == torch.int8 and sv.dtype == torch.int8 and sk.is_cuda and sv.is_cuda
            assert sk.is_contiguous() and sv.is_contiguous() and sk.shape == sv.shape
            p._host_counts = None
        else:
            hk = np.ascontiguousarray(state_k, dtype=np.int8)
            hv = np.ascontiguousarray(state_v, dtype=np.int8)
            if hk.shape != hv.shape or hk.min() < 0 or hk.max() > 2 or hv.min() < 0 or hv.max() > 2 \
                    or ((hk == SKIP) != (hv == SKIP)).any():
                raise HsError("explicit tile states: values must be SKIP / DENSE / SPARSE24 and a tile must be "
                              "skipped in K and V alike")
            n = [int((a == v).sum(-1).max()) for a, v in ((hk, SKIP), (hk, DENSE), (hk, SPARSE24), (hv, DENSE), (hv, SPARSE24))]
            p._host_counts = n
            sk, sv = torch.from_numpy(hk).to(device), torch.from_numpy(hv).to(device)
        flag = torch.zeros(1, dtype=torch.int32, device=sk.device)
        p.state_k, p.state_v, p.state_flag = sk.data_ptr(), sv.data_ptr(), flag.data_ptr()
        p._keep = (sk, sv, flag)
    return p


def check_state_flag(policy):
    """Reads the device flag that calls with explicit states raise (this synchronises): raises if a
    pool capacity was exceeded or a state pair was not valid; clears the flag."""
    if not policy.state_k:
        return
    flag = policy._keep[2]
    v = int(flag.item())
    flag.zero_()
    if v:
        raise HsError("explicit tile states: " + " and ".join(
            m for b, m in ((1, "a row needed more slots than a pool has (those tiles were stored as SKIP)"),
                           (2, "a state pair was not valid (those tiles were stored as SKIP)")) if v & b))


def tile_counts(shape, policy):
    """Pool capacities per (b, kv head) row for a policy.  Explicit states given as host arrays: their
    per-row maxima; given as device tensors: the always-sufficient T per pool."""
    if policy.state_k:
        T = shape.L // TILE
        return list(policy._host_counts) if policy._host_counts is not None else [0, T, T, T, T]
    c = (C.c_int32 * 5)()
    _check(lib().hs_tile_counts(C.byref(shape), C.byref(policy), c))
    return list(c)


def kv_bytes(shape, counts):
    c = (C.c_int32 * 5)(*counts)
    b = (C.c_size_t * 8)()
    _check(lib().hs_kv_bytes(C.byref(shape), c, b))
    return list(b)


def workspace_bytes(shape, op, arg=0):
    out = C.c_size_t(0)
    _check(lib().hs_workspace_bytes(C.byref(shape), op, arg, C.byref(out)))
    return out.value


def decode_auto_splits(shape):
    return lib().hs_decode_auto_splits(C.byref(shape))


class PackedKV:
    """Caller-owned device buffers of a packed cache (torch uint8 / int32 tensors)."""

    def __init__(self, shape, counts, device="cuda"):
        self.shape = shape
        self.counts = list(counts)
        nb = kv_bytes(shape, counts)
        rows_T = (shape.B, shape.Hkv, shape.L // TILE)

        def buf(n):
            return torch.empty(n, dtype=torch.uint8, device=device) if n else None

        self.k_dense, self.k_nnz, self.k_meta = buf(nb[0]), buf(nb[1]), buf(nb[2])
        self.v_dense, self.v_nnz, self.v_meta = buf(nb[4]), buf(nb[5]), buf(nb[6])
        self.k_map = torch.empty(rows_T, dtype=torch.int32, device=device)
        self.v_map = torch.empty(rows_T, dtype=torch.int32, device=device)
        self.nbytes = sum(nb)
        T = shape.L // TILE
        # slot == tile index: nothing skipped, one kind of tile per tensor
        self.uniform = int(counts[0] == 0 and (counts[1] == 0 or counts[2] == 0) and (counts[3] == 0 or counts[4] == 0)
                           and max(counts[1], counts[2]) == T and max(counts[3], counts[4]) == T)

    def struct(self):
        return HsKV(_ptr(self.k_dense), _ptr(self.k_nnz), _ptr(self.k_meta), _ptr(self.k_map),
                    _ptr(self.v_dense), _ptr(self.v_nnz), _ptr(self.v_meta), _ptr(self.v_map),
                    self.counts[1], self.counts[2], self.counts[3], self.counts[4], self.uniform)


def _workspace(nbytes, device):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)


def compress_kv(shape, policy, K, V, out=None, workspace=None):
    """K, V: bf16 device tensors [B, Hkv, L, D] (last dim contiguous).  Returns PackedKV."""
    assert K.dtype == torch_dtype(shape) and V.dtype == K.dtype and K.is_cuda and V.is_cuda
    assert K.stride(-1) == 1 and V.stride(-1) == 1 and K.stride() == V.stride()
    if out is None:
        out = PackedKV(shape, tile_counts(shape, policy), K.device)
    if workspace is None:
        workspace = _workspace(workspace_bytes(shape, 0), K.device)
    strides = (C.c_int64 * 3)(K.stride(0), K.stride(1), K.stride(2))
    if policy.state_k:
        out.uniform = 0      # explicit states may skip tiles or mix kinds: no "slot == tile" promise
    kvs = out.struct()
    _check(lib().hs_compress_kv(C.byref(shape), C.byref(policy), _ptr(K), _ptr(V), strides, C.byref(kvs),
                                _ptr(workspace), _stream()))
    return out


def append_tile(shape, kv, tile, K_tile, V_tile, state_k=SPARSE24, state_v=SPARSE24, element_rule=RULE_MAGNITUDE,
                overflow=None):
    """K_tile, V_tile: bf16 device tensors [B, Hkv, 64 n, D] (last dim contiguous); fills tiles tile .. tile + n - 1
    of kv.  overflow: optional int32 device tensor (1 element) raised when a row's pool is full."""
    assert K_tile.dtype == torch_dtype(shape) and V_tile.dtype == K_tile.dtype and K_tile.stride() == V_tile.stride()
    n = K_tile.shape[2] // TILE
    assert K_tile.stride(-1) == 1 and tuple(K_tile.shape) == (shape.B, shape.Hkv, TILE * n, shape.D) and n >= 1
    strides = (C.c_int64 * 3)(K_tile.stride(0), K_tile.stride(1), K_tile.stride(2))
    kvs = kv.struct()
    if torch.is_tensor(tile):        # one tile index per batch row (int32 device tensor [B])
        assert n == 1 and tile.dtype == torch.int32 and tile.is_cuda and tile.numel() == shape.B and tile.is_contiguous()
        _check(lib().hs_append_tile_rows(C.byref(shape), _ptr(tile), int(state_k), int(state_v), int(element_rule),
                                         _ptr(K_tile), _ptr(V_tile), strides, C.byref(kvs), _ptr(overflow), _stream()))
    elif n == 1:
        _check(lib().hs_append_tile(C.byref(shape), int(tile), int(state_k), int(state_v), int(element_rule), _ptr(K_tile),
                                    _ptr(V_tile), strides, C.byref(kvs), _ptr(overflow), _stream()))
    else:
        _check(lib().hs_append_tiles(C.byref(shape), int(tile), n, int(state_k), int(state_v), int(element_rule),
                                     _ptr(K_tile), _ptr(V_tile), strides, C.byref(kvs), _ptr(overflow), _stream()))


def recompress_kv(shape, kv, target, counts=None, overflow=None, out=None, workspace=None):
    """Prune the packed cache `kv` further towards the policy `target` (make_policy: explicit states,
    fractions 0 / 1 with protected end tiles, or any fractions together with tile_scores).  Returns a new PackedKV; counts = capacities of
    the new pools as [_, dense K, 2:4 K, dense V, 2:4 V] (default: enough for any outcome); out: a
    PackedKV to fill instead of a new one."""
    T = shape.L // TILE
    if counts is None:
        counts = [0, kv.counts[1], min(T, kv.counts[1] + kv.counts[2]), kv.counts[3], min(T, kv.counts[3] + kv.counts[4])]
        if not target.state_k:
            prot = min(T, target.dense_first_tiles + target.dense_last_tiles)
            if target.sparse_frac_k == 1.0:
                counts[1] = min(counts[1], prot)
            if target.sparse_frac_v == 1.0:
                counts[3] = min(counts[3], prot)
    if out is None:
        out = PackedKV(shape, counts, kv.k_map.device)
    counts = out.counts
    # slot == tile survives when nothing was skipped before and each tensor ends up in one kind
    whole = not target.state_k and target.skip_frac == 0.0 and target.sparse_frac_k in (0.0, 1.0) and target.sparse_frac_v in (0.0, 1.0)
    out.uniform = int(bool(kv.uniform) and whole and counts[1] * counts[2] == 0 and counts[3] * counts[4] == 0
                      and max(counts[1], counts[2]) == T and max(counts[3], counts[4]) == T)
    if workspace is None and target.tile_scores:
        workspace = _workspace(workspace_bytes(shape, 3), kv.k_map.device)
    a, b = kv.struct(), out.struct()
    _check(lib().hs_recompress_kv(C.byref(shape), C.byref(target), C.byref(a), C.byref(b), _ptr(workspace), _ptr(overflow),
                                  _stream()))
    return out


def score_tiles(shape, K, V, element_rule=RULE_MAGNITUDE):
    """Tile scores [3, B, Hkv, T] float64 (energy, pruning loss of K, of V) of K, V [B, Hkv, L, D]."""
    assert K.dtype == torch_dtype(shape) and V.dtype == K.dtype and K.stride() == V.stride() and K.stride(-1) == 1
    out = torch.empty((3, shape.B, shape.Hkv, shape.L // TILE), dtype=torch.float64, device=K.device)
    strides = (C.c_int64 * 3)(K.stride(0), K.stride(1), K.stride(2))
    _check(lib().hs_score_tiles(C.byref(shape), _ptr(K), _ptr(V), strides, int(element_rule), _ptr(out), _stream()))
    return out


def probe_mfma_rate(kind, iters, sink):
    """Launches the register-resident matrix-instruction loop (kind 0 dense, 1 sparse; sink: 4 int64 on the device); returns the
    dense-equivalent flops of the launch.  Time it with events around the call."""
    flop = C.c_double(0.0)
    _check(lib().hs_probe_mfma_rate(int(kind), int(iters), _ptr(sink), C.byref(flop), _stream()))
    return flop.value


def probe_stream_read(buf, n_tiles, n_workgroups, with_epilogue, sink):
    """Launches the load-only kernel with the decode kernel's access pattern over buf (uint8, n_tiles * 18432 bytes);
    sink: float32 device tensor of at least 16 + 512 * n_workgroups elements.  Time it with events around the call."""
    assert buf.is_cuda and buf.numel() * buf.element_size() >= n_tiles * 18432
    assert sink.dtype == torch.float32 and sink.numel() >= 16 + 512 * n_workgroups
    _check(lib().hs_probe_stream_read(_ptr(buf), int(n_tiles), int(n_workgroups), int(bool(with_epilogue)), _ptr(sink),
                                      _stream()))


def unpack_kv(shape, kv):
    K = torch.empty((shape.B, shape.Hkv, shape.L, shape.D), dtype=torch_dtype(shape), device=kv.k_map.device)
    V = torch.empty_like(K)
    kvs = kv.struct()
    _check(lib().hs_unpack_kv(C.byref(shape), C.byref(kvs), _ptr(K), _ptr(V), _stream()))
    return K, V


def prefill_attn(shape, Q, kv, causal=True, scale=0.0, want_lse=True, out=None, lse=None, q_start=None):
    """Q: bf16 [B, Hq, Lq, D] contiguous.  Returns (O bf16 [B, Hq, Lq, D], LSE fp32 [B, Hq, Lq] or None).
    q_start: position in the cache of the first query (default: the queries are the last Lq tokens)."""
    assert Q.dtype == torch_dtype(shape) and Q.is_contiguous() and Q.is_cuda
    Lq = Q.shape[2]
    O = torch.empty_like(Q) if out is None else out
    if lse is None and want_lse:
        lse = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    kvs = kv.struct()
    if q_start is None:
        _check(lib().hs_prefill_attn(C.byref(shape), Lq, float(scale), int(bool(causal)), _ptr(Q), C.byref(kvs), _ptr(O),
                                     _ptr(lse), None, _stream()))
    else:
        _check(lib().hs_prefill_attn_at(C.byref(shape), Lq, int(q_start), float(scale), int(bool(causal)), _ptr(Q),
                                        C.byref(kvs), _ptr(O), _ptr(lse), None, _stream()))
    return O, lse


def decode_attn(shape, Q, kv, scale=0.0, n_splits=0, want_lse=True, out=None, lse=None, workspace=None, phases=3,
                tail_k=None, tail_v=None, tail_len=None):
    """Q: bf16 [B, Hq, D] contiguous.  Returns (O bf16 [B, Hq, D], LSE fp32 [B, Hq] or None).
    phases: 3 = whole call; 1 = split-KV kernel only, 2 = merge kernel only (benchmarking).
    tail_k, tail_v (bf16 [B, Hkv, 64, D]) with tail_len: dense tail of not yet compressed tokens."""
    assert Q.dtype == torch_dtype(shape) and Q.is_contiguous() and Q.is_cuda
    O = torch.empty_like(Q) if out is None else out
    if lse is None and want_lse:
        lse = torch.empty(Q.shape[:2], dtype=torch.float32, device=Q.device)
    kvs = kv.struct()
    if tail_len is not None:
        assert phases == 3
        n = n_splits if n_splits else decode_auto_splits(shape)
        if workspace is None:
            workspace = _workspace(workspace_bytes(shape, 2, n + 1), Q.device)
        for t in (tail_k, tail_v):
            assert t is None or (t.dtype == Q.dtype and t.is_contiguous() and tuple(t.shape) == (shape.B, shape.Hkv, 64, shape.D))
        if torch.is_tensor(tail_len):    # one length per batch row (int32 device tensor [B])
            assert tail_len.dtype == torch.int32 and tail_len.is_cuda and tail_len.numel() == shape.B and tail_len.is_contiguous()
            _check(lib().hs_decode_attn_tail_rows(C.byref(shape), float(scale), int(n_splits), _ptr(Q), C.byref(kvs),
                                                  _ptr(tail_k), _ptr(tail_v), _ptr(tail_len), _ptr(O), _ptr(lse),
                                                  _ptr(workspace), _stream()))
            return O, lse
        _check(lib().hs_decode_attn_tail(C.byref(shape), float(scale), int(n_splits), _ptr(Q), C.byref(kvs), _ptr(tail_k),
                                         _ptr(tail_v), int(tail_len), _ptr(O), _ptr(lse), _ptr(workspace), _stream()))
        return O, lse
    if workspace is None:
        workspace = _workspace(workspace_bytes(shape, 2, n_splits), Q.device)
    if phases == 3:
        _check(lib().hs_decode_attn(C.byref(shape), float(scale), int(n_splits), _ptr(Q), C.byref(kvs), _ptr(O),
                                    _ptr(lse), _ptr(workspace), _stream()))
    else:
        _check(lib().hs_decode_attn_phases(C.byref(shape), float(scale), int(n_splits), _ptr(Q), C.byref(kvs), _ptr(O),
                                           _ptr(lse), _ptr(workspace), _stream(), int(phases)))
    return O, lse


STATIC_SCRATCH_BYTES = 4 << 20


def decode_attn_static(shape, Q, kv, scale=0.0, n_splits=0, out=None, lse=None):
    """hs_decode_attn_static: decode attention whose split partials live in the library's static device
    array.  out (bf16 [B, Hq, D]) and lse (fp32 [B, Hq] or None) are the caller's: nothing is allocated."""
    assert Q.dtype == torch_dtype(shape) and Q.is_contiguous() and Q.is_cuda and out is not None
    kvs = kv.struct()
    _check(lib().hs_decode_attn_static(C.byref(shape), float(scale), int(n_splits), _ptr(Q), C.byref(kvs), _ptr(out),
                                       _ptr(lse), _stream()))
    return out, lse


def bits_to_bf16_tensor(bits, device="cuda", dtype=torch.bfloat16):
    """numpy uint16 bit patterns -> torch bf16 (or fp16) tensor on the device (same bits)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(dtype)


def bf16_tensor_to_bits(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
