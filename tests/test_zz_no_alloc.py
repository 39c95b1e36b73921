"""The entry point that allocates nothing (hs_decode_attn_static: split partials in the library's
static device array) against hs_decode_attn with a caller-supplied workspace, through the C ABI:
two calls in a row, the second on a smaller input, so that what the first call left in the array
is seen not to leak into the second; both also against the oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import hs_oracle as orc
from paper_2604_16864_amd import binding as hb
from paper_2604_16864_amd import workloads as wl

pytestmark = pytest.mark.gpu

MAX_TOL, MEAN_TOL = 1e-2, 2e-3


def _dev(bits):
    return hb.bits_to_bf16_tensor(bits, "cuda")


def _case(B, Hq, Hkv, L, seed, n_splits, **pol):
    Q, K, V = wl.make_qkv(B, Hq, Hkv, L, 128, 1, seed=seed, k_outliers=True)
    q = Q[:, :, 0, :].copy()
    sh = hb.make_shape(B, Hq, Hkv, L)
    kv = hb.compress_kv(sh, hb.make_policy(**pol), _dev(K), _dev(V))
    qd = _dev(q)
    O_ref, LSE_ref = hb.decode_attn(sh, qd, kv, n_splits=n_splits)          # existing entry point, own workspace
    torch.cuda.synchronize()
    O = torch.full_like(O_ref, float("nan"))
    LSE = torch.full_like(LSE_ref, float("nan"))
    before = torch.cuda.memory_allocated()
    print(f"[no-alloc] B{B} Hq{Hq} Hkv{Hkv} L{L} splits {n_splits} {sorted(pol)}", flush=True)
    hb.decode_attn_static(sh, qd, kv, n_splits=n_splits, out=O, lse=LSE)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    # same kernels, same split count: the two entry points agree bit for bit
    assert torch.equal(O.view(torch.int16), O_ref.view(torch.int16))
    assert torch.equal(LSE, LSE_ref)
    pk, pv, _ = orc.compress_kv(K, V, Bt=64, **pol)
    Or, Lr = orc.attention_decode(q, pk, pv)
    got = O.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - Or)
    assert err.max() <= MAX_TOL * np.abs(Or).max() and err.mean() <= MEAN_TOL * np.abs(Or).mean()
    assert np.allclose(LSE.cpu().numpy(), Lr, rtol=1e-4, atol=1e-4)


def test_static_scratch_decode_two_calls_second_smaller():
    _case(2, 16, 4, 64 * 40, seed=400, n_splits=0, skip_frac=0.25)           # 2 x 16 heads, auto splits
    _case(1, 8, 2, 64 * 9, seed=401, n_splits=3)                             # smaller: fewer heads, fewer splits
    _case(1, 4, 1, 64 * 2, seed=402, n_splits=1, sparse_frac_k=0.0)          # smaller again, one split, dense keys


def test_static_scratch_rejects_what_does_not_fit():
    sh = hb.make_shape(8, 32, 8, 131072)
    c = [0, 0, 4, 0, 4]
    kv = hb.HsKV()
    # 8 * 32 heads * 65535 splits * 516 B is far beyond the 4 MiB array: refused before anything is looked at
    assert hb.lib().hs_decode_attn_static(C.byref(sh), 0.0, 65535, None, C.byref(kv), None, None, None) == -4
    assert b"static" in hb.lib().hs_strerror(-4)
    need = hb.workspace_bytes(sh, 2, 0)
    assert need <= hb.STATIC_SCRATCH_BYTES                                    # the benchmark's largest decode shape fits
