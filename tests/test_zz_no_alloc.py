"""GPU test of si_indexer_topk_static, the entry point that allocates nothing (its scratch is a
static array inside the library): through the C ABI, against si_indexer_topk_fused on the same
inputs, bit for bit, on two calls in a row, the second with a smaller input (the array still
holds the first call's candidates and counters), then a third at the largest k it accepts.
Collected last (file name), so that a failure here hides no other test."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_02568_amd as P
from paper_2605_02568_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _problem(seed, B, S, H, D, T):
    g = torch.Generator(device="cpu").manual_seed(seed)
    q = torch.randn((B, S, H, D), generator=g).to(torch.bfloat16).to(DEV)
    K = torch.randn((B, T, D), generator=g).to(torch.bfloat16).to(DEV)
    w = (torch.randn((B, S, H), generator=g) / np.sqrt(H)).to(DEV)
    return q, K, w


def _fused(q, K, w, m, k, mask):
    B, S, H, D = q.shape
    T = K.shape[1]
    oi = torch.full((B, S, k), -7, dtype=torch.int32, device=DEV)
    os_ = torch.full((B, S, k), 123.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(P.si_fused_workspace_bytes(B, S, H, D, T, k), dtype=torch.uint8, device=DEV)
    P.si_indexer_topk_fused(q, K, w, m, k, mask, 0, oi, os_, ws)
    torch.cuda.synchronize()
    return oi, os_


def _static_through_the_abi(q, K, w, m, k, mask):
    """Calls the C symbol directly with raw device pointers; the outputs exist before the call and
    nothing is allocated between the call and the synchronisation."""
    B, S, H, D = q.shape
    oi = torch.full((B, S, k), -7, dtype=torch.int32, device=DEV)
    os_ = torch.full((B, S, k), 123.0, dtype=torch.float32, device=DEV)
    dims = binding.si_dims(B, S, H, D, K.shape[1])
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = P.load().si_indexer_topk_static(
        ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(K.data_ptr()), ctypes.c_void_p(w.data_ptr()),
        ctypes.byref(dims), m, k, mask, ctypes.c_void_p(oi.data_ptr()), ctypes.c_void_p(os_.data_ptr()),
        ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == P.SI_OK, P.si_strerror(rc)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return oi, os_


def _same(a, b):
    return torch.equal(a[0], b[0]) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


def test_static_scratch_entry_point_matches_the_workspace_one():
    # first call: V4 head shape, rows that merge several times (2k candidates reached repeatedly)
    print("static: call 1 (S=1500, T=3000, k=512)", flush=True)
    q, K, w = _problem(41, 1, 1500, 64, 128, 3000)
    ref = _fused(q, K, w, 1, 512, P.SI_MASK_CAUSAL_BLOCK)
    got = _static_through_the_abi(q, K, w, 1, 512, P.SI_MASK_CAUSAL_BLOCK)
    assert _same(ref, got)
    # second call, smaller in every dimension, batch of 2, other head shape
    print("static: call 2 (B=2, S=203, T=50, k=16)", flush=True)
    q2, K2, w2 = _problem(42, 2, 203, 33, 64, 50)
    ref2 = _fused(q2, K2, w2, 4, 16, P.SI_MASK_CAUSAL_BLOCK)
    got2 = _static_through_the_abi(q2, K2, w2, 4, 16, P.SI_MASK_CAUSAL_BLOCK)
    assert _same(ref2, got2)
    assert int((got2[0] >= 0).sum()) > 0
    # third call: the largest k it accepts, no mask
    print("static: call 3 (S=300, T=5000, k=1024)", flush=True)
    q3, K3, w3 = _problem(43, 1, 300, 16, 32, 5000)
    ref3 = _fused(q3, K3, w3, 1, 1024, P.SI_MASK_NONE)
    got3 = _static_through_the_abi(q3, K3, w3, 1, 1024, P.SI_MASK_NONE)
    assert _same(ref3, got3)
    # and the first problem again: nothing of calls 2 and 3 leaks into it
    assert _same(ref, _static_through_the_abi(q, K, w, 1, 512, P.SI_MASK_CAUSAL_BLOCK))


def test_static_entry_point_rejects_what_its_array_cannot_hold():
    q, K, w = _problem(44, 1, 64, 4, 32, 4000)
    dims = binding.si_dims(1, 64, 4, 32, 4000)
    oi = torch.empty((1, 64, 1025), dtype=torch.int32, device=DEV)
    os_ = torch.empty((1, 64, 1025), dtype=torch.float32, device=DEV)
    args = lambda k: (ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(K.data_ptr()),  # noqa: E731
                      ctypes.c_void_p(w.data_ptr()), ctypes.byref(dims), 1, k, 0,
                      ctypes.c_void_p(oi.data_ptr()), ctypes.c_void_p(os_.data_ptr()), None)
    assert P.load().si_indexer_topk_static(*args(1025)) == P.SI_ERR_UNSUPPORTED_SHAPE
    assert P.load().si_indexer_topk_static(*args(0)) == P.SI_ERR_INVALID_ARG
    with pytest.raises(P.StreamIndexError):
        P.si_indexer_topk_static(q, K, w, 1, 1025, 0, oi, os_)
