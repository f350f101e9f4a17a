"""GPU parity of the index lists' consumer (si_sparse_attention: attention over TopK(t) U Window(t),
Section 3, step 4) against the CPU oracle, element by element, through the C ABI's binding."""
import os

import numpy as np
import pytest
import torch

import paper_2605_02568_amd as P
import workloads as W
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _problem(seed, B, S, H, D, T):
    g = torch.Generator(device="cpu").manual_seed(seed)
    qa = torch.randn((B, S, H, D), generator=g).to(torch.bfloat16)
    K = torch.randn((B, T, D), generator=g).to(torch.bfloat16)
    return qa, K


def _random_lists(rng, B, S, T, k, m, mask):
    """Distinct legal entries in random slots, pads elsewhere (what a caller may hand over)."""
    idx = np.full((B, S, k), -1, dtype=np.int32)
    for b in range(B):
        for t in range(S):
            L = T if mask == 0 else min(T, (t + 1) // m)
            n = int(rng.integers(0, min(k, L) + 1))
            if n:
                idx[b, t, rng.permutation(k)[:n]] = rng.choice(L, size=n, replace=False)
    return idx


def _check(oracle, qa, K, idx, m, mask, n_win, scale, rows=None):
    B, S, H, D = qa.shape
    k = idx.shape[2]
    out = torch.full((B, S, H, D), float("nan"), dtype=torch.float32, device=DEV)
    P.si_sparse_attention(qa.to(DEV), K.to(DEV), torch.from_numpy(idx).to(DEV), m, mask, n_win, scale, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(B * S, H, D)
    if rows is None:
        rows = np.arange(B * S)
    ref = oracle.sparse_attention_rows(
        W.bf16_bits(qa).reshape(B * S, H, D)[rows], W.bf16_bits(K), idx.reshape(B * S, k)[rows],
        (rows // S).astype(np.int32), (rows % S).astype(np.int64), m, mask, n_win, scale,
        n_threads=parity.host_threads())
    err = np.abs(got[rows] - ref)
    assert np.all(np.isfinite(got)), "non-finite output"
    assert np.all(err <= parity.tol(ref)), float(err.max())
    assert np.all(err <= 2e-4 * (np.abs(ref) + 1.0)), float(err.max())  # fp32-level in practice
    return float((err / (np.abs(ref) + 1.0)).max())


@pytest.mark.parametrize("B,S,H,D,T,m,k,mask,n_win", [
    (1, 64, 8, 64, 16, 4, 8, 1, 3),        # one wave per query, small everything
    (2, 45, 33, 128, 90, 1, 16, 1, 5),     # two waves per query, ragged heads, batch 2
    (1, 40, 64, 128, 300, 1, 100, 0, 0),   # no window, no mask, k not a multiple of anything
    (1, 30, 64, 128, 400, 2, 96, 1, 64),   # window longer than most rows' legal range
    (1, 24, 1, 64, 500, 1, 257, 0, 31),    # single head
    (3, 20, 32, 64, 77, 3, 7, 1, 1),       # m does not divide S, window of one
    (1, 16, 64, 128, 2000, 1, 1024, 0, 128),  # V4 head shape, k = 1024 + window
])
def test_random_lists_all_rows(oracle, B, S, H, D, T, m, k, mask, n_win):
    print(f"attention B={B} S={S} H={H} D={D} T={T} m={m} k={k} mask={mask} n_win={n_win}", flush=True)
    qa, K = _problem(17 + S, B, S, H, D, T)
    idx = _random_lists(np.random.default_rng(S), B, S, T, k, m, mask)
    worst = _check(oracle, qa, K, idx, m, mask, n_win, 1.0 / np.sqrt(D))
    print(f"  max scaled error {worst:.2e}", flush=True)


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        T = int(rng.integers(1, 700))
        cases.append(dict(
            B=int(rng.integers(1, 3)), S=int(rng.integers(1, 40)), H=int(rng.choice([1, 7, 32, 33, 64])),
            D=int(rng.choice([64, 128])), T=T, m=int(rng.choice([1, 2, 4, 16])),
            k=int(rng.choice([1, 5, 31, 32, 33, 64, 100, 257])), mask=int(rng.integers(0, 2)),
            n_win=int(rng.choice([0, 1, 31, 32, 33, 64, 200])),
            scale=float(rng.choice([0.09, -0.2, 1.5, 0.0, 1e-4])), seed=500 + i))
    return cases


# 16 seeded cases by default; SI_FUZZ_CASES=N runs the first N of the same seeded sequence
@pytest.mark.parametrize("c", _random_cases(int(os.environ.get("SI_FUZZ_CASES", "16")), 20260601),
                         ids=lambda c: f"S{c['S']}T{c['T']}H{c['H']}D{c['D']}k{c['k']}w{c['n_win']}s{c['seed']}")
def test_random_shapes_windows_and_scales(oracle, c):
    """Seeded shapes: set sizes on both sides of the 32-key tile and of the two-tile unrolling of
    the kernel's loop, every head split, both masks, scales of either sign and zero."""
    print("attention", c, flush=True)
    qa, K = _problem(c["seed"], c["B"], c["S"], c["H"], c["D"], c["T"])
    idx = _random_lists(np.random.default_rng(c["seed"]), c["B"], c["S"], c["T"], c["k"], c["m"], c["mask"])
    _check(oracle, qa, K, idx, c["m"], c["mask"], c["n_win"], c["scale"])


def test_lists_from_the_indexer(oracle):
    """The real producer: si_indexer_topk's lists (sorted by score, pads last) feed the consumer."""
    B, S, H, D, m, k, n_win = 1, 512, 64, 128, 4, 64, 16
    T = S // m
    g = torch.Generator(device="cpu").manual_seed(5)
    q = torch.randn((B, S, H, D), generator=g).to(torch.bfloat16)
    K = torch.randn((B, T, D), generator=g).to(torch.bfloat16)
    w = torch.randn((B, S, H), generator=g) / np.sqrt(H)
    qa = torch.randn((B, S, H, D), generator=g).to(torch.bfloat16)
    out_idx = torch.empty((B, S, k), dtype=torch.int32, device=DEV)
    out_score = torch.empty((B, S, k), dtype=torch.float32, device=DEV)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device=DEV)
    P.si_indexer_topk(q.to(DEV), K.to(DEV), w.to(DEV), m, k, 1, out_idx, out_score, ws)
    torch.cuda.synchronize()
    idx = out_idx.cpu().numpy()
    assert (idx[0, :m - 1] == -1).all() and (idx[0, -1] >= 0).all()
    _check(oracle, qa, K, idx, m, 1, n_win, 0.11)


def test_degenerate_rows_and_scales(oracle):
    B, S, H, D, m, k = 1, 48, 16, 64, 4, 8
    T = S // m
    qa, K = _problem(3, B, S, H, D, T)
    pads = np.full((B, S, k), -1, dtype=np.int32)
    # nothing selected, no window: every set is empty -> exact zeros
    out = torch.full((B, S, H, D), float("nan"), dtype=torch.float32, device=DEV)
    P.si_sparse_attention(qa.to(DEV), K.to(DEV), torch.from_numpy(pads).to(DEV), m, 1, 0, 1.0, out)
    torch.cuda.synchronize()
    assert torch.all(out == 0)
    # window only; rows t < m - 1 have no legal key and stay zero
    _check(oracle, qa, K, pads, m, 1, 4, 0.25)
    # a list that repeats what the window holds: counted once
    idx = pads.copy()
    for t in range(S):
        L = (t + 1) // m
        if L >= 2:
            idx[0, t, :2] = [L - 1, 0]
    _check(oracle, qa, K, idx, m, 1, 3, 0.25)
    # sharp and flat softmax, zero queries
    _check(oracle, qa, K, idx, m, 1, 3, 30.0)
    _check(oracle, qa, K, idx, m, 1, 3, 1e-6)
    _check(oracle, torch.zeros_like(qa), K, idx, m, 1, 3, 1.0)
    # negative scale (the kernel moves its sign into the query operand), zero scale (uniform weights
    # over a ragged last tile: the rows past the end must still weigh nothing), a vanishing one
    _check(oracle, qa, K, idx, m, 1, 3, -0.3)
    _check(oracle, qa, K, idx, m, 1, 3, 0.0)
    _check(oracle, qa, K, idx, m, 1, 3, -0.0)
    _check(oracle, qa, K, idx, m, 1, 3, 1e-30)
    # logits far apart between tiles: the reference maximum has to be raised late in the list
    T2 = 200
    qa2, K2 = _problem(4, 1, 4, 8, 64, T2)
    K2 = (K2.float() * torch.linspace(0.05, 3.0, T2)[None, :, None]).to(torch.bfloat16)
    idx2 = np.tile(np.arange(T2, dtype=np.int32), (1, 4, 1))
    _check(oracle, qa2, K2, idx2, 1, 0, 0, 2.0)
    _check(oracle, qa2, K2, np.ascontiguousarray(idx2[:, :, ::-1]), 1, 0, 0, 2.0)


def test_argument_errors():
    qa, K = _problem(1, 1, 8, 4, 64, 8)
    idx = torch.zeros((1, 8, 4), dtype=torch.int32, device=DEV)
    out = torch.empty((1, 8, 4, 64), dtype=torch.float32, device=DEV)
    with pytest.raises(P.StreamIndexError) as e:
        P.si_sparse_attention(qa.to(DEV), K.to(DEV), idx, 0, 1, 0, 1.0, out)
    assert e.value.status == P.SI_ERR_INVALID_ARG
    with pytest.raises(P.StreamIndexError) as e:
        P.si_sparse_attention(qa.to(DEV), K.to(DEV), idx, 1, 1, 0, float("inf"), out)
    assert e.value.status == P.SI_ERR_INVALID_ARG
    q32, K32 = _problem(1, 1, 8, 4, 32, 8)
    with pytest.raises(P.StreamIndexError) as e:
        P.si_sparse_attention(q32.to(DEV), K32.to(DEV), idx, 1, 1, 0, 1.0,
                              torch.empty((1, 8, 4, 32), dtype=torch.float32, device=DEV))
    assert e.value.status == P.SI_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(ValueError):
        P.si_sparse_attention(qa.to(DEV), K.to(DEV), idx, 1, 1, 0, 1.0, out[:, :4])
