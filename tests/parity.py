"""GPU-vs-oracle comparison rule for the indexer top-k (used by the gpu tests, smoke and
bench).  Scores: |gpu - ref| <= 2e-3 * (|ref| + 1).  Index sets: equal, except for swaps
whose oracle scores lie within that tolerance of the oracle's k-th score.  Pads exact."""
from __future__ import annotations

import os

import numpy as np

REL = 2e-3


def tol(x):
    return REL * (np.abs(x) + 1.0)


def host_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def check_rows(oracle, q_rows, w_rows, K_bits, b_of_row, t_of_row, m, k, mask_mode,
               gpu_idx, gpu_score, n_threads=None, oracle_out=None):
    """q_rows [n,H,D] uint16, w_rows [n,H] f32, K_bits [B,T,D] uint16, gpu_idx/gpu_score [n,k].
    Raises AssertionError on the first violated rule; returns a stats dict."""
    n_threads = n_threads or host_threads()
    n = q_rows.shape[0]
    T = K_bits.shape[1]
    if oracle_out is None:
        oracle_out = oracle.topk_rows(q_rows, w_rows, K_bits, b_of_row, t_of_row, m, k,
                                      mask_mode, n_threads=n_threads)
    ora_idx, ora_score = oracle_out
    recalls, swaps, max_err, exact_rows, checked_pairs = [], 0, 0.0, 0, 0
    for r in range(n):
        t = int(t_of_row[r])
        L = oracle.legal_count(t, T, m, mask_mode)  # Section 4.2, from the oracle itself
        checked_pairs += L
        ke = min(k, L)
        gi, gs = gpu_idx[r], gpu_score[r]
        where = f"row {r} (b={int(b_of_row[r])}, t={t}, legal={L})"
        # pads
        assert np.all(gi[ke:] == -1), f"{where}: pad idx"
        assert np.all(np.isneginf(gs[ke:])), f"{where}: pad score"
        assert np.all(ora_idx[r, ke:] == -1)
        if ke == 0:
            continue
        G = gi[:ke].astype(np.int64)
        assert G.min() >= 0 and G.max() < L, f"{where}: illegal key index"
        assert np.unique(G).size == ke, f"{where}: duplicate key index"
        # slots ordered by (score desc, idx asc) on the GPU's own scores
        d = np.diff(gs[:ke].astype(np.float64))
        assert np.all(d <= 0), f"{where}: scores not sorted"
        tie = d == 0
        assert np.all(np.diff(G)[tie] > 0), f"{where}: tie not broken towards the lower index"
        O = ora_idx[r, :ke].astype(np.int64)
        if np.array_equal(G, O):
            sig_G = ora_score[r, :ke]
            exact_rows += 1
            recalls.append(1.0)
        else:
            pos_in_O = {int(s): j for j, s in enumerate(O)}
            sig_G = np.empty(ke)
            missing = [j for j, s in enumerate(G) if int(s) not in pos_in_O]
            for j, s in enumerate(G):
                if int(s) in pos_in_O:
                    sig_G[j] = ora_score[r, pos_in_O[int(s)]]
            if missing:
                sig_G[missing] = oracle.score_at(q_rows[r], K_bits[int(b_of_row[r])], w_rows[r],
                                                 G[missing].astype(np.int32))
            theta = ora_score[r, ke - 1]
            gset = set(int(s) for s in G)
            for j in missing:  # in G, not in O: must be within tolerance of the boundary
                assert sig_G[j] >= theta - tol(theta), \
                    f"{where}: key {G[j]} score {sig_G[j]} too far below k-th score {theta}"
            for j, s in enumerate(O):
                if int(s) not in gset:
                    assert ora_score[r, j] <= theta + tol(theta), \
                        f"{where}: missed key {s} score {ora_score[r, j]} vs k-th {theta}"
            swaps += len(missing)
            if not missing:
                exact_rows += 1  # same set, order differs only among near-equal scores
            recalls.append(1.0 - len(missing) / ke)
        err = np.abs(gs[:ke].astype(np.float64) - sig_G)
        bad = err > tol(sig_G)
        assert not bad.any(), f"{where}: score error {err[bad].max()} at slot {np.argmax(bad)}"
        max_err = max(max_err, float((err / (np.abs(sig_G) + 1.0)).max()))
    return {
        "rows": n,
        "rows_with_keys": len(recalls),
        "mean_recall": float(np.mean(recalls)) if recalls else 1.0,
        "min_recall": float(np.min(recalls)) if recalls else 1.0,
        "rows_exact_set": exact_rows,
        "boundary_swaps": swaps,
        "max_scaled_err": max_err,
        "checked_pairs": checked_pairs,
    }
