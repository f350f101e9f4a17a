"""Pins for the oracle of the index lists' consumer (Section 3, step 4: attention over
TopK(t) U Window(t), keys = values = the compressed cache rows): what the definition and
the mathematics fix, none of it the oracle's own output.  CPU only."""
import numpy as np
import pytest

import workloads as W

NINF = -np.inf


def _case(rng, B, S, H, D, T, k, integer=False):
    if integer:
        qa = rng.integers(-2, 3, size=(B, S, H, D)).astype(np.float32)
        K = rng.integers(-2, 3, size=(B, T, D)).astype(np.float32)
    else:
        qa = rng.standard_normal((B, S, H, D)).astype(np.float32)
        K = rng.standard_normal((B, T, D)).astype(np.float32)
    return W.float_to_bf16_bits(qa), W.float_to_bf16_bits(K)


def _random_lists(rng, B, S, T, k, m, mask_mode):
    """Index lists with pads, in random order, entries legal for their query."""
    idx = np.full((B, S, k), -1, dtype=np.int32)
    for b in range(B):
        for t in range(S):
            L = T if mask_mode == 0 else min(T, (t + 1) // m)
            n = int(rng.integers(0, min(k, L) + 1))
            pick = rng.choice(L, size=n, replace=False) if n else np.zeros(0, dtype=np.int64)
            slots = rng.permutation(k)[:n]
            idx[b, t, slots] = pick
    return idx


def _brute(qab, Kb, idx, m, mask_mode, n_win, scale):
    """Dense masked softmax attention with numpy: membership mask [B,S,T] from the lists and the
    window, logits for all (t, s), -inf outside the mask, softmax, P @ K."""
    qa, K = W.bits_to_float(qab), W.bits_to_float(Kb)
    B, S, H, D = qa.shape
    T = K.shape[1]
    member = np.zeros((B, S, T), dtype=bool)
    for b in range(B):
        for t in range(S):
            L = T if mask_mode == 0 else min(T, (t + 1) // m)
            for s in idx[b, t]:
                if s >= 0:
                    member[b, t, s] = True
            member[b, t, max(0, L - n_win):L] = True
    logits = scale * np.einsum("bshd,btd->bsht", qa, K)
    logits = np.where(member[:, :, None, :], logits, NINF)
    top = logits.max(axis=3, keepdims=True)
    top = np.where(np.isfinite(top), top, 0.0)
    e = np.exp(logits - top)
    den = e.sum(axis=3, keepdims=True)
    p = np.divide(e, den, out=np.zeros_like(e), where=den > 0)
    return np.einsum("bsht,btd->bshd", p, K), member


def _all_rows(oracle, qab, Kb, idx, m, mask_mode, n_win, scale, n_threads=1):
    B, S, H, D = qab.shape
    k = idx.shape[2]
    b = np.repeat(np.arange(B, dtype=np.int32), S)
    t = np.tile(np.arange(S, dtype=np.int64), B)
    out = oracle.sparse_attention_rows(qab.reshape(B * S, H, D), Kb, idx.reshape(B * S, k), b, t, m,
                                       mask_mode, n_win, scale, n_threads)
    return out.reshape(B, S, H, D)


@pytest.mark.parametrize("mask_mode", [0, 1])
@pytest.mark.parametrize("n_win", [0, 1, 5, 64])
def test_dense_masked_attention_brute_force(oracle, mask_mode, n_win):
    rng = np.random.default_rng(31 + n_win)
    B, S, H, D, m, k = 2, 30, 3, 8, 2, 6
    T = S // m
    qab, Kb = _case(rng, B, S, H, D, T, k)
    idx = _random_lists(rng, B, S, T, k, m, mask_mode)
    ref, member = _brute(qab, Kb, idx, m, mask_mode, n_win, 0.37)
    got = _all_rows(oracle, qab, Kb, idx, m, mask_mode, n_win, 0.37)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-13)
    # rows from a shuffled list of (batch, position) pairs: the batch offset of K and of the lists
    n = 40
    b_of = rng.integers(0, B, size=n).astype(np.int32)
    t_of = rng.integers(0, S, size=n).astype(np.int64)
    part = oracle.sparse_attention_rows(qab[b_of, t_of], Kb, idx[b_of, t_of], b_of, t_of, m, mask_mode, n_win, 0.37)
    assert np.allclose(part, ref[b_of, t_of], rtol=1e-12, atol=1e-13)
    if mask_mode == 1 and n_win == 0:  # some sets are empty: exact zeros
        empty = ~member.any(axis=2)
        assert empty.any() and np.all(got[empty] == 0.0)


def test_weights_sum_to_one_constant_value_rows(oracle):
    # every key row equals v  =>  out = v whatever the logits are (they are all equal here, but the
    # next test varies them): the softmax weights sum to 1
    rng = np.random.default_rng(32)
    B, S, H, D, T, k = 1, 12, 2, 8, 12, 4
    qab, _ = _case(rng, B, S, H, D, T, k)
    v = rng.standard_normal(D).astype(np.float32)
    Kb = W.float_to_bf16_bits(np.tile(v, (B, T, 1)))
    idx = _random_lists(rng, B, S, T, k, 1, 1)
    got = _all_rows(oracle, qab, Kb, idx, 1, 1, 3, 1.0)
    vb = W.bits_to_float(W.float_to_bf16_bits(v))
    assert np.allclose(got, vb[None, None, None, :], rtol=1e-14, atol=1e-15)


def test_values_in_a_line_give_the_weighted_mean_position(oracle):
    # K[s] = a + s*u with integer-valued a, u: out = a + (sum_s p_s s) u, so every output component
    # lies on that line at the same parameter: pins that the SAME weights multiply every component
    B, S, H, D, T, k = 1, 6, 2, 8, 16, 5
    rng = np.random.default_rng(33)
    a = rng.integers(-3, 4, size=D).astype(np.float64)
    u = np.array([1, -1, 2, 0, 1, 1, -2, 1], dtype=np.float64)
    K = a[None, :] + np.arange(T)[:, None] * u[None, :]
    Kb = W.float_to_bf16_bits(K[None].astype(np.float32))
    assert np.array_equal(W.bits_to_float(Kb)[0], K)  # exactly representable
    qab, _ = _case(rng, B, S, H, D, T, k)
    idx = _random_lists(rng, B, S, T, k, 1, 0)
    idx[0, :, 0] = 3  # never empty
    got = _all_rows(oracle, qab, Kb, idx, 1, 0, 0, 0.05)
    lam = (got[..., 0] - a[0]) / u[0]
    for d in range(D):
        assert np.allclose(got[..., d], a[d] + lam * u[d], rtol=1e-12, atol=1e-12)
    assert np.all(lam >= 0) and np.all(lam <= T - 1)


def test_zero_queries_give_the_mean_of_the_selected_rows(oracle):
    rng = np.random.default_rng(34)
    B, S, H, D, m, k = 1, 20, 2, 8, 2, 5
    T = S // m
    _, Kb = _case(rng, B, S, H, D, T, k)
    qab = np.zeros((B, S, H, D), dtype=np.uint16)
    idx = _random_lists(rng, B, S, T, k, m, 1)
    got = _all_rows(oracle, qab, Kb, idx, m, 1, 2, 3.0)
    K = W.bits_to_float(Kb)[0]
    for t in range(S):
        L = min(T, (t + 1) // m)
        U = sorted(set(int(s) for s in idx[0, t] if s >= 0) | set(range(max(0, L - 2), L)))
        want = K[U].mean(axis=0) if U else np.zeros(D)
        assert np.allclose(got[0, t], want[None, :], rtol=1e-13, atol=1e-14)


def test_window_only_is_local_attention(oracle):
    # all pads: attention over the last n_win legal keys, written out separately here
    rng = np.random.default_rng(35)
    B, S, H, D, m, n_win = 1, 40, 2, 8, 4, 3
    T = S // m
    qab, Kb = _case(rng, B, S, H, D, T, 4)
    idx = np.full((B, S, 4), -1, dtype=np.int32)
    got = _all_rows(oracle, qab, Kb, idx, m, 1, n_win, 0.5)
    qa, K = W.bits_to_float(qab)[0], W.bits_to_float(Kb)[0]
    for t in range(S):
        L = (t + 1) // m
        lo = max(0, L - n_win)
        for h in range(H):
            if L == 0:
                assert np.all(got[0, t, h] == 0)
                continue
            z = 0.5 * (K[lo:L] @ qa[t, h])
            p = np.exp(z - z.max())
            p /= p.sum()
            assert np.allclose(got[0, t, h], p @ K[lo:L], rtol=1e-13, atol=1e-14)


def test_list_order_duplicates_and_overlap_with_the_window_do_not_matter(oracle):
    rng = np.random.default_rng(36)
    B, S, H, D, T, k, n_win = 1, 1, 3, 8, 50, 8, 6
    qab, Kb = _case(rng, B, S, H, D, T, k)
    b, t = np.zeros(1, dtype=np.int32), np.zeros(1, dtype=np.int64)
    base = np.array([[3, 17, 40, 9, -1, -1, 22, 5]], dtype=np.int32)
    ref = oracle.sparse_attention_rows(qab[0], Kb, base, b, t, 1, 0, n_win, 0.3)
    for variant in (base[:, ::-1], base[:, rng.permutation(k)],
                    np.array([[3, 17, 40, 9, 9, 3, 22, 5]], dtype=np.int32),        # repeats in the list
                    np.array([[3, 17, 40, 9, 47, 49, 22, 5]], dtype=np.int32)):    # 47, 49 are window keys too
        got = oracle.sparse_attention_rows(qab[0], Kb, np.ascontiguousarray(variant), b, t, 1, 0, n_win, 0.3)
        assert np.array_equal(got, ref)  # same set, visited in the same (ascending) order: same bits
    # a different set is a different result (the test above is not vacuous)
    other = oracle.sparse_attention_rows(qab[0], Kb, np.array([[3, 17, 41, 9, -1, -1, 22, 5]], dtype=np.int32),
                                         b, t, 1, 0, n_win, 0.3)
    assert not np.allclose(other, ref)


def test_huge_scale_selects_the_best_matching_row(oracle):
    rng = np.random.default_rng(37)
    B, S, H, D, T, k = 1, 10, 2, 8, 30, 6
    qab, Kb = _case(rng, B, S, H, D, T, k)
    idx = _random_lists(rng, B, S, T, k, 1, 0)
    idx[0, :, 0] = np.arange(S)  # never empty
    got = _all_rows(oracle, qab, Kb, idx, 1, 0, 0, 1e4)
    qa, K = W.bits_to_float(qab)[0], W.bits_to_float(Kb)[0]
    for t in range(S):
        U = sorted(set(int(s) for s in idx[0, t] if s >= 0))
        for h in range(H):
            best = U[int(np.argmax(K[U] @ qa[t, h]))]
            assert np.allclose(got[0, t, h], K[best], rtol=1e-9, atol=1e-9)


def test_logit_shift_invariance_and_scale(oracle):
    # softmax is invariant to adding a constant to all logits of a row: appending a component that
    # is 1 for every key and c in the query adds scale*c to every logit; the first D outputs stay
    rng = np.random.default_rng(38)
    B, S, H, D, T, k = 1, 5, 2, 8, 20, 4
    qa = rng.integers(-2, 3, size=(B, S, H, D)).astype(np.float32)
    K = rng.integers(-2, 3, size=(B, T, D)).astype(np.float32)
    idx = _random_lists(rng, B, S, T, k, 1, 0)
    idx[0, :, 0] = 1
    base = _all_rows(oracle, W.float_to_bf16_bits(qa), W.float_to_bf16_bits(K), idx, 1, 0, 2, 0.25)
    qa2 = np.concatenate([qa, np.full((B, S, H, 1), 7.0, dtype=np.float32)], axis=3)
    K2 = np.concatenate([K, np.ones((B, T, 1), dtype=np.float32)], axis=2)
    ext = _all_rows(oracle, W.float_to_bf16_bits(qa2), W.float_to_bf16_bits(K2), idx, 1, 0, 2, 0.25)
    assert np.allclose(ext[..., :D], base, rtol=1e-12, atol=1e-13)
    assert np.allclose(ext[..., D], 1.0, rtol=1e-14)  # the weights sum to 1
    # halving the scale and doubling the queries is the same logits (exact in binary)
    dbl = _all_rows(oracle, W.float_to_bf16_bits(qa * 2), W.float_to_bf16_bits(K), idx, 1, 0, 2, 0.125)
    assert np.array_equal(dbl, base)


def test_fan_out_and_bad_indices(oracle):
    rng = np.random.default_rng(39)
    B, S, H, D, m, k = 2, 17, 2, 8, 1, 5
    T = 9
    qab, Kb = _case(rng, B, S, H, D, T, k)
    idx = _random_lists(rng, B, S, T, k, m, 1)
    one = _all_rows(oracle, qab, Kb, idx, m, 1, 2, 0.2, n_threads=1)
    many = _all_rows(oracle, qab, Kb, idx, m, 1, 2, 0.2, n_threads=5)
    assert np.array_equal(one.view(np.int64), many.view(np.int64))
    bad = idx.copy()
    bad[0, 3, 0] = T
    with pytest.raises(ValueError):
        _all_rows(oracle, qab, Kb, bad, m, 1, 2, 0.2)
