"""Pins for the CPU oracle: things the paper and the mathematics fix, none of which
is the oracle's own output.  CPU only."""
import os

import numpy as np
import pytest

import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
NINF = -np.inf


def _read_hand_case():
    d = {}
    with open(os.path.join(GOLDEN, "hand_case.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, *vals = line.split()
                d[key] = np.array([float(v) for v in vals])
    return d


def _read_figures():
    d = {}
    with open(os.path.join(GOLDEN, "paper_figures.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, val = line.split()
                d[key] = float(val)
    return d


def _rand_case(rng, S, H, D, m, integer=False):
    T = S // m
    if integer:
        q = rng.integers(-3, 4, size=(1, S, H, D)).astype(np.float32)
        K = rng.integers(-3, 4, size=(1, T, D)).astype(np.float32)
        w = rng.integers(-2, 3, size=(1, S, H)).astype(np.float32) * 0.5
    else:
        q = rng.standard_normal((1, S, H, D)).astype(np.float32)
        K = rng.standard_normal((1, T, D)).astype(np.float32)
        w = (rng.standard_normal((1, S, H)) / np.sqrt(H)).astype(np.float32)
    return W.float_to_bf16_bits(q), W.float_to_bf16_bits(K), w


def _brute(qb, Kb, w, m, k, mask_mode):
    """Materialize-then-sort with numpy (Section 3, the two-line einsum form)."""
    q = W.bits_to_float(qb)
    K = W.bits_to_float(Kb)
    B, S, H, D = q.shape
    T = K.shape[1]
    full = np.einsum("bshd,btd->bsht", q, K)
    score = (np.maximum(full, 0.0) * w.astype(np.float64)[..., None]).sum(axis=2)  # [B,S,T]
    idx = np.full((B, S, k), -1, dtype=np.int32)
    sc = np.full((B, S, k), NINF)
    for b in range(B):
        for t in range(S):
            L = T if mask_mode == 0 else min(T, (t + 1) // m)
            order = np.lexsort((np.arange(L), -score[b, t, :L]))  # score desc, then index asc
            keep = min(k, L)
            idx[b, t, :keep] = order[:keep]
            sc[b, t, :keep] = score[b, t, order[:keep]]
    return idx, sc, score


# ----------------------------------------------------------------------------- hand case
def test_hand_worked_scores_and_order(oracle):
    g = _read_hand_case()
    H, D = int(g["H"][0]), int(g["D"][0])
    q = W.float_to_bf16_bits(g["q"].reshape(H, D))
    K = W.float_to_bf16_bits(g["K"].reshape(-1, D))
    w = g["w"].astype(np.float32)
    sc = oracle.score_row(q, K, w)
    assert np.array_equal(sc, g["scores"])
    n = len(g["scores"])
    idx, s = oracle.sort_topk(sc, n)
    assert np.array_equal(idx, g["order"].astype(np.int32))
    # k smaller than the tie group: lower indices survive
    idx2, _ = oracle.sort_topk(sc, 2)
    assert list(idx2) == [0, 4]
    # end to end through the row driver, no mask, k larger than T -> pads
    oi, os_ = oracle.topk_rows(q[None], w[None], K[None], [0], [0], m=1, k=8, mask_mode=0)
    assert list(oi[0]) == [0, 4, 5, 2, 3, 1, -1, -1]
    assert np.array_equal(os_[0][:6], [1.5, 1.5, 1.5, 0.0, -2.0, -6.0])
    assert np.all(os_[0][6:] == NINF)


# ----------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("mask_mode", [0, 1])
@pytest.mark.parametrize("integer", [False, True])
def test_brute_force_small(oracle, mask_mode, integer):
    rng = np.random.default_rng(11 + mask_mode)
    qb, Kb, w = _rand_case(rng, S=96, H=3, D=8, m=3, integer=integer)
    k = 7
    bi, bs, _ = _brute(qb, Kb, w, 3, k, mask_mode)
    oi, os_ = oracle.topk_all(qb, Kb, w, 3, k, mask_mode)
    if integer:  # exact arithmetic, heavy ties: must agree to the bit
        assert np.array_equal(oi, bi)
        assert np.array_equal(os_, bs)
    else:
        assert np.array_equal(oi, bi)
        assert np.allclose(os_, bs, rtol=1e-13, atol=1e-13)


def test_brute_force_tiny_config(oracle):
    wl = W.CONFIGS["tiny"]
    q, K, w, info = W.make_inputs(wl)
    qb, Kb = W.bf16_bits(q), W.bf16_bits(K)
    bi, bs, _ = _brute(qb, Kb, w.numpy(), wl.m, wl.k, wl.mask_mode)
    oi, os_ = oracle.topk_all(qb, Kb, w.numpy(), wl.m, wl.k, wl.mask_mode)
    assert np.array_equal(oi, bi)
    assert np.allclose(os_, bs, rtol=1e-13, atol=1e-13)


# ----------------------------------------------------------------------------- batch offset, row fan-out, score_at
def _rand_case_batched(rng, B, S, H, D, T, integer=False):
    if integer:
        q = rng.integers(-3, 4, size=(B, S, H, D)).astype(np.float32)
        K = rng.integers(-3, 4, size=(B, T, D)).astype(np.float32)
        w = rng.integers(-2, 3, size=(B, S, H)).astype(np.float32) * 0.5
    else:
        q = rng.standard_normal((B, S, H, D)).astype(np.float32)
        K = rng.standard_normal((B, T, D)).astype(np.float32)
        w = (rng.standard_normal((B, S, H)) / np.sqrt(H)).astype(np.float32)
    return W.float_to_bf16_bits(q), W.float_to_bf16_bits(K), w


@pytest.mark.parametrize("mask_mode", [0, 1])
@pytest.mark.parametrize("integer", [False, True])
def test_brute_force_three_batches_rows_in_mixed_order(oracle, mask_mode, integer):
    """Rows from every batch, listed in a shuffled order with repeated positions: each row must
    be scored against its own batch's keys (a dropped or transposed batch offset picks another
    batch's K, whose values differ)."""
    rng = np.random.default_rng(21 + mask_mode)
    B, S, H, D, m, k = 3, 40, 3, 8, 2, 6
    T = S // m
    qb, Kb, w = _rand_case_batched(rng, B, S, H, D, T, integer=integer)
    bi, bs, _ = _brute(qb, Kb, w, m, k, mask_mode)
    # whole problem through the all-rows driver
    oi, os_ = oracle.topk_all(qb, Kb, w, m, k, mask_mode)
    assert np.array_equal(oi, bi)
    assert np.array_equal(os_, bs) if integer else np.allclose(os_, bs, rtol=1e-13, atol=1e-13)
    # a shuffled list of (batch, position) pairs, some twice
    n = 70
    b_of = rng.integers(0, B, size=n).astype(np.int32)
    t_of = rng.integers(0, S, size=n).astype(np.int64)
    assert set(b_of) == {0, 1, 2}
    ri, rs = oracle.topk_rows(qb[b_of, t_of], w[b_of, t_of], Kb, b_of, t_of, m, k, mask_mode)
    assert np.array_equal(ri, bi[b_of, t_of])
    assert np.array_equal(rs, bs[b_of, t_of]) if integer else np.allclose(rs, bs[b_of, t_of], rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("n_threads", [2, 5, 16])
def test_row_fan_out_over_threads_changes_nothing(oracle, n_threads):
    """n_threads > 1 must return, bit for bit, what one thread returns, and that must be the
    brute-force result: more threads than rows, a row count that does not divide, ties."""
    rng = np.random.default_rng(23)
    B, S, H, D, m, k = 2, 37, 4, 16, 3, 5
    T = 12
    for integer in (False, True):
        qb, Kb, w = _rand_case_batched(rng, B, S, H, D, T, integer=integer)
        bi, bs, _ = _brute(qb, Kb, w, m, k, 1)
        for n in (1, 3, B * S):
            sel = rng.permutation(B * S)[:n]
            b_of = (sel // S).astype(np.int32)
            t_of = (sel % S).astype(np.int64)
            one = oracle.topk_rows(qb[b_of, t_of], w[b_of, t_of], Kb, b_of, t_of, m, k, 1, n_threads=1)
            many = oracle.topk_rows(qb[b_of, t_of], w[b_of, t_of], Kb, b_of, t_of, m, k, 1,
                                    n_threads=n_threads)
            assert np.array_equal(one[0], many[0])
            assert np.array_equal(one[1].view(np.int64), many[1].view(np.int64))
            assert np.array_equal(many[0], bi[b_of, t_of])
            if integer:
                assert np.array_equal(many[1], bs[b_of, t_of])


def test_score_at_listed_keys(oracle):
    """Scores at a shuffled list of key indices (with repeats): equal to the materialized
    einsum row at those indices, and a negative index gives NaN in exactly that place."""
    rng = np.random.default_rng(24)
    S, H, D, T = 5, 6, 16, 90
    for integer in (False, True):
        qb, Kb, w = _rand_case_batched(rng, 1, S, H, D, T, integer=integer)
        _, _, full = _brute(qb, Kb, w, 1, 1, 0)  # [1, S, T] fp64 scores
        for t in range(S):
            idx = rng.integers(0, T, size=40).astype(np.int32)
            idx[[3, 17, 39]] = -1
            idx[5] = idx[6] = T - 1
            idx[7] = 0
            got = oracle.score_at(qb[0, t], Kb[0], w[0, t], idx)
            hole = idx < 0
            assert np.array_equal(np.isnan(got), hole)
            ref = full[0, t, idx[~hole]]
            if integer:
                assert np.array_equal(got[~hole], ref)
            else:
                assert np.allclose(got[~hole], ref, rtol=1e-13, atol=1e-13)
            # and bit-equal to the whole-row routine at the same places
            assert np.array_equal(got[~hole], oracle.score_row(qb[0, t], Kb[0], w[0, t])[idx[~hole]])
        assert oracle.score_at(qb[0, 0], Kb[0], w[0, 0], np.zeros(0, dtype=np.int32)).size == 0


# ----------------------------------------------------------------------------- planted keys
def test_planted_keys_are_the_top(oracle):
    wl = W.CONFIGS["tiny"]
    q, K, w, info = W.make_inputs(wl)
    oi, os_ = oracle.topk_all(W.bf16_bits(q), W.bf16_bits(K), w.numpy(), wl.m, wl.k, wl.mask_mode)
    t = info["t_star"]
    assert set(oi[0, t, :wl.planted]) == set(info["planted_keys"])
    margin = os_[0, t, wl.planted - 1] / os_[0, t, wl.planted]
    assert margin > 2.0, margin
    # the own-head term alone: 3 * w * |q_j|^2 with w = 0.5 is a lower bound (other heads add >= 0)
    qf = W.bits_to_float(W.bf16_bits(q))[0, t]
    for j, s in enumerate(info["planted_keys"]):
        pos = list(oi[0, t]).index(s)
        Kf = W.bits_to_float(W.bf16_bits(K))[0, s]
        assert os_[0, t, pos] >= 0.5 * float(qf[j] @ Kf) - 1e-9
        assert float(qf[j] @ Kf) > 2.5 * float(qf[j] @ qf[j])  # K row is ~3 q_j after rounding


# ----------------------------------------------------------------------------- tie order
def test_zero_weights_give_index_order(oracle):
    rng = np.random.default_rng(3)
    qb, Kb, w = _rand_case(rng, S=64, H=4, D=16, m=2)
    w[:] = 0.0
    oi, os_ = oracle.topk_all(qb, Kb, w, 2, 5, 1)
    for t in range(64):
        keep = min(5, (t + 1) // 2)
        assert list(oi[0, t, :keep]) == list(range(keep))
        assert np.all(os_[0, t, :keep] == 0.0)
        assert np.all(oi[0, t, keep:] == -1) and np.all(os_[0, t, keep:] == NINF)


def test_all_dots_negative_give_index_order(oracle):
    # K = -c * (a positive vector), q positive  => every dot < 0 => ReLU kills every term
    rng = np.random.default_rng(4)
    q = np.abs(rng.standard_normal((1, 8, 3, 16))).astype(np.float32) + 0.1
    K = -np.abs(rng.standard_normal((1, 8, 16))).astype(np.float32) - 0.1
    w = rng.standard_normal((1, 8, 3)).astype(np.float32)
    oi, os_ = oracle.topk_all(W.float_to_bf16_bits(q), W.float_to_bf16_bits(K), w, 1, 4, 0)
    assert np.all(oi == np.arange(4)[None, None]) and np.all(os_ == 0.0)


def test_duplicate_keys_lower_index_first(oracle):
    rng = np.random.default_rng(5)
    qb, Kb, w = _rand_case(rng, S=32, H=4, D=16, m=1)
    Kb[0, 20] = Kb[0, 3]  # key 20 is a copy of key 3
    oi, os_ = oracle.topk_all(qb, Kb, w, 1, 32, 0)
    for t in range(32):
        row = list(oi[0, t])
        a, b = row.index(3), row.index(20)
        assert a < b  # lower index first
        assert np.all(os_[0, t, a:b + 1] == os_[0, t, a])  # only equal scores in between ...
        assert row[a:b + 1] == sorted(row[a:b + 1])  # ... and those in index order
    # k cuts between the two copies: only the lower index survives
    for t in range(32):
        pos = list(oi[0, t]).index(3)
        oi2, _ = oracle.topk_all(qb[:, t:t + 1], Kb, w[:, t:t + 1], 1, pos + 1, 0)
        assert oi2[0, 0, -1] == 3 and 20 not in oi2[0, 0]


# ----------------------------------------------------------------------------- pads / legal count
def test_pad_structure_and_closed_form_count(oracle):
    rng = np.random.default_rng(6)
    S, m, k = 200, 4, 9
    qb, Kb, w = _rand_case(rng, S=S, H=2, D=8, m=m)
    oi, os_ = oracle.topk_all(qb, Kb, w, m, k, 1)
    T = S // m
    total = 0
    for t in range(S):
        L = min(T, (t + 1) // m)  # Section 4.2
        keep = min(k, L)
        total += keep
        assert np.all(oi[0, t, :keep] >= 0) and np.all(oi[0, t, :keep] < L)
        assert len(set(oi[0, t, :keep])) == keep
        assert np.all(oi[0, t, keep:] == -1) and np.all(os_[0, t, keep:] == NINF)
        assert np.all(np.diff(os_[0, t, :keep]) <= 0)
    assert np.all(oi[0, :m - 1] == -1)  # rows with no complete block in their past
    # closed form of sum_t min(k, floor((t+1)/m)): the first k*m-1 rows ramp up m at a time
    ramp = m * (k - 1) * k // 2 + k  # rows t = m-1 .. k*m-1 inclusive: m rows per level 1..k-1, then 1
    closed = ramp + (S - k * m) * k
    assert int((oi >= 0).sum()) == total == closed


def test_legal_count_matches_both_forms_of_the_mask(oracle):
    # Section 4.2: floor((t+1)/m); Section 5 / config text: key s visible iff (s+1)*m <= t+1
    for m in (1, 2, 3, 4, 7):
        for T in (1, 5, 64):
            for t in range(0, 300):
                L = oracle.legal_count(t, T, m, 1)
                vis = sum(1 for s in range(T) if (s + 1) * m <= t + 1)
                assert L == vis == min(T, (t + 1) // m)
                assert oracle.legal_count(t, T, m, 0) == T


def test_k_at_least_legal_returns_everything_sorted(oracle):
    rng = np.random.default_rng(7)
    qb, Kb, w = _rand_case(rng, S=40, H=2, D=8, m=2)
    oi, os_ = oracle.topk_all(qb, Kb, w, 2, 64, 1)
    for t in range(40):
        L = (t + 1) // 2
        assert sorted(oi[0, t, :L]) == list(range(L)) and np.all(oi[0, t, L:] == -1)


# ----------------------------------------------------------------------------- identities
def test_relu_identity_against_matvec(oracle):
    # ReLU(x) - ReLU(-x) = x  =>  I(q,K,w) - I(q,-K,w) = (sum_h w_h q_h) . K
    rng = np.random.default_rng(8)
    qb, Kb, w = _rand_case(rng, S=4, H=8, D=32, m=1)
    Kneg = Kb ^ np.uint16(0x8000)
    q = W.bits_to_float(qb)[0]
    K = W.bits_to_float(Kb)[0]
    for t in range(4):
        a = oracle.score_row(qb[0, t], Kb[0], w[0, t])
        b = oracle.score_row(qb[0, t], Kneg[0], w[0, t])
        lin = (w[0, t].astype(np.float64)[:, None] * q[t]).sum(axis=0) @ K.T
        assert np.allclose(a - b, lin, rtol=1e-12, atol=1e-12)
        # and the sum is sum_h w_h |x_h|
        absum = (np.abs(q[t] @ K.T) * w[0, t].astype(np.float64)[:, None]).sum(axis=0)
        assert np.allclose(a + b, absum, rtol=1e-12, atol=1e-12)


def test_power_of_two_scaling_is_exact(oracle):
    rng = np.random.default_rng(9)
    qb, Kb, w = _rand_case(rng, S=8, H=4, D=16, m=1)
    base_i, base_s = oracle.topk_all(qb, Kb, w, 1, 6, 0)
    i2, s2 = oracle.topk_all(qb, Kb, w * np.float32(4.0), 1, 6, 0)
    assert np.array_equal(i2, base_i) and np.array_equal(s2, base_s * 4.0)
    K8 = W.float_to_bf16_bits(W.bits_to_float(Kb) * 0.125)
    i3, s3 = oracle.topk_all(qb, K8, w, 1, 6, 0)
    assert np.array_equal(i3, base_i) and np.array_equal(s3, base_s * 0.125)


def test_single_head_nonnegative_reduces_to_matmul_and_sort(oracle):
    rng = np.random.default_rng(10)
    q = np.abs(rng.standard_normal((1, 16, 1, 32))).astype(np.float32)
    K = np.abs(rng.standard_normal((1, 50, 32))).astype(np.float32)
    w = np.ones((1, 16, 1), dtype=np.float32)
    qb, Kb = W.float_to_bf16_bits(q), W.float_to_bf16_bits(K)
    oi, os_ = oracle.topk_all(qb, Kb, w, 1, 10, 0)
    P = W.bits_to_float(qb)[0, :, 0] @ W.bits_to_float(Kb)[0].T  # [16, 50]
    for t in range(16):
        order = np.argsort(-P[t], kind="stable")[:10]
        assert np.array_equal(oi[0, t], order)
        assert np.allclose(os_[0, t], P[t, order], rtol=1e-13)


def test_head_and_weight_pairing(oracle):
    # one-hot weights pick out single heads: catches a w/head mismatch or a transposed operand
    rng = np.random.default_rng(12)
    qb, Kb, w = _rand_case(rng, S=1, H=5, D=8, m=1)
    q = W.bits_to_float(qb)[0, 0]
    K = W.bits_to_float(Kb)[0]
    for h in range(5):
        wh = np.zeros(5, dtype=np.float32)
        wh[h] = -1.5
        sc = oracle.score_row(qb[0, 0], Kb[0], wh)
        assert np.allclose(sc, -1.5 * np.maximum(K @ q[h], 0.0), rtol=1e-13, atol=1e-13)


def test_key_permutation_invariance(oracle):
    rng = np.random.default_rng(13)
    qb, Kb, w = _rand_case(rng, S=12, H=4, D=16, m=1)
    T = Kb.shape[1]
    perm = rng.permutation(T)
    Kp = Kb[:, perm]  # new key j is old key perm[j]
    i0, s0 = oracle.topk_all(qb, Kb, w, 1, 5, 0)
    i1, s1 = oracle.topk_all(qb, Kp, w, 1, 5, 0)
    assert np.array_equal(perm[i1], i0)  # tie-free with continuous inputs
    assert np.array_equal(s1, s0)


# ----------------------------------------------------------------------------- Algorithms 1 and 2
def _tie_heavy_scores(rng, n):
    return rng.integers(-4, 5, size=n).astype(np.float64) * 0.25


@pytest.mark.parametrize("ties", [False, True])
def test_algorithm1_any_order_equals_full_sort(oracle, ties):
    rng = np.random.default_rng(14)
    for L, k in [(0, 3), (1, 3), (5, 5), (50, 7), (333, 64), (64, 100)]:
        sc = _tie_heavy_scores(rng, L) if ties else rng.standard_normal(L)
        ref_i, ref_s = oracle.sort_topk(sc, k)
        for perm in (np.arange(L), np.arange(L)[::-1].copy(), rng.permutation(L), rng.permutation(L)):
            i, s = oracle.stream_topk(sc, perm, k)
            assert np.array_equal(i, ref_i) and np.array_equal(s, ref_s)


@pytest.mark.parametrize("ties", [False, True])
def test_algorithm2_chunked_equals_full_sort(oracle, ties):
    rng = np.random.default_rng(15)
    T = 700
    for legal in (0, 1, 13, 256, 511, 700):
        sc = _tie_heavy_scores(rng, T) if ties else rng.standard_normal(T)
        for k in (1, 16, 100):
            ref_i, ref_s = oracle.sort_topk(sc[:legal], k)
            for c_T in (1, 7, 64, 99, 256, 700, 4096):  # includes c_T < k (saturated tiles)
                i, s = oracle.chunked_topk_row(sc, legal, k, c_T, 0)
                assert np.array_equal(i, ref_i), (legal, k, c_T)
                assert np.array_equal(s, ref_s)


def _recall(i, ref_i):
    valid = ref_i[ref_i >= 0]
    if valid.size == 0:
        return None
    return len(set(i[i >= 0]) & set(valid)) / valid.size


def test_ablation_mutants_match_table6(oracle):
    """Table 6: recall is a rank statistic, so iid continuous scores reproduce it.
    A1 (later tiles never merged) at S=16384, T=4096, k=512, c_T=1024;
    A2 (tiles narrower than k skipped) at c_T=256; A2 control = production at c_T=256."""
    fig = _read_figures()
    rng = np.random.default_rng(16)
    S, T, m, k = 16384, 4096, 4, 512
    rows = np.arange(3, S, 16)  # every 16th row keeps the CPU time small
    rec_a1, rec_a2 = [], []
    for t in rows:
        L = min(T, (t + 1) // m)
        if L == 0:
            continue
        sc = rng.standard_normal(T)
        ref_i, _ = oracle.sort_topk(sc[:L], k)
        a1, _ = oracle.chunked_topk_row(sc, L, k, 1024, 1)
        rec_a1.append(_recall(a1, ref_i))
        if t % 64 == 3:
            a2, _ = oracle.chunked_topk_row(sc, L, k, 256, 2)
            rec_a2.append(_recall(a2, ref_i))
            ctrl, _ = oracle.chunked_topk_row(sc, L, k, 256, 0)
            assert np.array_equal(ctrl, ref_i)  # A2 control: exact
    rec_a1 = np.array(rec_a1)
    assert abs(rec_a1.mean() - fig["A1_mean_recall"]) < 0.01, rec_a1.mean()
    assert abs(100.0 * (rec_a1 == 1.0).mean() - fig["A1_pct_perfect"]) < 0.5
    assert abs(rec_a1.min() - fig["A1_min_recall"]) < 0.04, rec_a1.min()
    assert np.mean(rec_a2) <= fig["A2_mean_recall"] + 1e-12  # everything skipped


# ----------------------------------------------------------------------------- footprints
def test_footprint_figures(oracle):
    fig = _read_figures()
    GiB = 1 << 30
    assert oracle.materialize_bytes(1, 65536, 64, 16384) == fig["materialize_S65536_GiB"] * GiB
    assert oracle.materialize_bytes(1, 131072, 64, 32768) == fig["materialize_S131072_GiB"] * GiB
    assert oracle.materialize_bytes(1, 262144, 64, 65536) == fig["materialize_S262144_GiB"] * GiB
    assert oracle.materialize_bytes(1, 32768, 64, 8192) == fig["materialize_S32768_GiB"] * GiB
    assert oracle.materialize_bytes(1, 32768, 1, 8192) == fig["headsum_S32768_GiB"] * GiB
    assert oracle.mask_bytes(1, 131072, 32768) == fig["mask_S131072_GiB"] * GiB
    assert oracle.mask_bytes(1, 1048576, 262144) == fig["mask_S1048576_GiB"] * GiB


def test_workload_table_matches_closed_forms():
    # legal pairs of the causal block mask: m*T*(T-1)/2 + T when S = m*T
    for name in ("flash_4k", "flash_64k"):
        wl = W.CONFIGS[name]
        T = wl.T
        assert wl.legal_pairs() == wl.m * T * (T - 1) // 2 + T
    assert W.CONFIGS["tiny"].legal_pairs() == 1024 * 256
    assert W.CONFIGS["flash_4k"].flop_per_pair() == 16384


def test_workload_pair_accounting_agrees_with_the_oracle_mask(oracle):
    # the FLOP accounting of the benchmark counts legal pairs; it must count what the oracle masks
    for wl in (W.CONFIGS["tiny"], W.CONFIGS["flash_4k"],
               W.Workload("odd", B=2, S=103, H=4, D=32, m=3, k=5, mask_mode=W.MASK_CAUSAL_BLOCK)):
        per_row = [oracle.legal_count(t, wl.T, wl.m, wl.mask_mode) for t in range(wl.S)]
        assert per_row == [wl.legal_count(t) for t in range(wl.S)]
        assert wl.legal_pairs() == wl.B * sum(per_row)
