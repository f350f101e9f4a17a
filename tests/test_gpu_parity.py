"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Run with `-m gpu` on an MI355X."""
import numpy as np
import pytest
import torch

import paper_2605_02568_amd as P
import workloads as W
from tests import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def _workspace(nbytes):
    return torch.empty(int(nbytes), dtype=torch.uint8, device=DEV)


def _run_tiled(q, K, w, wl_m, k, mask_mode, c_S, c_T):
    B, S, H, D = q.shape
    T = K.shape[1]
    out_idx = torch.full((B, S, k), -7, dtype=torch.int32, device=DEV)
    out_score = torch.full((B, S, k), 123.0, dtype=torch.float32, device=DEV)
    ws = _workspace(P.si_workspace_bytes(B, S, H, D, T, k, c_S, c_T))
    P.si_indexer_topk_tiled(q, K, w, wl_m, k, mask_mode, c_S, c_T, out_idx, out_score, ws)
    torch.cuda.synchronize()
    return out_idx, out_score


def _rand_problem(seed, B, S, H, D, T):
    g = torch.Generator(device="cpu").manual_seed(seed)
    q = torch.randn((B, S, H, D), generator=g).to(torch.bfloat16)
    K = torch.randn((B, T, D), generator=g).to(torch.bfloat16)
    w = torch.randn((B, S, H), generator=g) / np.sqrt(H)
    return q, K, w


# ------------------------------------------------------------------ step a1/a2: score tile
@pytest.mark.parametrize("B,S,H,D,T,s0,t0,c_S,c_T", [
    (1, 64, 4, 32, 48, 0, 0, 64, 48),       # tiny head shape, one tile
    (2, 37, 33, 64, 200, 5, 32, 19, 131),   # ragged everything, two head blocks, batch 2
    (1, 300, 64, 128, 700, 8, 128, 280, 512),  # V4 head shape, several key chunks + ragged tail
    (1, 16, 17, 128, 40, 3, 7, 9, 33),      # tile origin not aligned to anything
])
def test_score_tile_matches_oracle(oracle, B, S, H, D, T, s0, t0, c_S, c_T):
    _say(f"score_tile B={B} S={S} H={H} D={D} T={T} s0={s0} t0={t0} c_S={c_S} c_T={c_T}")
    q, K, w = _rand_problem(1, B, S, H, D, T)
    tile = torch.full((B, c_S, c_T), float("nan"), dtype=torch.float32, device=DEV)
    P.si_score_tile(q.to(DEV), K.to(DEV), w.to(DEV), 1, P.SI_MASK_NONE, s0, t0, c_S, c_T, tile)
    torch.cuda.synchronize()
    got = tile.cpu().numpy()
    qb, Kb, wn = W.bf16_bits(q), W.bf16_bits(K), w.numpy()
    rows = min(c_S, S - s0)
    width = min(c_T, T - t0)
    for b in range(B):
        for r in range(rows):
            ref = oracle.score_row(qb[b, s0 + r], Kb[b], wn[b, s0 + r])[t0:t0 + width]
            err = np.abs(got[b, r, :width] - ref)
            assert np.all(err <= parity.tol(ref)), (b, r, err.max())
            assert np.all(err <= 1e-4 * (np.abs(ref) + 1)), (b, r, err.max())  # fp32-level in practice
    # nothing outside the live part of the tile is written
    assert np.isnan(got[:, rows:, :]).all() and np.isnan(got[:, :, width:]).all()


def test_score_tile_causal_covers_every_legal_entry(oracle):
    B, S, H, D, m = 1, 96, 8, 32, 4
    T = S // m
    q, K, w = _rand_problem(2, B, S, H, D, T)
    tile = torch.full((B, S, T), float("nan"), dtype=torch.float32, device=DEV)
    P.si_score_tile(q.to(DEV), K.to(DEV), w.to(DEV), m, P.SI_MASK_CAUSAL_BLOCK, 0, 0, S, T, tile)
    torch.cuda.synchronize()
    got = tile.cpu().numpy()
    qb, Kb, wn = W.bf16_bits(q), W.bf16_bits(K), w.numpy()
    for t in range(S):
        L = (t + 1) // m
        ref = oracle.score_row(qb[0, t], Kb[0], wn[0, t], L)
        assert np.all(np.abs(got[0, t, :L] - ref) <= parity.tol(ref))


def test_score_does_not_depend_on_tile_position():
    """The same (query, key) pair must get the same bits wherever it falls in a tile."""
    B, S, H, D, T = 1, 40, 64, 128, 300
    q, K, w = _rand_problem(3, B, S, H, D, T)
    qd, Kd, wd = q.to(DEV), K.to(DEV), w.to(DEV)
    full = torch.zeros((B, S, T), dtype=torch.float32, device=DEV)
    P.si_score_tile(qd, Kd, wd, 1, P.SI_MASK_NONE, 0, 0, S, T, full)
    for (s0, t0, c_S, c_T) in [(1, 1, 17, 100), (7, 33, 33, 267), (13, 129, 8, 31)]:
        part = torch.zeros((B, c_S, c_T), dtype=torch.float32, device=DEV)
        P.si_score_tile(qd, Kd, wd, 1, P.SI_MASK_NONE, s0, t0, c_S, c_T, part)
        torch.cuda.synchronize()
        rows, width = min(c_S, S - s0), min(c_T, T - t0)
        a = full[0, s0:s0 + rows, t0:t0 + width].cpu().numpy().view(np.uint32)
        b = part[0, :rows, :width].cpu().numpy().view(np.uint32)
        assert np.array_equal(a, b), (s0, t0)


# ------------------------------------------------------------------ steps a3-a5: select, merge, write-out
def _score_cases():
    rng = np.random.default_rng(5)
    R, n = 24, 3000
    cases = {}
    cases["normal"] = rng.standard_normal((R, n)).astype(np.float32)
    cases["ties"] = (rng.integers(-3, 4, size=(R, n)) * 0.5).astype(np.float32)
    cases["ascending"] = np.tile(np.arange(n, dtype=np.float32), (R, 1))
    cases["descending"] = np.tile(-np.arange(n, dtype=np.float32), (R, 1))
    cases["all_equal"] = np.full((R, n), 2.5, dtype=np.float32)
    z = np.zeros((R, n), dtype=np.float32)
    z[:, ::2] = -0.0  # +0 and -0 tie: index order decides
    z[:, 5::7] = 1e-30
    cases["signed_zero"] = z
    big = rng.standard_normal((R, n)).astype(np.float32)
    big[:, ::3] *= 1e30
    big[:, 1::5] *= 1e-30
    cases["wide_range"] = big
    return cases


@pytest.mark.parametrize("name", ["normal", "ties", "ascending", "descending", "all_equal",
                                  "signed_zero", "wide_range"])
def test_topk_from_scores_is_bit_exact(oracle, name):
    sc = _score_cases()[name]
    R, n = sc.shape
    rng = np.random.default_rng(6)
    legal = rng.integers(0, n + 1, size=R).astype(np.int32)
    legal[:4] = [0, 1, n, n - 1]
    scd = torch.from_numpy(sc).to(DEV)
    for k, c_T in [(1, 64), (16, 7), (100, 256), (512, 300), (512, 3000), (1024, 1024), (4096, 1000)]:
        for lg in (None, legal):
            _say(f"topk_from_scores {name} k={k} c_T={c_T} legal={'yes' if lg is not None else 'no'}")
            out_idx = torch.full((R, k), -7, dtype=torch.int32, device=DEV)
            out_score = torch.full((R, k), 9.0, dtype=torch.float32, device=DEV)
            ws = _workspace(P.si_workspace_bytes(1, R, 1, 32, n, k, R, c_T))
            lgd = None if lg is None else torch.from_numpy(lg).to(DEV)
            P.si_topk_from_scores(scd, lgd, k, c_T, out_idx, out_score, ws)
            torch.cuda.synchronize()
            gi, gs = out_idx.cpu().numpy(), out_score.cpu().numpy()
            for r in range(R):
                L = n if lg is None else int(lg[r])
                ri, rs = oracle.sort_topk(sc[r, :L].astype(np.float64), k)
                assert np.array_equal(gi[r], ri), (name, k, c_T, r, L)
                ke = min(k, L)
                # scores come back bit for bit, except that -0 may be returned as +0
                assert np.array_equal(gs[r, :ke] + 0.0, rs[:ke].astype(np.float32) + 0.0)
                assert np.all(np.isneginf(gs[r, ke:]))


# ------------------------------------------------------------------ whole path
def _check_all_rows(oracle, wl, q, K, w, out_idx, out_score):
    B, S, H, D = q.shape
    qb = W.bf16_bits(q).reshape(B * S, H, D)
    Kb = W.bf16_bits(K)
    wn = w.cpu().numpy().reshape(B * S, H)
    b = np.repeat(np.arange(B, dtype=np.int32), S)
    t = np.tile(np.arange(S, dtype=np.int64), B)
    return parity.check_rows(oracle, qb, wn, Kb, b, t, wl.m, wl.k, wl.mask_mode,
                             out_idx.cpu().numpy().reshape(B * S, wl.k),
                             out_score.cpu().numpy().reshape(B * S, wl.k))


def test_tiny_config_all_rows_and_planted_keys(oracle):
    wl = W.CONFIGS["tiny"]
    q, K, w, info = W.make_inputs(wl)
    qd, Kd, wd = q.to(DEV), K.to(DEV), w.to(DEV)
    ref = None
    for c_S, c_T in [(1024, 256), (64, 32), (100, 7), (8, 256), (333, 100)]:
        _say(f"tiny c_S={c_S} c_T={c_T}")
        oi, os_ = _run_tiled(qd, Kd, wd, wl.m, wl.k, wl.mask_mode, c_S, c_T)
        if ref is None:
            stats = _check_all_rows(oracle, wl, q, K, w, oi, os_)
            _say(f"tiny stats {stats}")
            assert stats["min_recall"] == 1.0
            t = info["t_star"]
            assert set(oi[0, t, :wl.planted].cpu().tolist()) == set(info["planted_keys"])
            ref = (oi, os_)
        else:  # bit-identical across tilings
            assert torch.equal(oi, ref[0]) and torch.equal(os_.view(torch.int32), ref[1].view(torch.int32))


def test_flash_4k_all_rows(oracle):
    wl = W.CONFIGS["flash_4k"]
    q, K, w, _ = W.make_inputs(wl)
    qd, Kd, wd = q.to(DEV), K.to(DEV), w.to(DEV)
    ref = None
    for c_S, c_T in [(4096, 1024), (512, 256), (1000, 333), (2048, 512)]:  # 256 < k: saturated tiles
        _say(f"flash_4k c_S={c_S} c_T={c_T}")
        oi, os_ = _run_tiled(qd, Kd, wd, wl.m, wl.k, wl.mask_mode, c_S, c_T)
        if ref is None:
            stats = _check_all_rows(oracle, wl, q, K, w, oi, os_)
            _say(f"flash_4k stats {stats}")
            assert stats["mean_recall"] > 0.9999
            ref = (oi, os_)
        else:
            assert torch.equal(oi, ref[0]) and torch.equal(os_.view(torch.int32), ref[1].view(torch.int32))
    # the planned entry point gives the same bits
    out_idx = torch.empty_like(ref[0])
    out_score = torch.empty_like(ref[1])
    ws = _workspace(64 << 20)
    P.si_indexer_topk(qd, Kd, wd, wl.m, wl.k, wl.mask_mode, out_idx, out_score, ws)
    torch.cuda.synchronize()
    assert torch.equal(out_idx, ref[0]) and torch.equal(out_score.view(torch.int32), ref[1].view(torch.int32))


@pytest.mark.parametrize("B,S,H,D,m,k,mask", [
    (2, 203, 4, 32, 4, 16, 1),     # batch 2, ragged S
    (3, 64, 33, 64, 1, 70, 0),     # k > T: pads without a mask
    (1, 129, 64, 128, 3, 5, 1),    # m does not divide S
    (1, 50, 1, 32, 4, 4096, 1),    # largest k, single head
])
def test_odd_shapes_all_rows(oracle, B, S, H, D, m, k, mask):
    T = max(1, S // m)
    q, K, w = _rand_problem(7, B, S, H, D, T)
    wl = W.Workload("odd", B, S, H, D, m, k, mask)
    ref = None
    for c_S, c_T in [(S, T), (13, 11), (8, 1)]:
        _say(f"odd B={B} S={S} H={H} D={D} m={m} k={k} c_S={c_S} c_T={c_T}")
        oi, os_ = _run_tiled(q.to(DEV), K.to(DEV), w.to(DEV), m, k, mask, c_S, c_T)
        if ref is None:
            B_, S_, H_, D_ = q.shape
            stats = parity.check_rows(
                oracle, W.bf16_bits(q).reshape(B * S, H, D), w.numpy().reshape(B * S, H),
                W.bf16_bits(K), np.repeat(np.arange(B, dtype=np.int32), S),
                np.tile(np.arange(S, dtype=np.int64), B), m, k, mask,
                oi.cpu().numpy().reshape(B * S, k), os_.cpu().numpy().reshape(B * S, k))
            assert stats["min_recall"] == 1.0, stats
            ref = (oi, os_)
        else:
            assert torch.equal(oi, ref[0]) and torch.equal(os_.view(torch.int32), ref[1].view(torch.int32))


def _random_shapes(n, seed):
    """Seeded shapes that mix every supported head dimension, ragged sizes, T != S/m, k above
    and below the number of legal keys, and tilings that cut rows and key chunks anywhere."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        B = int(rng.integers(1, 4))
        S = int(rng.integers(1, 260))
        H = int(rng.choice([1, 3, 8, 31, 32, 33, 48, 64]))
        D = int(rng.choice([32, 64, 128]))
        m = int(rng.choice([1, 2, 4, 7]))
        mask = int(rng.integers(0, 2))
        T = int(rng.integers(1, 600))           # explicit T: not tied to S/m
        k = int(rng.choice([1, 2, 7, 32, 100, 257, 1024]))
        c_S = int(rng.integers(1, S + 8))
        c_T = int(rng.integers(1, T + 40))
        cases.append((B, S, H, D, T, m, k, mask, c_S, c_T))
    return cases


@pytest.mark.parametrize("B,S,H,D,T,m,k,mask,c_S,c_T", _random_shapes(16, 20260513))
def test_random_shapes_all_rows(oracle, B, S, H, D, T, m, k, mask, c_S, c_T):
    q, K, w = _rand_problem(B * 1000 + S, B, S, H, D, T)
    _say(f"random B={B} S={S} H={H} D={D} T={T} m={m} k={k} mask={mask} c_S={c_S} c_T={c_T}")
    oi, os_ = _run_tiled(q.to(DEV), K.to(DEV), w.to(DEV), m, k, mask, c_S, c_T)
    stats = parity.check_rows(
        oracle, W.bf16_bits(q).reshape(B * S, H, D), w.numpy().reshape(B * S, H),
        W.bf16_bits(K), np.repeat(np.arange(B, dtype=np.int32), S),
        np.tile(np.arange(S, dtype=np.int64), B), m, k, mask,
        oi.cpu().numpy().reshape(B * S, k), os_.cpu().numpy().reshape(B * S, k))
    assert stats["min_recall"] == 1.0, stats
    # the planned tiling (whatever fits a small budget) must give the same bits
    ws = _workspace(P.si_workspace_bytes(B, S, H, D, T, k, S, T))
    oi2 = torch.empty_like(oi)
    os2 = torch.empty_like(os_)
    P.si_indexer_topk(q.to(DEV), K.to(DEV), w.to(DEV), m, k, mask, oi2, os2, ws)
    torch.cuda.synchronize()
    assert torch.equal(oi, oi2) and torch.equal(os_.view(torch.int32), os2.view(torch.int32))


def test_duplicate_keys_and_zero_weights_tie_break(oracle):
    B, S, H, D, m, k = 1, 64, 8, 32, 1, 12
    T = 64
    q, K, w = _rand_problem(8, B, S, H, D, T)
    K[0, 40] = K[0, 9]
    K[0, 41] = K[0, 9]
    w[0, 5] = 0.0  # row 5: every score is 0 -> keys 0..k-1
    oi, os_ = _run_tiled(q.to(DEV), K.to(DEV), w.to(DEV), m, k, 0, 16, 16)
    ri, rs = oracle.topk_all(W.bf16_bits(q), W.bf16_bits(K), w.numpy(), m, k, 0)
    assert oi[0, 5].cpu().tolist() == list(range(k))
    assert torch.all(os_[0, 5] == 0)
    got = oi.cpu().numpy()
    for t in range(S):
        row = list(got[0, t])
        present = [s for s in (9, 40, 41) if s in row]
        assert present == sorted(present) and present == [9, 40, 41][:len(present)]
    assert np.array_equal(got, ri)  # this small case has no near-ties besides the planted exact ones


# ------------------------------------------------------------------ the paper's other sweeps, at V4 head shape
@pytest.mark.parametrize("B,S,m,k,mask", [
    (1, 2048, 4, 64, 1),      # k sweep of Section 6.5 (Table 5): 64 ... 2048
    (1, 2048, 4, 256, 1),
    (1, 4096, 2, 2048, 1),    # k = 2048 needs T >= 2048 to fill a row
    (2, 1536, 4, 128, 1),     # batch 2
    (1, 1024, 4, 512, 0),     # no mask: every query sees all T keys, k > T pads
])
def test_v4_head_shape_sweeps(oracle, B, S, m, k, mask):
    H, D = 64, 128
    T = S // m
    q, K, w = _rand_problem(9, B, S, H, D, T)
    qd, Kd, wd = q.to(DEV), K.to(DEV), w.to(DEV)
    ref = None
    for c_S, c_T in [(S, T), (520, 192)]:
        _say(f"v4 sweep B={B} S={S} m={m} k={k} mask={mask} c_S={c_S} c_T={c_T}")
        oi, os_ = _run_tiled(qd, Kd, wd, m, k, mask, c_S, c_T)
        if ref is None:
            rows = np.arange(0, B * S, 3)  # every third row keeps the CPU time small
            stats = parity.check_rows(
                oracle, W.bf16_bits(q).reshape(B * S, H, D)[rows], w.numpy().reshape(B * S, H)[rows],
                W.bf16_bits(K), (rows // S).astype(np.int32), (rows % S).astype(np.int64), m, k, mask,
                oi.cpu().numpy().reshape(B * S, k)[rows], os_.cpu().numpy().reshape(B * S, k)[rows])
            _say(f"  {stats}")
            assert stats["mean_recall"] > 0.9999 and stats["min_recall"] >= 1.0 - 2.0 / k
            ref = (oi, os_)
        else:
            assert torch.equal(oi, ref[0]) and torch.equal(os_.view(torch.int32), ref[1].view(torch.int32))


def _pattern_problem(dist, seed, B, S, H, D, T):
    """dist 0: iid normal; 1: scores that rise with the key index for every query (nothing can be
    filtered); 2: small integers (many exact ties: the index half of the order decides)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    q = torch.randn((B, S, H, D), generator=g)
    K = torch.randn((B, T, D), generator=g)
    w = torch.randn((B, S, H), generator=g) / np.sqrt(H)
    if dist == 1:
        K = K.abs() * torch.linspace(0.5, 4.0, T)[None, :, None]
        q, w = q.abs(), w.abs()
    elif dist == 2:
        K = torch.randint(-1, 2, (B, T, D), generator=g).float()
        q = torch.randint(-1, 2, (B, S, H, D), generator=g).float()
        w = torch.ones((B, S, H))
    return q.to(torch.bfloat16), K.to(torch.bfloat16), w


@pytest.mark.parametrize("k", [2049, 3000, 4096])
@pytest.mark.parametrize("dist", [0, 1, 2])
def test_k_above_2048_with_more_than_k_legal_keys(oracle, k, dist):
    """The upper end of the advertised k range (the k sweep of Section 6.5 continued): every row
    has far more than k legal keys, so the radix cut at k, the streamed (not register-held) rows
    of the compaction and the write-out's largest sort all decide the result.  All rows against
    the oracle, two tilings and the planned entry point bit-identical."""
    B, S, H, D, T, m = 1, 48, 8, 32, 12000, 1
    q, K, w = _pattern_problem(dist, 77 + k, B, S, H, D, T)
    qd, Kd, wd = q.to(DEV), K.to(DEV), w.to(DEV)
    _say(f"large k={k} dist={dist}")
    a = _run_tiled(qd, Kd, wd, m, k, 0, S, T)
    stats = parity.check_rows(
        oracle, W.bf16_bits(q).reshape(B * S, H, D), w.numpy().reshape(B * S, H), W.bf16_bits(K),
        np.zeros(S, dtype=np.int32), np.arange(S, dtype=np.int64), m, k, 0,
        a[0].cpu().numpy().reshape(S, k), a[1].cpu().numpy().reshape(S, k))
    _say(f"  {stats}")
    assert stats["min_recall"] >= 1.0 - 2.0 / k, stats
    if dist == 2:  # exactly representable scores: sets, order and ties must be the oracle's
        ri, rs = oracle.topk_all(W.bf16_bits(q), W.bf16_bits(K), w.numpy(), m, k, 0, n_threads=parity.host_threads())
        assert np.array_equal(a[0].cpu().numpy(), ri)
        assert np.array_equal(a[1].cpu().numpy(), rs.astype(np.float32))
    b = _run_tiled(qd, Kd, wd, m, k, 0, 16, 1500)   # key tiles narrower than k: saturated tiles
    assert torch.equal(a[0], b[0]) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))
    oi, os_ = torch.empty_like(a[0]), torch.empty_like(a[1])
    P.si_indexer_topk(qd, Kd, wd, m, k, 0, oi, os_, _workspace(256 << 20))
    torch.cuda.synchronize()
    assert torch.equal(a[0], oi) and torch.equal(a[1].view(torch.int32), os_.view(torch.int32))


def test_adversarial_score_order_through_the_whole_path(oracle):
    """Keys sorted so that every later key scores higher for every query: nothing can be filtered,
    every tile floods the row buffers, compaction runs on its streaming path."""
    B, S, H, D, m, k = 1, 256, 1, 32, 1, 64
    T = 6000
    g = torch.Generator(device="cpu").manual_seed(10)
    base = torch.randn((D,), generator=g).abs() + 0.1
    q = (base[None, None, None, :] * (1.0 + torch.rand((B, S, H, D), generator=g))).to(torch.bfloat16)
    scale = torch.linspace(0.5, 4.0, T)
    K = (base[None, None, :] * scale[None, :, None]).to(torch.bfloat16)
    w = torch.ones((B, S, H))
    ref = None
    for c_S, c_T in [(S, T), (S, 4096), (64, 1000)]:
        _say(f"adversarial c_S={c_S} c_T={c_T}")
        oi, os_ = _run_tiled(q.to(DEV), K.to(DEV), w.to(DEV), m, k, 0, c_S, c_T)
        if ref is None:
            stats = parity.check_rows(
                oracle, W.bf16_bits(q).reshape(S, H, D), w.numpy().reshape(S, H), W.bf16_bits(K),
                np.zeros(S, dtype=np.int32), np.arange(S, dtype=np.int64), m, k, 0,
                oi.cpu().numpy().reshape(S, k), os_.cpu().numpy().reshape(S, k))
            assert stats["mean_recall"] > 0.999, stats
            ref = (oi, os_)
        else:
            assert torch.equal(oi, ref[0]) and torch.equal(os_.view(torch.int32), ref[1].view(torch.int32))


def test_profile_counters_follow_the_launches():
    """Per-kernel timing facility: one score launch and one compaction per key tile, one init and
    one finalize per query tile; durations are positive; disabled means nothing is recorded."""
    B, S, H, D, m, k = 1, 512, 64, 128, 1, 32
    T = 4096
    q, K, w = _rand_problem(11, B, S, H, D, T)
    qd, Kd, wd = q.to(DEV), K.to(DEV), w.to(DEV)
    P.si_profile_reset()
    P.si_profile_enable(True)
    _run_tiled(qd, Kd, wd, m, k, 0, 256, 2048)  # 2 query tiles; key tiles 1024, 1024, 2048
    prof = P.si_profile_read()
    P.si_profile_enable(False)
    assert prof["score_tile"][1] == 2 * 3 and prof["compact"][1] == 2 * 3
    assert prof["init"][1] == 2 and prof["finalize"][1] == 2 and prof["filter_scores"][1] == 0
    assert all(ms > 0 for name, (ms, n) in prof.items() if n > 0)
    P.si_profile_reset()
    _run_tiled(qd, Kd, wd, m, k, 0, 256, 2048)
    assert all(n == 0 for _, n in P.si_profile_read().values())
