"""CPU-only: the C-ABI library loads, exports what include/streamindex.h declares, and its
host-side logic (planning, sizes, argument checks before any launch) behaves."""
import ctypes
import os
import re

import pytest

import paper_2605_02568_amd as P
from paper_2605_02568_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GiB = 1 << 30


def test_library_exports_every_declared_symbol():
    hdr = "".join(open(os.path.join(ROOT, "include", f)).read()
                  for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(si_[a-z_]+)\s*\(", hdr))
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)
    lib = ctypes.CDLL(P.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert P.si_version() >= 100


def test_strerror_and_sizes():
    assert P.si_strerror(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert P.si_strerror(code) not in ("ok", "unknown status")
    # Section 1: 256 GB at S=65536 with H_I=64, T=S/4
    assert P.si_materialize_bytes(1, 65536, 64, 128, 16384) == 256 * GiB
    # workspace = per row (2k + c_T) u64 keys + a count + a threshold
    ws = P.si_workspace_bytes(1, 1 << 20, 64, 128, 1 << 18, 1024, 2048, 8192)
    expect = 2048 * (2 * 1024 + 8192) * 8 + 2 * 2048 * 4
    assert expect <= ws <= expect + 5 * 256
    assert P.si_workspace_bytes(1, 100, 4, 32, 25, 16, 4096, 4096) == \
        P.si_workspace_bytes(1, 100, 4, 32, 25, 16, 100, 25)  # clamped to the problem
    assert P.si_workspace_bytes(1, 100, 4, 32, 25, 0, 8, 8) == 0


def test_plan_respects_budget_and_shapes():
    dims = (1, 1 << 20, 64, 128, 1 << 18)
    # 1M context under 8 GB (headline configuration): large, balanced tiles
    c_S, c_T, ws = P.si_plan_tiles(*dims, 4, 1024, 1, 8 * 10**9)
    assert ws <= 8 * 10**9 and c_S % 8 == 0 and c_S >= c_T >= 16384
    assert ws == P.si_workspace_bytes(*dims, 1024, c_S, c_T)
    # the tile area never grows when the budget shrinks, and the plan always fits it
    prev = (c_S, c_T)
    for budget in (4 * 10**9, 10**9, 64 << 20, 8 << 20, 200 << 10):
        s_, t_, w_ = P.si_plan_tiles(*dims, 4, 1024, 1, budget)
        assert w_ <= budget and w_ == P.si_workspace_bytes(*dims, 1024, s_, t_)
        assert s_ * t_ <= prev[0] * prev[1] and s_ >= 8 and s_ % 8 == 0 and t_ >= 32
        prev = (s_, t_)
    with pytest.raises(P.StreamIndexError) as e:
        P.si_plan_tiles(*dims, 4, 1024, 1, 1024)
    assert e.value.status == P.SI_ERR_WORKSPACE_TOO_SMALL
    # small problems are clamped to their own size
    c_S, c_T, _ = P.si_plan_tiles(1, 1024, 4, 32, 256, 4, 16, 0, 1 << 30)
    assert (c_S, c_T) == (1024, 256)
    # batch entries share the budget
    s4, t4, w4 = P.si_plan_tiles(4, 65536, 64, 128, 16384, 4, 512, 1, 8 * 10**9)
    assert w4 <= 8 * 10**9 and s4 * 4 <= 32768 and t4 == 16384


@pytest.mark.parametrize("bad,status", [
    (dict(D=48), P.SI_ERR_UNSUPPORTED_SHAPE),
    (dict(H_I=65), P.SI_ERR_UNSUPPORTED_SHAPE),
    (dict(k=4097), P.SI_ERR_UNSUPPORTED_SHAPE),
    (dict(T=1 << 24, D=128), P.SI_ERR_UNSUPPORTED_SHAPE),  # one batch of keys must stay below 4 GiB
    (dict(k=0), P.SI_ERR_INVALID_ARG),
    (dict(m=0), P.SI_ERR_INVALID_ARG),
    (dict(S=0), P.SI_ERR_INVALID_ARG),
    (dict(mask=2), P.SI_ERR_INVALID_ARG),
])
def test_argument_errors_are_reported_before_any_launch(bad, status):
    a = dict(B=1, S=64, H_I=4, D=32, T=16, m=4, k=8, mask=1)
    a.update(bad)
    lib = P.load()
    dims = binding.si_dims(a["B"], a["S"], a["H_I"], a["D"], a["T"])
    plan = binding.si_plan()
    assert lib.si_plan_tiles(ctypes.byref(dims), a["m"], a["k"], a["mask"], 1 << 30,
                             ctypes.byref(plan)) == status
    # the compute entry point rejects the same arguments on the host (pointers are never used)
    fake = ctypes.c_void_p(256)
    rc = lib.si_indexer_topk(fake, fake, fake, ctypes.byref(dims), a["m"], a["k"], a["mask"],
                             fake, fake, fake, 1 << 30, None)
    assert rc == status


def test_null_pointers_and_small_workspace_rejected():
    lib = P.load()
    dims = binding.si_dims(1, 64, 4, 32, 16)
    fake = ctypes.c_void_p(256)
    assert lib.si_indexer_topk(None, fake, fake, ctypes.byref(dims), 4, 8, 1, fake, fake, fake,
                               1 << 30, None) == P.SI_ERR_INVALID_ARG
    assert lib.si_indexer_topk_tiled(fake, fake, fake, ctypes.byref(dims), 4, 8, 1, 64, 16, fake,
                                     fake, fake, 16, None) == P.SI_ERR_WORKSPACE_TOO_SMALL
    assert lib.si_indexer_topk_tiled(fake, fake, fake, ctypes.byref(dims), 4, 8, 1, 64, 16, fake,
                                     fake, ctypes.c_void_p(264), 1 << 30, None) == P.SI_ERR_INVALID_ARG
    assert lib.si_topk_from_scores(None, 4, 4, None, 2, 2, fake, fake, fake, 1 << 20, None) \
        == P.SI_ERR_INVALID_ARG
    assert lib.si_profile_read(None, None) == P.SI_ERR_INVALID_ARG


def test_single_pass_workspace_and_argument_checks():
    dims = (1, 1 << 20, 64, 128, 1 << 18)
    # 256 resident workgroups x 8 rows x (2k + 384) keys, plus one counter per launch
    ws = P.si_fused_workspace_bytes(*dims, 1024)
    expect = 256 * 8 * (2 * 1024 + 384) * 8
    assert expect <= ws <= expect + 2 * 256
    # independent of the problem size, growing with k only
    assert abs(P.si_fused_workspace_bytes(1, 4096, 64, 128, 1024, 1024) - ws) <= 256
    assert P.si_fused_workspace_bytes(*dims, 2048) > ws > P.si_fused_workspace_bytes(*dims, 64)
    assert P.si_fused_workspace_bytes(*dims, 2049) == 0 and P.si_fused_workspace_bytes(*dims, 0) == 0
    # more launches, more counters
    assert P.si_fused_workspace_bytes(*dims, 1024, 8) >= ws
    lib = P.load()
    d = binding.si_dims(1, 64, 4, 32, 16)
    fake = ctypes.c_void_p(256)
    call = lambda k, ws_bytes, q=fake, wsp=fake: lib.si_indexer_topk_fused(  # noqa: E731
        q, fake, fake, ctypes.byref(d), 4, k, 1, 0, fake, fake, wsp, ws_bytes, None)
    assert call(2049, 1 << 30) == P.SI_ERR_UNSUPPORTED_SHAPE
    assert call(8, 16) == P.SI_ERR_WORKSPACE_TOO_SMALL
    assert call(8, 1 << 30, q=None) == P.SI_ERR_INVALID_ARG
    assert call(8, 1 << 30, wsp=ctypes.c_void_p(264)) == P.SI_ERR_INVALID_ARG
    # si_indexer_topk falls back to the tiled plan when the single-pass workspace does not fit
    small = P.si_workspace_bytes(1, 64, 4, 32, 16, 8, 8, 16)
    assert small < P.si_fused_workspace_bytes(1, 64, 4, 32, 16, 8)
    assert lib.si_indexer_topk(None, fake, fake, ctypes.byref(d), 4, 8, 1, fake, fake, fake, small,
                               None) == P.SI_ERR_INVALID_ARG


def test_static_scratch_entry_point_rejects_on_the_host():
    """si_indexer_topk_static: what its static array cannot hold is refused before any GPU call."""
    lib = P.load()
    fake = ctypes.c_void_p(256)
    d = binding.si_dims(1, 64, 4, 32, 16)
    call = lambda dims, k, q=fake: lib.si_indexer_topk_static(  # noqa: E731
        q, fake, fake, ctypes.byref(dims), 4, k, 1, fake, fake, None)
    assert call(d, 1025) == P.SI_ERR_UNSUPPORTED_SHAPE
    assert call(d, 0) == P.SI_ERR_INVALID_ARG
    assert call(d, 8, q=None) == P.SI_ERR_INVALID_ARG
    assert call(binding.si_dims(1, 64, 4, 48, 16), 8) == P.SI_ERR_UNSUPPORTED_SHAPE
    too_long = binding.si_dims(1, 64 * 131072 + 1, 4, 32, 16)  # more launches than it has counters for
    assert call(too_long, 8) == P.SI_ERR_UNSUPPORTED_SHAPE


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_02568_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no cpu fallback", ""), (dirpath, f)


def test_wrong_output_shape_raises_before_the_library_is_called(monkeypatch):
    """Every whole-step wrapper checks the output shapes first: a too-small output must never
    reach a kernel.  Host tensors suffice, since the shape check comes before the device check."""
    import torch

    class Untouchable:
        def __getattr__(self, name):
            raise AssertionError(f"library entry {name} was reached with a mis-shaped output")

    monkeypatch.setattr(binding, "_lib", Untouchable())
    B, S, H, D, T, k = 1, 16, 4, 32, 8, 4
    q = torch.zeros((B, S, H, D), dtype=torch.bfloat16)
    K = torch.zeros((B, T, D), dtype=torch.bfloat16)
    w = torch.zeros((B, S, H))
    ws = torch.zeros(1 << 20, dtype=torch.uint8)
    good_i = torch.zeros((B, S, k), dtype=torch.int32)
    for bad_i, bad_s in [
        (torch.zeros((B, S, k - 1), dtype=torch.int32), torch.zeros((B, S, k - 1))),
        (good_i, torch.zeros((B, S - 1, k))),
        (torch.zeros((B * S, k), dtype=torch.int32), torch.zeros((B * S, k))),
    ]:
        with pytest.raises(ValueError):
            P.si_indexer_topk(q, K, w, 4, k, 1, bad_i, bad_s, ws)
        with pytest.raises(ValueError):
            P.si_indexer_topk_tiled(q, K, w, 4, k, 1, 8, 8, bad_i, bad_s, ws)
        with pytest.raises(ValueError):
            P.si_indexer_topk_fused(q, K, w, 4, k, 1, 0, bad_i, bad_s, ws)
