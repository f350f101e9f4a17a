"""Seeded synthetic inputs for the indexer top-k path.

This module only draws random tensors and rounds them to the storage types of
the interface; it contains none of the method's arithmetic.  It is the one
piece that both the oracle-side tests and the HIP-side tests import, so that
the two paths see the same bits.

Configurations follow the evaluation shapes of the paper (Section 6: B=1,
H_I=64, d_h=128, m=4, causal block mask, k in {512, 1024}) with the value
distribution q, K ~ N(0,1) stored as bfloat16 and w ~ N(0, 1/H_I) (variance)
stored as float32.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch

MASK_NONE = 0
MASK_CAUSAL_BLOCK = 1

# separate random streams per tensor, all derived from the config seed
_STREAM_Q, _STREAM_K, _STREAM_W, _STREAM_ROWS = 1, 2, 3, 4


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    S: int
    H: int
    D: int
    m: int
    k: int
    mask_mode: int
    seed: int = 0
    planted: int = 0  # number of planted keys (tiny parity case only)

    @property
    def T(self) -> int:
        return self.S // self.m

    def legal_count(self, t: int) -> int:
        return self.T if self.mask_mode == MASK_NONE else min(self.T, (t + 1) // self.m)

    def legal_pairs(self) -> int:
        if self.mask_mode == MASK_NONE:
            return self.B * self.S * self.T
        t = np.arange(self.S, dtype=np.int64)
        return int(self.B * np.minimum(self.T, (t + 1) // self.m).sum())

    def flop_per_pair(self) -> int:
        return 2 * self.H * self.D

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS = {
    "tiny": Workload("tiny", B=1, S=1024, H=4, D=32, m=4, k=16, mask_mode=MASK_NONE, planted=4),
    "flash_4k": Workload("flash_4k", B=1, S=4096, H=64, D=128, m=4, k=512,
                         mask_mode=MASK_CAUSAL_BLOCK),
    "flash_64k": Workload("flash_64k", B=1, S=65536, H=64, D=128, m=4, k=512,
                          mask_mode=MASK_CAUSAL_BLOCK),
    "flash_256k": Workload("flash_256k", B=1, S=262144, H=64, D=128, m=4, k=1024,
                           mask_mode=MASK_CAUSAL_BLOCK),
    "flash_1m": Workload("flash_1m", B=1, S=1048576, H=64, D=128, m=4, k=1024,
                         mask_mode=MASK_CAUSAL_BLOCK),
}


def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + stream)
    return g


def _randn_bf16(shape, gen, device, chunk_rows=4096):
    """N(0,1) drawn in float32 and rounded once (nearest-even) to bfloat16, chunked over dim 0
    of the flattened [rows, cols] view so that the float32 temporary stays small."""
    total = int(np.prod(shape))
    cols = int(np.prod(shape[-2:])) if len(shape) >= 2 else total
    rows = total // cols
    out = torch.empty((rows, cols), dtype=torch.bfloat16, device=device)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = torch.randn((r1 - r0, cols), generator=gen, device=device,
                                 dtype=torch.float32).to(torch.bfloat16)
    return out.view(*shape)


def make_inputs(wl: Workload, device="cpu"):
    """Returns (q [B,S,H,D] bf16, K [B,T,D] bf16, w [B,S,H] f32, info dict) on `device`.

    The same (workload, device type) always gives the same bits.  CPU and GPU
    generators give different streams; a test draws once and hands the same
    tensors to both paths.
    """
    device = torch.device(device)
    q = _randn_bf16((wl.B, wl.S, wl.H, wl.D), _gen(wl.seed, _STREAM_Q, device), device)
    K = _randn_bf16((wl.B, wl.T, wl.D), _gen(wl.seed, _STREAM_K, device), device)
    w = torch.randn((wl.B, wl.S, wl.H), generator=_gen(wl.seed, _STREAM_W, device),
                    device=device, dtype=torch.float32) * (1.0 / np.sqrt(wl.H))
    info = {"sigma_w": float(1.0 / np.sqrt(wl.H)), "seed": wl.seed}
    if wl.planted:
        # Planted keys: pick one query t*, overwrite `planted` distinct key rows
        # with 3x that query's head vectors (one head each) and give that query equal
        # positive weights, so these keys are its best-scoring ones by construction
        # (own-head term 3*w*|q_j|^2 ~ 48 against ~15 for the best unplanted key).
        assert wl.planted <= wl.H and wl.B == 1
        t_star = wl.S // 2 + 1
        slots = [(7 + 61 * j) % wl.T for j in range(wl.planted)]
        assert len(set(slots)) == wl.planted
        for j, s in enumerate(slots):
            K[0, s] = (3.0 * q[0, t_star, j].float()).to(torch.bfloat16)
        w[0, t_star] = 0.5
        info.update({"t_star": t_star, "planted_keys": slots})
    return q, K, w, info


def sample_rows(wl: Workload, n: int):
    """Seeded sample of query positions for the large configurations, plus the edge rows:
    first rows with no / few legal keys, the rows around the point where k legal keys
    first exist, and the last row."""
    rng = np.random.default_rng(wl.seed * 1000003 + _STREAM_ROWS)
    rows = set(int(x) for x in rng.integers(0, wl.S, size=n))
    km = wl.k * wl.m
    for t in (0, wl.m - 2, wl.m - 1, wl.m, km - 2, km - 1, km, wl.S - 2, wl.S - 1):
        if 0 <= t < wl.S:
            rows.add(int(t))
    return np.array(sorted(rows), dtype=np.int64)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """bfloat16 tensor -> host uint16 array of its bit patterns."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def float_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32/64 host array -> bfloat16 bit patterns (nearest-even), for hand-made cases."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return bf16_bits(t)


def bits_to_float(a: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> float64 host array (exact)."""
    u = a.astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)
