"""Seeded synthetic workloads: shapes and random tensors only, none of the method's arithmetic.

The five configurations are the long-context shapes this library is measured on.  The paper's own
benchmark (Sec. 5.1.2) is a grid of random tensors (batch 1-128, sequence 3K-1M, bf16), so seeded
normal tensors of the listed shapes stand in for it.  Both the CPU oracle's tests and the GPU tests
draw their inputs from here so that the two sides see the same bits.
"""
from dataclasses import dataclass, replace

import torch

BASE_SEED = 250926541
FULL = 0
ZIGZAG_CAUSAL = 1


@dataclass(frozen=True)
class Workload:
    name: str
    n_ranks: int
    rank: int
    S: int                 # total sequence length
    Hq: int
    Hkv: int
    d: int
    dtype: str             # "fp32" or "bf16"
    mask_mode: int
    k_scale: float = 1.0   # applied after the cast (a power of two, so exact)
    outlier_frac: float = 0.0
    outlier_scale: float = 8.0
    seed: int = BASE_SEED

    @property
    def L(self):
        return self.S // self.n_ranks

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def scaled(self, S, **kw):
        """Same recipe at another sequence length (for tests the oracle can finish)."""
        return replace(self, S=S, **kw)


CONFIGS = [
    Workload("cfg1_n4_s1k_fp32_full", 4, 0, 1024, 4, 4, 64, "fp32", FULL, seed=BASE_SEED + 1),
    Workload("cfg2_n8_s128k_bf16_zigzag", 8, 3, 131072, 32, 8, 128, "bf16", ZIGZAG_CAUSAL, seed=BASE_SEED + 2),
    Workload("cfg3_n8_s256k_bf16_full_k2", 8, 0, 262144, 32, 8, 128, "bf16", FULL, k_scale=2.0, seed=BASE_SEED + 3),
    Workload("cfg4_n16_s512k_bf16_zigzag", 16, 5, 524288, 64, 8, 128, "bf16", ZIGZAG_CAUSAL, seed=BASE_SEED + 4),
    Workload("cfg5_n8_s1m_bf16_zigzag_outliers", 8, 7, 1048576, 32, 8, 128, "bf16", ZIGZAG_CAUSAL,
             outlier_frac=0.01, seed=BASE_SEED + 5),
]


def paper_grid(heads, seq, n_ranks=8, rank=3, mask_mode=ZIGZAG_CAUSAL, seed_offset=0):
    """One sequence of the paper's own benchmark grid (Sec. 5.1.2): multi-head attention with 4, 12 or
    20 heads of dimension 64 in bf16, sequence length `seq` (3K-1M there); the grid's batch dimension
    is the `batch` argument of the attention call (sequences seeded seed, seed + 1000, ...)."""
    name = "grid_n%d_h%d_s%d_d64_%s" % (n_ranks, heads, seq, "zigzag" if mask_mode == ZIGZAG_CAUSAL else "full")
    return Workload(name, n_ranks, rank, seq, heads, heads, 64, "bf16", mask_mode, seed=BASE_SEED + 100 + heads + seed_offset)


def _normal(shape, gen, dtype, rows_per_pass=1 << 16):
    """N(0,1) in fp32 from `gen`, cast (round to nearest even) to dtype; drawn in fixed-size row
    blocks so that the bits do not depend on available memory."""
    out = torch.empty(shape, dtype=dtype)
    for r0 in range(0, shape[0], rows_per_pass):
        r1 = min(shape[0], r0 + rows_per_pass)
        out[r0:r1] = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=gen, dtype=torch.float32).to(dtype)
    return out


def make_qkv(w):
    """Returns CPU tensors q [L, Hq, d] (the rank's local rows), k, v [S, Hkv, d] (whole sequence)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed)
    dt = w.torch_dtype
    q = _normal((w.L, w.Hq, w.d), gen, dt)
    k = _normal((w.S, w.Hkv, w.d), gen, dt)
    v = _normal((w.S, w.Hkv, w.d), gen, dt)
    if w.k_scale != 1.0:
        k *= w.k_scale
    if w.outlier_frac > 0.0:
        n_out = int(w.outlier_frac * w.S)
        idx = torch.randperm(w.S, generator=gen)[:n_out]
        k[idx] *= w.outlier_scale
    return q, k, v


def make_dout(w):
    """Upstream gradient of the local output, [L, Hq, d]: N(0,1) in the workload's dtype."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed + 104729)
    return _normal((w.L, w.Hq, w.d), gen, w.torch_dtype)


def sample_rows(w, n_random, seed_offset=0):
    """Local row indices worth checking: ends of each half, rows next to 32/64/128/256-row tile
    edges, plus seeded random rows.  Sorted, unique."""
    L = w.L
    H = L // 2 if w.mask_mode == ZIGZAG_CAUSAL else L
    rows = {0, L - 1, H - 1, H % L, min(L - 1, H + 1)}
    for t in (31, 32, 63, 64, 127, 128, 255, 256):
        for base in (0, H % L):
            if base + t < L:
                rows.add(base + t)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed + 7919 + seed_offset)
    rows.update(int(x) for x in torch.randint(0, L, (n_random,), generator=gen))
    return sorted(rows)
