"""Seeded synthetic inputs for the structured-sparse INT8 SpMM.

This module only draws random tensors with the shapes, sparsity structure and
value distributions of the paper's workloads (Table 4 weight shapes, sparsity
ratios 70-90 %, sequence lengths 16-384).  It holds none of the method's
arithmetic: no products, no epilogue, no packing.  Both the CPU oracle's tests
and the HIP path's tests/bench draw their inputs from here so that the two
sides provably consume the same bytes (see `sha256`).

Axis names (the paper swaps letters between paragraphs, so they are fixed here):
    N  output channels = rows of W = rows of out
    K  reduction dim   = cols of W = rows of X
    M  tokens          = cols of X = cols of out
W is int8 [N, K] row-major, X is uint8 [K, M] row-major (tokens contiguous).
"""
from __future__ import annotations

import hashlib
import math
from dataclasses import dataclass, field, replace
from typing import Dict, Iterator, List, Optional, Tuple

import numpy as np

BASE_SEED = 230616601

# Block orientations of the "4x1" pattern (Section 3.1, Figure 1).
N4K1 = "n4k1"  # 4 consecutive output rows x 1 k  (sparsity dimension on N)
N1K4 = "n1k4"  # 1 output row x 4 consecutive k   (alternative wording)

# Output types / post-ops, as plain strings (the binding and the oracle wrapper
# each map them to their own enums).
OUT_S32, OUT_F32, OUT_S8, OUT_U8 = "s32", "f32", "s8", "u8"
POST_NONE, POST_GELU = "none", "gelu"

# Tensor ids for the per-tensor random sub-streams.
_T_W, _T_X, _T_WSCALE, _T_BIAS, _T_JITTER, _T_CLUSTER = 1, 2, 3, 4, 5, 6

X_SCALE = 0.02  # scalar activation scale used by every config


def rng_for(*keys: int) -> np.random.Generator:
    """Independent generator for (BASE_SEED, *keys)."""
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED, *[int(k) for k in keys]]))


def sha256(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def round_half_up(x: float) -> int:
    return int(math.floor(x + 0.5))


def block_counts(n_units: int, positions: int, density: float, jitter: float,
                 rng: np.random.Generator) -> np.ndarray:
    """Number of non-zero blocks for each of `n_units` block-rows.

    Without jitter every unit gets exactly floor(density*positions + 0.5).
    With jitter j the count is floor(c*(1+u)+0.5), u ~ U[-j, j], clipped to
    [0, positions] (load-imbalance exercise of the shape-grid config).
    """
    c = density * positions
    if jitter <= 0.0:
        return np.full(n_units, min(positions, round_half_up(c)), dtype=np.int64)
    u = rng.uniform(-jitter, jitter, size=n_units)
    cnt = np.floor(c * (1.0 + u) + 0.5).astype(np.int64)
    return np.clip(cnt, 0, positions)


def sparse_weight(N: int, K: int, sparsity: float, orientation: str = N4K1,
                  jitter: float = 0.0, keys: Tuple[int, ...] = (), clusters: int = 0) -> np.ndarray:
    """int8 [N, K] weight pruned in constant 4x1 blocks.

    N4K1: a block covers output rows 4b..4b+3 at one k; each block-row (4 rows)
    keeps `count` k positions chosen uniformly at random.
    N1K4: a block covers one row at k = 4c..4c+3; each row keeps `count` of the
    K/4 aligned K-blocks.
    Kept blocks are filled with values uniform in [-127, 127] without 0.
    N (N4K1) or K (N1K4) need not be multiples of 4: the last, partial block
    row/column is treated as a block of fewer elements.

    clusters > 0 gives the pattern a structure that an offline row ordering can find: that
    many prototype position sets are drawn, every block-row (in random order) follows one of
    them, keeping about 90 % of its positions and drawing the rest at random.
    """
    density = 1.0 - sparsity
    rng_w = rng_for(*keys, _T_W)
    rng_j = rng_for(*keys, _T_JITTER)
    W = np.zeros((N, K), dtype=np.int8)
    if orientation == N4K1:
        units, positions = (N + 3) // 4, K
    elif orientation == N1K4:
        units, positions = N, (K + 3) // 4
    else:
        raise ValueError(orientation)
    counts = block_counts(units, positions, density, jitter, rng_j)
    # random position order per unit: rank of uniform keys
    rank_key = rng_w.random((units, positions))
    if clusters > 0:
        rng_c = rng_for(*keys, _T_CLUSTER)
        proto_count = min(positions, round_half_up(density * positions))
        proto_order = np.argsort(rng_c.random((clusters, positions)), axis=1)
        member = np.zeros((clusters, positions), dtype=bool)
        np.put_along_axis(member, proto_order[:, :proto_count], True, axis=1)
        follows = rng_c.integers(0, clusters, size=units)
        dropped = rng_c.random((units, positions)) < 0.1
        # positions of the followed prototype (minus the dropped tenth) rank before all others
        rank_key = rank_key + np.where(member[follows] & ~dropped, 0.0, 1.0)
    order = np.argsort(rank_key, axis=1)
    keep = np.zeros((units, positions), dtype=bool)
    cols = np.arange(positions)[None, :]
    np.put_along_axis(keep, order, cols < counts[:, None], axis=1)
    mag = rng_w.integers(1, 128, size=(N, K), dtype=np.int16)
    sign = rng_w.integers(0, 2, size=(N, K), dtype=np.int16) * 2 - 1
    vals = (mag * sign).astype(np.int8)
    if orientation == N4K1:
        mask = np.repeat(keep, 4, axis=0)[:N, :]
    else:
        mask = np.repeat(keep, 4, axis=1)[:, :K]
    W[mask] = vals[mask]
    return W


def activations(K: int, M: int, keys: Tuple[int, ...] = ()) -> np.ndarray:
    """uint8 [K, M] uniform in [0, 255]."""
    return rng_for(*keys, _T_X).integers(0, 256, size=(K, M), dtype=np.uint8)


def channel_params(N: int, keys: Tuple[int, ...] = ()) -> Tuple[np.ndarray, np.ndarray]:
    """(w_scale [N] fp32 ~ U[1e-3, 1e-2], bias [N] fp32 ~ N(0, 1))."""
    w_scale = rng_for(*keys, _T_WSCALE).uniform(1e-3, 1e-2, size=N).astype(np.float32)
    bias = rng_for(*keys, _T_BIAS).standard_normal(N).astype(np.float32)
    return w_scale, bias


def preact_sigma(K: int, sparsity: float) -> float:
    """Analytic standard deviation of the dequantised pre-activation for the
    value distributions above (used only to choose quantisation scales, the
    way a calibration run would): var = nnz_row * E[w^2] * E[x^2] * E[s^2] + 1.
    """
    nnz_row = (1.0 - sparsity) * K
    e_w2 = 128.0 * 255.0 / 6.0            # uniform on +-{1..127}
    e_x2 = 255.0 * 511.0 / 6.0            # uniform on {0..255}
    e_s2 = (X_SCALE ** 2) * (1e-6 + 1e-5 + 1e-4) / 3.0
    return math.sqrt(nnz_row * e_w2 * e_x2 * e_s2 + 1.0)


def quant_scales(K: int, sparsity: float) -> Tuple[float, float]:
    """(mid_scale, out_scale): symmetric int8 scales clipping at 4 sigma,
    rounded to fp32 (what the boundary carries)."""
    s = np.float32(4.0 * preact_sigma(K, sparsity) / 127.0)
    return float(s), float(s)


@dataclass(frozen=True)
class Case:
    """One SpMM problem: shapes, sparsity structure and epilogue."""
    name: str
    N: int
    K: int
    M: int
    sparsity: float
    orientation: str = N4K1
    out_type: str = OUT_S32
    postop: str = POST_NONE
    with_bias: bool = True
    jitter: float = 0.0
    x_zero_point: int = 0
    out_zero_point: int = 0
    keys: Tuple[int, ...] = field(default_factory=tuple)
    clusters: int = 0

    def with_(self, **kw) -> "Case":
        return replace(self, **kw)


def make(case: Case) -> Dict[str, object]:
    """Draw every input tensor of `case` (host numpy arrays + scalar params)."""
    W = sparse_weight(case.N, case.K, case.sparsity, case.orientation, case.jitter, case.keys, case.clusters)
    X = activations(case.K, case.M, case.keys)
    w_scale, bias = channel_params(case.N, case.keys)
    mid_scale, out_scale = quant_scales(case.K, case.sparsity)
    return dict(W=W, X=X, w_scale=w_scale, bias=bias if case.with_bias else None,
                x_scale=X_SCALE, x_zero_point=case.x_zero_point,
                mid_scale=mid_scale, out_scale=out_scale, out_zero_point=case.out_zero_point)


def realised_block_sparsity(W: np.ndarray, orientation: str = N4K1) -> Tuple[int, int]:
    """(non-zero blocks, total blocks) of W under the given orientation, counted
    directly on the dense-with-zeros matrix."""
    N, K = W.shape
    nz = (W != 0)
    if orientation == N4K1:
        pad = (-N) % 4
        nz = np.pad(nz, ((0, pad), (0, 0)))
        blk = nz.reshape(-1, 4, K).any(axis=1)
    else:
        pad = (-K) % 4
        nz = np.pad(nz, ((0, 0), (0, pad)))
        blk = nz.reshape(N, -1, 4).any(axis=2)
    return int(blk.sum()), int(blk.size)


# --------------------------------------------------------------------------
# The five configurations
# --------------------------------------------------------------------------
SPARSITIES = (0.70, 0.75, 0.80, 0.85, 0.90)

BERT_MINI_SHAPES = ((1024, 256), (256, 1024))
BERT_BASE_SHAPES = ((768, 768), (3072, 768), (768, 3072))
BERT_LARGE_SHAPES = ((1024, 1024), (4096, 1024), (1024, 4096))


def _pct(s: float) -> int:
    return int(round(s * 100))


def tiny_cases(orientation: str = N4K1) -> List[Case]:
    """Config 1: 256x256 at 90 %, X 256x128, int32 output."""
    return [Case("tiny_256x256_m128_s90", 256, 256, 128, 0.90, orientation, OUT_S32,
                 POST_NONE, keys=(1, 256, 256, 128, 90))]


def mini_cases(orientation: str = N4K1) -> List[Case]:
    """Config 2: BERT-Mini FFN pair at 80 %, M = 8*128; W1 bias+GELU -> fp32,
    W2 requant -> int8."""
    M = 8 * 128
    return [
        Case("mini_ffn1_1024x256_m1024_s80", 1024, 256, M, 0.80, orientation, OUT_F32,
             POST_GELU, keys=(2, 1024, 256, M, 80)),
        Case("mini_ffn2_256x1024_m1024_s80", 256, 1024, M, 0.80, orientation, OUT_S8,
             POST_NONE, keys=(2, 256, 1024, M, 80)),
    ]


def chain_cases(orientation: str = N4K1, large: bool = False) -> List[Case]:
    """Config 2 as a chained pair (Figure 3 / Algorithm 2: a quantised operator feeding the next one with
    no fp32 tensor between them): W1 bias + GELU -> uint8 code with a zero point (the table chain), whose
    output IS the activation matrix of W2 -> int8.  Inputs of the pair come from make_chain().
    large: the same pair with the feed-forward shapes and token count of config 4 (BERT-Large, 90 %)."""
    if large:
        M = 16 * 384
        return [
            Case("chain_ffn1_4096x1024_m%d_s90" % M, 4096, 1024, M, 0.90, orientation, OUT_U8,
                 POST_GELU, keys=(7, 4096, 1024, M, 90)),
            Case("chain_ffn2_1024x4096_m%d_s90" % M, 1024, 4096, M, 0.90, orientation, OUT_S8,
                 POST_NONE, keys=(7, 1024, 4096, M, 90)),
        ]
    M = 8 * 128
    return [
        Case("chain_ffn1_1024x256_m1024_s80", 1024, 256, M, 0.80, orientation, OUT_U8,
             POST_GELU, keys=(2, 1024, 256, M, 80)),
        Case("chain_ffn2_256x1024_m1024_s80", 256, 1024, M, 0.80, orientation, OUT_S8,
             POST_NONE, keys=(2, 256, 1024, M, 80)),
    ]


def make_chain(cases: List[Case]) -> List[Dict[str, object]]:
    """Inputs of chain_cases(): the first stage's uint8 output scale / zero point (GELU output lies in
    [-0.17, ~4 sigma]: the code covers that range) are the second stage's activation scale / zero
    point; the second stage has no X of its own (d["X"] is None)."""
    c1, c2 = cases
    d1, d2 = make(c1), make(c2)
    sigma1 = preact_sigma(c1.K, c1.sparsity)
    h_scale = float(np.float32((4.0 * sigma1 + 0.17) / 255.0))
    h_zp = int(round_half_up(0.17 / h_scale))
    d1["out_scale"], d1["out_zero_point"] = h_scale, h_zp
    # second stage: E[(h - zp)^2 h_scale^2] ~ E[GELU(y)^2] ~ sigma1^2 / 2 for y ~ N(0, sigma1^2)
    nnz_row = (1.0 - c2.sparsity) * c2.K
    e_w2 = 128.0 * 255.0 / 6.0
    e_s2 = (1e-6 + 1e-5 + 1e-4) / 3.0
    sigma2 = math.sqrt(nnz_row * e_w2 * (sigma1 ** 2 / 2.0) * e_s2 + 1.0)
    d2["X"] = None
    d2["x_scale"], d2["x_zero_point"] = h_scale, h_zp
    d2["out_scale"] = float(np.float32(4.0 * sigma2 / 127.0))
    return [d1, d2]


def base_cases(orientation: str = N4K1, batches=(1, 8, 32), sparsities=SPARSITIES) -> List[Case]:
    """Config 3: BERT-Base layer shapes x sparsity sweep x M = 128*batch, fp32 output."""
    out = []
    for (N, K) in BERT_BASE_SHAPES:
        for s in sparsities:
            for b in batches:
                M = 128 * b
                out.append(Case(f"base_{N}x{K}_m{M}_s{_pct(s)}", N, K, M, s, orientation,
                                OUT_F32, POST_NONE, keys=(3, N, K, M, _pct(s))))
    return out


def large_cases(orientation: str = N4K1, sparsities=(0.90, 0.80), M: int = 16 * 384) -> List[Case]:
    """Config 4: BERT-Large layer shapes, M = 16*384, bias+GELU with int8 requant."""
    out = []
    for (N, K) in BERT_LARGE_SHAPES:
        for s in sparsities:
            out.append(Case(f"large_{N}x{K}_m{M}_s{_pct(s)}", N, K, M, s, orientation,
                            OUT_S8, POST_GELU, keys=(4, N, K, M, _pct(s))))
    return out


GRID_DIMS = (256, 512, 768, 1024, 2048, 3072, 4096)
GRID_M = (128, 384, 1024, 4096)


def clustered_cases(orientation: str = N4K1, clusters: int = 32, M: int = 16 * 384) -> List[Case]:
    """The 4096x1024 BERT-Large layer at 90 and 80 % with block-rows that follow `clusters`
    prototype patterns in random order (exercise for offline row ordering; not one of the five
    configurations: pruned checkpoints are not available, this only shows what structure is worth)."""
    out = []
    for s in (0.90, 0.80):
        out.append(Case("clustered%d_4096x1024_m%d_s%d" % (clusters, M, _pct(s)), 4096, 1024, M, s, orientation,
                        OUT_S8, POST_GELU, keys=(6, 4096, 1024, M, _pct(s), clusters), clusters=clusters))
    return out


def grid_shapes() -> List[Tuple[int, int]]:
    """(N, K) pairs of the shape grid: both dims from GRID_DIMS with aspect
    ratio N/K in {1, 2, 4, 1/2, 1/4} (the ratios Transformer layers use)."""
    pairs = []
    for N in GRID_DIMS:
        for K in GRID_DIMS:
            if N == K or N == 2 * K or N == 4 * K or K == 2 * N or K == 4 * N:
                pairs.append((N, K))
    return pairs


def grid_cases(orientation: str = N4K1, out_type: str = OUT_S32,
               sparsities=SPARSITIES, Ms=GRID_M) -> List[Case]:
    """Config 5: the shape grid x 5 sparsities with +-20 % per-block-row count jitter."""
    out = []
    for (N, K) in grid_shapes():
        for M in Ms:
            for s in sparsities:
                out.append(Case(f"grid_{N}x{K}_m{M}_s{_pct(s)}", N, K, M, s, orientation,
                                out_type, POST_NONE, jitter=0.2, keys=(5, N, K, M, _pct(s))))
    return out
