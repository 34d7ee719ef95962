"""Seeded synthetic inputs for the low-precision MoE expert layer.

This module only draws numbers and lays them out; it performs none of the layer's
arithmetic (no rotation, no quantization, no routing, no decode), so that the CPU oracle
and the HIP path can both be fed the very same bytes without sharing any of the method.

The shapes follow the MoE models the paper evaluates (Mixtral-8x7B, DeepSeek-V2-Lite,
Qwen3-30B-A3B; Experiments section) and the deployed weight format of the ACCF section:
for every weight row a 16-entry centroid table (Eq. W_c: W_c[i,j] = sum_k C[i,k] A[i,j,k])
and, for every weight, the 4-bit position of its single non-zero A[i,j,:] entry.

Layouts produced (all numpy, host memory):
  X        [T, H]        float32   hidden states, a few channels scaled up (activation outliers)
  R        [H, H]        float32   orthogonal matrix (Q factor of a Gaussian matrix, sign-fixed)
  Wr       [E, H]        float32   router weight, already expressed in the rotated basis
  bias     [E] or None   float32   router bias (only the Zipf-popularity config has one)
  experts[e]["gate"|"up"|"down"] = (idx, cent)
      idx  [N, K/2]      uint8     byte j of a row = index of weight 2j (bits 0-3) and 2j+1 (bits 4-7)
      cent [N, 16]       uint16    bf16 bit patterns, ascending within a row (embedding-wise tables), or
           [N, ceil(K/g), 16]      one table per group of g consecutive weights of the row (block-wise
                                   setting of the experimental setup; LayerConfig.group_k = g)
  with (N, K) = (I, H) for gate and up and (H, I) for down.  Experts E .. E+S-1 are the
  always-on shared experts.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import numpy as np

SEED_BASE = 20260410 * 10
N_CENTROIDS = 16


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    index: int          # position in the list of benchmark configurations (seeds derive from it)
    E: int              # routed experts
    top_k: int
    S: int              # shared (always-on) experts
    H: int              # hidden size (d_in)
    I: int              # expert intermediate size
    T: int              # tokens
    act_bits: int       # 8 or 4
    outlier_channels: Tuple[int, ...]   # explicit channel ids, or () to draw n_outliers of them
    n_outliers: int
    outlier_scale: float
    zipf_s: float = 0.0  # > 0: router bias makes expert popularity follow Zipf(s)
    h_bits: int = 0      # 4 or 8: online-Hadamard variant (the intermediate is rotated and quantized)
    group_k: int = 0     # > 0: block-wise centroid tables, one per group_k consecutive weights of a row
    r_hadamard: bool = False  # the rotation is the Hadamard matrix H/sqrt(H): no R is drawn (callers that
                              # need the dense matrix build it themselves and pass it as R_override)
    index_bits: int = 4  # 2: the W2 budget of the ablation on centroid budgets -- idx [N, K/4] (2-bit stream,
                         # weight j in bits 2(j%4).. of byte j/4), cent [N, 4]

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def n_groups(self) -> int:
        return self.E + self.S


CONFIGS: Dict[str, LayerConfig] = {
    c.name: c
    for c in [
        LayerConfig("tiny", 0, E=4, top_k=2, S=0, H=256, I=512, T=64, act_bits=8,
                    outlier_channels=(3, 77), n_outliers=2, outlier_scale=50.0),
        LayerConfig("mixtral_decode", 1, E=8, top_k=2, S=0, H=4096, I=14336, T=16, act_bits=8,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0),
        LayerConfig("mixtral_prefill", 2, E=8, top_k=2, S=0, H=4096, I=14336, T=4096, act_bits=4,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0),
        LayerConfig("dsv2lite", 3, E=64, top_k=6, S=2, H=2048, I=1408, T=512, act_bits=8,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0),
        LayerConfig("qwen3_zipf", 4, E=128, top_k=8, S=0, H=2048, I=768, T=2048, act_bits=4,
                    outlier_channels=(), n_outliers=4, outlier_scale=100.0, zipf_s=1.1),
        # online-Hadamard variants of the two Mixtral-shaped workloads (same inputs as configurations 1, 2)
        LayerConfig("mixtral_decode_had", 1, E=8, top_k=2, S=0, H=4096, I=14336, T=16, act_bits=8,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0, h_bits=8, r_hadamard=True),
        LayerConfig("mixtral_prefill_had", 2, E=8, top_k=2, S=0, H=4096, I=14336, T=4096, act_bits=4,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0, h_bits=4, r_hadamard=True),
        # block-wise centroid tables (g = 1024) on the same two workloads
        LayerConfig("mixtral_decode_blockwise", 1, E=8, top_k=2, S=0, H=4096, I=14336, T=16, act_bits=8,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0, group_k=1024),
        LayerConfig("mixtral_prefill_blockwise", 2, E=8, top_k=2, S=0, H=4096, I=14336, T=4096, act_bits=4,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0, group_k=1024),
        # the decode workload with the W2 budget (four centroids per row, 2-bit indices streamed as stored)
        LayerConfig("mixtral_decode_w2", 1, E=8, top_k=2, S=0, H=4096, I=14336, T=16, act_bits=8,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0, index_bits=2),
        # the decode workload with 4-bit activations (what the lookup formulation of the product needs)
        LayerConfig("mixtral_decode_a4", 1, E=8, top_k=2, S=0, H=4096, I=14336, T=16, act_bits=4,
                    outlier_channels=(), n_outliers=8, outlier_scale=100.0),
    ]
}


def small_variant(cfg: LayerConfig, **overrides) -> LayerConfig:
    """A config with some fields replaced (used for reduced-size parity cases)."""
    return dataclasses.replace(cfg, **overrides)


# ----------------------------------------------------------------------------------------------
# number formats (data formatting only)
# ----------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = u + 0x7FFF + lsb
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------------------------
# pieces
# ----------------------------------------------------------------------------------------------
def draw_tokens(cfg: LayerConfig, rng: np.random.Generator, n_rows: int,
                channels: np.ndarray) -> np.ndarray:
    x = rng.standard_normal((n_rows, cfg.H), dtype=np.float32)
    x[:, channels] *= np.float32(cfg.outlier_scale)
    return x


def draw_orthogonal(rng: np.random.Generator, H: int) -> np.ndarray:
    g = rng.standard_normal((H, H))
    q, r = np.linalg.qr(g)
    q = q * np.sign(np.diag(r))[None, :]
    return q.astype(np.float32)


def draw_centroids(rng: np.random.Generator, N: int, outlier_row_frac: float = 0.01,
                   n_blocks: int = 0) -> np.ndarray:
    """[N, 16] tables, or [N, n_blocks, 16] when n_blocks > 0 (every table drawn like a row's)."""
    if n_blocks > 0:
        return draw_centroids(rng, N * n_blocks, outlier_row_frac).reshape(N, n_blocks, N_CENTROIDS)
    c = np.sort(rng.standard_normal((N, N_CENTROIDS)).astype(np.float32) * np.float32(0.02), axis=1)
    n_out = int(math.ceil(outlier_row_frac * N))
    rows = rng.permutation(N)[:n_out]
    # the largest-magnitude centroid sits at one end of the sorted table: scaling it keeps the order
    left_bigger = np.abs(c[rows, 0]) >= np.abs(c[rows, -1])
    col = np.where(left_bigger, 0, N_CENTROIDS - 1)
    c[rows, col] *= np.float32(20.0)
    return f32_to_bf16_bits(c)


def n_blocks(K: int, group_k: int) -> int:
    """Tables per weight row: 0 stands for the embedding-wise layout [N, 16]."""
    return -(-K // group_k) if group_k > 0 else 0


def zipf_bias(cfg: LayerConfig, rng: np.random.Generator) -> np.ndarray:
    """Router bias tau*log p_rank(e), p_r ~ r^-s over a seeded ranking of the experts.

    tau matches the spread of the logits: for a token x and Wr ~ N(0, 1/H) a logit has variance
    |x|^2/H, which for N(0,1) channels with n_outliers channels scaled by outlier_scale equals
    (H - n + n*scale^2)/H; tau = std*sqrt(6)/pi is the Gumbel scale with that standard deviation.
    """
    n = cfg.n_outliers
    logit_std = math.sqrt((cfg.H - n + n * cfg.outlier_scale ** 2) / cfg.H)
    tau = logit_std * math.sqrt(6.0) / math.pi
    rank = rng.permutation(cfg.E)  # rank[e] = popularity rank of expert e (0 = most popular)
    p = (np.arange(1, cfg.E + 1, dtype=np.float64)) ** (-cfg.zipf_s)
    p /= p.sum()
    return (tau * np.log(p[rank])).astype(np.float32)


# ----------------------------------------------------------------------------------------------
# a whole layer
# ----------------------------------------------------------------------------------------------
@dataclasses.dataclass
class LayerInputs:
    cfg: LayerConfig
    X: np.ndarray
    channels: np.ndarray
    R: np.ndarray
    Wr: np.ndarray
    bias: Optional[np.ndarray]
    experts: List[Dict[str, Tuple[np.ndarray, np.ndarray]]]  # E routed then S shared
    redrawn_rows: int = 0


def make_layer(cfg: LayerConfig, with_experts: bool = True,
               R_override: Optional[np.ndarray] = None) -> LayerInputs:
    """Draw every input of one layer in a fixed order from one seeded generator.

    Order: X, outlier channels, R, Wr, bias, then per expert gate idx, up idx, down idx,
    gate centroids, up centroids, down centroids (routed experts first, then shared ones).
    """
    rng = np.random.default_rng(cfg.seed)
    X = rng.standard_normal((cfg.T, cfg.H), dtype=np.float32)
    if cfg.outlier_channels:
        channels = np.asarray(cfg.outlier_channels, dtype=np.int64)
    else:
        channels = np.sort(rng.permutation(cfg.H)[: cfg.n_outliers])
    X[:, channels] *= np.float32(cfg.outlier_scale)
    if R_override is not None:
        R = R_override.astype(np.float32)
    else:
        R = None if cfg.r_hadamard else draw_orthogonal(rng, cfg.H)
    Wr = (rng.standard_normal((cfg.E, cfg.H)) / math.sqrt(cfg.H)).astype(np.float32)
    bias = zipf_bias(cfg, rng) if cfg.zipf_s > 0 else None
    experts: List[Dict[str, Tuple[np.ndarray, np.ndarray]]] = []
    if with_experts:
        per_byte = 8 // cfg.index_bits   # weights per index byte: uniform bytes are uniform indices at any width
        for _ in range(cfg.E + cfg.S):
            gi = rng.integers(0, 256, size=(cfg.I, cfg.H // per_byte), dtype=np.uint8)
            ui = rng.integers(0, 256, size=(cfg.I, cfg.H // per_byte), dtype=np.uint8)
            di = rng.integers(0, 256, size=(cfg.H, cfg.I // per_byte), dtype=np.uint8)
            gc = draw_centroids(rng, cfg.I, n_blocks=n_blocks(cfg.H, cfg.group_k))
            uc = draw_centroids(rng, cfg.I, n_blocks=n_blocks(cfg.H, cfg.group_k))
            dc = draw_centroids(rng, cfg.H, n_blocks=n_blocks(cfg.I, cfg.group_k))
            if cfg.index_bits == 2:
                # four of the sixteen sorted draws, the two ends left out: the x20 outlier of 1 % of the rows is always
                # an end, and with uniform 2-bit indices a quarter of such a row's weights would carry it -- the
                # intermediate h would leave the f16 range (a real 4-centroid clustering has no such centroid)
                gc, uc, dc = (np.ascontiguousarray(c[..., [1, 5, 10, 14]]) for c in (gc, uc, dc))
            experts.append({"gate": (gi, gc), "up": (ui, uc), "down": (di, dc)})
    return LayerInputs(cfg, X, channels, R, Wr, bias, experts)


def redraw_rows(inputs: LayerInputs, rows: np.ndarray, attempt: int) -> None:
    """Replace the given token rows of X by fresh draws from a seed derived from (seed, attempt).

    Callers use it to move tokens whose k-th and (k+1)-th router logits are too close to call
    in single precision; which rows those are is the caller's business (it needs the method).
    """
    rows = np.asarray(rows, dtype=np.int64)
    if rows.size == 0:
        return
    cfg = inputs.cfg
    rng = np.random.default_rng([cfg.seed, 7919, attempt])
    inputs.X[rows] = draw_tokens(cfg, rng, rows.size, inputs.channels)
    inputs.redrawn_rows += int(rows.size)


def pack_indices_bits(idx: np.ndarray, bits: int) -> np.ndarray:
    """[N, K] indices in [0, 2^bits) -> [N, K*bits/8] bytes: weight j at bits [j*bits, (j+1)*bits) of the row's
    little-endian bit stream (pure layout; with bits = 4, weight 2j is the low nibble of byte j)."""
    idx = np.asarray(idx, dtype=np.uint64)
    N, K = idx.shape
    assert (K * bits) % 8 == 0 and int(idx.max(initial=0)) < (1 << bits)
    out = np.zeros((N, K * bits // 8), dtype=np.uint8)
    for j in range(K):
        for i in range(bits):
            pos = j * bits + i
            out[:, pos >> 3] |= (((idx[:, j] >> np.uint64(i)) & np.uint64(1)) << np.uint64(pos & 7)).astype(np.uint8)
    return out


def interleave_gate_up(gate: Tuple[np.ndarray, np.ndarray],
                       up: Tuple[np.ndarray, np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Fused [2I, ...] matrix whose row 2i is gate row i and row 2i+1 is up row i (pure layout)."""
    gi, gc = gate
    ui, uc = up
    I = gi.shape[0]
    idx = np.empty((2 * I, gi.shape[1]), dtype=np.uint8)
    idx[0::2] = gi
    idx[1::2] = ui
    cent = np.empty((2 * I,) + gc.shape[1:], dtype=np.uint16)
    cent[0::2] = gc
    cent[1::2] = uc
    return idx, cent


def stack_experts(inputs: LayerInputs) -> Dict[str, np.ndarray]:
    """Stack per-expert matrices into the [G, N, K/2] / [G, N, (blocks,) 16] arrays the library takes."""
    gu = [interleave_gate_up(e["gate"], e["up"]) for e in inputs.experts]
    return {
        "gate_up_idx": np.stack([g[0] for g in gu]),
        "gate_up_cent": np.stack([g[1] for g in gu]),
        "down_idx": np.stack([e["down"][0] for e in inputs.experts]),
        "down_cent": np.stack([e["down"][1] for e in inputs.experts]),
    }
