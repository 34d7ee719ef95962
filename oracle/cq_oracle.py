"""CPU oracle for the forward pass of a low-precision MoE expert layer (CodeQuant deployment).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, float64 definition that the HIP
library is checked against.  Only the tests, the smoke check and the cpu_baseline leg of the
benchmark may import it; the product path never does.  It shares no code with the HIP path
and imports nothing from it.

The forward pass is exact, not approximate: looking weights up through the per-row centroid
table gives precisely the dense matrix W_c of the ACCF section (Eq. W_c), so every function
here is the textbook definition written out in numpy float64.

What follows which passage of the paper
  rotate            X_R = X R                         AOS section (definition of X_R)
  quantize          Q(.) integer quantization          AOS section (objective ||X_R - Q(X_R)||^2),
                                                       kernel section (16 four-bit activation values)
  router_logits     the router is a linear layer       AOS section
  route_topk        Top-K experts and weights Pi       ACCF section (MoE weighted sum), appendix (Top-K)
  permute_by_expert X_t = tokens assigned to expert    AOS section (definition of X_t)
  decode_*          W_c[i,j] = sum_k C[i,k] A[i,j,k]   ACCF section (Eq. W_c)
  expert_ffn        (phi(X W_gate) . X W_up) W_down    AOS section (rotation-invariance equation)
  moe_forward       sum_i Pi_i X_R W_c (+ shared)      ACCF section (Eq. L, MoE case), appendix (shared expert)

Readings taken where the paper is silent (each is also listed in the design notes):
  * quantization is symmetric and per token: s_t = max_j |X_R[t,j]| / qmax, qmax = 2^(b-1)-1,
    q = clip(rint(X_R / s_t), -qmax, qmax) with round-half-to-even; an all-zero row has s_t = 1;
  * the router reads the un-quantized rotated activations;
  * routing weights are the softmax over the k selected logits (they sum to 1); ids are in
    descending logit order and equal logits go to the lower expert id;
  * tokens are grouped by expert with a stable sort of the assignment number a = t*k + j;
  * the intermediate h is not re-quantized before the down projection;
  * phi is SiLU; the output stays in the rotated basis (no R^T is applied);
  * shared experts see every token with weight 1 and are added after the routed sum.

Parity pins for every function are in tests/test_oracle_pins.py; none is unpinned, but the
paper prints no numeric example for this path, so the pins are closed forms, invariants,
brute force on tiny inputs and reductions to library routines.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

N_CENTROIDS = 16


# ------------------------------------------------------------------------------------------
# number formats
# ------------------------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """A bfloat16 bit pattern is the upper half of the float32 with the same value."""
    u32 = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u32.view(np.float32).astype(np.float64)


def unpack_indices(idx_packed: np.ndarray) -> np.ndarray:
    """[N, K/2] bytes -> [N, K] indices in [0,16): byte j holds weight 2j (low nibble), 2j+1 (high)."""
    p = np.asarray(idx_packed, dtype=np.uint8)
    out = np.empty((p.shape[0], p.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = p & 0x0F
    out[:, 1::2] = p >> 4
    return out


# ------------------------------------------------------------------------------------------
# a1 / a2: rotation and per-token quantization
# ------------------------------------------------------------------------------------------
def rotate(X: np.ndarray, R: np.ndarray) -> np.ndarray:
    return np.asarray(X, dtype=np.float64) @ np.asarray(R, dtype=np.float64)


def quantize(XR: np.ndarray, act_bits: int) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric per-token integer quantization.  Returns (codes int32 [T,H], scale float64 [T])."""
    qmax = float(2 ** (act_bits - 1) - 1)
    XR = np.asarray(XR, dtype=np.float64)
    amax = np.max(np.abs(XR), axis=1)
    scale = np.where(amax == 0.0, 1.0, amax / qmax)
    q = np.clip(np.rint(XR / scale[:, None]), -qmax, qmax)
    return q.astype(np.int32), scale


def tie_distance(XR: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """|frac(|x/s|) - 0.5| per element: small values are the rounding ties where +-1 is tolerated."""
    r = np.abs(np.asarray(XR, dtype=np.float64) / scale[:, None])
    return np.abs((r - np.floor(r)) - 0.5)


# ------------------------------------------------------------------------------------------
# a3 / a4 / a5: router, top-k, permutation by expert
# ------------------------------------------------------------------------------------------
def router_logits(XR: np.ndarray, Wr: np.ndarray, bias: Optional[np.ndarray]) -> np.ndarray:
    L = np.asarray(XR, dtype=np.float64) @ np.asarray(Wr, dtype=np.float64).T
    if bias is not None:
        L = L + np.asarray(bias, dtype=np.float64)[None, :]
    return L


def route_topk(L: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """ids [T,k] (descending logit, equal logits -> lower id) and softmax weights over the k chosen."""
    L = np.asarray(L, dtype=np.float64)
    order = np.argsort(-L, axis=1, kind="stable")  # stable: equal keys keep ascending expert id
    ids = order[:, :k].astype(np.int32)
    sel = np.take_along_axis(L, ids.astype(np.int64), axis=1)
    ex = np.exp(sel - sel[:, :1])
    w = ex / ex.sum(axis=1, keepdims=True)
    return ids, w


def permute_by_expert(ids: np.ndarray, n_experts: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Stable grouping of assignments a = t*k + j by expert.

    Returns expert_offsets [E+1], perm [T*k] (sorted position -> a), inv_perm [T*k] (a -> position).
    """
    flat = np.asarray(ids, dtype=np.int64).reshape(-1)
    perm = np.argsort(flat, kind="stable").astype(np.int32)
    counts = np.bincount(flat, minlength=n_experts)
    offsets = np.zeros(n_experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size, dtype=np.int32)
    return offsets, perm, inv


# ------------------------------------------------------------------------------------------
# a6 / a7: codebook weights
# ------------------------------------------------------------------------------------------
def decode_weights(idx_packed: np.ndarray, cent_bits: np.ndarray) -> np.ndarray:
    """W_c [N, K] float64: every weight is the centroid its 4-bit index points at (Eq. W_c)."""
    idx = unpack_indices(idx_packed).astype(np.int64)
    C = bf16_bits_to_f64(cent_bits)
    return np.take_along_axis(C, idx, axis=1)


def decode_weights_bf16_bits(idx_packed: np.ndarray, cent_bits: np.ndarray) -> np.ndarray:
    """Same decode, returning the bf16 bit patterns (what a bit-exact decode check compares)."""
    idx = unpack_indices(idx_packed).astype(np.int64)
    return np.take_along_axis(np.asarray(cent_bits, dtype=np.uint16), idx, axis=1)


def decode_weights_onehot(idx_packed: np.ndarray, cent_bits: np.ndarray) -> np.ndarray:
    """Eq. W_c taken literally: build the one-hot assignment tensor A and contract it with C."""
    idx = unpack_indices(idx_packed)
    N, K = idx.shape
    A = np.zeros((N, K, N_CENTROIDS), dtype=np.float64)
    n, j = np.meshgrid(np.arange(N), np.arange(K), indexing="ij")
    A[n, j, idx] = 1.0
    assert np.all(A.sum(axis=2) == 1.0)
    C = bf16_bits_to_f64(cent_bits)
    return np.einsum("nk,njk->nj", C, A)


def codebook_matmul(A_rows: np.ndarray, idx_packed: np.ndarray, cent_bits: np.ndarray) -> np.ndarray:
    """[M, K] activations times W_c^T -> [M, N]."""
    return np.asarray(A_rows, dtype=np.float64) @ decode_weights(idx_packed, cent_bits).T


def product_lut_matmul(codes: np.ndarray, idx_packed: np.ndarray, cent_bits: np.ndarray,
                       act_bits: int = 4) -> np.ndarray:
    """The lookup formulation of the kernel section, for integer activation codes.

    For one weight row the table has one sub-table per centroid holding centroid * v for every
    representable activation value v; a (weight index, activation code) pair selects one product
    and the products are accumulated.  Pure-Python loops: tiny inputs only.
    """
    idx = unpack_indices(idx_packed)
    C = bf16_bits_to_f64(cent_bits)
    N, K = idx.shape
    lo = -(2 ** (act_bits - 1))
    values = np.arange(lo, -lo, dtype=np.float64)            # all 2^b representable codes
    M = codes.shape[0]
    out = np.zeros((M, N), dtype=np.float64)
    for n in range(N):
        lut = C[n][:, None] * values[None, :]                 # [16 sub-tables, 2^b entries]
        for m in range(M):
            acc = 0.0
            for j in range(K):
                acc += lut[idx[n, j], int(codes[m, j]) - lo]
            out[m, n] = acc
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def expert_ffn(a_rows: np.ndarray, expert: Dict[str, Tuple[np.ndarray, np.ndarray]]) -> Dict[str, np.ndarray]:
    """SwiGLU expert on de-quantized rows a = s*q: returns g, u, h, o (all float64)."""
    g = codebook_matmul(a_rows, *expert["gate"])
    u = codebook_matmul(a_rows, *expert["up"])
    h = silu(g) * u
    o = codebook_matmul(h, *expert["down"])
    return {"g": g, "u": u, "h": h, "o": o}


# ------------------------------------------------------------------------------------------
# the whole layer
# ------------------------------------------------------------------------------------------
def moe_forward(X: np.ndarray, R: np.ndarray, Wr: np.ndarray, bias: Optional[np.ndarray],
                experts: Sequence[Dict[str, Tuple[np.ndarray, np.ndarray]]],
                n_routed: int, top_k: int, act_bits: int,
                only_tokens: Optional[np.ndarray] = None,
                keep_expert_outputs: bool = False) -> Dict[str, np.ndarray]:
    """Forward pass of one layer.  experts = n_routed routed experts followed by shared experts.

    only_tokens: if given, expert FFNs and Y are evaluated for these token rows only (the front
    end -- rotation, codes, routing, permutation -- is always computed for every token).
    """
    T = X.shape[0]
    XR = rotate(X, R)
    q, scale = quantize(XR, act_bits)
    L = router_logits(XR, Wr, bias)
    ids, w = route_topk(L, top_k)
    offsets, perm, inv_perm = permute_by_expert(ids, n_routed)
    a = scale[:, None] * q.astype(np.float64)

    tok_mask = np.ones(T, dtype=bool)
    if only_tokens is not None:
        tok_mask[:] = False
        tok_mask[np.asarray(only_tokens)] = True

    Y = np.zeros((T, X.shape[1]), dtype=np.float64)
    n_assign = T * top_k
    o_sorted = np.zeros((n_assign, X.shape[1]), dtype=np.float64) if keep_expert_outputs else None
    # routed experts, in the order j = 0..k-1 per token (fixed summation order)
    contrib = np.zeros((T, top_k, X.shape[1]), dtype=np.float64)
    for e in range(n_routed):
        pos = np.arange(offsets[e], offsets[e + 1])
        assign = perm[pos]
        toks = assign // top_k
        keep = tok_mask[toks]
        if not np.any(keep):
            continue
        res = expert_ffn(a[toks[keep]], experts[e])
        contrib[toks[keep], assign[keep] % top_k] = res["o"]
        if keep_expert_outputs:
            o_sorted[pos[keep]] = res["o"]
    for j in range(top_k):
        Y += w[:, j:j + 1] * contrib[:, j]
    shared_o = []
    for s in range(n_routed, len(experts)):
        rows = np.nonzero(tok_mask)[0]
        res = expert_ffn(a[rows], experts[s])
        Y[rows] += res["o"]
        if keep_expert_outputs:
            full = np.zeros((T, X.shape[1]), dtype=np.float64)
            full[rows] = res["o"]
            shared_o.append(full)
    Y[~tok_mask] = 0.0
    out = {"XR": XR, "q": q, "scale": scale, "logits": L, "ids": ids, "w": w,
           "offsets": offsets, "perm": perm, "inv_perm": inv_perm, "Y": Y}
    if keep_expert_outputs:
        out["o_sorted"] = o_sorted
        out["o_shared"] = shared_o
    return out


def unquantized_ffn(X: np.ndarray, Wg: np.ndarray, Wu: np.ndarray, Wd: np.ndarray) -> np.ndarray:
    """Dense SwiGLU FFN with weights in [out, in] layout, no quantization (for invariance pins)."""
    X = np.asarray(X, dtype=np.float64)
    return (silu(X @ Wg.T) * (X @ Wu.T)) @ Wd.T
