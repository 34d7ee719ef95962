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
  decode_*          W_c[i,j] = sum_k C[i,k] A[i,j,k]   ACCF section (Eq. W_c); embedding-wise or block-wise
                                                       tables (experimental setup, g = 1024); budgets of 4 or 8
                                                       centroids (ablation on centroid budgets, W2 / W3)
  expert_ffn        (phi(X W_gate) . X W_up) W_down    AOS section (rotation-invariance equation)
  moe_forward       sum_i Pi_i X_R W_c (+ shared)      ACCF section (Eq. L, MoE case), appendix (shared expert)
  hadamard_*        online Hadamard transform          evaluation section (the "had" variant)

Readings taken where the paper is silent (each is also listed in the design notes):
  * quantization is symmetric and per token: s_t = max_j |X_R[t,j]| / qmax, qmax = 2^(b-1)-1,
    q = clip(rint(X_R / s_t), -qmax, qmax) with round-half-to-even; an all-zero row has s_t = 1;
  * the router reads the un-quantized rotated activations;
  * routing weights are the softmax over the k selected logits (they sum to 1); ids are in
    descending logit order and equal logits go to the lower expert id;
  * tokens are grouped by expert with a stable sort of the assignment number a = t*k + j;
  * the intermediate h is not re-quantized before the down projection, except in the online-Hadamard
    variant (h_bits > 0): there h is multiplied by H_I / sqrt(I), H_I = H_m (x) H_{2^k} with a Paley matrix
    of order m in {12, 28, 44} when I is not a power of two, and quantized per row exactly like X_R;
  * block-wise clustering groups g consecutive weights of a row along d_in; when g does not divide d_in
    the last group of the row is shorter;
  * 2- and 3-bit indices (budgets of 4 and 8 centroids) are packed as a little-endian bit stream per row;
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


def unpack_indices_bits(idx_packed: np.ndarray, bits: int, K: int) -> np.ndarray:
    """[N, K*bits/8] bytes -> [N, K] indices in [0, 2^bits) for the smaller centroid budgets (W2: 4
    centroids, W3: 8; ablation on centroid budgets).  The indices of a row form one little-endian bit
    stream: weight j occupies bits [j*bits, (j+1)*bits) of the row, bit i of the stream being bit i%8 of
    byte i//8.  With bits = 4 this is the nibble order of unpack_indices."""
    p = np.asarray(idx_packed, dtype=np.uint8)
    assert p.shape[1] * 8 == K * bits
    stream = np.unpackbits(p, axis=1, bitorder="little")            # [N, K*bits], stream bit i at column i
    fields = stream.reshape(p.shape[0], K, bits).astype(np.uint8)   # field j = bits j*bits .. j*bits+bits-1
    weights = (np.uint8(1) << np.arange(bits, dtype=np.uint8))
    return (fields * weights[None, None, :]).sum(axis=2).astype(np.uint8)


def decode_weights_budget(idx_packed: np.ndarray, cent_bits: np.ndarray, bits: int, K: int,
                          group_k: int = 0) -> np.ndarray:
    """W_c [N, K] float64 for a budget of 2^bits centroids per table (Eq. W_c with fewer columns in C):
    cent_bits is [N, 2^bits] or, block-wise, [N, ceil(K/g), 2^bits]."""
    idx = unpack_indices_bits(idx_packed, bits, K).astype(np.int64)
    cent = np.asarray(cent_bits)
    C = bf16_bits_to_f64(cent if group_k > 0 else cent[:, None, :])
    assert C.shape[2] == 2 ** bits and C.shape[1] == (-(-K // group_k) if group_k > 0 else 1)
    W = np.empty(idx.shape, dtype=np.float64)
    for b, j0, j1 in _column_groups(K, group_k):
        W[:, j0:j1] = np.take_along_axis(C[:, b], idx[:, j0:j1], axis=1)
    return W


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
def _column_groups(K: int, group_k: int):
    """(table number, first column, end column) of every clustering group along d_in.

    Embedding-wise (group_k = 0; centroids [N, 16]): one table per output row over all of d_in.
    Block-wise (group_k = g > 0; centroids [N, ceil(K/g), 16]): weights are clustered in groups of g
    consecutive values along d_in (experimental setup, g = 1024), so column j of row n uses table
    j // g of that row; the last group of a row is shorter when g does not divide K.
    """
    g = group_k if group_k > 0 else K
    return [(b, j0, min(K, j0 + g)) for b, j0 in enumerate(range(0, K, g))]


def _tables(cent: np.ndarray, K: int, group_k: int) -> np.ndarray:
    """The centroid array as [N, groups, 16] (a view; checks the shape against the grouping)."""
    cent = np.asarray(cent)
    if group_k <= 0:
        assert cent.ndim == 2 and cent.shape[1] == N_CENTROIDS
        return cent[:, None, :]
    assert cent.ndim == 3 and cent.shape[1] == -(-K // group_k) and cent.shape[2] == N_CENTROIDS
    return cent


def decode_weights(idx_packed: np.ndarray, cent_bits: np.ndarray, group_k: int = 0) -> np.ndarray:
    """W_c [N, K] float64: every weight is the centroid its 4-bit index points at (Eq. W_c).
    Tables of 4 or 8 entries (the smaller budgets of the ablation on centroid budgets) mean 2- / 3-bit index
    streams: those go through decode_weights_budget."""
    n_cent = np.asarray(cent_bits).shape[-1]
    if n_cent != N_CENTROIDS:
        bits = {4: 2, 8: 3}[n_cent]
        return decode_weights_budget(idx_packed, cent_bits, bits, np.asarray(idx_packed).shape[1] * 8 // bits, group_k)
    idx = unpack_indices(idx_packed).astype(np.int64)
    K = idx.shape[1]
    C = bf16_bits_to_f64(_tables(cent_bits, K, group_k))
    W = np.empty(idx.shape, dtype=np.float64)
    for b, j0, j1 in _column_groups(K, group_k):
        W[:, j0:j1] = np.take_along_axis(C[:, b], idx[:, j0:j1], axis=1)
    return W


def decode_weights_bf16_bits(idx_packed: np.ndarray, cent_bits: np.ndarray, group_k: int = 0) -> np.ndarray:
    """Same decode, returning the bf16 bit patterns (what a bit-exact decode check compares)."""
    idx = unpack_indices(idx_packed).astype(np.int64)
    K = idx.shape[1]
    C = _tables(np.asarray(cent_bits, dtype=np.uint16), K, group_k)
    W = np.empty(idx.shape, dtype=np.uint16)
    for b, j0, j1 in _column_groups(K, group_k):
        W[:, j0:j1] = np.take_along_axis(C[:, b], idx[:, j0:j1], axis=1)
    return W


def decode_weights_onehot(idx_packed: np.ndarray, cent_bits: np.ndarray, group_k: int = 0) -> np.ndarray:
    """Eq. W_c taken literally: build the one-hot assignment tensor A and contract it with C."""
    idx = unpack_indices(idx_packed)
    N, K = idx.shape
    A = np.zeros((N, K, N_CENTROIDS), dtype=np.float64)
    n, j = np.meshgrid(np.arange(N), np.arange(K), indexing="ij")
    A[n, j, idx] = 1.0
    assert np.all(A.sum(axis=2) == 1.0)
    # one contraction per clustering group of columns, each with its own centroid matrix
    C = bf16_bits_to_f64(_tables(cent_bits, K, group_k))
    W = np.empty((N, K), dtype=np.float64)
    for b, j0, j1 in _column_groups(K, group_k):
        W[:, j0:j1] = np.einsum("nk,njk->nj", C[:, b], A[:, j0:j1])
    return W


def codebook_matmul(A_rows: np.ndarray, idx_packed: np.ndarray, cent_bits: np.ndarray,
                    group_k: int = 0) -> np.ndarray:
    """[M, K] activations times W_c^T -> [M, N]."""
    return np.asarray(A_rows, dtype=np.float64) @ decode_weights(idx_packed, cent_bits, group_k).T


def product_lut_matmul(codes: np.ndarray, idx_packed: np.ndarray, cent_bits: np.ndarray,
                       act_bits: int = 4, group_k: int = 0) -> np.ndarray:
    """The lookup formulation of the kernel section, for integer activation codes.

    For one weight group (a row, or g consecutive columns of a row) the table has one sub-table per
    centroid holding centroid * v for every representable activation value v; a (weight index,
    activation code) pair selects one product and the products are accumulated.  Pure-Python loops:
    tiny inputs only.
    """
    idx = unpack_indices(idx_packed)
    N, K = idx.shape
    g = group_k if group_k > 0 else K
    C = bf16_bits_to_f64(cent_bits).reshape(N, -1, N_CENTROIDS)   # [N, groups, 16]
    lo = -(2 ** (act_bits - 1))
    values = np.arange(lo, -lo, dtype=np.float64)            # all 2^b representable codes
    M = codes.shape[0]
    out = np.zeros((M, N), dtype=np.float64)
    for n in range(N):
        luts = [C[n, b][:, None] * values[None, :] for b in range(C.shape[1])]  # [16 sub-tables, 2^b entries] each
        for m in range(M):
            acc = 0.0
            for j in range(K):
                acc += luts[j // g][idx[n, j], int(codes[m, j]) - lo]
            out[m, n] = acc
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


# ------------------------------------------------------------------------------------------
# online Hadamard transform of the intermediate (the "had" variant of the evaluation section:
# an online Hadamard rotation in front of the down projection, whose input is then quantized
# like any other activation)
# ------------------------------------------------------------------------------------------
def _legendre(x: int, q: int) -> int:
    """Quadratic character of x modulo the odd prime q: 0, +1 (non-zero square) or -1."""
    x %= q
    if x == 0:
        return 0
    return 1 if any((y * y) % q == x for y in range(1, q)) else -1


def paley_hadamard(n: int) -> np.ndarray:
    """Hadamard matrix of order 12 or 44 (Paley's first construction, q = n-1 = 3 mod 4) or 28
    (Paley's second construction, q = 13 = 1 mod 4), entries +-1, int64.

    First construction: H = I + S with the skew matrix S = [[0, 1^T], [-1, Q]], Q[i,j] = chi(j - i).
    Second: H = S (x) [[1,1],[1,-1]] + I (x) [[1,-1],[-1,-1]] with the symmetric 14 x 14 matrix
    S = [[0, 1^T], [1, Q]], Q[i,j] = chi(i - j).
    """
    if n in (12, 44):
        q = n - 1
        S = np.zeros((n, n), dtype=np.int64)
        S[0, 1:] = 1
        S[1:, 0] = -1
        for i in range(q):
            for j in range(q):
                S[1 + i, 1 + j] = _legendre(j - i, q)
        return np.eye(n, dtype=np.int64) + S
    if n == 28:
        q = 13
        S = np.zeros((q + 1, q + 1), dtype=np.int64)
        S[0, 1:] = 1
        S[1:, 0] = 1
        for i in range(q):
            for j in range(q):
                S[1 + i, 1 + j] = _legendre(i - j, q)
        A = np.array([[1, 1], [1, -1]], dtype=np.int64)
        B = np.array([[1, -1], [-1, -1]], dtype=np.int64)
        return np.kron(S, A) + np.kron(np.eye(q + 1, dtype=np.int64), B)
    raise ValueError("no Paley matrix of that order here")


def sylvester_hadamard(n: int) -> np.ndarray:
    """H[i,j] = (-1)^popcount(i & j) for n a power of two (Sylvester's construction, natural order)."""
    assert n >= 1 and n & (n - 1) == 0
    i = np.arange(n)
    bits = i[:, None] & i[None, :]
    par = np.zeros((n, n), dtype=np.int64)
    while np.any(bits):
        par ^= bits & 1
        bits >>= 1
    return 1 - 2 * par


def hadamard_split(n: int) -> Tuple[int, int]:
    """n = m * 2^k with m in {1, 12, 28, 44}: m is 1 for a power of two, else four times the odd part."""
    odd = n
    while odd % 2 == 0:
        odd //= 2
    if odd == 1:
        return 1, n
    m = 4 * odd
    if m not in (12, 28, 44) or n % m != 0:
        raise ValueError(f"no Hadamard matrix of order {n} here")
    return m, n // m


def hadamard_matrix(n: int) -> np.ndarray:
    """H_m (x) H_{2^k} (Kronecker product: index i = a*2^k + b), entries +-1."""
    m, p = hadamard_split(n)
    Hm = np.ones((1, 1), dtype=np.int64) if m == 1 else paley_hadamard(m)
    return np.kron(Hm, sylvester_hadamard(p))


def hadamard_rows(h: np.ndarray) -> np.ndarray:
    """h' = h H_n / sqrt(n) for every row of h (n = row length): an orthogonal change of basis."""
    h = np.asarray(h, dtype=np.float64)
    n = h.shape[1]
    return (h @ hadamard_matrix(n).astype(np.float64)) / np.sqrt(float(n))


def expert_ffn(a_rows: np.ndarray, expert: Dict[str, Tuple[np.ndarray, np.ndarray]],
               h_bits: int = 0, group_k: int = 0) -> Dict[str, np.ndarray]:
    """SwiGLU expert on de-quantized rows a = s*q: returns g, u, h, o (all float64).

    h_bits = 4 or 8: the online-Hadamard variant.  The intermediate is rotated, h' = h H / sqrt(I),
    quantized per row to h_bits like the layer's input, and the down projection (whose weights are
    clustered in that rotated basis) reads the de-quantized codes; hq, hs are returned too.
    group_k > 0: block-wise centroid tables for all three matrices (see centroid_per_weight).
    """
    g = codebook_matmul(a_rows, *expert["gate"], group_k)
    u = codebook_matmul(a_rows, *expert["up"], group_k)
    h = silu(g) * u
    if h_bits:
        hr = hadamard_rows(h)
        hq, hs = quantize(hr, h_bits)
        o = codebook_matmul(hs[:, None] * hq.astype(np.float64), *expert["down"], group_k)
        return {"g": g, "u": u, "h": h, "hr": hr, "hq": hq, "hs": hs, "o": o}
    o = codebook_matmul(h, *expert["down"], group_k)
    return {"g": g, "u": u, "h": h, "o": o}


# ------------------------------------------------------------------------------------------
# the whole layer
# ------------------------------------------------------------------------------------------
def moe_forward(X: np.ndarray, R: np.ndarray, Wr: np.ndarray, bias: Optional[np.ndarray],
                experts: Sequence[Dict[str, Tuple[np.ndarray, np.ndarray]]],
                n_routed: int, top_k: int, act_bits: int,
                only_tokens: Optional[np.ndarray] = None,
                keep_expert_outputs: bool = False, h_bits: int = 0, group_k: int = 0) -> Dict[str, np.ndarray]:
    """Forward pass of one layer.  experts = n_routed routed experts followed by shared experts.

    only_tokens: if given, expert FFNs and Y are evaluated for these token rows only (the front
    end -- rotation, codes, routing, permutation -- is always computed for every token).
    h_bits: 0, or the bit width of the online-Hadamard variant's second quantization (see expert_ffn);
    with keep_expert_outputs the rotated intermediates and their codes come back per sorted row.
    group_k: 0 (one centroid table per weight row) or the block-wise group size g.
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
    n_shared = len(experts) - n_routed
    keep_h = keep_expert_outputs and h_bits
    I = experts[0]["down"][0].shape[1] * 2 if experts else 0
    h_sorted = np.zeros((n_assign + n_shared * T, I), dtype=np.float64) if keep_h else None
    hr_sorted = np.zeros((n_assign + n_shared * T, I), dtype=np.float64) if keep_h else None
    hq_sorted = np.zeros((n_assign + n_shared * T, I), dtype=np.int32) if keep_h else None
    hs_sorted = np.ones(n_assign + n_shared * T, dtype=np.float64) if keep_h else None
    # routed experts, in the order j = 0..k-1 per token (fixed summation order)
    contrib = np.zeros((T, top_k, X.shape[1]), dtype=np.float64)
    for e in range(n_routed):
        pos = np.arange(offsets[e], offsets[e + 1])
        assign = perm[pos]
        toks = assign // top_k
        keep = tok_mask[toks]
        if not np.any(keep):
            continue
        res = expert_ffn(a[toks[keep]], experts[e], h_bits, group_k)
        contrib[toks[keep], assign[keep] % top_k] = res["o"]
        if keep_expert_outputs:
            o_sorted[pos[keep]] = res["o"]
        if keep_h:
            hr_sorted[pos[keep]], hq_sorted[pos[keep]], hs_sorted[pos[keep]] = res["hr"], res["hq"], res["hs"]
            h_sorted[pos[keep]] = res["h"]
    for j in range(top_k):
        Y += w[:, j:j + 1] * contrib[:, j]
    shared_o = []
    for s in range(n_routed, len(experts)):
        rows = np.nonzero(tok_mask)[0]
        res = expert_ffn(a[rows], experts[s], h_bits, group_k)
        Y[rows] += res["o"]
        if keep_h:
            base = n_assign + (s - n_routed) * T
            hr_sorted[base + rows], hq_sorted[base + rows], hs_sorted[base + rows] = res["hr"], res["hq"], res["hs"]
            h_sorted[base + rows] = res["h"]
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
    if keep_h:
        out["hr_sorted"], out["hq_sorted"], out["hs_sorted"] = hr_sorted, hq_sorted, hs_sorted
        out["h_sorted"] = h_sorted
    return out


def unquantized_ffn(X: np.ndarray, Wg: np.ndarray, Wu: np.ndarray, Wd: np.ndarray) -> np.ndarray:
    """Dense SwiGLU FFN with weights in [out, in] layout, no quantization (for invariance pins)."""
    X = np.asarray(X, dtype=np.float64)
    return (silu(X @ Wg.T) * (X @ Wu.T)) @ Wd.T
