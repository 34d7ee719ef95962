"""Pins for the CPU oracle: closed forms, invariants, brute force on tiny inputs, and reductions
to library routines.  The paper prints no numeric example for the forward path, so nothing here
is a quoted value; each test names the passage whose statement it checks.

All of these run without a GPU.
"""
import math

import numpy as np
import pytest
import scipy.linalg
import scipy.special

from oracle import cq_oracle as O
from paper_2604_10496_amd import synth


def _rng(seed=0):
    return np.random.default_rng(seed)


def _bf16(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _pack(idx):
    """[N,K] indices -> packed bytes, written independently of the oracle's unpacker."""
    idx = np.asarray(idx, dtype=np.uint8)
    return (idx[:, 0::2] | (idx[:, 1::2] << 4)).astype(np.uint8)


def _small_expert(rng, H, I):
    def mat(N, K):
        return rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8), synth.draw_centroids(rng, N)
    return {"gate": mat(I, H), "up": mat(I, H), "down": mat(H, I)}


# ------------------------------------------------------------------------------------------
# rotation (AOS section: X_R = X R with R orthogonal; Cayley construction; invariance equation)
# ------------------------------------------------------------------------------------------
def _cayley(rng, H):
    M = rng.standard_normal((H, H))
    S = 0.5 * (M - M.T)
    return (np.eye(H) - S) @ np.linalg.inv(np.eye(H) + S)


@pytest.mark.parametrize("family", ["qr", "cayley", "hadamard"])
def test_rotation_preserves_norms(family):
    rng = _rng(1)
    H = 64
    if family == "qr":
        R = synth.draw_orthogonal(rng, H).astype(np.float64)
        tol = 1e-5  # R was rounded to float32
    elif family == "cayley":
        R = _cayley(rng, H)
        tol = 1e-10
    else:
        R = scipy.linalg.hadamard(H) / math.sqrt(H)
        tol = 1e-12
    X = rng.standard_normal((9, H)) * 10
    XR = O.rotate(X, R)
    assert np.allclose(np.linalg.norm(XR, axis=1), np.linalg.norm(X, axis=1), rtol=tol)
    assert np.allclose(R @ R.T, np.eye(H), atol=max(tol, 1e-12) * 10)


def test_rotation_identity_and_orientation():
    rng = _rng(2)
    X = rng.standard_normal((5, 8)).astype(np.float32)
    assert np.array_equal(O.rotate(X, np.eye(8, dtype=np.float32)), X.astype(np.float64))
    # X R, not X R^T and not R X: a single 1 at R[2,5] moves channel 2 into channel 5
    R = np.zeros((8, 8)); R[2, 5] = 1.0
    XR = O.rotate(X, R)
    assert np.array_equal(XR[:, 5], X[:, 2].astype(np.float64))
    assert np.count_nonzero(XR[:, np.arange(8) != 5]) == 0


def test_rotation_invariance_of_ffn():
    """(phi(X R R^T Wg) . X R R^T Wu) Wd = (phi(X Wg) . X Wu) Wd: fold R^T into dense weights."""
    rng = _rng(3)
    H, I = 32, 48
    R = _cayley(rng, H)
    X = rng.standard_normal((7, H))
    Wg, Wu, Wd = rng.standard_normal((I, H)), rng.standard_normal((I, H)), rng.standard_normal((H, I))
    ref = O.unquantized_ffn(X, Wg, Wu, Wd)
    # weights in [out,in] layout: (R^T W)^T in the paper's [in,out] layout is W_oi R
    rot = O.unquantized_ffn(O.rotate(X, R), Wg @ R, Wu @ R, Wd)
    assert np.allclose(rot, ref, rtol=1e-10, atol=1e-10)


# ------------------------------------------------------------------------------------------
# quantization (integer quantization Q; symmetric per token, round-half-to-even)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_closed_forms(bits):
    rng = _rng(4)
    qmax = 2 ** (bits - 1) - 1
    XR = rng.standard_normal((11, 40)) * rng.uniform(0.1, 30, size=(11, 1))
    q, s = O.quantize(XR, bits)
    j = np.argmax(np.abs(XR), axis=1)
    r = np.arange(11)
    assert np.array_equal(q[r, j], (np.sign(XR[r, j]) * qmax).astype(np.int32))
    assert np.allclose(s, np.abs(XR[r, j]) / qmax, rtol=1e-15)
    assert np.all(np.abs(s[:, None] * q - XR) <= s[:, None] / 2 * (1 + 1e-12))
    assert q.min() >= -qmax and q.max() <= qmax
    # idempotence and homogeneity
    q2, s2 = O.quantize(s[:, None] * q, bits)
    assert np.array_equal(q2, q) and np.allclose(s2, s, rtol=1e-15)
    q3, s3 = O.quantize(2.0 * XR, bits)
    assert np.array_equal(q3, q) and np.allclose(s3, 2 * s, rtol=1e-15)


@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_grid_rows_are_exact(bits):
    rng = _rng(5)
    qmax = 2 ** (bits - 1) - 1
    m = rng.integers(-qmax, qmax + 1, size=(6, 50))
    m[:, 0] = qmax * np.where(rng.random(6) < 0.5, -1, 1)
    c = np.array([0.25, 0.5, 1.0, 3.0, 0.125, 8.0])
    q, s = O.quantize(m * c[:, None], bits)
    assert np.array_equal(q, m)
    assert np.allclose(s, c)


def test_quantize_ties_round_to_even_and_zero_row():
    # scale is exactly 1 (amax = qmax = 7): halves must go to the even neighbour
    row = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 6.5]])
    q, s = O.quantize(row, 4)
    assert s[0] == 1.0
    assert q[0].tolist() == [7, 0, 2, 2, 0, -2, -2, 4, 6]
    q0, s0 = O.quantize(np.zeros((1, 5)), 8)
    assert s0[0] == 1.0 and not q0.any()
    d = O.tie_distance(row, s)
    assert np.all(d[0, 1:] == 0.0) and d[0, 0] == 0.5


def test_rotation_tames_outliers():
    """Why R is there: un-rotated rows have amax far above the typical magnitude, rotated rows do not."""
    L = synth.make_layer(synth.CONFIGS["tiny"], with_experts=False)
    X = L.X.astype(np.float64)
    XR = O.rotate(L.X, L.R)
    ratio_raw = np.max(np.abs(X), axis=1) / np.median(np.abs(X), axis=1)
    ratio_rot = np.max(np.abs(XR), axis=1) / np.median(np.abs(XR), axis=1)
    assert np.median(ratio_raw) > 5 * np.median(ratio_rot)


# ------------------------------------------------------------------------------------------
# routing (router = linear layer, Top-K, weights that sum to one, grouping by expert)
# ------------------------------------------------------------------------------------------
def test_router_logits_is_linear_layer():
    rng = _rng(6)
    XR, Wr, b = rng.standard_normal((5, 12)), rng.standard_normal((7, 12)), rng.standard_normal(7)
    L = O.router_logits(XR, Wr, b)
    for t in range(5):
        for e in range(7):
            assert math.isclose(L[t, e], sum(XR[t, j] * Wr[e, j] for j in range(12)) + b[e],
                                rel_tol=1e-12, abs_tol=1e-12)
    assert np.array_equal(O.router_logits(XR, Wr, None), L - b[None, :]) or \
        np.allclose(O.router_logits(XR, Wr, None), L - b[None, :], atol=1e-13)


def test_topk_brute_force_and_weights():
    rng = _rng(7)
    T, E, k = 40, 12, 5
    L = rng.standard_normal((T, E))
    L[3, 4] = L[3, 9] = L[3].max() + 1.0        # an exact tie at the top: lower id first
    L[5, :] = 0.25                               # all equal: ids 0..k-1
    ids, w = O.route_topk(L, k)
    for t in range(T):
        chosen = []
        avail = list(range(E))
        for _ in range(k):                       # repeated arg-max, first occurrence wins
            best = avail[0]
            for e in avail:
                if L[t, e] > L[t, best]:
                    best = e
            chosen.append(best)
            avail.remove(best)
        assert ids[t].tolist() == chosen
        z = [math.exp(L[t, e]) for e in chosen]
        assert np.allclose(w[t], np.array(z) / sum(z), rtol=1e-12)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-12)
    assert ids[3, :2].tolist() == [4, 9] and ids[5].tolist() == list(range(k))
    # k = E: the weights are the ordinary softmax of all logits
    ids_all, w_all = O.route_topk(L, E)
    sm = scipy.special.softmax(L, axis=1)
    assert np.allclose(w_all, np.take_along_axis(sm, ids_all.astype(np.int64), axis=1), rtol=1e-12)


def test_permutation_is_stable_counting_sort():
    rng = _rng(8)
    T, E, k = 37, 9, 3
    ids = rng.integers(0, E - 1, size=(T, k)).astype(np.int32)   # expert E-1 stays empty
    off, perm, inv = O.permute_by_expert(ids, E)
    flat = ids.reshape(-1)
    expect = []
    for e in range(E):                           # brute force: scan assignments in order per expert
        expect += [a for a in range(T * k) if flat[a] == e]
    assert perm.tolist() == expect
    assert off[0] == 0 and off[E] == T * k and off[E] == off[E - 1]
    assert np.array_equal(np.diff(off), np.bincount(flat, minlength=E))
    assert np.array_equal(inv[perm], np.arange(T * k)) and sorted(perm.tolist()) == list(range(T * k))
    for e in range(E):
        seg = perm[off[e]:off[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)


# ------------------------------------------------------------------------------------------
# index decode (Eq. W_c) and the codebook product
# ------------------------------------------------------------------------------------------
def test_nibble_order_and_bf16_bits():
    # byte 0x3A: weight 0 has index 0xA, weight 1 has index 0x3
    idx = np.array([[0x3A, 0xF0]], dtype=np.uint8)
    assert O.unpack_indices(idx).tolist() == [[0xA, 0x3, 0x0, 0xF]]
    cent = _bf16(np.arange(16, dtype=np.float32)[None, :] * 0.5 - 2.0)
    assert O.decode_weights(idx, cent).tolist() == [[3.0, -0.5, -2.0, 5.5]]
    # bf16 pattern 0x3F80 is 1.0, 0xC000 is -2.0, 0x3DCD is 0.10009765625
    assert O.bf16_bits_to_f64(np.array([0x3F80, 0xC000, 0x3DCD], dtype=np.uint16)).tolist() == \
        [1.0, -2.0, 0.10009765625]


def test_three_decode_formulations_agree():
    rng = _rng(9)
    N, K, M = 6, 16, 3
    idx = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    packed = _pack(idx)
    cent = synth.draw_centroids(rng, N)
    W1 = O.decode_weights(packed, cent)
    W2 = O.decode_weights_onehot(packed, cent)
    C = O.bf16_bits_to_f64(cent)
    W3 = np.array([[C[n, idx[n, j]] for j in range(K)] for n in range(N)])
    assert np.array_equal(W1, W2) and np.array_equal(W1, W3)
    assert np.array_equal(O.decode_weights_bf16_bits(packed, cent),
                          np.array([[cent[n, idx[n, j]] for j in range(K)] for n in range(N)]))
    codes = rng.integers(-7, 8, size=(M, K))
    lut = O.product_lut_matmul(codes, packed, cent, act_bits=4)
    gemm = O.codebook_matmul(codes, packed, cent)
    assert np.allclose(lut, gemm, rtol=1e-12, atol=1e-15)


def test_blockwise_tables():
    """Block-wise clustering (experimental setup): column j of a row uses that row's table j // g."""
    rng = _rng(19)
    N, K, M, g = 5, 40, 3, 16                    # three groups per row, the last one of 8 columns
    idx = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    packed = _pack(idx)
    cent = synth.draw_centroids(rng, N, n_blocks=3)
    assert cent.shape == (N, 3, 16)
    C = O.bf16_bits_to_f64(cent)
    brute = np.array([[C[n, j // g, idx[n, j]] for j in range(K)] for n in range(N)])
    W = O.decode_weights(packed, cent, g)
    assert np.array_equal(W, brute)
    assert np.array_equal(O.decode_weights_onehot(packed, cent, g), brute)
    assert np.array_equal(O.decode_weights_bf16_bits(packed, cent, g),
                          np.array([[cent[n, j // g, idx[n, j]] for j in range(K)] for n in range(N)]))
    # a block-wise product is the sum of embedding-wise products over the column groups
    A = rng.standard_normal((M, K))
    parts = sum(O.codebook_matmul(A[:, j0:j0 + g], packed[:, j0 // 2:(j0 + g) // 2], cent[:, b])
                for b, j0 in enumerate(range(0, K, g)))
    assert np.allclose(O.codebook_matmul(A, packed, cent, g), parts, rtol=1e-12, atol=1e-15)
    # the same table in every group, or one group spanning the row, is the embedding-wise setting
    rep = np.repeat(cent[:, :1], 3, axis=1)
    assert np.array_equal(O.decode_weights(packed, rep, g), O.decode_weights(packed, cent[:, 0]))
    assert np.array_equal(O.decode_weights(packed, cent[:, :1], K), O.decode_weights(packed, cent[:, 0]))
    # changing one group's table changes exactly that group's columns
    other = cent.copy()
    other[:, 1] = synth.draw_centroids(rng, N)
    diff = O.decode_weights(packed, other, g) != W
    assert not diff[:, :g].any() and not diff[:, 2 * g:].any() and diff[:, g:2 * g].any()
    # lookup formulation with one product table per (row, group)
    codes = rng.integers(-7, 8, size=(M, K))
    assert np.allclose(O.product_lut_matmul(codes, packed, cent, act_bits=4, group_k=g),
                       O.codebook_matmul(codes, packed, cent, g), rtol=1e-12, atol=1e-15)


def test_blockwise_layer_matches_dense():
    """The block-wise layer equals the dense SwiGLU FFN on brute-force decoded matrices."""
    cfg = synth.small_variant(synth.CONFIGS["tiny"], H=64, I=96, T=5, E=2, top_k=1, group_k=32,
                              outlier_channels=(3,), n_outliers=1)
    L = synth.make_layer(cfg)
    assert L.experts[0]["gate"][1].shape == (96, 2, 16) and L.experts[0]["down"][1].shape == (64, 3, 16)
    res = O.moe_forward(L.X, L.R, L.Wr, L.bias, L.experts, cfg.E, cfg.top_k, cfg.act_bits, group_k=32)
    a = res["scale"][:, None] * res["q"]
    def dense(mat, K):
        idx = O.unpack_indices(mat[0])
        C = O.bf16_bits_to_f64(mat[1])
        return np.array([[C[n, j // 32, idx[n, j]] for j in range(K)] for n in range(idx.shape[0])])
    for t in range(cfg.T):
        e = L.experts[int(res["ids"][t, 0])]
        y = O.unquantized_ffn(a[t:t + 1], dense(e["gate"], 64), dense(e["up"], 64), dense(e["down"], 96))
        assert np.allclose(res["Y"][t], y[0], rtol=1e-10, atol=1e-12)


def test_smaller_centroid_budgets():
    """W2 / W3: 4 or 8 centroids, indices as a little-endian bit stream per row."""
    # hand-made bytes.  2 bits: 0b11_10_01_00 = 0xE4 holds weights 0,1,2,3 = 0,1,2,3.
    assert O.unpack_indices_bits(np.array([[0xE4, 0x1B]], dtype=np.uint8), 2, 8).tolist() == [[0, 1, 2, 3, 3, 2, 1, 0]]
    # 3 bits: weights 0..7 = 0..7 -> stream 000 100 010 110 001 101 011 111 (LSB first) = bytes 0x88 0xC6 0xFA
    assert O.unpack_indices_bits(np.array([[0x88, 0xC6, 0xFA]], dtype=np.uint8), 3, 8).tolist() == \
        [[0, 1, 2, 3, 4, 5, 6, 7]]
    rng = _rng(23)
    N, K = 5, 64
    for bits in (2, 3, 4):
        idx = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
        packed = synth.pack_indices_bits(idx, bits)
        assert packed.shape == (N, K * bits // 8)
        assert np.array_equal(O.unpack_indices_bits(packed, bits, K), idx)
        # brute force over the bit stream
        for n in (0, N - 1):
            big = int.from_bytes(packed[n].tobytes(), "little")
            assert [(big >> (j * bits)) & ((1 << bits) - 1) for j in range(K)] == idx[n].tolist()
    # 4 bits: the same bytes as the nibble packing used everywhere else
    idx4 = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    assert np.array_equal(synth.pack_indices_bits(idx4, 4), _pack(idx4))
    assert np.array_equal(O.unpack_indices_bits(_pack(idx4), 4, K), O.unpack_indices(_pack(idx4)))
    # decode: brute force, embedding-wise and block-wise
    for bits, g in ((2, 0), (3, 0), (3, 32), (2, 48)):
        nblk = -(-K // g) if g else 0
        idx = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
        cent = synth.draw_centroids(rng, N, n_blocks=nblk)[..., :1 << bits]
        C = O.bf16_bits_to_f64(cent)
        brute = np.array([[(C[n, j // g, idx[n, j]] if g else C[n, idx[n, j]]) for j in range(K)] for n in range(N)])
        assert np.array_equal(O.decode_weights_budget(synth.pack_indices_bits(idx, bits), cent, bits, K, g), brute)
    # a 4-bit table whose upper entries are never addressed decodes to the same matrix
    idx = rng.integers(0, 4, size=(N, K), dtype=np.uint8)
    cent16 = synth.draw_centroids(rng, N)
    assert np.array_equal(O.decode_weights_budget(synth.pack_indices_bits(idx, 2), cent16[:, :4], 2, K),
                          O.decode_weights(_pack(idx), cent16))


def test_codebook_matmul_special_cases():
    rng = _rng(10)
    N, K, M = 10, 64, 4
    packed = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    A = rng.standard_normal((M, K))
    # (i) every centroid of a row equal -> W_c = c 1^T -> rank one: out[m,n] = c_n * sum_j A[m,j]
    c = rng.standard_normal(N).astype(np.float32)
    cent = np.repeat(_bf16(c)[:, None], 16, axis=1)
    cv = O.bf16_bits_to_f64(cent[:, 0])
    assert np.allclose(O.codebook_matmul(A, packed, cent), A.sum(axis=1)[:, None] * cv[None, :], rtol=1e-12)
    # (iii) every index equal k0 -> same thing with column k0 of the table
    cent2 = synth.draw_centroids(rng, N)
    k0 = 11
    same = np.full((N, K // 2), k0 | (k0 << 4), dtype=np.uint8)
    assert np.allclose(O.codebook_matmul(A, same, cent2),
                       A.sum(axis=1)[:, None] * O.bf16_bits_to_f64(cent2[:, k0])[None, :], rtol=1e-12)
    # (ii) integer centroids k-8 and integer codes: exact integer result
    cent3 = np.repeat(_bf16(np.arange(16, dtype=np.float32) - 8.0)[None, :], N, axis=0)
    codes = rng.integers(-127, 128, size=(M, K))
    idx = O.unpack_indices(packed).astype(np.int64)
    expect = np.array([[int(sum(int(codes[m, j]) * (int(idx[n, j]) - 8) for j in range(K)))
                        for n in range(N)] for m in range(M)])
    assert np.array_equal(O.codebook_matmul(codes, packed, cent3), expect.astype(np.float64))
    # orientation: out[m, n] pairs activation row m with weight row n
    out = O.codebook_matmul(A, packed, cent2)
    W = O.decode_weights(packed, cent2)
    assert math.isclose(out[2, 7], float(np.dot(A[2], W[7])), rel_tol=1e-12)


# ------------------------------------------------------------------------------------------
# SwiGLU expert, weighted combine, shared experts
# ------------------------------------------------------------------------------------------
def test_silu_closed_forms():
    x = np.array([-30.0, -2.0, 0.0, 1.0, 5.0])
    y = O.silu(x)
    assert y[2] == 0.0
    assert np.allclose(y - O.silu(-x), x, rtol=1e-12)           # silu(x) - silu(-x) = x
    assert math.isclose(y[3], 1.0 / (1.0 + math.exp(-1.0)), rel_tol=1e-15)
    assert np.allclose(y, x * scipy.special.expit(x), rtol=1e-12)


def test_hand_worked_layer():
    """A two-token layer small enough to evaluate by hand; the expected values are closed forms."""
    R = np.array([[0.0, 1.0], [-1.0, 0.0]], dtype=np.float32)
    X = np.array([[7.0, 0.0], [0.0, -3.5]], dtype=np.float32)
    # X R = [[0, 7], [3.5, 0]]; 4-bit codes [[0, 7], [7, 0]] with scales 1 and 0.5
    Wr = np.eye(2, dtype=np.float32)            # logits = X R: token 0 -> expert 1, token 1 -> expert 0
    table = (np.arange(16, dtype=np.float32) - 8.0) / 4.0     # index i <-> value (i-8)/4
    cent = np.repeat(_bf16(table)[None, :], 2, axis=0)

    def mat(values):                             # dense [N,K] of table values -> (packed idx, cent)
        idx = (np.asarray(values) * 4 + 8).astype(np.uint8)
        return _pack(idx), cent

    Wg = [[1.0, 0.0], [0.5, -1.0]]
    Wu = [[0.25, 1.0], [-0.5, 0.75]]
    Wd = [[1.0, -1.0], [0.5, 0.25]]
    e0 = {"gate": mat(Wg), "up": mat(Wu), "down": mat(Wd)}
    e1 = {"gate": mat(Wu), "up": mat(Wg), "down": mat(Wd)}
    out = O.moe_forward(X, R, Wr, None, [e0, e1], n_routed=2, top_k=1, act_bits=4)
    assert out["XR"].tolist() == [[0.0, 7.0], [3.5, 0.0]]
    assert out["q"].tolist() == [[0, 7], [7, 0]] and out["scale"].tolist() == [1.0, 0.5]
    assert out["ids"].tolist() == [[1], [0]] and out["w"].tolist() == [[1.0], [1.0]]
    assert out["offsets"].tolist() == [0, 1, 2] and out["perm"].tolist() == [1, 0]

    def sl(v):
        return v / (1.0 + math.exp(-v))
    # token 1 -> expert 0 with a = (3.5, 0): g = (3.5, 1.75), u = (0.875, -1.75)
    h = [sl(3.5) * 0.875, sl(1.75) * -1.75]
    y1 = [h[0] - h[1], 0.5 * h[0] + 0.25 * h[1]]
    # token 0 -> expert 1 (gate and up swapped) with a = (0, 7): g = (7, 5.25), u = (0, -7)
    h = [sl(7.0) * 0.0, sl(5.25) * -7.0]
    y0 = [h[0] - h[1], 0.5 * h[0] + 0.25 * h[1]]
    assert np.allclose(out["Y"], np.array([y0, y1]), rtol=1e-14)


def _brute_layer(L, cfg, act_bits):
    """Token-by-token evaluation with Python-level control flow (independent of moe_forward)."""
    X, R = L.X.astype(np.float64), L.R.astype(np.float64)
    qmax = 2 ** (act_bits - 1) - 1
    dense = [{m: O.decode_weights_onehot(*e[m]) for m in ("gate", "up", "down")} for e in L.experts]
    Y = np.zeros((cfg.T, cfg.H))
    for t in range(cfg.T):
        xr = X[t] @ R
        s = np.max(np.abs(xr)) / qmax
        a = s * np.clip(np.rint(xr / s), -qmax, qmax)
        logit = L.Wr.astype(np.float64) @ xr
        if L.bias is not None:
            logit = logit + L.bias
        order = sorted(range(cfg.E), key=lambda e: (-logit[e], e))[: cfg.top_k]
        z = np.exp(logit[order] - logit[order[0]])
        wts = z / z.sum()

        def ffn(e):
            g, u = dense[e]["gate"] @ a, dense[e]["up"] @ a
            return dense[e]["down"] @ (g * scipy.special.expit(g) * u)
        for wt, e in zip(wts, order):
            Y[t] += wt * ffn(e)
        for s_id in range(cfg.E, cfg.E + cfg.S):
            Y[t] += ffn(s_id)
    return Y


@pytest.mark.parametrize("shared,bits,k", [(0, 8, 2), (2, 4, 3), (0, 4, 1)])
def test_moe_forward_against_token_loop(shared, bits, k):
    cfg = synth.small_variant(synth.CONFIGS["tiny"], E=5, top_k=k, S=shared, H=32, I=48, T=9,
                              act_bits=bits, outlier_channels=(3, 7))
    L = synth.make_layer(cfg)
    out = O.moe_forward(L.X, L.R, L.Wr, L.bias, L.experts, cfg.E, cfg.top_k, bits, keep_expert_outputs=True)
    Y = _brute_layer(L, cfg, bits)
    assert np.allclose(out["Y"], Y, rtol=1e-11, atol=1e-13)
    if k == 1 and shared == 0:                   # k = 1: the output is the single expert's output
        assert np.allclose(out["Y"], out["o_sorted"][out["inv_perm"]], rtol=1e-14)
    # only_tokens evaluates a subset of rows to the same values
    sub = O.moe_forward(L.X, L.R, L.Wr, L.bias, L.experts, cfg.E, cfg.top_k, bits, only_tokens=np.array([1, 4]))
    assert np.allclose(sub["Y"][[1, 4]], out["Y"][[1, 4]], rtol=1e-13)
    assert not sub["Y"][[0, 2, 3]].any()


# ------------------------------------------------------------------------------------------
# online Hadamard variant
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n", [12, 28, 44])
def test_paley_matrices_are_hadamard(n):
    """Defining property H H^T = n I in exact integers; Paley I gives I + skew, Paley II a symmetric matrix."""
    H = O.paley_hadamard(n)
    assert H.shape == (n, n) and set(np.unique(H).tolist()) == {-1, 1}
    assert np.array_equal(H @ H.T, n * np.eye(n, dtype=np.int64))
    S = H - np.eye(n, dtype=np.int64)
    if n == 28:
        assert np.array_equal(H, H.T)
    else:
        assert np.array_equal(S, -S.T) and np.all(H[0] == 1)


def test_sylvester_matches_library_and_recursion():
    for n in (1, 2, 8, 64, 512):
        H = O.sylvester_hadamard(n)
        assert np.array_equal(H, scipy.linalg.hadamard(n))          # library routine
        if n > 1:
            h = O.sylvester_hadamard(n // 2)
            assert np.array_equal(H, np.block([[h, h], [h, -h]]))    # textbook recursion


@pytest.mark.parametrize("n,split", [(512, (1, 512)), (768, (12, 64)), (1408, (44, 32)), (14336, (28, 512))])
def test_hadamard_split_and_kronecker_structure(n, split):
    assert O.hadamard_split(n) == split
    if n <= 1408:
        H = O.hadamard_matrix(n)
        assert np.array_equal(H @ H.T, n * np.eye(n, dtype=np.int64))
        m, p = split
        a, b, a2, b2 = 3 % m, 5 % p, 7 % m, 11 % p
        Hm = np.ones((1, 1), dtype=np.int64) if m == 1 else O.paley_hadamard(m)
        assert H[a * p + b, a2 * p + b2] == Hm[a, a2] * (-1) ** bin(b & b2).count("1")
    with pytest.raises(ValueError):
        O.hadamard_split(5 * 64)


def _fwht_loop(v):
    """Fast Walsh-Hadamard transform written as the textbook butterfly loop (power-of-two length)."""
    v = [float(x) for x in v]
    h = 1
    while h < len(v):
        for i in range(0, len(v), 2 * h):
            for j in range(i, i + h):
                v[j], v[j + h] = v[j] + v[j + h], v[j] - v[j + h]
        h *= 2
    return v


def test_hadamard_rows_against_butterfly_and_orthogonality():
    rng = np.random.default_rng(11)
    h = rng.standard_normal((3, 64))
    got = O.hadamard_rows(h)
    for r in range(3):
        assert np.allclose(got[r], np.asarray(_fwht_loop(h[r])) / 8.0, rtol=0, atol=1e-12)
    assert np.allclose(O.hadamard_rows(got), h, atol=1e-12)              # symmetric orthogonal: an involution
    for n in (768, 1408):
        x = rng.standard_normal((2, n))
        y = O.hadamard_rows(x)
        assert np.allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)
        # mixed order: block a of the result = sum_a' Hm[a', a] * FWHT(block a') / sqrt(n)
        m, p = O.hadamard_split(n)
        Hm = O.paley_hadamard(m)
        blocks = np.stack([np.asarray(_fwht_loop(x[0, a * p:(a + 1) * p])) for a in range(m)])
        want = (Hm.T.astype(np.float64) @ blocks).reshape(-1) / math.sqrt(n)
        assert np.allclose(y[0], want, atol=1e-10)
    e = np.zeros((1, 768)); e[0, 5] = 1.0                                  # a unit vector picks out a row of H
    assert np.allclose(O.hadamard_rows(e)[0] * math.sqrt(768), O.hadamard_matrix(768)[5])


def test_online_hadamard_ffn_reduces_to_plain_ffn_without_rounding():
    """With a down projection whose dense weights are W H / sqrt(I) the rotation cancels (orthogonality):
    the had variant evaluated without the second rounding equals the plain FFN on W."""
    rng = np.random.default_rng(12)
    I, H, n = 64, 8, 5
    h = rng.standard_normal((n, I))
    W = rng.standard_normal((H, I))
    Wrot = O.hadamard_rows(W)                 # rows of W in the rotated basis
    assert np.allclose(O.hadamard_rows(h) @ Wrot.T, h @ W.T, atol=1e-12)


@pytest.mark.parametrize("h_bits", [4, 8])
def test_online_hadamard_expert_and_layer_consistency(h_bits):
    cfg = synth.small_variant(synth.CONFIGS["tiny"], T=6, H=64, I=96, E=3, top_k=2, outlier_channels=(3, 41))   # I = 12 * 8
    L = synth.make_layer(cfg)
    a = np.random.default_rng(13).standard_normal((4, cfg.H))
    res = O.expert_ffn(a, L.experts[0], h_bits)
    plain = O.expert_ffn(a, L.experts[0])
    assert np.array_equal(res["h"], plain["h"])
    hq, hs = O.quantize(O.hadamard_rows(plain["h"]), h_bits)
    assert np.array_equal(res["hq"], hq) and np.array_equal(res["hs"], hs)
    W = O.decode_weights(*L.experts[0]["down"])
    assert np.allclose(res["o"], (hs[:, None] * hq) @ W.T, rtol=1e-12, atol=1e-12)
    qmax = 2 ** (h_bits - 1) - 1
    assert np.abs(hq).max() == qmax
    # the layer: token-by-token evaluation with the same functions
    out = O.moe_forward(L.X, L.R, L.Wr, L.bias, L.experts, cfg.E, cfg.top_k, cfg.act_bits, h_bits=h_bits,
                        keep_expert_outputs=True)
    aq = out["scale"][:, None] * out["q"]
    for t in range(cfg.T):
        y = np.zeros(cfg.H)
        for j in range(cfg.top_k):
            y += out["w"][t, j] * O.expert_ffn(aq[t:t + 1], L.experts[out["ids"][t, j]], h_bits)["o"][0]
        assert np.allclose(out["Y"][t], y, rtol=1e-12, atol=1e-12)
    assert out["hq_sorted"].shape == (cfg.T * cfg.top_k, cfg.I) and np.abs(out["hq_sorted"]).max() == qmax


@pytest.mark.parametrize("h_bits", [4, 8])
def test_online_hadamard_expert_against_a_dense_ffn_with_the_quantizer_bound(h_bits):
    """The h_bits branch of expert_ffn as a whole, against quantities built WITHOUT the oracle's Hadamard,
    quantizer or decode routines: SciPy's Hadamard matrix, a loop-decoded dense down matrix and plain matmuls.
    With h' = h H / sqrt(I) exact, every de-quantized code is within s/2 of h'_i (s = max|h'| / qmax), so
    |o[n] - sum_i W[n,i] h'_i| <= (s/2) sum_i |W[n,i]|; the arg-max element is represented exactly, the bound is
    not vacuous (the rounding really happens), and the variant differs from the plain FFN on the same weights
    (the rotation really is applied in front of the down projection)."""
    import scipy.linalg
    cfg = synth.small_variant(synth.CONFIGS["tiny"], T=4, H=64, I=128, E=2, top_k=1, outlier_channels=(3, 41))   # I a power of two
    L = synth.make_layer(cfg)
    rng = np.random.default_rng(99)
    a = rng.standard_normal((5, cfg.H))
    res = O.expert_ffn(a, L.experts[1], h_bits)

    def dense(pair):   # Eq. W_c by loops: row n, weight j -> centroid table entry of its 4-bit index
        idx, cent = pair
        c = synth.bf16_bits_to_f32(cent).astype(np.float64)
        W = np.empty((idx.shape[0], idx.shape[1] * 2))
        for n in range(idx.shape[0]):
            for j in range(idx.shape[1]):
                W[n, 2 * j], W[n, 2 * j + 1] = c[n, idx[n, j] & 15], c[n, idx[n, j] >> 4]
        return W
    Wg, Wu, Wd = dense(L.experts[1]["gate"]), dense(L.experts[1]["up"]), dense(L.experts[1]["down"])
    g, u = a @ Wg.T, a @ Wu.T
    h = g / (1.0 + np.exp(-g)) * u
    hr = h @ scipy.linalg.hadamard(cfg.I).astype(np.float64) / math.sqrt(cfg.I)
    o_exact = hr @ Wd.T
    qmax = 2 ** (h_bits - 1) - 1
    s = np.abs(hr).max(axis=1) / qmax
    bound = 0.5 * s[:, None] * np.abs(Wd).sum(axis=1)[None, :]
    dev = np.abs(res["o"] - o_exact)
    assert np.all(dev <= bound * (1 + 1e-9) + 1e-12)
    assert dev.max() > 1e-3 * bound.max()                       # the second quantizer is really there
    assert np.allclose(res["hs"], s, rtol=1e-12)
    assert np.all(np.abs(res["hs"][:, None] * res["hq"] - hr) <= 0.5 * s[:, None] * (1 + 1e-9))
    assert np.array_equal(np.abs(res["hq"]).max(axis=1), np.full(5, qmax))
    # without the rotation the same weights give something else entirely
    assert np.abs(res["o"] - h @ Wd.T).max() > 2 * bound.max()


def test_decode_weights_takes_the_smaller_budgets_by_table_width():
    """Tables of four entries = the W2 budget, 2-bit indices as a little-endian bit stream: checked against
    loops over bytes and bit fields, and through the layer generator's W2 variant (expert_ffn on such weights
    equals the dense FFN on the loop-decoded matrices)."""
    rng = np.random.default_rng(202)
    N, K = 6, 32
    packed = rng.integers(0, 256, size=(N, K // 4), dtype=np.uint8)
    cent = synth.f32_to_bf16_bits(rng.standard_normal((N, 4)).astype(np.float32))
    W = O.decode_weights(packed, cent)
    c = synth.bf16_bits_to_f32(cent).astype(np.float64)
    for n in range(N):
        for j in range(K):
            want = c[n, (int(packed[n, j // 4]) >> (2 * (j % 4))) & 3]
            assert W[n, j] == want
    cfg = synth.small_variant(synth.CONFIGS["tiny"], T=4, H=64, I=128, E=2, top_k=1, outlier_channels=(3, 41),
                              index_bits=2)
    L = synth.make_layer(cfg)
    gi, gc = L.experts[0]["gate"]
    assert gi.shape == (cfg.I, cfg.H // 4) and gc.shape == (cfg.I, 4) and np.all(np.diff(synth.bf16_bits_to_f32(gc), axis=1) >= 0)

    def dense(pair):
        idx, cb = pair
        cc = synth.bf16_bits_to_f32(cb).astype(np.float64)
        Wd = np.empty((idx.shape[0], idx.shape[1] * 4))
        for n in range(idx.shape[0]):
            for j in range(Wd.shape[1]):
                Wd[n, j] = cc[n, (int(idx[n, j // 4]) >> (2 * (j % 4))) & 3]
        return Wd
    a = rng.standard_normal((3, cfg.H))
    g, u = a @ dense(L.experts[0]["gate"]).T, a @ dense(L.experts[0]["up"]).T
    want = (g / (1.0 + np.exp(-g)) * u) @ dense(L.experts[0]["down"]).T
    assert np.allclose(O.expert_ffn(a, L.experts[0])["o"], want, rtol=1e-12, atol=1e-12)


def test_generator_properties():
    cfg = synth.CONFIGS["tiny"]
    L = synth.make_layer(cfg)
    L2 = synth.make_layer(cfg)
    assert np.array_equal(L.X, L2.X) and np.array_equal(L.experts[3]["down"][0], L2.experts[3]["down"][0])
    cent = synth.bf16_bits_to_f32(L.experts[0]["gate"][1])
    assert np.all(np.diff(cent, axis=1) >= 0)                   # tables stay sorted
    big = np.max(np.abs(cent), axis=1) > 0.2
    assert 1 <= big.sum() <= math.ceil(0.01 * cfg.I) + 1        # about 1 % outlier rows
    assert np.allclose(L.R.astype(np.float64) @ L.R.astype(np.float64).T, np.eye(cfg.H), atol=1e-5)
    # bf16 rounding is to nearest even
    x = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20], dtype=np.float32)
    assert synth.f32_to_bf16_bits(x).tolist() == [0x3F80, 0x3F82, 0x3F81]
    z = synth.make_layer(synth.small_variant(synth.CONFIGS["qwen3_zipf"], T=4, H=64, I=64, E=16), with_experts=False)
    assert z.bias is not None and z.bias.shape == (16,) and np.all(z.bias <= 0)
