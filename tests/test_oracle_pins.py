"""Pins of the CPU oracle to things other than itself (no GPU).

The oracle (oracle/gemm_oracle.c) is the definition the GPU library is graded
against, so it is checked here against: hand-worked products, exact integer
brute force written independently in pure Python, identity matrices, the
transpose identity, linearity, closed forms, finite differences of the forward
product (ties both backward products to the one forward definition) and numpy's
fp64 matmul.  Each test is chosen so that a wrong index map, a transposed
operand, a dropped k term or a wrong mode would fail it.
"""
import os

import numpy as np
import pytest

from paper_2502_08145_amd import synth

LAYOUTS = ["NN", "NT", "TN"]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tiny_products.txt")


def bits(x):
    """Exact small-integer / power-of-two valued array -> bf16 bits (asserts exactness)."""
    x = np.asarray(x, dtype=np.float32)
    b = synth.f32_to_bf16_bits(x)
    assert np.array_equal(synth.bf16_bits_to_f32(b), x), "test value not exact in bf16"
    return b.reshape(x.shape)


def store(a_mk, b_kn, layout):
    """Store logical A[M,K], B[K,N] (bit arrays) the way `layout` wants them."""
    if layout == "NN":
        return a_mk, b_kn
    if layout == "NT":
        return a_mk, np.ascontiguousarray(b_kn.T)
    return np.ascontiguousarray(a_mk.T), b_kn


def brute_force_int(a, b):
    """Pure-Python exact integer product of integer lists-of-lists: no numpy, no oracle."""
    M, K, N = len(a), len(b), len(b[0])
    out = [[0] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            s = 0
            for k in range(K):
                s += int(a[i][k]) * int(b[k][j])
            out[i][j] = s
    return out


# ---------------------------------------------------------------- golden file
def _parse_golden():
    cases, cur = {}, None
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            if line.startswith("case"):
                cur = {}
                cases[line.split()[1]] = cur
                continue
            name, rhs = line.split("=")
            cur[name.strip()] = np.array([[float(v) for v in row.split()] for row in rhs.split(";")])
    return cases


@pytest.mark.parametrize("case", sorted(_parse_golden()))
def test_hand_worked_products(oracle_mod, case):
    g = _parse_golden()[case]
    I, W, dO = bits(g["I"]), bits(g["W"]), bits(g["dO"])
    T, d_in = I.shape
    d_out = W.shape[1]
    # natural modes with the cached buffers: fwd NN, bwd_data NT, bwd_weight TN
    assert np.array_equal(oracle_mod.linear_fwd(T, d_out, d_in, "NN", I, W), g["O"])
    assert np.array_equal(oracle_mod.linear_bwd_data(T, d_in, d_out, "NT", dO, W), g["dI"])
    assert np.array_equal(oracle_mod.linear_bwd_weight(d_in, d_out, T, "TN", I, dO), g["dW"])


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 2, 2), (3, 5, 7), (17, 1, 33), (1, 64, 1), (5, 3, 2)])
def test_brute_force_exact_integers(oracle_mod, layout, shape):
    M, N, K = shape
    a = synth.bf16_bits_to_f32(synth.integer_bf16(11 + M, (M, K), -7, 7)).astype(int)
    b = synth.bf16_bits_to_f32(synth.integer_bf16(23 + N, (K, N), -7, 7)).astype(int)
    want = np.array(brute_force_int(a.tolist(), b.tolist()), dtype=np.float64)
    A, B = store(bits(a), bits(b), layout)
    got = oracle_mod.gemm(M, N, K, layout, A, B)
    assert got.shape == (M, N)
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- identity
@pytest.mark.parametrize("layout", LAYOUTS)
def test_identity_right_and_left(oracle_mod, layout):
    M, K = 5, 9
    a_bits = synth.normal_bf16(7, (M, K))           # asymmetric, M != K
    a = synth.bf16_bits_to_f32(a_bits).astype(np.float64)
    eye_k = bits(np.eye(K))
    A, B = store(a_bits, eye_k, layout)
    assert np.array_equal(oracle_mod.gemm(M, K, K, layout, A, B), a)          # A . I = A
    eye_m = bits(np.eye(M))
    A, B = store(eye_m, a_bits, layout)
    assert np.array_equal(oracle_mod.gemm(M, K, M, layout, A, B), a)          # I . A = A


@pytest.mark.parametrize("layout", LAYOUTS)
def test_shifted_identity_catches_transposed_operand(oracle_mod, layout):
    # P is a cyclic shift (not symmetric): (A.P)[i,j] = A[i, j-1].  Using P^T instead gives j+1.
    M, K = 4, 6
    a_bits = synth.normal_bf16(8, (M, K))
    a = synth.bf16_bits_to_f32(a_bits).astype(np.float64)
    P = np.roll(np.eye(K), 1, axis=1)
    A, B = store(a_bits, bits(P), layout)
    assert np.array_equal(oracle_mod.gemm(M, K, K, layout, A, B), np.roll(a, 1, axis=1))


# ---------------------------------------------------------------- transpose identity
def test_transpose_identity_and_mode_agreement(oracle_mod):
    M, N, K = 13, 7, 29
    a_bits = synth.normal_bf16(31, (M, K))
    b_bits = synth.normal_bf16(32, (K, N), 0.02)
    c_nn = oracle_mod.gemm(M, N, K, "NN", a_bits, b_bits)
    # (A.B)^T = B^T . A^T : same terms in the same k order -> bit-identical fp64
    c_t = oracle_mod.gemm(N, M, K, "NN", np.ascontiguousarray(b_bits.T), np.ascontiguousarray(a_bits.T))
    assert np.array_equal(c_nn.T, c_t)
    for layout in ("NT", "TN"):
        A, B = store(a_bits, b_bits, layout)
        assert np.array_equal(oracle_mod.gemm(M, N, K, layout, A, B), c_nn)
    # and the mixed-mode forms of the transposed product: C^T = B^T A^T
    # NT call with first = B^T [N,K], second stored [M,K] = A
    assert np.array_equal(oracle_mod.gemm(N, M, K, "NT", np.ascontiguousarray(b_bits.T), a_bits), c_nn.T)
    # TN call with first stored [K,N] = B, second [K,M] = A^T
    assert np.array_equal(oracle_mod.gemm(N, M, K, "TN", b_bits, np.ascontiguousarray(a_bits.T)), c_nn.T)


# ---------------------------------------------------------------- linearity
@pytest.mark.parametrize("layout", LAYOUTS)
def test_linearity_exact(oracle_mod, layout):
    M, N, K = 6, 5, 11
    a1 = synth.bf16_bits_to_f32(synth.integer_bf16(41, (M, K), -3, 3))
    a2 = synth.bf16_bits_to_f32(synth.integer_bf16(42, (M, K), -3, 3))
    b = synth.integer_bf16(43, (K, N), -3, 3)
    alpha, beta = 4.0, 0.5
    comb = alpha * a1 + beta * a2          # multiples of 0.5 up to 13.5: exact in bf16

    def run(a):
        A, B = store(bits(a), b, layout)
        return oracle_mod.gemm(M, N, K, layout, A, B)

    assert np.array_equal(run(comb), alpha * run(a1) + beta * run(a2))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_linearity_in_second_operand_random(oracle_mod, layout):
    M, N, K = 9, 8, 37
    a = synth.normal_bf16(51, (M, K))
    b1 = synth.bf16_bits_to_f32(synth.normal_bf16(52, (K, N)))
    b2 = synth.bf16_bits_to_f32(synth.normal_bf16(53, (K, N)))
    # b1 + b2 is not bf16-exact in general: use 2*b1 and (2*b1 - b1) style power-of-two scalings
    def run(bm):
        A, B = store(a, bits(bm), layout)
        return oracle_mod.gemm(M, N, K, layout, A, B)
    r1, r2 = run(b1), run(b2)
    assert np.array_equal(run(2.0 * b1), 2.0 * r1)
    assert np.array_equal(run(-0.25 * b2), -0.25 * r2)


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("layout", LAYOUTS)
def test_closed_forms(oracle_mod, layout):
    M, N, K = 7, 4, 50
    ones_a, ones_b = bits(np.ones((M, K))), bits(np.ones((K, N)))
    A, B = store(ones_a, ones_b, layout)
    assert np.array_equal(oracle_mod.gemm(M, N, K, layout, A, B), np.full((M, N), float(K)))
    # rank one: A = u 1^T, B = 1 v^T  ->  C_ij = K u_i v_j
    u = np.arange(1, M + 1, dtype=np.float64)            # 1..7
    v = np.array([1.0, -2.0, 0.5, 3.0])
    A, B = store(bits(np.outer(u, np.ones(K))), bits(np.outer(np.ones(K), v)), layout)
    assert np.array_equal(oracle_mod.gemm(M, N, K, layout, A, B), K * np.outer(u, v))
    # one-hot selection: A = e_p e_q^T picks row q of B into row p of C
    E = np.zeros((M, K)); E[2, 31] = 1.0
    b_bits = synth.normal_bf16(61, (K, N))
    A, B = store(bits(E), b_bits, layout)
    want = np.zeros((M, N)); want[2] = synth.bf16_bits_to_f32(b_bits)[31]
    assert np.array_equal(oracle_mod.gemm(M, N, K, layout, A, B), want)
    # k-dependent weights: A_ik = k (same for all i), B_kj = 1 -> C = sum k = K(K-1)/2
    A, B = store(bits(np.tile(np.arange(K, dtype=np.float64), (M, 1))), ones_b, layout)
    assert np.array_equal(oracle_mod.gemm(M, N, K, layout, A, B), np.full((M, N), K * (K - 1) / 2.0))


def test_diagonal_scaling(oracle_mod):
    M, K = 6, 6
    a_bits = synth.normal_bf16(71, (M, K))
    a = synth.bf16_bits_to_f32(a_bits).astype(np.float64)
    d = np.array([1.0, 2.0, -4.0, 0.5, 8.0, -0.25])
    for layout in LAYOUTS:
        A, B = store(a_bits, bits(np.diag(d)), layout)
        assert np.array_equal(oracle_mod.gemm(M, K, K, layout, A, B), a * d[None, :])
        A, B = store(bits(np.diag(d)), a_bits, layout)
        assert np.array_equal(oracle_mod.gemm(M, K, M, layout, A, B), d[:, None] * a)


# ---------------------------------------------------------------- finite differences
def test_backward_products_are_gradients_of_forward(oracle_mod):
    """L(X,W) = sum_ij G_ij (X W)_ij is linear in X and in W, so a central difference with any
    step equals dL/dW = X^T G and dL/dX = G W^T exactly (up to fp64 round-off)."""
    T, d_in, d_out = 9, 6, 5
    X = synth.bf16_bits_to_f32(synth.integer_bf16(81, (T, d_in), -4, 4))
    W = synth.bf16_bits_to_f32(synth.integer_bf16(82, (d_in, d_out), -4, 4))
    G = synth.bf16_bits_to_f32(synth.integer_bf16(83, (T, d_out), -4, 4)).astype(np.float64)

    def loss(Xm, Wm):
        return float((G * oracle_mod.linear_fwd(T, d_out, d_in, "NN", bits(Xm), bits(Wm))).sum())

    dW = oracle_mod.linear_bwd_weight(d_in, d_out, T, "TN", bits(X), bits(G))
    dX = oracle_mod.linear_bwd_data(T, d_in, d_out, "NT", bits(G), bits(W))
    eps = 1.0                                        # W +- 1 stays an exact bf16 integer
    for (a, b) in [(0, 0), (5, 4), (2, 3), (3, 1)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[a, b] += eps; Wm[a, b] -= eps
        fd = (loss(X, Wp) - loss(X, Wm)) / (2 * eps)
        assert fd == dW[a, b]
    for (t, a) in [(0, 0), (8, 5), (4, 2), (1, 3)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[t, a] += eps; Xm[t, a] -= eps
        fd = (loss(Xp, W) - loss(Xm, W)) / (2 * eps)
        assert fd == dX[t, a]


# ---------------------------------------------------------------- numpy fp64 matmul
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", [(96, 130, 257), (300, 64, 520)])
def test_against_numpy_fp64_matmul(oracle_mod, layout, shape):
    M, N, K = shape
    a_bits = synth.normal_bf16(91, (M, K))
    b_bits = synth.normal_bf16(92, (K, N), 0.02)
    a = synth.bf16_bits_to_f32(a_bits).astype(np.float64)
    b = synth.bf16_bits_to_f32(b_bits).astype(np.float64)
    want = a @ b
    A, B = store(a_bits, b_bits, layout)
    got = oracle_mod.gemm(M, N, K, layout, A, B)
    scale = (np.abs(a) @ np.abs(b)).max()
    assert np.abs(got - want).max() <= 1e-12 * scale


@pytest.mark.parametrize("layout", LAYOUTS)
def test_sampled_entry_points_match_full(oracle_mod, layout):
    M, N, K = 37, 41, 129
    a_bits = synth.normal_bf16(101, (M, K))
    b_bits = synth.normal_bf16(102, (K, N))
    A, B = store(a_bits, b_bits, layout)
    full = oracle_mod.gemm(M, N, K, layout, A, B)
    ii = np.array([0, 36, 5, 17, 36, 0], dtype=np.int64)
    jj = np.array([0, 40, 40, 3, 0, 39], dtype=np.int64)
    # the sampled form sums the same terms in the same k order for NT, and the same
    # mathematical sum otherwise: exact equality in NT, round-off equality elsewhere
    got = oracle_mod.gemm_at(M, N, K, layout, A, B, ii, jj)
    assert np.allclose(got, full[ii, jj], rtol=0, atol=1e-12 * np.abs(full).max())
    # brute-force the samples independently in exact rational arithmetic via integers:
    a = synth.bf16_bits_to_f32(a_bits).astype(np.float64)
    b = synth.bf16_bits_to_f32(b_bits).astype(np.float64)
    for s in range(len(ii)):
        want = sum(a[ii[s], k] * b[k, jj[s]] for k in range(K))
        assert abs(got[s] - want) <= 1e-12 * np.abs(full).max()


def test_thread_count_does_not_change_bits(oracle_mod):
    M, N, K = 33, 17, 65
    a_bits, b_bits = synth.normal_bf16(111, (M, K)), synth.normal_bf16(112, (K, N))
    c1 = oracle_mod.gemm(M, N, K, "NN", a_bits, b_bits, threads=1)
    c8 = oracle_mod.gemm(M, N, K, "NN", a_bits, b_bits, threads=8)
    assert np.array_equal(c1, c8)


def test_empty_and_bad_arguments(oracle_mod):
    z = np.zeros((0, 4), dtype=np.uint16)
    b = synth.normal_bf16(1, (4, 3))
    assert oracle_mod.gemm(0, 3, 4, "NN", z, b).shape == (0, 3)
    # K = 0: empty sum is zero
    c = oracle_mod.gemm(2, 3, 0, "NN", np.zeros((2, 0), np.uint16), np.zeros((0, 3), np.uint16))
    assert np.array_equal(c, np.zeros((2, 3)))
    with pytest.raises(ValueError):
        oracle_mod.gemm(2, 3, 4, "NN", np.zeros((2, 5), np.uint16), b)
    with pytest.raises(ValueError):
        oracle_mod.gemm(2, 3, 4, "TT", np.zeros((2, 4), np.uint16), b)
    with pytest.raises(RuntimeError):
        oracle_mod.gemm_at(2, 3, 4, "NN", np.zeros((2, 4), np.uint16), b, [2], [0])


# ------------------------------------------------------------------ operand re-storage (Sec. IV-C)
def test_transpose_hand_example_and_shapes(oracle_mod):
    # worked by hand from the definition dst[c][r] = src[r][c]
    src = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.uint16)
    assert oracle_mod.transpose(src).tolist() == [[1, 4], [2, 5], [3, 6]]
    row = np.arange(7, dtype=np.uint16).reshape(1, 7)
    assert oracle_mod.transpose(row).tolist() == [[v] for v in range(7)]
    assert oracle_mod.transpose(oracle_mod.transpose(row)).tolist() == row.tolist()
    assert oracle_mod.transpose(np.zeros((0, 5), np.uint16)).shape == (5, 0)
    with pytest.raises(TypeError):
        oracle_mod.transpose(np.zeros((2, 2), np.float32))


@pytest.mark.parametrize("shape", [(3, 5), (64, 64), (65, 130), (257, 31), (1000, 8)])
def test_transpose_position_code_involution_and_numpy(oracle_mod, shape):
    rows, cols = shape
    # every element carries its own (row, col): a wrong index map cannot pass
    src = ((np.arange(rows)[:, None] * 251 + np.arange(cols)[None, :] * 7) % 65521).astype(np.uint16)
    dst = oracle_mod.transpose(src)
    assert dst.shape == (cols, rows)
    for r, c in [(0, 0), (rows - 1, 0), (0, cols - 1), (rows - 1, cols - 1), (rows // 2, cols // 3)]:
        assert dst[c, r] == src[r, c]
    assert np.array_equal(dst, src.T)                       # the library routine it must reduce to
    assert np.array_equal(oracle_mod.transpose(dst), src)   # involution


def test_transposed_operand_gives_the_same_product_in_the_other_mode(oracle_mod):
    # the reason the re-storage exists: NN on (A, B) == NT on (A, B^T) == TN on (A^T, B), bit for bit
    M, N, K = 9, 14, 11
    a = synth.normal_bf16(901, (M, K))
    b = synth.normal_bf16(902, (K, N))
    ref = oracle_mod.gemm(M, N, K, "NN", a, b)
    assert np.array_equal(oracle_mod.gemm(M, N, K, "NT", a, oracle_mod.transpose(b)), ref)
    assert np.array_equal(oracle_mod.gemm(M, N, K, "TN", oracle_mod.transpose(a), b), ref)
