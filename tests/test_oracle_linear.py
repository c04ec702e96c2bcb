"""Pins for oracle/linear.py: Eq. 2 written out term by term, scalar triple
loops on tiny shapes, the k = 0 reduction, and losslessly-representable inputs
for which all three products must equal the plain products."""
import numpy as np

from oracle import decompose as dec
from oracle import linear as lin
from oracle import quant


def _split(rs, M, N, k, g=(2.0 ** -11, 2.0 ** -11, 2.0 ** -6)):
    A = rs.standard_normal((M, N)) + np.outer(rs.standard_normal(M), rs.standard_normal(N)) * 3
    U, S, V = dec.decompose(A, k, 4, 1.0, seed=M + N)
    return A, lin.split_quantize(A, U, S, V, *g)


def test_eq2_expansion_equals_assembled_product():
    rs = np.random.default_rng(0)
    _, xq = _split(rs, 48, 64, 4)
    _, wq = _split(rs, 32, 64, 4)
    Y = lin.linear_fwd(xq, wq)
    assert np.allclose(Y, lin.linear_fwd_expanded(xq, wq), rtol=1e-12, atol=1e-12)


def test_triple_loop_tiny():
    rs = np.random.default_rng(1)
    _, xq = _split(rs, 16, 32, 2)
    _, wq = _split(rs, 16, 32, 2)
    _, gq = _split(rs, 16, 16, 2)
    Xb, Wb = lin.assemble(xq), lin.assemble(wq)
    Y = lin.linear_fwd(xq, wq)
    ref = np.zeros((16, 16))
    for l in range(16):
        for n in range(16):
            for kk in range(32):
                ref[l, n] += Xb[l, kk] * Wb[n, kk]
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-12)
    # dgrad: dX[l,k] = sum_n Gbar[l,n] Wbar_t[n,k], with W's residual blocked along N
    Gb, Wt = lin.assemble(gq), lin.assemble(wq, transposed_residual=True)
    dX = lin.linear_dgrad(gq, wq)
    ref = np.zeros((16, 32))
    for l in range(16):
        for kk in range(32):
            for n in range(16):
                ref[l, kk] += Gb[l, n] * Wt[n, kk]
    assert np.allclose(dX, ref, rtol=1e-12, atol=1e-12)
    Gt, Xt = lin.assemble(gq, True), lin.assemble(xq, True)
    dW = lin.linear_wgrad(gq, xq)
    ref = np.zeros((16, 32))
    for n in range(16):
        for kk in range(32):
            for l in range(16):
                ref[n, kk] += Gt[l, n] * Xt[l, kk]
    assert np.allclose(dW, ref, rtol=1e-12, atol=1e-12)


def test_assemble_element_by_element():
    rs = np.random.default_rng(2)
    A, sq = _split(rs, 32, 48, 3)
    Ab = lin.assemble(sq)
    Ud = quant.dequantize(*sq.Ut)       # [k, M]
    Vd = quant.dequantize(*sq.Vt)       # [k, N]
    Rd = quant.dequantize(*sq.R)
    for (i, j) in [(0, 0), (5, 17), (31, 47)]:
        v = sum(Ud[c, i] * sq.S[c] * Vd[c, j] for c in range(3)) + Rd[i, j]
        assert np.isclose(Ab[i, j], v, rtol=1e-13)
    # S is not quantized: it is carried verbatim
    U, S, V = dec.decompose(A, 3, 4, 1.0, seed=32 + 48)
    assert np.array_equal(sq.S, S)
    # the quantized operand approximates A
    assert np.linalg.norm(Ab - A) / np.linalg.norm(A) < 0.15


def test_k0_is_plain_quantized_gemm():
    rs = np.random.default_rng(3)
    X, W = rs.standard_normal((16, 32)), rs.standard_normal((32, 32))
    xq = lin.split_quantize(X, None, None, None, 1, 1, 2.0 ** -6)
    wq = lin.split_quantize(W, None, None, None, 1, 1, 2.0 ** -6)
    ref = quant.dequantize(*quant.quantize(X, 2.0 ** -6), 2.0 ** -6) @ \
        quant.dequantize(*quant.quantize(W, 2.0 ** -6), 2.0 ** -6).T
    assert np.array_equal(lin.linear_fwd(xq, wq), ref)
    assert np.array_equal(lin.linear_fwd_expanded(xq, wq), ref)


def test_lossless_inputs_give_plain_products():
    # entries on the E2M1 grid with a common power-of-two scale quantize without
    # error along either axis, so all three products equal the plain ones
    rs = np.random.default_rng(4)
    grid = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])

    def lossless(m, n):
        a = grid[rs.integers(0, 8, (m, n))] * rs.choice([-1, 1], (m, n))
        a[:, ::16] = 6.0
        a[::16, :] = 6.0
        return a * 0.25
    X, W, G = lossless(32, 48), lossless(16, 48), lossless(32, 16)
    q = lambda a: lin.split_quantize(a, None, None, None, 1, 1, 1.0)
    xq, wq, gq = q(X), q(W), q(G)
    assert np.array_equal(lin.assemble(xq), X) and np.array_equal(lin.assemble(xq, True), X)
    assert np.array_equal(lin.linear_fwd(xq, wq), X @ W.T)
    assert np.array_equal(lin.linear_dgrad(gq, wq), G @ W)
    assert np.array_equal(lin.linear_wgrad(gq, xq), G.T @ X)


def test_residual_is_narrower_and_quantizes_with_less_error():
    # the paper's premise (Sec. 2.2, 2.3): removing the dominant components narrows the
    # distribution (residual one to two orders of magnitude narrower), so the long-tail
    # part is quantized with far smaller absolute error than under direct quantization
    rs = np.random.default_rng(5)
    q_, _ = np.linalg.qr(rs.standard_normal((128, 64)))
    p_, _ = np.linalg.qr(rs.standard_normal((256, 64)))
    s = 100.0 * np.arange(1, 65) ** -2.0
    A = (q_ * s) @ p_.T
    U, S, V = dec.decompose(A, 8, 8, 1.0, seed=1)
    R = dec.residual(A, U, S, V)
    assert np.abs(R).max() < 0.1 * np.abs(A).max()
    g = quant.tensor_scale_for(np.abs(A).max())
    err_r = np.linalg.norm(quant.dequantize(*quant.quantize(R, g), g) - R)
    err_a = np.linalg.norm(quant.dequantize(*quant.quantize(A, g), g) - A)
    assert err_r < 0.2 * err_a


def test_split_quantize_sr_is_unbiased_where_nearest_rounding_is_not():
    """Sec. 4: stochastic rounding removes the quantization bias.  Averaged over seeds, the split
    quantized with SR reproduces A far better than any single draw and than nearest rounding's
    systematic error allows."""
    odec, olin, oq = dec, lin, quant
    rng = np.random.default_rng(3)
    A = rng.standard_normal((64, 8)) @ rng.standard_normal((8, 96)) + 0.3 * rng.standard_normal((64, 96))
    U, S, V = odec.decompose(A, 8, 8, 1.0, 5)
    g = oq.tensor_scale_for(np.abs(A).max())
    one = olin.assemble(olin.split_quantize_sr(A, U, S, V, 2.0 ** -11, 2.0 ** -11, g, seed=0))
    mean = np.zeros_like(A)
    n = 48
    for seed in range(n):
        sq = olin.split_quantize_sr(A, U, S, V, 2.0 ** -11, 2.0 ** -11, g, seed=10 * seed)
        # the residual part alone is unbiased; factors enter as a product, so average the residual term
        mean += oq.dequantize(*sq.R)
    mean /= n
    R = odec.residual(A, U, S, V)
    rne = oq.dequantize(*(oq.quantize(R, g) + (g,)))
    err_one = np.linalg.norm(oq.dequantize(*olin.split_quantize_sr(A, U, S, V, 2.0 ** -11, 2.0 ** -11, g, seed=0).R) - R)
    err_mean = np.linalg.norm(mean - R)
    assert err_mean < err_one / 4                   # ~1/sqrt(48) of a single draw
    assert err_mean < np.linalg.norm(rne - R) / 2   # below what deterministic rounding leaves
    assert np.isfinite(one).all()
    # distinct tensors draw from distinct keys: U^T and R^T codes are not produced from shared words
    a = olin.split_quantize_sr(A, U, S, V, 2.0 ** -11, 2.0 ** -11, g, seed=1)
    b = olin.split_quantize_sr(A, U, S, V, 2.0 ** -11, 2.0 ** -11, g, seed=2)
    assert not np.array_equal(a.R[0], b.R[0]) and not np.array_equal(a.Ut[0], b.Ut[0])


def test_factor_grads_match_finite_differences_of_the_quantized_forward():
    """L(U, S, V) = <G, X (U S V^T + R)^T> is linear in each factor: its gradient at the dequantized
    factors must equal factor_grads fed dW = G^T X (central differences are exact for a bilinear form up
    to rounding)."""
    rng = np.random.default_rng(11)
    L_, N, K, k = 24, 32, 48, 4
    X = rng.standard_normal((L_, K)); G = rng.standard_normal((L_, N))
    W = rng.standard_normal((N, k)) @ rng.standard_normal((k, K)) + 0.1 * rng.standard_normal((N, K))
    U, S, V = dec.decompose(W, k, 4, 1.0, 3)
    wq = lin.split_quantize(W, U, S, V, 2.0 ** -11, 2.0 ** -11, quant.tensor_scale_for(np.abs(W).max()))
    Ub, Vb = quant.dequantize(*wq.Ut).T, quant.dequantize(*wq.Vt).T
    Rb = quant.dequantize(*wq.R)
    dW = G.T @ X
    dU, dS, dV = lin.factor_grads(dW, wq)
    assert dU.shape == (N, k) and dS.shape == (k, k) and dV.shape == (K, k)

    def loss(Uc, Sm, Vc):
        return float(np.sum(G * (X @ (Uc @ Sm @ Vc.T + Rb).T)))
    Sm = np.diag(wq.S)
    h = 1e-3
    for (i, j) in [(0, 0), (5, 2), (N - 1, k - 1)]:
        E = np.zeros_like(Ub); E[i, j] = h
        assert np.isclose((loss(Ub + E, Sm, Vb) - loss(Ub - E, Sm, Vb)) / (2 * h), dU[i, j], rtol=1e-8, atol=1e-9)
    for (i, j) in [(0, 0), (7, 1), (K - 1, k - 1)]:
        E = np.zeros_like(Vb); E[i, j] = h
        assert np.isclose((loss(Ub, Sm, Vb + E) - loss(Ub, Sm, Vb - E)) / (2 * h), dV[i, j], rtol=1e-8, atol=1e-9)
    for (i, j) in [(0, 0), (1, 3), (k - 1, k - 1)]:
        E = np.zeros_like(Sm); E[i, j] = h
        assert np.isclose((loss(Ub, Sm + E, Vb) - loss(Ub, Sm - E, Vb)) / (2 * h), dS[i, j], rtol=1e-8, atol=1e-9)
    # and dW itself is the gradient with respect to the residual (the hot path's wgrad)
    E = np.zeros_like(Rb); E[3, 9] = h
    f = lambda Rm: float(np.sum(G * (X @ (Ub @ Sm @ Vb.T + Rm).T)))
    assert np.isclose((f(Rb + E) - f(Rb - E)) / (2 * h), dW[3, 9], rtol=1e-8)


def test_split_from_parts_stores_the_parts_it_is_given():
    # Sec. 3.2: a weight's factors and residual are stored variables.  Pins: (i) parts on the
    # E2M1 grid come back exactly, in both orientations of the residual and with each factor
    # transposed (a swapped U/V or a missing transpose changes the assembled matrix);
    # (ii) with W_R = W - U S V^T it is the same split as split_quantize of W;
    # (iii) for general parts every assembled element is within the quantizer's half-step bound.
    rs = np.random.default_rng(11)
    grid = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])

    def lossless(m, n):
        a = grid[rs.integers(0, 8, (m, n))] * rs.choice([-1, 1], (m, n))
        a[:, ::16] = 6.0
        a[::16, :] = 6.0
        return a
    N, K, k = 48, 32, 16
    U, V, WR = lossless(N, k), lossless(K, k), lossless(N, K) * 0.5
    S = rs.uniform(0.5, 2.0, k)
    sq = lin.split_from_parts(WR, U, S, V, 1.0, 1.0, 1.0)
    ref = (U * S) @ V.T + WR
    assert np.array_equal(lin.assemble(sq), ref) and np.array_equal(lin.assemble(sq, True), ref)
    assert sq.Ut[0].shape == (k, N // 2) and sq.Vt[0].shape == (k, K // 2)
    assert sq.R[0].shape == (N, K // 2) and sq.Rt[0].shape == (K, N // 2)

    W = rs.standard_normal((N, K))
    Uo, So, Vo = dec.decompose(W, 8, 8, 1.0, seed=2)
    a = lin.split_quantize(W, Uo, So, Vo, 2.0 ** -11, 2.0 ** -11, 2.0 ** -6)
    b = lin.split_from_parts(dec.residual(W, Uo, So, Vo), Uo, So, Vo, 2.0 ** -11, 2.0 ** -11, 2.0 ** -6)
    for x, y in ((a.Ut, b.Ut), (a.Vt, b.Vt), (a.R, b.R), (a.Rt, b.Rt)):
        assert np.array_equal(x[0], y[0]) and np.array_equal(x[1], y[1]) and x[2] == y[2]

    g = 2.0 ** -6
    WR2 = 0.05 * rs.standard_normal((N, K))
    c = lin.split_from_parts(WR2, Uo, So, Vo, 2.0 ** -11, 2.0 ** -11, g, seed=None)
    err = np.abs(quant.dequantize(*c.R) - WR2)
    amax = np.abs(WR2).reshape(N, K // 16, 16).max(axis=2)
    # step of a block <= its amax/6 rounded up to the next E4M3 value (<= 1.125x, or the smallest scale);
    # the widest grid gap is 2 steps
    bound = np.maximum(amax / 6.0 * 1.125, 2.0 ** -9 * g)
    assert (err.reshape(N, K // 16, 16) <= bound[:, :, None] + 1e-15).all()
    d = lin.split_from_parts(WR2, Uo, So, Vo, 2.0 ** -11, 2.0 ** -11, g, seed=5)
    e = lin.split_quantize_sr(WR2 + (Uo * So) @ Vo.T, Uo, So, Vo, 2.0 ** -11, 2.0 ** -11, g, 5)
    assert np.array_equal(d.Ut[0], e.Ut[0]) and np.array_equal(d.Vt[0], e.Vt[0])   # same keys as the recomputed split


def test_row_subsets_are_rows_of_the_full_products():
    rs = np.random.default_rng(11)
    _, xq = _split(rs, 48, 64, 4)
    _, wq = _split(rs, 32, 64, 4)
    _, gq = _split(rs, 48, 32, 4)
    rows = np.array([0, 5, 17, 31])
    # (a library matmul may sum in another order for another shape: compare to rounding)
    assert np.allclose(lin.linear_fwd(xq, wq, rows), lin.linear_fwd(xq, wq)[rows], rtol=1e-13, atol=1e-13)
    assert np.allclose(lin.linear_dgrad(gq, wq, rows), lin.linear_dgrad(gq, wq)[rows], rtol=1e-13, atol=1e-13)
    assert np.allclose(lin.linear_wgrad(gq, xq, rows), lin.linear_wgrad(gq, xq)[rows], rtol=1e-13, atol=1e-13)
