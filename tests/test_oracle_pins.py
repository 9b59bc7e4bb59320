"""Pins for the float64 oracle: closed forms, invariants, special cases and
brute force.  None of these re-call the oracle's own library routines to build
the expected value; helper algorithms (one-sided Jacobi SVD, Gram–Schmidt,
scalar loops) are written out here independently."""
import math

import numpy as np
import pytest

import oracle
import workloads as wl


# ----------------------------- independent helpers ------------------------- #
def jacobi_svd(A, sweeps=60, tol=1e-15):
    """One-sided (Hestenes) Jacobi SVD: returns U (m×n), s (n), V (n×n)."""
    A = np.array(A, dtype=np.float64, copy=True)
    m, n = A.shape
    V = np.eye(n)
    for _ in range(sweeps):
        off = 0.0
        for p in range(n - 1):
            for q in range(p + 1, n):
                a = A[:, p] @ A[:, p]
                b = A[:, q] @ A[:, q]
                g = A[:, p] @ A[:, q]
                if abs(g) <= tol * math.sqrt(a * b) or g == 0.0:
                    continue
                off = max(off, abs(g) / math.sqrt(a * b))
                zeta = (b - a) / (2.0 * g)
                t = math.copysign(1.0, zeta) / (abs(zeta) + math.sqrt(1.0 + zeta * zeta))
                c = 1.0 / math.sqrt(1.0 + t * t)
                s = c * t
                Ap, Aq = A[:, p].copy(), A[:, q].copy()
                A[:, p], A[:, q] = c * Ap - s * Aq, s * Ap + c * Aq
                Vp, Vq = V[:, p].copy(), V[:, q].copy()
                V[:, p], V[:, q] = c * Vp - s * Vq, s * Vp + c * Vq
        if off < tol:
            break
    s = np.sqrt((A * A).sum(axis=0))
    order = np.argsort(-s)
    s, A, V = s[order], A[:, order], V[:, order]
    U = A / np.where(s > 0, s, 1.0)
    return U, s, V


def mgs2(Z):
    """Modified Gram–Schmidt applied twice; R has a positive diagonal by construction."""
    Z = np.array(Z, dtype=np.float64, copy=True)
    n, r = Z.shape
    Q = np.zeros((n, r))
    for j in range(r):
        v = Z[:, j].copy()
        for _ in range(2):
            for i in range(j):
                v -= (Q[:, i] @ v) * Q[:, i]
        Q[:, j] = v / math.sqrt(v @ v)
    return Q


def sin_theta(Ua, Ub):
    """Sine of the largest principal angle between span(Ua) and span(Ub) (same dim)."""
    return np.linalg.norm(Ub - Ua @ (Ua.T @ Ub), 2)


def constructed(L, d, s, seed, sigma=0.0):
    return wl.make_X(L, d, np.asarray(s, dtype=np.float64), sigma, seed, return_factors=True)


# ----------------------------- qf ------------------------------------------ #
def test_qf_matches_gram_schmidt_and_has_positive_diagonal():
    rng = np.random.default_rng(1)
    Z = rng.standard_normal((37, 9)) * (10.0 ** -np.arange(9))[None, :]
    Q = oracle.qf(Z)
    assert np.abs(Q.T @ Q - np.eye(9)).max() < 1e-13            # P-1
    R = Q.T @ Z
    assert np.all(np.diag(R) > 0)
    assert np.abs(np.tril(R, -1)).max() < 1e-12 * np.abs(R).max()
    assert np.abs(Q @ R - Z).max() < 1e-12
    assert np.abs(Q - mgs2(Z)).max() < 1e-9


def test_qf_is_invariant_to_positive_upper_triangular_right_factor():
    # the property that lets any intermediate orthonormalisation be used (closed form of the iteration)
    rng = np.random.default_rng(2)
    Z = rng.standard_normal((20, 6))
    T = np.triu(rng.standard_normal((6, 6)))
    T[np.diag_indices(6)] = np.abs(np.diag(T)) + 0.5
    assert np.abs(oracle.qf(Z @ T) - oracle.qf(Z)).max() < 1e-10
    # a sign flip of a column (not positive diagonal) must flip the basis vector
    D = np.eye(6); D[2, 2] = -1
    Qf = oracle.qf(Z @ D)
    assert np.abs(Qf[:, 2] + oracle.qf(Z)[:, 2]).max() < 1e-12


# ----------------------------- principal_bases ----------------------------- #
def test_orthonormal_and_coefficients():                         # P-1, Eq.5
    c = wl.CONFIGS["tiny"]
    X = c.X()
    U, B = oracle.principal_bases(X, c.omega(), c.iters)
    assert U.shape == (128, 32) and B.shape == (32, 64)
    assert np.abs(U.T @ U - np.eye(32)).max() < 1e-12
    assert np.abs(B - U.T @ X).max() < 1e-12


def test_eckart_young_tail_energy():                             # P-2, Eq.9
    s = np.concatenate([np.linspace(9, 5, 6), np.linspace(0.05, 0.01, 10)])
    X, Us, Vs = constructed(40, 24, s, 11)
    Om = wl.make_omega(24, 6, 11)
    U, B = oracle.principal_bases(X, Om, 30)
    res = np.linalg.norm(X - U @ B, "fro") ** 2
    assert abs(res - np.sum(s[6:] ** 2)) < 1e-10
    # and no other rank-6 subspace tried does better (energy ratio, P-5 / Fig.5's quantity)
    assert abs(np.linalg.norm(B, "fro") ** 2 / np.linalg.norm(X, "fro") ** 2
               - np.sum(s[:6] ** 2) / np.sum(s ** 2)) < 1e-12
    assert sin_theta(Us[:, :6], U) < 1e-10


def test_projector_matches_bruteforce_jacobi_svd():              # P-3
    rng = np.random.default_rng(5)
    s = np.array([7.0, 5.0, 3.0, 0.2, 0.1, 0.05, 0.02, 0.01])
    X, _, _ = constructed(12, 8, s, 5)
    Uj, sj, Vj = jacobi_svd(X)
    assert np.abs(sj - s).max() < 1e-12                         # the helper itself is right
    U, B = oracle.principal_bases(X, rng.standard_normal((8, 3)), 25)
    P_orc = U @ U.T
    P_ref = Uj[:, :3] @ Uj[:, :3].T
    assert np.abs(P_orc - P_ref).max() < 1e-10


def test_exact_rank_r_reconstruction_and_commutation_any_iters():  # P-4, Eq.5-6
    rng = np.random.default_rng(7)
    s = np.array([3.0, 2.0, 1.5, 1.0, 0.5])
    X, _, _ = constructed(30, 16, s, 7)                          # rank exactly 5
    W = rng.standard_normal((16, 10))
    for k in (0, 1, 3):
        U, B = oracle.principal_bases(X, rng.standard_normal((16, 5)), k)
        assert np.abs(U @ B - X).max() < 1e-11
        assert np.abs(U @ oracle.lowrank_linear(B, W) - X @ W).max() < 1e-11


def test_iteration_closed_form_and_meaning_of_iters():           # P-6
    rng = np.random.default_rng(9)
    X = rng.standard_normal((14, 9)) + 0.5                       # well conditioned, tiny
    Om = rng.standard_normal((9, 4))
    G = X.T @ X
    for k in (0, 1, 2):
        M = X @ np.linalg.matrix_power(G, k) @ Om
        expect = mgs2(M)
        U, _ = oracle.principal_bases(X, Om, k)
        assert np.abs(U - expect).max() < 1e-8, k
    # one more iteration really changes the answer (iters is not ignored / off by one)
    U0, _ = oracle.principal_bases(X, Om, 0)
    U1, _ = oracle.principal_bases(X, Om, 1)
    assert np.abs(U0 - U1).max() > 1e-3


def test_convergence_rate_of_subspace_iteration():
    # textbook: sin(theta) contracts by (s_{r+1}/s_r)^2 per iteration
    s = np.array([4.0, 3.0, 2.0, 0.2, 0.1, 0.05])
    X, Us, _ = constructed(25, 10, s, 13)
    Om = wl.make_omega(10, 3, 13)
    e = [sin_theta(Us[:, :3], oracle.principal_bases(X, Om, k)[0]) for k in range(4)]
    for a, b in zip(e[:-1], e[1:]):
        assert b < a * (0.2 / 2.0) ** 2 * 3.0


# ----------------------------- lowrank_linear ------------------------------ #
def test_lowrank_linear_bruteforce_and_swiglu_values():
    rng = np.random.default_rng(3)
    B = rng.standard_normal((5, 7)); W = rng.standard_normal((7, 6))
    ref = np.zeros((5, 6))
    for i in range(5):
        for j in range(6):
            for t in range(7):
                ref[i, j] += B[i, t] * W[t, j]
    assert np.abs(oracle.lowrank_linear(B, W) - ref).max() < 1e-13
    g = oracle.lowrank_linear(B, W, "swiglu")
    assert g.shape == (5, 3)
    for i in range(5):
        for j in range(3):
            x, u = ref[i, j], ref[i, j + 3]
            assert abs(g[i, j] - x * (1.0 / (1.0 + math.exp(-x))) * u) < 1e-13
    # closed-form SiLU values: SiLU(0)=0, SiLU(1)=1/(1+1/e), SiLU(-x)=SiLU(x)-x, SiLU(30)≈30
    one = np.array([[0.0, 1.0, -1.0, 30.0]])
    eye = np.concatenate([np.eye(4), np.eye(4)], axis=1)          # gate = up = input
    out = oracle.lowrank_linear(one, eye, "swiglu")[0]
    assert out[0] == 0.0
    assert abs(out[1] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(out[2] - (-1.0) * (1.0 / (1.0 + math.e)) * (-1.0)) < 1e-15
    assert abs(out[3] - 900.0) < 1e-9


# ----------------------------- attention ----------------------------------- #
def brute_attention(Q, K, V, heads, scale=None):
    L, dq = Q.shape; r = K.shape[0]; dh = dq // heads
    sc = 1.0 / math.sqrt(dh) if scale is None else scale
    O = np.zeros((L, dq))
    for h in range(heads):
        for i in range(L):
            sco = [sc * sum(Q[i, h * dh + c] * K[j, h * dh + c] for c in range(dh)) for j in range(r)]
            m = max(sco)
            e = [math.exp(x - m) for x in sco]
            z = sum(e)
            for c in range(dh):
                O[i, h * dh + c] = sum(e[j] / z * V[j, h * dh + c] for j in range(r))
    return O


def test_attention_bruteforce_multihead():
    rng = np.random.default_rng(4)
    Q = rng.standard_normal((6, 8)); K = rng.standard_normal((5, 8)); V = rng.standard_normal((5, 8))
    for heads in (1, 2, 4):
        assert np.abs(oracle.attention(Q, K, V, heads) - brute_attention(Q, K, V, heads)).max() < 1e-13
    assert np.abs(oracle.attention(Q, K, V, 2, scale=0.3) - brute_attention(Q, K, V, 2, 0.3)).max() < 1e-13


def test_attention_special_cases():                              # P-7
    rng = np.random.default_rng(6)
    L, r, dq, H = 9, 7, 12, 3
    Q = rng.standard_normal((L, dq)); K = rng.standard_normal((r, dq)); V = rng.standard_normal((r, dq))
    # (a) equal keys → mean of values
    Keq = np.tile(K[:1], (r, 1))
    assert np.abs(oracle.attention(Q, Keq, V, H) - V.mean(axis=0)[None]).max() < 1e-13
    # (b) r = 1 → that value row
    assert np.abs(oracle.attention(Q, K[:1], V[:1], H) - V[:1]).max() < 1e-14
    # (c) scale → 0 → uniform average
    assert np.abs(oracle.attention(Q, K, V, H, scale=1e-12) - V.mean(axis=0)[None]).max() < 1e-9
    # (d) one dominant key per head → that value row (per head)
    Kd = K.copy(); Qd = np.abs(Q) + 0.1
    Kd[3] = 1e3
    assert np.abs(oracle.attention(Qd, Kd, V, H) - V[3][None]).max() < 1e-12
    # (e) joint permutation of keys and values
    p = rng.permutation(r)
    assert np.abs(oracle.attention(Q, K[p], V[p], H) - oracle.attention(Q, K, V, H)).max() < 1e-13
    # (f) heads are independent column slices
    full = oracle.attention(Q, K, V, H)
    dh = dq // H
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        assert np.abs(full[:, c] - oracle.attention(Q[:, c], K[:, c], V[:, c], 1)).max() < 1e-14
    # shift invariance of softmax: adding a constant vector to every key along q changes nothing
    # (large scores must not overflow)
    big = oracle.attention(50 * Q, 50 * K, V, H)
    assert np.isfinite(big).all()
    # default scale is 1/sqrt(d_h), not 1/sqrt(dq)
    assert np.abs(oracle.attention(Q, K, V, H) - oracle.attention(Q, K, V, H, scale=1 / math.sqrt(dh))).max() == 0
    assert np.abs(oracle.attention(Q, K, V, H) - oracle.attention(Q, K, V, H, scale=1 / math.sqrt(dq))).max() > 1e-3


def test_lowrank_attention_identity_eq7():                        # P-8
    # exp(q·Kᵀ)·V with K = U·K', V = U·V' equals exp(q·K'ᵀ·Uᵀ)·U·V' (unnormalised)
    rng = np.random.default_rng(8)
    s = np.array([2.0, 1.0, 0.7, 0.4])
    X, _, _ = constructed(15, 10, s, 8)
    Wq, Wk, Wv = (0.3 * rng.standard_normal((10, 6)) for _ in range(3))
    U, B = oracle.principal_bases(X, rng.standard_normal((10, 4)), 1)
    Qp, Kp, Vp = (oracle.lowrank_linear(B, W) for W in (Wq, Wk, Wv))
    Q, K, V = X @ Wq, X @ Wk, X @ Wv
    assert np.abs(U @ Qp - Q).max() < 1e-12                      # Eq.6
    lhs = np.exp(Q @ K.T) @ V
    rhs = np.exp(Q @ Kp.T @ U.T) @ U @ Vp
    assert np.abs(lhs - rhs).max() < 1e-10 * np.abs(lhs).max()
    # first-order term of Eq.8 does not depend on the basis chosen
    R, _ = np.linalg.qr(rng.standard_normal((4, 4)))
    U2, B2 = U @ R, R.T @ B
    t1 = (Q @ Kp.T) @ Vp
    t2 = (Q @ oracle.lowrank_linear(B2, Wk).T) @ oracle.lowrank_linear(B2, Wv)
    assert np.abs(t1 - t2).max() < 1e-11
    # ... but softmax over principal keys does (why the basis convention must be shared)
    a1 = oracle.attention(Q, Kp, Vp, 1)
    a2 = oracle.attention(Q, oracle.lowrank_linear(B2, Wk), oracle.lowrank_linear(B2, Wv), 1)
    assert np.abs(a1 - a2).max() > 1e-6


def test_linearised_attention_matches_dense_first_order_expansion():   # Eq.8
    # For an input of exact rank r, (1·U + s·q·K'ᵀ)·V' must equal the token-by-token sum
    # Σ_j (1 + s·q·k_j)·v_j over all L tokens, and the "taylor" normaliser the sum Σ_j (1 + s·q·k_j):
    # both written here as scalar loops over tokens, per head.
    rng = np.random.default_rng(18)
    L, d, r, H = 14, 8, 3, 2
    X, _, _ = constructed(L, d, np.array([3.0, 1.5, 0.8]), 18)
    Wq, Wk, Wv = (0.4 * rng.standard_normal((d, d)) for _ in range(3))
    U, B = oracle.principal_bases(X, rng.standard_normal((d, r)), 1)
    Qp, Kp, Vp = (oracle.lowrank_linear(B, W) for W in (Wq, Wk, Wv))
    Q, K, V = X @ Wq, X @ Wk, X @ Wv                      # dense, = U·Q' etc. because rank(X) = r
    dh = d // H
    sc = 0.37
    want = np.zeros((L, d))
    for h in range(H):
        for i in range(L):
            num = np.zeros(dh)
            den = 0.0
            for j in range(L):
                w = 1.0 + sc * sum(Q[i, h * dh + c] * K[j, h * dh + c] for c in range(dh))
                den += w
                for c in range(dh):
                    num[c] += w * V[j, h * dh + c]
            want[i, h * dh:(h + 1) * dh] = num / den
    got = oracle.linearised_attention(U @ Qp, Kp, Vp, U, H, scale=sc, norm="taylor")
    assert np.abs(got - want).max() < 1e-11
    # the result does not depend on the orthonormal basis chosen for the subspace
    R, _ = np.linalg.qr(rng.standard_normal((r, r)))
    U2, B2 = U @ R, R.T @ B
    got2 = oracle.linearised_attention(U2 @ oracle.lowrank_linear(B2, Wq), oracle.lowrank_linear(B2, Wk),
                                       oracle.lowrank_linear(B2, Wv), U2, H, scale=sc, norm="taylor")
    assert np.abs(got2 - want).max() < 1e-11
    # scale -> 0: every token gets weight 1: the output is the mean value row for every query
    flat = oracle.linearised_attention(U @ Qp, Kp, Vp, U, H, scale=1e-12, norm="taylor")
    assert np.abs(flat - V.mean(axis=0)[None, :]).max() < 1e-9
    # "rowsum" reading: same numerator, denominator = sum of the r entries of A' (scalar loops again)
    ones_U = [sum(U[i, j] for i in range(L)) for j in range(r)]
    want_rs = np.zeros((L, d))
    for h in range(H):
        for i in range(L):
            a = [ones_U[j] + sc * sum((U @ Qp)[i, h * dh + c] * Kp[j, h * dh + c] for c in range(dh)) for j in range(r)]
            for c in range(dh):
                want_rs[i, h * dh + c] = sum(a[j] * Vp[j, h * dh + c] for j in range(r)) / sum(a)
    got_rs = oracle.linearised_attention(U @ Qp, Kp, Vp, U, H, scale=sc, norm="rowsum")
    assert np.abs(got_rs - want_rs).max() < 1e-10 * max(1.0, np.abs(want_rs).max())


def test_rope_properties():
    rng = np.random.default_rng(31)
    L, H, dh = 9, 2, 8
    Y = rng.standard_normal((L, H * dh))
    R = oracle.rope(Y, H, base=100.0, pos0=0)
    # position 0 is not rotated; every pair keeps its length
    assert np.abs(R[0] - Y[0]).max() < 1e-15
    for h in range(H):
        for j in range(dh // 2):
            a, b = h * dh + j, h * dh + j + dh // 2
            assert np.abs(R[:, a] ** 2 + R[:, b] ** 2 - (Y[:, a] ** 2 + Y[:, b] ** 2)).max() < 1e-12
    # d_h = 2: one pair per head, a plain 2×2 rotation by the angle pos·base^0 = pos
    y = rng.standard_normal((4, 2))
    r = oracle.rope(y, 1, base=7.0, pos0=3)
    for i in range(4):
        t = 3 + i
        want = np.array([y[i, 0] * math.cos(t) - y[i, 1] * math.sin(t), y[i, 0] * math.sin(t) + y[i, 1] * math.cos(t)])
        assert np.abs(r[i] - want).max() < 1e-14
    # relative-position property: <R_i q, R_j k> depends on i - j only (per head)
    q, k = rng.standard_normal((1, dh)), rng.standard_normal((1, dh))
    def dot_at(i, j):
        qi = oracle.rope(q, 1, base=50.0, pos0=i)[0]
        kj = oracle.rope(k, 1, base=50.0, pos0=j)[0]
        return qi @ kj
    assert abs(dot_at(5, 2) - dot_at(11, 8)) < 1e-12 and abs(dot_at(5, 2) - dot_at(3, 0)) < 1e-12
    # principal keys of the rotated keys: U·K' is the projection of RoPE(K) on the subspace
    X, _, _ = constructed(12, 8, np.array([2.0, 1.0, 0.5]), 32)
    U, B = oracle.principal_bases(X, rng.standard_normal((8, 3)), 2)
    Kp0 = B @ (0.3 * rng.standard_normal((8, 8)))
    Kr = oracle.rope(U @ Kp0, 2, 100.0)
    Kp = oracle.rope_principal_keys(U, Kp0, 2, 100.0)
    assert np.abs(U @ Kp - U @ (U.T @ Kr)).max() < 1e-12
    assert np.abs(U.T @ (Kr - U @ Kp)).max() < 1e-12        # residual orthogonal to the subspace


def test_rope_frequencies_closed_form():
    # Sec. "Combine with Position Encoding" / RoFormer angles: pair j of a head of width d_h turns by
    # pos·base^(-2j/d_h).  d_h = 4: pair 0 = coordinates (0, 2), angle pos; pair 1 = (1, 3), angle
    # pos·base^(-1/2).  d_h = 8: pair j = (j, j + 4), angle pos·base^(-j/4).  Values worked by hand.
    base, pos = 16.0, 3
    y = np.array([[1.0, 2.0, -0.5, 0.25]])
    got = oracle.rope(y, 1, base=base, pos0=pos)[0]
    t0, t1 = 3.0, 3.0 / 4.0                       # 3·16^0, 3·16^(-1/2)
    want = np.array([1.0 * math.cos(t0) + 0.5 * math.sin(t0), 2.0 * math.cos(t1) - 0.25 * math.sin(t1),
                     1.0 * math.sin(t0) - 0.5 * math.cos(t0), 2.0 * math.sin(t1) + 0.25 * math.cos(t1)])
    assert np.abs(got - want).max() < 1e-14
    # a wrong exponent (base^(-j/d_h) = 3/2 instead of 3/4) must not pass
    wrong = 3.0 / 2.0
    assert abs(got[1] - (2.0 * math.cos(wrong) - 0.25 * math.sin(wrong))) > 0.1
    base = 81.0
    y8 = np.zeros((1, 16))
    y8[0, :8] = [1, 0, 0, 0, 0, 0, 0, 0]          # head 0: unit vector on pair 0
    y8[0, 8:] = [0, 0, 0, 1, 0, 0, 0, 0]          # head 1: unit vector on the first half of pair 3
    g8 = oracle.rope(y8, 2, base=base, pos0=2)[0]
    a0, a3 = 2.0, 2.0 * 81.0 ** (-0.75)            # 2·81^0 and 2·81^(-3/4) = 2/27
    assert abs(a3 - 2.0 / 27.0) < 1e-15
    want8 = np.zeros(16)
    want8[0], want8[4] = math.cos(a0), math.sin(a0)
    want8[8 + 3], want8[8 + 7] = math.cos(a3), math.sin(a3)
    assert np.abs(g8 - want8).max() < 1e-14
    # second rows take the next position
    y2 = np.array([[0.0, 1.0, 0.0, 0.0], [0.0, 1.0, 0.0, 0.0]])
    g2 = oracle.rope(y2, 1, base=4.0, pos0=5)
    assert abs(g2[0, 1] - math.cos(2.5)) < 1e-14 and abs(g2[1, 3] - math.sin(3.0)) < 1e-14


def test_full_rank_limit_recovers_dense_layer():
    # r = L = rank(X): U is square orthogonal, so softmax over "principal keys" is a
    # different function; but Q = U·Q' = X·W^Q exactly and K', V' span the same rows.
    rng = np.random.default_rng(10)
    X = rng.standard_normal((6, 9))
    Wq, Wk, Wv = (rng.standard_normal((9, 4)) for _ in range(3))
    out = oracle.atp_layer(X, rng.standard_normal((9, 6)), 0, Wq, Wk, Wv, 2)
    assert np.abs(out["Q"] - X @ Wq).max() < 1e-11
    assert np.abs(out["U"] @ out["Kp"] - X @ Wk).max() < 1e-11
    # with U = I (identity start block, L = d = r) the ATP layer IS the dense layer
    Xs = rng.standard_normal((5, 5))
    Xs = np.triu(Xs); Xs[np.diag_indices(5)] = np.abs(np.diag(Xs)) + 1.0   # qf(Xs) = I
    W3 = [rng.standard_normal((5, 4)) for _ in range(3)]
    o = oracle.atp_layer(Xs, np.eye(5), 0, *W3, 2)
    assert np.abs(o["U"] - np.eye(5)).max() < 1e-12
    assert np.abs(o["O"] - oracle.dense_attention_layer(Xs, *W3, 2)).max() < 1e-11


def test_layer_chain_shapes_and_factored_tail():
    c = wl.CONFIGS["tiny"]
    rng = np.random.default_rng(12)
    X = c.X()
    W = [wl.make_weight(64, 64, 100 + i) for i in range(4)]
    Wg, Wu, Wd = wl.make_weight(64, 96, 200), wl.make_weight(64, 96, 201), wl.make_weight(96, 64, 202)
    o = oracle.atp_layer(X, c.omega(), 2, W[0], W[1], W[2], 1, None, W[3], None, Wg, Wu, Wd)
    assert o["O"].shape == (128, 64) and o["A"].shape == (32, 64) and o["F"].shape == (32, 64)
    assert np.abs(o["Bo"] - o["Uo"].T @ o["O"]).max() < 1e-12
    A = o["A"]
    G = (A @ Wg) / (1 + np.exp(-(A @ Wg))) * (A @ Wu)
    assert np.abs(o["F"] - G @ Wd).max() < 1e-12


def test_factored_residual_and_norm_match_the_dense_definitions():      # Fig.3: residual + Norm on factored pairs
    rng = np.random.default_rng(77)
    L, d, r1, r2 = 7, 6, 2, 3
    U1, C1 = rng.standard_normal((L, r1)), rng.standard_normal((r1, d))
    U2, C2 = rng.standard_normal((L, r2)), rng.standard_normal((r2, d))
    P, C = oracle.concat_factors(U1, C1, U2, C2)
    assert P.shape == (L, r1 + r2) and C.shape == (r1 + r2, d)
    H = U1 @ C1 + U2 @ C2
    assert np.abs(P @ C - H).max() < 1e-13                       # the residual sum, in factored form
    g = rng.uniform(0.5, 1.5, d)
    eps = 1e-5
    for center in (False, True):
        Pn, Cn = oracle.norm_factored(P, C, g, eps, center)
        got = Pn @ Cn
        want = np.empty((L, d))
        for i in range(L):                                        # textbook row-wise normalisation with scalar loops
            row = [H[i, j] for j in range(d)]
            mean = sum(row) / d if center else 0.0
            row = [x - mean for x in row]
            ms = sum(x * x for x in row) / d
            for j in range(d):
                want[i, j] = row[j] / math.sqrt(ms + eps) * g[j]
        assert np.abs(got - want).max() < 1e-12
        assert Pn.shape == P.shape and Cn.shape == C.shape
    # unit gain, eps = 0: every row has unit mean square; scaling H does not change the result
    Pn, Cn = oracle.norm_factored(P, C, np.ones(d), 0.0, False)
    assert np.abs(np.mean((Pn @ Cn) ** 2, axis=1) - 1.0).max() < 1e-12
    Pn2, Cn2 = oracle.norm_factored(3.0 * P, C, np.ones(d), 0.0, False)
    assert np.abs(Pn2 @ Cn2 - Pn @ Cn).max() < 1e-12
    # centred variant: rows sum to zero
    Pn, Cn = oracle.norm_factored(P, C, np.ones(d), 0.0, True)
    assert np.abs((Pn @ Cn).sum(axis=1)).max() < 1e-12


def test_block_with_residuals_and_two_block_chain():
    c = wl.CONFIGS["tiny"]
    X = c.X()
    d, f = 64, 96
    W = [wl.make_weight(d, d, 300 + i) for i in range(4)]
    Wg, Wu, Wd = wl.make_weight(d, f, 310), wl.make_weight(d, f, 311), wl.make_weight(f, d, 312)
    g = np.linspace(0.8, 1.2, d)
    o = oracle.atp_block(X, c.omega(), 2, W[0], W[1], W[2], W[3], 1, g, Wg, Wu, Wd, eps=1e-6)
    r = c.r
    assert o["P"].shape == (128, 2 * r) and o["C"].shape == (2 * r, d) and o["Y"].shape == (128, d)
    H = o["U"] @ o["B"] + o["Uo"] @ o["A"]                        # first residual: rank-r input + attention branch
    assert np.abs(o["P"] @ o["C"] - H).max() < 1e-11
    N = H / np.sqrt(np.mean(H * H, axis=1, keepdims=True) + 1e-6) * g[None, :]
    assert np.abs(o["Pn"] @ o["Cn"] - N).max() < 1e-11           # Norm of the residual stream
    Cn = o["Cn"]
    F = ((Cn @ Wg) / (1 + np.exp(-(Cn @ Wg))) * (Cn @ Wu)) @ Wd   # feed-forward on the 2r coefficient rows
    assert np.abs(o["F2"] - F).max() < 1e-11
    assert np.abs(o["Y"] - (H + o["Pn"] @ F)).max() < 1e-10       # second residual
    # chaining: the next block extracts the principal components of Y
    o2 = oracle.atp_block(o["Y"], c.omega(), 2, W[0], W[1], W[2], W[3], 1, g, Wg, Wu, Wd, eps=1e-6)
    assert np.isfinite(o2["Y"]).all()
    assert np.abs(o2["U"].T @ o2["U"] - np.eye(r)).max() < 1e-12
    assert np.abs(o2["B"] - o2["U"].T @ o["Y"]).max() < 1e-10


# ----------------------------- variants ------------------------------------ #
def test_rayleigh_ritz_gives_singular_pairs():
    s = np.array([6.0, 4.0, 2.5, 0.03, 0.02, 0.01])
    X, Us, Vs = constructed(18, 11, s, 21)
    U, B = oracle.principal_bases(X, wl.make_omega(11, 3, 21), 40)
    Uc, Bc, sig = oracle.rayleigh_ritz(U, B)
    assert np.abs(sig - s[:3]).max() < 1e-10
    assert np.abs(Uc @ Bc - U @ B).max() < 1e-12                 # same rank-r approximation
    T = Bc @ Bc.T
    assert np.abs(T - np.diag(np.diag(T))).max() < 1e-10         # rows are sigma_i v_iᵀ: orthogonal
    for i in range(3):
        assert Uc[:, i].sum() >= 0
        assert min(np.abs(Bc[i] / s[i] - Vs[:, i]).max(), np.abs(Bc[i] / s[i] + Vs[:, i]).max()) < 1e-8


def test_rayleigh_ritz_fallback_sign_on_centred_input():
    # Hand-built centred example (every column of U sums to zero, so the rule 1ᵀu_i >= 0 decides
    # nothing and the largest-magnitude entry of each row of X' must come out positive).
    # X = 3·u1·v1ᵀ + 1·u2·v2ᵀ,  u1 = (1,-1,1,-1)/2, u2 = (1,1,-1,-1)/2, v1 = (0.6,-0.8,0), v2 = (0,0,-1).
    u1, u2 = np.array([1.0, -1, 1, -1]) / 2, np.array([1.0, 1, -1, -1]) / 2
    v1, v2 = np.array([0.6, -0.8, 0.0]), np.array([0.0, 0.0, -1.0])
    X = 3.0 * np.outer(u1, v1) + 1.0 * np.outer(u2, v2)
    # canonical form worked by hand: row 1 = ±3·v1 with its largest entry (-2.4) made positive,
    # row 2 = ±v2 with -1 made positive; the u_i follow the same sign
    want_B = np.array([[-1.8, 2.4, 0.0], [0.0, 0.0, 1.0]])
    want_U = np.stack([-u1, -u2], axis=1)
    c, s_ = math.cos(0.5), math.sin(0.5)
    G = np.array([[c, -s_], [s_, c]])                  # any rotation of the basis gives the same answer
    for rot in (np.eye(2), G, -np.eye(2)):
        U = np.stack([u1, u2], axis=1) @ rot
        B = U.T @ X
        assert np.abs(U.sum(axis=0)).max() < 1e-15
        Uc, Bc, sig = oracle.rayleigh_ritz(U, B)
        assert np.abs(sig - np.array([3.0, 1.0])).max() < 1e-12
        assert np.abs(Bc - want_B).max() < 1e-12
        assert np.abs(Uc - want_U).max() < 1e-12
    # and the primary rule where the sums are not zero: u = (1,1,1,1)/2 must keep a positive sum
    w1 = np.array([1.0, 1, 1, 1]) / 2
    X2 = 2.0 * np.outer(w1, v1) + 0.5 * np.outer(u2, v2)
    U = np.stack([-w1, u2], axis=1)
    Uc, Bc, _ = oracle.rayleigh_ritz(U, U.T @ X2)
    assert np.abs(Uc[:, 0] - w1).max() < 1e-12 and np.abs(Bc[0] - 2.0 * v1).max() < 1e-12
    assert np.abs(Bc[1] - np.array([0.0, 0.0, 0.5])).max() < 1e-12   # centred column: fallback rule


def test_alternating_rank1_invariants():                          # P-9 (Alg.1)
    rng = np.random.default_rng(14)
    s = np.array([5.0, 3.0, 2.0, 1.0, 0.5, 0.2])
    X, _, _ = constructed(16, 9, s, 14, sigma=0.01)
    U, B = oracle.alternating_rank1(X, rng.standard_normal((9, 4)), 2)
    assert np.abs(U.T @ U - np.eye(4)).max() < 1e-10             # deflation makes the u_i orthogonal
    assert np.abs(B - U.T @ X).max() < 1e-10                     # sum u_i v_iᵀ = P_U · X
    # many sweeps on a gapped spectrum: converges to the leading singular pairs
    Xg, Ug, _ = constructed(16, 9, np.array([5.0, 2.0, 0.8, 0.01, 0.005]), 15)
    U2, B2 = oracle.alternating_rank1(Xg, rng.standard_normal((9, 3)), 60)
    assert sin_theta(Ug[:, :3], U2) < 1e-8
    assert np.abs(np.linalg.norm(B2, axis=1) - np.array([5.0, 2.0, 0.8])).max() < 1e-8


def test_alternating_rank1_two_sweeps_worked_by_hand():          # Alg.1 with its 2 alternations
    # X = [[2,1],[0,1]], start vectors e1, e2.  Component 1 by hand:
    #   sweep 1: u = X·v/|v|² = (2,0);  v = Xᵀu/|u|² = (4,2)/4 = (1, 1/2)
    #   sweep 2: u = (5/2, 1/2)/(5/4) = (2, 2/5);  v = (4, 12/5)/(104/25) = (25/26, 15/26)
    # deflation: X − u·vᵀ = (1/26)·[[2,−4],[−10,20]] = (1/26)·(1,−5)ᵀ(2,−4), rank one, so component 2
    # is u ∝ −(1,−5) (from v0 = e2: (2,−4)·e2 < 0) and ‖u‖·vᵀ = U[:,1]ᵀ·(X − u·vᵀ) = (−2, 4)/√26.
    X = np.array([[2.0, 1.0], [0.0, 1.0]])
    U, B = oracle.alternating_rank1(X, np.eye(2), 2)
    n1 = math.sqrt(104.0 / 25.0)
    want_U = np.array([[2.0 / n1, -1.0 / math.sqrt(26.0)], [0.4 / n1, 5.0 / math.sqrt(26.0)]])
    want_B = np.array([[n1 * 25.0 / 26.0, n1 * 15.0 / 26.0], [-2.0 / math.sqrt(26.0), 4.0 / math.sqrt(26.0)]])
    assert np.abs(U - want_U).max() < 1e-14
    assert np.abs(B - want_B).max() < 1e-14
    # one sweep gives a different first component: u = (2,0), v = (1,1/2)
    U1, B1 = oracle.alternating_rank1(X, np.eye(2), 1)
    assert np.abs(U1[:, 0] - np.array([1.0, 0.0])).max() < 1e-14 and np.abs(B1[0] - np.array([2.0, 1.0])).max() < 1e-14
    # three sweeps: u = X·v/|v|² with v = (25,15)/26: (65/26, 15/26)/(850/676) = (169/85, 39/85)
    U3, _ = oracle.alternating_rank1(X, np.eye(2), 3)
    u3 = np.array([169.0, 39.0]) / 85.0
    assert np.abs(U3[:, 0] - u3 / np.linalg.norm(u3)).max() < 1e-14
    assert np.abs(U3[:, 0] - want_U[:, 0]).max() > 1e-3


def test_svd_entropy_closed_forms():                              # Eq.4
    mu, n = oracle.svd_entropy(np.ones(8))
    assert abs(mu - 3.0) < 1e-14 and n == 8                       # flat spectrum: all 8 needed
    mu, n = oracle.svd_entropy(np.array([1.0, 0, 0, 0]))
    assert abs(mu) < 1e-14 and n == 1                             # rank one
    mu, n = oracle.svd_entropy(np.array([3.0, 1.0]))
    assert abs(mu + math.log2((9 + 1) / 16.0)) < 1e-14 and n == 2


# ----------------------------- generators ---------------------------------- #
def test_generator_spectrum_and_rounding():
    c = wl.CONFIGS["tiny"]
    X, U, V = c.X(return_factors=True)
    assert np.abs(U.T @ U - np.eye(32)).max() < 1e-12
    sv = jacobi_svd(X - 0 * X)[1]
    assert abs(sv[0] - 10.0) < 0.01 and abs(sv[1] - 8.0) < 0.01
    b = wl.round_to_bf16(np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -0.3], dtype=np.float32))
    assert b[0] == 1.0 and b[1] == 1.0 + 2 ** -6                  # ties to even
    assert abs(b[2] + 0.3) < 0.3 * 2 ** -8
    s = wl.spectrum("power", 4096, 4096, 4096, alpha=1.2)
    assert abs(np.sum(s * s) - 4096 * 4096) < 1e-3 and s[0] > s[1]
