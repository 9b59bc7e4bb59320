"""Plain float64 CPU oracle of the ATP hot path (numpy).  TEST INFRASTRUCTURE.

Only `tests/`, `__graft_entry__.smoke()` and `bench.py`'s `cpu_baseline` leg may
import this module; the product path never does.  It shares no code with the
HIP kernels.  Every function is the definition written out (a library matmul or
LAPACK factorisation serves as one step); there is no blocking, fusion or
reordering, so it can be checked against the paper by eye.

Notation follows the paper: X (L×d) hidden state, U (L×r) orthonormal basis,
X' = B_r (r×d) principal components, W (d×d') projection, Q', K', V' (r×d')
principal queries/keys/values.

Pin status (see tests/test_oracle_pins.py):
  qf, principal_bases, lowrank_linear, attention, linearised_attention,
  alternating_rank1 (including a two-sweep example worked by hand),
  rayleigh_ritz (both sign rules on hand-built examples), rope (angles at
  d_h = 2, 4, 8 in closed form), svd_entropy, concat_factors, norm_factored
  (against the dense row-wise normalisation written with loops): pinned by
  closed forms, invariants, brute force and special cases.
  atp_block: every step is a pinned function; the way residuals and Norm are
  carried in factored form is a reading of Fig.3 — parity unpinned.
  atp_layer: each step is a pinned function; WHICH basis the layer should use,
  and the meaning of the output projection / FFN "on the r bases", are fixed by
  convention only (the paper gives no equation for them) — parity unpinned for
  those two conventions.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- #
# Orthonormalisation: Q factor of the thin QR with positive-diagonal R.
# The paper requires UᵀU = I (text after Eq.8) without naming a method; the
# positive-diagonal convention makes the factor unique for full column rank.
# --------------------------------------------------------------------------- #
def qf(Z: np.ndarray) -> np.ndarray:
    Z = np.asarray(Z, dtype=np.float64)
    Q, R = np.linalg.qr(Z, mode="reduced")
    sgn = np.where(np.diag(R) < 0.0, -1.0, 1.0)
    return Q * sgn[None, :]


# --------------------------------------------------------------------------- #
# Principal bases: X ≈ U_r · B_r  (Eq.5), B_r targets the best rank-r
# approximation of Eq.9.  Block orthogonal iteration:
#   U ← qf(X·Ω);  repeat iters times { V ← qf(Xᵀ·U);  U ← qf(X·V) };
#   B_r = U_rᵀ·X.
# In exact arithmetic U_r = qf( X (XᵀX)^iters Ω ).
# --------------------------------------------------------------------------- #
def principal_bases(X: np.ndarray, Omega: np.ndarray, iters: int):
    X = np.asarray(X, dtype=np.float64)
    Omega = np.asarray(Omega, dtype=np.float64)
    L, d = X.shape
    assert Omega.shape[0] == d
    r = Omega.shape[1]
    assert 1 <= r <= min(L, d) and iters >= 0
    U = qf(X @ Omega)
    for _ in range(iters):
        V = qf(X.T @ U)
        U = qf(X @ V)
    B = U.T @ X
    return U, B


# --------------------------------------------------------------------------- #
# Low-rank linear layer: Q', K', V' = X'·{W^Q, W^K, W^V}  (Eq.6, Tab.1 row
# "Projection").  epilogue "swiglu": SiLU(first half) ⊙ second half, the gated
# feed-forward used when the FFN also runs on the r bases (end of Sec.4.3).
# --------------------------------------------------------------------------- #
def lowrank_linear(B: np.ndarray, W: np.ndarray, epilogue: str = "none") -> np.ndarray:
    B = np.asarray(B, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    out = B @ W
    if epilogue == "none":
        return out
    if epilogue == "swiglu":
        n = out.shape[-1]
        assert n % 2 == 0
        g, u = out[..., : n // 2], out[..., n // 2:]
        return g / (1.0 + np.exp(-g)) * u
    raise ValueError(epilogue)


# --------------------------------------------------------------------------- #
# Attention of all L queries over the r principal keys/values (Fig.2b, Tab.1
# row "Attention"): the standard procedure of Eq.1 with K', V' in place of K, V.
# Heads are column slices of width d_h; scale defaults to 1/sqrt(d_h).
# --------------------------------------------------------------------------- #
def attention(Q: np.ndarray, K_r: np.ndarray, V_r: np.ndarray, heads: int,
              scale: float | None = None) -> np.ndarray:
    Q = np.asarray(Q, dtype=np.float64)
    K_r = np.asarray(K_r, dtype=np.float64)
    V_r = np.asarray(V_r, dtype=np.float64)
    L, dq = Q.shape
    r = K_r.shape[0]
    assert K_r.shape == (r, dq) and V_r.shape == (r, dq) and dq % heads == 0
    dh = dq // heads
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(dh)
    O = np.empty((L, dq), dtype=np.float64)
    for h in range(heads):
        c = slice(h * dh, (h + 1) * dh)
        S = scale * (Q[:, c] @ K_r[:, c].T)          # L×r scores
        S = S - S.max(axis=1, keepdims=True)
        P = np.exp(S)
        P = P / P.sum(axis=1, keepdims=True)           # row softmax over r keys
        O[:, c] = P @ V_r[:, c]
    return O


# --------------------------------------------------------------------------- #
# First-order ("linearised") attention over the principal keys (Eq.8): with exp
# replaced by its first-order Taylor expansion the unnormalised attention of a
# query q on all L tokens becomes A'·V' with the 1×r map
#     A' = 1·U + scale·q·K'ᵀ            (1 ∈ R^{1×L}: 1·U = column sums of U).
# The text after Eq.8 asks for a row-wise normalisation of A' without giving a formula; it is read in
# two ways (`norm`):
#   "taylor": divide by the same expansion of the softmax denominator,
#             Σ_j (1 + scale·q·k_j) = L + scale·(q·K'ᵀ)·(1·U)ᵀ  (sum over tokens j);
#   "rowsum": divide by the sum of the r entries of A'.
# Heads are column slices of width d_h; 1·U is shared by the heads.
# --------------------------------------------------------------------------- #
def linearised_attention(Q: np.ndarray, K_r: np.ndarray, V_r: np.ndarray, U: np.ndarray, heads: int,
                         scale: float | None = None, norm: str = "taylor") -> np.ndarray:
    Q = np.asarray(Q, dtype=np.float64)
    K_r = np.asarray(K_r, dtype=np.float64)
    V_r = np.asarray(V_r, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    L, dq = Q.shape
    r = K_r.shape[0]
    assert K_r.shape == (r, dq) and V_r.shape == (r, dq) and U.shape[1] == r and dq % heads == 0
    assert norm in ("taylor", "rowsum")
    n_tokens = U.shape[0]
    dh = dq // heads
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(dh)
    ones_U = U.sum(axis=0)                               # 1·U, length r
    O = np.empty((L, dq), dtype=np.float64)
    for h in range(heads):
        c = slice(h * dh, (h + 1) * dh)
        S = scale * (Q[:, c] @ K_r[:, c].T)              # L×r
        A = ones_U[None, :] + S                           # A'
        if norm == "taylor":
            den = n_tokens + S @ ones_U
        else:
            den = A.sum(axis=1)
        O[:, c] = (A @ V_r[:, c]) / den[:, None]
    return O


# --------------------------------------------------------------------------- #
# Rotary position encoding and principal keys under it (Sec. "Combine with
# Position Encoding"): k_i = x_i·W^K·R_i with R_i the rotary matrix of position i;
# the r principal keys are then the coordinates of the rotated key matrix in the
# basis U: K' = Uᵀ·RoPE(U·K'_0), K'_0 = X'·W^K.
# The paper does not fix the layout of R_i; the half-split pairing of the Llama
# family is used: within a head of width d_h, coordinate j < d_h/2 is paired with
# j + d_h/2 and the pair is rotated by the angle (pos0 + i)·base^(-2j/d_h).
# --------------------------------------------------------------------------- #
def rope(Y: np.ndarray, heads: int, base: float = 10000.0, pos0: int = 0) -> np.ndarray:
    Y = np.asarray(Y, dtype=np.float64)
    L, dq = Y.shape
    assert dq % heads == 0 and (dq // heads) % 2 == 0
    dh = dq // heads
    half = dh // 2
    out = np.empty_like(Y)
    pos = pos0 + np.arange(L, dtype=np.float64)
    for h in range(heads):
        for j in range(half):
            ang = pos * base ** (-2.0 * j / dh)
            c, s = np.cos(ang), np.sin(ang)
            a, b = Y[:, h * dh + j], Y[:, h * dh + j + half]
            out[:, h * dh + j] = a * c - b * s
            out[:, h * dh + j + half] = a * s + b * c
    return out


def project_onto_bases(U: np.ndarray, Y: np.ndarray) -> np.ndarray:
    """Coordinates of the rows-space projection of Y on the basis U: Uᵀ·Y (r×dq)."""
    return np.asarray(U, dtype=np.float64).T @ np.asarray(Y, dtype=np.float64)


def rope_principal_keys(U: np.ndarray, Kp0: np.ndarray, heads: int, base: float = 10000.0, pos0: int = 0):
    """K' = Uᵀ·RoPE(U·K'_0): principal keys of the rotated key matrix."""
    return project_onto_bases(U, rope(np.asarray(U, dtype=np.float64) @ np.asarray(Kp0, dtype=np.float64),
                                      heads, base, pos0))


# --------------------------------------------------------------------------- #
# Standard self-attention layer (Eq.1-2): the dense comparator.
# --------------------------------------------------------------------------- #
def dense_attention_layer(X, Wq, Wk, Wv, heads: int, scale: float | None = None):
    X = np.asarray(X, dtype=np.float64)
    return attention(X @ Wq, X @ Wk, X @ Wv, heads, scale)


# --------------------------------------------------------------------------- #
# One ATP block (Fig.3): extraction → projections of the r bases (Eq.6) →
# Q = U·Q' (Eq.6) → attention over the r principal keys/values.  Optional
# continuation on the bases: second extraction on the attention output followed
# by the output projection, and a SwiGLU feed-forward applied row-wise to the
# r×d basis matrix; the result stays factored as (U_o, F).
# --------------------------------------------------------------------------- #
def atp_layer(X, Omega, iters, Wq, Wk, Wv, heads, scale=None,
              Wo=None, Omega_o=None, Wgate=None, Wup=None, Wdown=None, attention_kind="softmax"):
    U, B = principal_bases(X, Omega, iters)
    Qp = lowrank_linear(B, Wq)
    Kp = lowrank_linear(B, Wk)
    Vp = lowrank_linear(B, Wv)
    Q = U @ Qp
    if attention_kind == "softmax":
        O = attention(Q, Kp, Vp, heads, scale)
    else:   # first-order attention of Eq.8, normaliser expanded the same way
        assert attention_kind == "linearised"
        O = linearised_attention(Q, Kp, Vp, U, heads, scale, "taylor")
    out = {"U": U, "B": B, "Qp": Qp, "Kp": Kp, "Vp": Vp, "Q": Q, "O": O}
    if Wo is None:
        return out
    Uo, Bo = principal_bases(O, Omega if Omega_o is None else Omega_o, iters)
    A = lowrank_linear(Bo, Wo)
    out.update({"Uo": Uo, "Bo": Bo, "A": A})
    if Wgate is None:
        return out
    G = lowrank_linear(A, np.concatenate([Wgate, Wup], axis=1), "swiglu")
    F = lowrank_linear(G, Wdown)
    out.update({"G": G, "F": F})
    return out


# --------------------------------------------------------------------------- #
# Residual, Norm and block chaining in factored form (Fig.3 and the last
# paragraph of Sec.4.2).  Fig.3 draws one residual arrow from the rank-r
# representation X' around the attention into "Norm" and one around the
# feed-forward; it gives no equations, and X' (r×d) and the attention output
# (L×d') do not even have the same number of rows.  Reading used here:
#   * what the block holds of its input is the pair (U, X'), so the first residual adds
#     U·X' to the attention branch U_o·A:  H = U·X' + U_o·A = [U | U_o]·[X'; A] = P·C,
#     a factored matrix of rank <= 2r (concat_factors);
#   * "Norm" is the row-wise normalisation of the model family (RMSNorm for Llama;
#     with `center` the mean is removed first, LayerNorm without bias, for BERT), with
#     gain g.  It keeps the factored form: Norm(H) = (D·P)·((C − c̄·1ᵀ)·diag(g)),
#     c̄ = C·1/d, D = diag(1/sqrt(var_i + eps)), var_i the mean square of row i;
#   * the feed-forward acts row-wise on the coefficient matrix (as in atp_layer) and the
#     second residual gives Y = P·C + P̃·F = [P | P̃]·[C; F];
#   * the next block starts from the dense Y (it "first attains the principal
#     components of Y").
# Parity of these conventions with the paper is unpinned (no equation exists); the
# arithmetic of each function is pinned against the dense definitions.
# --------------------------------------------------------------------------- #
def concat_factors(U1, C1, U2, C2):
    """(U1, C1), (U2, C2) -> (P, C) with P·C = U1·C1 + U2·C2: P = [U1 | U2], C = [C1; C2]."""
    P = np.concatenate([np.asarray(U1, dtype=np.float64), np.asarray(U2, dtype=np.float64)], axis=1)
    C = np.concatenate([np.asarray(C1, dtype=np.float64), np.asarray(C2, dtype=np.float64)], axis=0)
    return P, C


def norm_factored(P, C, gain, eps: float = 1e-6, center: bool = False):
    """Row-wise normalisation of H = P·C returned as a factored pair (Pn, Cn), Pn·Cn = Norm(H)."""
    P = np.asarray(P, dtype=np.float64)
    C = np.asarray(C, dtype=np.float64)
    gain = np.asarray(gain, dtype=np.float64)
    H = P @ C                                            # the definition: statistics of the rows of H itself
    if center:
        H = H - H.mean(axis=1, keepdims=True)
        C = C - C.mean(axis=1, keepdims=True)            # rows of P·(C − c̄·1ᵀ) are the centred rows of H
    var = np.mean(H * H, axis=1)
    Pn = P / np.sqrt(var + eps)[:, None]
    Cn = C * gain[None, :]
    return Pn, Cn


def atp_block(X, Omega, iters, Wq, Wk, Wv, Wo, heads, gain, Wgate, Wup, Wdown, eps: float = 1e-6, center: bool = False,
              scale=None):
    """One ATP block with both residuals and the Norm in factored form; returns the dense output Y and the parts."""
    o = atp_layer(X, Omega, iters, Wq, Wk, Wv, heads, scale, Wo)
    P, C = concat_factors(o["U"], o["B"], o["Uo"], o["A"])           # H = U·X' + U_o·A
    Pn, Cn = norm_factored(P, C, gain, eps, center)
    G = lowrank_linear(Cn, np.concatenate([Wgate, Wup], axis=1), "swiglu")
    F = lowrank_linear(G, Wdown)
    Py, Cy = concat_factors(P, C, Pn, F)                               # Y = H + Norm(H)-branch
    o.update({"P": P, "C": C, "Pn": Pn, "Cn": Cn, "G2": G, "F2": F, "Py": Py, "Cy": Cy, "Y": Py @ Cy})
    return o


# --------------------------------------------------------------------------- #
# Canonical (singular) form of a basis pair: rotate (U, B) so that the rows of
# B are σ̃_i ṽ_iᵀ in descending order, the X' of Eq.9.  Rayleigh–Ritz on
# T = B·Bᵀ.  Sign rule: 1ᵀu_i ≥ 0 (the 1·U term of Eq.8), falling back to
# "largest-magnitude entry of b_i positive" when 1ᵀu_i is numerically zero.
# --------------------------------------------------------------------------- #
def rayleigh_ritz(U: np.ndarray, B: np.ndarray):
    U = np.asarray(U, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    lam, R = np.linalg.eigh(B @ B.T)
    order = np.argsort(-lam, kind="stable")
    lam, R = lam[order], R[:, order]
    Uc, Bc = U @ R, R.T @ B
    L = U.shape[0]
    for i in range(Uc.shape[1]):
        t = Uc[:, i].sum()
        if abs(t) < 1e-8 * np.sqrt(L):
            j = np.argmax(np.abs(Bc[i]))
            t = Bc[i, j]
        if t < 0:
            Uc[:, i] *= -1.0
            Bc[i] *= -1.0
    return Uc, Bc, np.sqrt(np.maximum(lam, 0.0))


# --------------------------------------------------------------------------- #
# The paper's own extractor (Alg.1, appendix "Alternating Optimization"):
# rank-1 alternating least squares with deflation, `sweeps` alternations per
# component (the paper uses 2).  Returns (U_r, B_r) with normalised u_i:
# U_r[:, i] = u_i/‖u_i‖, B_r[i] = ‖u_i‖·v_iᵀ.
# --------------------------------------------------------------------------- #
def _rank1_fit(R: np.ndarray, v: np.ndarray, sweeps: int):
    """Alternating least squares for R ≈ u·vᵀ: with v fixed the best u is R·v/(vᵀv), with u fixed the
    best v is Rᵀ·u/(uᵀu); one sweep does both, in that order."""
    u = None
    for _ in range(sweeps):
        u = R @ v / (v @ v)
        v = R.T @ u / (u @ u)
    return u, v


def alternating_rank1(X: np.ndarray, V0: np.ndarray, sweeps: int = 2):
    V0 = np.asarray(V0, dtype=np.float64)          # d×r start vectors, one per component
    R = np.array(X, dtype=np.float64, copy=True)   # what is left of X after the components found so far
    pairs = []
    for v0 in V0.T:
        u, v = _rank1_fit(R, v0.copy(), sweeps)
        R = R - np.outer(u, v)
        pairs.append((u, v))
    norms = [np.linalg.norm(u) for u, _ in pairs]
    U = np.stack([u / n for (u, _), n in zip(pairs, norms)], axis=1)
    B = np.stack([n * v for (_, v), n in zip(pairs, norms)], axis=0)
    return U, B


# --------------------------------------------------------------------------- #
# SVD-entropy "low-rankness" (Eq.4): mu = -log2( sum_i sbar_i² ),
# sbar_i = sigma_i / sum sigma;  ceil(2^mu) = components needed.
# --------------------------------------------------------------------------- #
def svd_entropy(sigma: np.ndarray):
    sigma = np.asarray(sigma, dtype=np.float64)
    sbar = sigma / sigma.sum()
    mu = -np.log2(np.sum(sbar * sbar))
    return mu, int(np.ceil(2.0 ** mu - 1e-12))
