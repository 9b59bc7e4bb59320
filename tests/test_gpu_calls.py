"""GPU-vs-oracle parity of the three C-ABI calls on identical (already rounded) inputs.
Tolerances: relative Frobenius error <= 1e-4 (fp32 storage path), <= 1e-2 (bf16 MFMA path)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from util import rel_fro, sin_theta, to_dev, to_host, tol

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def atp():
    import paper_2403_02352_amd as m
    return m


def rnd(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


# ------------------------------------------------------------------ lowrank_linear
LIN_CASES = [
    # batch, m, k, n
    (1, 32, 64, 64),        # config-1 size
    (2, 300, 256, 200),     # ragged m, n: partial tiles
    (3, 129, 72, 136),      # k not a multiple of the k-tile
    (1, 1024, 512, 768),    # several 256x256 tiles
    (2, 70, 100, 36),       # k % 8 != 0 -> generic kernel
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("case", LIN_CASES)
@pytest.mark.parametrize("layout", ["kn", "nk"])
def test_lowrank_linear(atp, dtype, case, layout):
    batch, m, k, n = case
    print(f"linear {dtype} {case} {layout}", flush=True)
    B = wl.round_to_dtype(rnd((batch, m, k), 1), dtype)
    W = wl.round_to_dtype(rnd((k, n), 2, 1 / np.sqrt(k)), dtype)
    ref = np.stack([oracle.lowrank_linear(B[b], W) for b in range(batch)])
    Wd = to_dev(W if layout == "kn" else W.T, dtype)
    out = atp.lowrank_linear(to_dev(B, dtype), Wd, atp.ATP_W_KN if layout == "kn" else atp.ATP_W_NK)
    torch.cuda.synchronize()
    e = rel_fro(to_host(out), ref)
    print("  rel", e)
    assert e <= tol(dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("case", [(2, 100, 64, 96), (1, 512, 256, 1024), (2, 40, 52, 30)])
def test_lowrank_linear_swiglu_and_per_sequence_weights(atp, dtype, case):
    batch, m, k, n = case
    print(f"swiglu {dtype} {case}", flush=True)
    B = wl.round_to_dtype(rnd((batch, m, k), 3), dtype)
    W = wl.round_to_dtype(rnd((k, n), 4, 1 / np.sqrt(k)), dtype)
    ref = np.stack([oracle.lowrank_linear(B[b], W, "swiglu") for b in range(batch)])
    for layout in ("kn", "nk"):
        Wd = to_dev(W if layout == "kn" else W.T, dtype)
        out = atp.lowrank_linear(to_dev(B, dtype), Wd, atp.ATP_W_KN if layout == "kn" else atp.ATP_W_NK,
                                 atp.ATP_EPI_SWIGLU)
        assert tuple(out.shape) == (batch, m, n // 2)
        e = rel_fro(to_host(out), ref)
        print("  swiglu rel", layout, e)
        assert e <= tol(dtype)
    # per-sequence weights (the query expansion Q = U·Q' of Eq.6)
    Wb = wl.round_to_dtype(rnd((batch, k, n), 5, 1 / np.sqrt(k)), dtype)
    ref = np.stack([oracle.lowrank_linear(B[b], Wb[b]) for b in range(batch)])
    out = atp.lowrank_linear(to_dev(B, dtype), to_dev(Wb, dtype), atp.ATP_W_KN)
    e = rel_fro(to_host(out), ref)
    print("  per-seq rel", e)
    assert e <= tol(dtype)


# ------------------------------------------------------------------ attention
ATT_CASES = [
    # batch, L, r, dq, heads
    (1, 128, 32, 64, 1),      # config-1 size
    (2, 300, 100, 256, 2),    # d_h = 128, ragged L and r
    (2, 200, 64, 128, 2),     # d_h = 64, exactly one key tile
    (1, 130, 65, 128, 1),     # one key past a tile boundary
    (1, 70, 1, 128, 2),       # r = 1: output rows equal the single value row
    (1, 257, 200, 384, 3),    # three heads of 128
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("case", ATT_CASES)
def test_attention(atp, dtype, case):
    batch, L, r, dq, heads = case
    print(f"attention {dtype} {case}", flush=True)
    Q = wl.round_to_dtype(rnd((batch, L, dq), 6), dtype)
    K = wl.round_to_dtype(rnd((batch, r, dq), 7), dtype)
    V = wl.round_to_dtype(rnd((batch, r, dq), 8), dtype)
    ref = np.stack([oracle.attention(Q[b], K[b], V[b], heads) for b in range(batch)])
    out = atp.attention(to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype), heads)
    torch.cuda.synchronize()
    e = rel_fro(to_host(out), ref)
    print("  rel", e)
    assert np.isfinite(to_host(out)).all()
    assert e <= tol(dtype)
    if r == 1:
        assert np.abs(to_host(out) - V.astype(np.float64)).max() <= (2e-2 if dtype == "bf16" else 1e-6)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_peaked_scores_and_scale(atp, dtype):
    # large score range: softmax must not overflow; explicit scale argument honoured
    batch, L, r, dq, heads = 1, 96, 80, 128, 1
    Q = wl.round_to_dtype(rnd((batch, L, dq), 9, 4.0), dtype)
    K = wl.round_to_dtype(rnd((batch, r, dq), 10, 4.0), dtype)
    V = wl.round_to_dtype(rnd((batch, r, dq), 11), dtype)
    for scale in (0.0, 0.5, 0.01):
        ref = oracle.attention(Q[0], K[0], V[0], heads, scale if scale > 0 else None)[None]
        out = atp.attention(to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype), heads, scale)
        e = rel_fro(to_host(out), ref)
        print("  peaked rel", scale, e, flush=True)
        assert np.isfinite(to_host(out)).all()
        assert e <= tol(dtype)


# ------------------------------------------------------------------ principal_bases
LIN_CASES = [
    # batch, L, r, dq, heads
    (1, 128, 32, 64, 1),
    (2, 300, 100, 256, 2),    # d_h = 128, ragged L and r
    (2, 200, 64, 128, 2),     # d_h = 64
    (1, 130, 65, 128, 1),     # one key past a tile boundary
    (1, 257, 200, 384, 3),
]


def orthonormal_with_positive_sums(batch, L, r, seed):
    """U [batch, L, r] with orthonormal columns whose sums are not tiny (so that both normalisers of
    the first-order attention stay away from zero): QR of a shifted Gaussian matrix, signs fixed."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(batch):
        q, _ = np.linalg.qr(0.6 + rng.standard_normal((L, r)))
        q = q * np.where(q.sum(axis=0) < 0, -1.0, 1.0)[None, :]
        out.append(q)
    return np.stack(out)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("norm", ["taylor", "rowsum"])
@pytest.mark.parametrize("case", LIN_CASES)
def test_attention_linearised(atp, dtype, norm, case):
    """First-order attention over the principal keys (Eq.8) against the float64 oracle."""
    batch, L, r, dq, heads = case
    print(f"linearised attention {dtype} {norm} {case}", flush=True)
    U = wl.round_to_dtype(orthonormal_with_positive_sums(batch, L, r, 31), dtype)
    Q = wl.round_to_dtype(rnd((batch, L, dq), 32), dtype)
    K = wl.round_to_dtype(np.abs(rnd((batch, r, dq), 33)) * 0.3, dtype)
    V = wl.round_to_dtype(rnd((batch, r, dq), 34), dtype)
    scale = 0.02
    ref = np.stack([oracle.linearised_attention(Q[b], K[b], V[b], U[b], heads, scale=scale, norm=norm)
                    for b in range(batch)])
    out = atp.attention_linearised(to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype), to_dev(U, dtype), heads,
                                   scale=scale, norm=atp.ATP_NORM_TAYLOR if norm == "taylor" else atp.ATP_NORM_ROWSUM)
    torch.cuda.synchronize()
    got = to_host(out)
    e = rel_fro(got, ref)
    print("  rel", e)
    assert np.isfinite(got).all()
    assert e <= tol(dtype)


def check_bases(atp, X, Om, r, iters, dtype, gap_cols=None, U_sig=None, elem_cols=None):
    """X [batch, L, d] float (already rounded); returns diagnostics dict.  elem_cols: number of leading basis
    columns compared element by element with the oracle (default all; columns that only noise determines
    are individually ill-conditioned and are compared through the subspace instead)."""
    batch, L, d = X.shape
    U, B, info, Um = atp.principal_bases(to_dev(X, dtype), r, iters, to_dev(Om, "f32"), want_master=True)
    torch.cuda.synchronize()
    U, B, Um, info = to_host(U), to_host(B), to_host(Um), info.cpu().numpy()
    out = {"info": info, "orth": 0.0, "orth_master": 0.0, "coef": 0.0, "recon": 0.0, "sin": 0.0, "elem": 0.0}
    for b in range(batch):
        Xb = X[b].astype(np.float64)
        Uo, Bo = oracle.principal_bases(Xb, Om.astype(np.float64), iters)
        out["orth"] = max(out["orth"], np.abs(U[b].T @ U[b] - np.eye(r)).max())
        out["orth_master"] = max(out["orth_master"], np.abs(Um[b].T @ Um[b] - np.eye(r)).max())
        out["coef"] = max(out["coef"], rel_fro(B[b], U[b].T @ Xb))
        rg = np.linalg.norm(Xb - U[b] @ B[b])
        ro = np.linalg.norm(Xb - Uo @ Bo)
        out["recon"] = max(out["recon"], abs(rg - ro) / np.linalg.norm(Xb))
        ec = r if elem_cols is None else elem_cols
        out["elem"] = max(out["elem"], rel_fro(Um[b][:, :ec], Uo[:, :ec]))
        if gap_cols is not None:
            out["sin"] = max(out["sin"], sin_theta(Uo[:, :gap_cols], Um[b][:, :gap_cols]))
        if U_sig is not None:
            Q, _ = np.linalg.qr(Um[b])
            out["sin"] = max(out["sin"], np.linalg.norm(U_sig[b] - Q @ (Q.T @ U_sig[b]), 2))
    print("  bases", {k: (v if k == "info" else float(f"{v:.3e}")) for k, v in out.items()}, flush=True)
    if dtype == "f32" and (info == 0).all():
        # same start block, same positive-diagonal convention: on the fp32 path the basis itself must
        # match the oracle's column by column
        assert out["elem"] <= 1e-4, out["elem"]
    return out


def test_principal_bases_config1_fp32(atp):
    c = wl.CONFIGS["tiny"]
    print("bases config1 f32", flush=True)
    X = wl.round_to_dtype(c.X()[None], "f32")
    o = check_bases(atp, X, c.omega(), c.r, c.iters, "f32")
    assert (o["info"] == 0).all()
    assert o["orth"] <= 1e-5
    assert o["coef"] <= 1e-4
    assert o["recon"] <= 1e-4


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("iters", [0, 1, 3])
def test_principal_bases_small_shapes(atp, dtype, iters):
    print(f"bases small {dtype} iters={iters}", flush=True)
    L, d, r, batch = 200, 136, 40, 2          # ragged: partial tiles everywhere
    s = wl.spectrum("exp", 100, L, d, tau=12.0)
    X = np.stack([wl.make_X(L, d, s, 1e-2, 77 + b) for b in range(batch)])
    X = wl.round_to_dtype(X, dtype)
    o = check_bases(atp, X, wl.make_omega(d, r, 5), r, iters, dtype)
    assert (o["info"] == 0).all()
    assert o["orth"] <= (5e-3 if dtype == "bf16" else 1e-5)
    assert o["coef"] <= tol(dtype)
    assert o["recon"] <= tol(dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_principal_bases_gap_projector(atp, dtype):
    # constructed rank-24 signal, 1e4 gap to the noise: the leading 24 columns' span is well defined
    print(f"bases gap {dtype}", flush=True)
    L, d, r, g = 384, 256, 48, 24
    s = np.linspace(40.0, 20.0, g)
    Xs, Us = [], []
    for b in range(2):
        X, U, V = wl.make_X(L, d, s, 1e-4, 900 + b, return_factors=True)
        Xs.append(X); Us.append(U)
    X = wl.round_to_dtype(np.stack(Xs), dtype)
    # leading g-dimensional left singular subspace of the rounded input (converged oracle run)
    Ug = [oracle.principal_bases(X[b].astype(np.float64), wl.make_omega(d, g, 10), 8)[0] for b in range(2)]
    o = check_bases(atp, X, wl.make_omega(d, r, 9), r, 2, dtype, U_sig=Ug, elem_cols=g)
    assert o["sin"] <= 1e-3
    assert o["orth"] <= (5e-3 if dtype == "bf16" else 1e-5)
    assert o["coef"] <= tol(dtype)


def test_principal_bases_bert_shape_bf16(atp):
    c = wl.CONFIGS["bert_r128"]
    print("bases bert bf16", flush=True)
    X = wl.round_to_dtype(np.stack([c.X(b) for b in range(2)]), "bf16")
    o = check_bases(atp, X, c.omega(), c.r, c.iters, "bf16")
    assert (o["info"] == 0).all()
    assert o["orth"] <= 5e-3 and o["coef"] <= 1e-2 and o["recon"] <= 1e-2


def test_principal_bases_rank_deficient_input(atp):
    # rank(X) < r: qf is not unique.  Either the call certifies its result (info == 0: then U_r is
    # orthonormal and its span contains range(X)), or it flags the breakdown (info > 0); never NaN.
    print("bases rank deficient", flush=True)
    L, d, r = 128, 96, 32
    X = wl.make_X(L, d, np.linspace(5, 1, 10), 0.0, 31)[None]      # rank 10 < r
    for dtype in ("f32", "bf16"):
        Xr = wl.round_to_dtype(X, dtype)
        U, B, info, Um = atp.principal_bases(to_dev(Xr, dtype), r, 1, to_dev(wl.make_omega(d, r, 3), "f32"),
                                             want_master=True)
        torch.cuda.synchronize()
        print("  info", info.cpu().numpy(), flush=True)
        assert torch.isfinite(U.float()).all() and torch.isfinite(B.float()).all()
        if int(info[0]) == 0:
            Uh, Bh = to_host(U)[0], to_host(B)[0]
            assert np.abs(Uh.T @ Uh - np.eye(r)).max() <= (5e-3 if dtype == "bf16" else 1e-5)
            assert rel_fro(Uh @ Bh, Xr[0].astype(np.float64)) <= tol(dtype)


def test_principal_bases_zero_input_sets_info(atp):
    print("bases zero input", flush=True)
    L, d, r = 128, 96, 32
    for dtype in ("f32", "bf16"):
        X = to_dev(np.zeros((2, L, d)), dtype)
        U, B, info, _ = atp.principal_bases(X, r, 1, to_dev(wl.make_omega(d, r, 3), "f32"))
        torch.cuda.synchronize()
        print("  info", info.cpu().numpy(), flush=True)
        assert torch.isfinite(U.float()).all() and torch.isfinite(B.float()).all()
        assert (info.cpu().numpy() > 0).all()


def test_principal_bases_generated_omega_is_deterministic(atp):
    print("bases generated omega", flush=True)
    c = wl.CONFIGS["tiny"]
    X = to_dev(c.X()[None], "f32")
    a = atp.principal_bases(X, c.r, 2, None, seed=1234)
    b = atp.principal_bases(X, c.r, 2, None, seed=1234)
    d = atp.principal_bases(X, c.r, 2, None, seed=1235)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert not torch.equal(a[0], d[0])
    U = to_host(a[0])[0]
    assert np.abs(U.T @ U - np.eye(c.r)).max() <= 1e-5


def test_principal_bases_generated_omega_reaches_the_gapped_subspace(atp):
    # Omega = NULL: the library draws the start block itself, so the basis cannot be compared column by
    # column; across a 1e4 spectral gap the 24-dimensional signal subspace must still be contained in
    # the returned span (sine of the largest principal angle <= 1e-3), for any seed.
    print("bases generated omega, gapped input", flush=True)
    L, d, r, g = 384, 256, 48, 24
    s = np.linspace(40.0, 20.0, g)
    for dtype in ("f32", "bf16"):
        X = wl.round_to_dtype(np.stack([wl.make_X(L, d, s, 1e-4, 910 + b) for b in range(2)]), dtype)
        Ug = [oracle.principal_bases(X[b].astype(np.float64), wl.make_omega(d, g, 11), 8)[0] for b in range(2)]
        for seed in (1, 77):
            U, B, info, Um = atp.principal_bases(to_dev(X, dtype), r, 2, None, seed=seed, want_master=True)
            torch.cuda.synchronize()
            assert (info.cpu().numpy() == 0).all()
            Um, Uh, Bh = to_host(Um), to_host(U), to_host(B)
            for b in range(2):
                Q, _ = np.linalg.qr(Um[b])
                sin = np.linalg.norm(Ug[b] - Q @ (Q.T @ Ug[b]), 2)
                orth = np.abs(Uh[b].T @ Uh[b] - np.eye(r)).max()
                coef = rel_fro(Bh[b], Uh[b].T @ X[b].astype(np.float64))
                print(f"  {dtype} seed {seed} item {b}: sin {sin:.2e} orth {orth:.2e} coef {coef:.2e}", flush=True)
                assert sin <= 1e-3
                assert orth <= (5e-3 if dtype == "bf16" else 1e-5) and coef <= tol(dtype)


# ------------------------------------------------------------------ chained layer, config 1
def test_layer_config1_fp32_chained(atp):
    c = wl.CONFIGS["tiny"]
    print("layer config1", flush=True)
    X = wl.round_to_dtype(c.X()[None], "f32")
    Wq, Wk, Wv = (wl.round_to_dtype(c.weight(w), "f32") for w in "qkv")
    ref = oracle.atp_layer(X[0], c.omega(), c.iters, Wq, Wk, Wv, c.heads)
    Xd = to_dev(X, "f32")
    U, B, info, _ = atp.principal_bases(Xd, c.r, c.iters, to_dev(c.omega(), "f32"))
    Qp, Kp, Vp = (atp.lowrank_linear(B, to_dev(W, "f32")) for W in (Wq, Wk, Wv))
    Q = atp.lowrank_linear(U, Qp)
    O = atp.attention(Q, Kp, Vp, c.heads)
    torch.cuda.synchronize()
    e = {k: rel_fro(to_host(v)[0], ref[n]) for k, v, n in
         (("U", U, "U"), ("B", B, "B"), ("Qp", Qp, "Qp"), ("Q", Q, "Q"), ("O", O, "O"))}
    print("  chained rel", {k: float(f"{v:.3e}") for k, v in e.items()}, flush=True)
    assert e["O"] <= 1e-4
    assert e["Q"] <= 1e-4


def test_layer_with_linearised_attention_chained(atp):
    """The block with the first-order attention of Eq.8 (AtpLayer(attention_kind="linearised")): the whole chain
    against the oracle, fp32 at config-1 size and bf16 at a BERT-like size.  With the expanded normaliser
    the attention output does not depend on the basis, so the chained comparison is meaningful on bf16 too."""
    for name, dtype, T in (("tiny", "f32", 1e-4), ("bert_r128", "bf16", 1e-2)):
        c = wl.CONFIGS[name]
        nb = min(c.batch, 2)
        X = np.stack([wl.round_to_dtype(c.X(b), dtype) for b in range(nb)])
        W = {k: wl.round_to_dtype(c.weight(k), dtype) for k in "qkv"}
        scale = 0.01
        layer = atp.AtpLayer(nb, c.L, c.d, c.heads, c.r, c.iters, torch.float32 if dtype == "f32" else torch.bfloat16,
                             *(to_dev(np.ascontiguousarray(W[k].T), dtype) for k in "qkv"), Omega=to_dev(c.omega(), "f32"),
                             attention_kind="linearised", scale=scale)
        O = layer.forward(to_dev(X, dtype))
        torch.cuda.synchronize()
        for b in range(nb):
            ref = oracle.atp_layer(X[b].astype(np.float64), c.omega(), c.iters, *(W[k].astype(np.float64) for k in "qkv"),
                                   c.heads, scale=scale, attention_kind="linearised")
            e = rel_fro(to_host(O[b]), ref["O"])
            print(f"  {name}[{b}] chained linearised layer rel {e:.2e}", flush=True)
            assert e <= T


ALT_CASES = [
    # batch, L, d, r
    (1, 128, 64, 32),     # config-1 size
    (2, 130, 52, 20),     # ragged L (two row blocks), d not a power of two
    (1, 64, 256, 8),
    (3, 200, 96, 40),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", ALT_CASES)
def test_alternating_bases(atp, dtype, case):
    """Alg.1 (two alternations per component, deflation) against the float64 oracle, element by element:
    the procedure is deterministic given the start vectors."""
    batch, L, d, r = case
    print(f"alternating bases {dtype} {case}", flush=True)
    rng = np.random.default_rng(77)
    X = np.stack([wl.round_to_dtype(wl.make_X(L, d, 10.0 * 0.8 ** np.arange(min(L, d, 48)), 1e-3, 500 + b), dtype)
                  for b in range(batch)])
    V0 = rng.standard_normal((d, r)).astype(np.float32)
    U, B, info = atp.alternating_bases(to_dev(X, dtype), r, 2, to_dev(V0, "f32"))
    torch.cuda.synchronize()
    assert (info.cpu().numpy() == 0).all()
    for b in range(batch):
        Uo, Bo = oracle.alternating_rank1(X[b].astype(np.float64), V0.astype(np.float64), 2)
        eu, eb = rel_fro(to_host(U[b]), Uo), rel_fro(to_host(B[b]), Bo)
        orth = np.abs(to_host(U[b]).T @ to_host(U[b]) - np.eye(r)).max()
        print(f"  [{b}] rel U {eu:.2e} rel B {eb:.2e} orth {orth:.2e}", flush=True)
        assert eu <= tol(dtype) and eb <= tol(dtype)
        assert orth <= (5e-3 if dtype == "bf16" else 1e-4)


def test_alternating_bases_zero_input_sets_info(atp):
    X = torch.zeros((1, 96, 64), dtype=torch.float32, device="cuda")
    U, B, info = atp.alternating_bases(X, 4, 2, seed=5)
    torch.cuda.synchronize()
    assert int(info[0]) == 1
    assert torch.isfinite(U).all() and torch.isfinite(B).all()
    assert float(U.abs().max()) == 0.0 and float(B.abs().max()) == 0.0


RITZ_CASES = [
    # batch, L, d, r
    (1, 128, 64, 32),
    (2, 130, 52, 20),     # ragged sizes, odd-free but not multiples of the tile sizes
    (1, 96, 80, 33),      # odd r: the round-robin schedule runs with one padding index
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", RITZ_CASES)
def test_rayleigh_ritz(atp, dtype, case):
    """Singular-basis canonicalisation against the oracle: same (U_r, B_r) in, compare σ̃, the basis pair
    element by element (distinct, well separated singular values) and the diagnostics."""
    batch, L, d, r = case
    print(f"rayleigh-ritz {dtype} {case}", flush=True)
    rng = np.random.default_rng(55)
    s = 10.0 * 0.8 ** np.arange(r + 8)
    Us, Bs = [], []
    for b in range(batch):
        X = wl.make_X(L, d, s, 1e-3, 900 + b)
        U, B = oracle.principal_bases(X, rng.standard_normal((d, r)), 2)
        Us.append(wl.round_to_dtype(U, dtype)); Bs.append(wl.round_to_dtype(B, dtype))
    U, B = np.stack(Us), np.stack(Bs)
    Uo, Bo, sig, diag = atp.rayleigh_ritz(to_dev(U, dtype), to_dev(B, dtype), 10)
    torch.cuda.synchronize()
    for b in range(batch):
        Ur, Br, sr = oracle.rayleigh_ritz(U[b].astype(np.float64), B[b].astype(np.float64))
        es = np.abs(sig[b].cpu().numpy() - sr).max() / sr.max()
        eu, eb = rel_fro(to_host(Uo[b]), Ur), rel_fro(to_host(Bo[b]), Br)
        mu, need = oracle.svd_entropy(sr)
        dg = diag[b].cpu().numpy()
        print(f"  [{b}] sigma {es:.2e} U {eu:.2e} B {eb:.2e} offdiag {dg[1]:.1e} mu {dg[2]:.4f} (oracle {mu:.4f}) "
              f"components {int(dg[3])} (oracle {need})", flush=True)
        assert es <= 1e-5 and dg[1] <= 1e-5
        assert eu <= tol(dtype) * 3 and eb <= tol(dtype) * 3   # eigenvector sensitivity ~ eps / relative gap (0.36)
        assert abs(dg[0] - (B[b].astype(np.float64) ** 2).sum()) <= 1e-5 * dg[0]
        assert abs(dg[2] - mu) <= 1e-4 and int(dg[3]) == need


def test_rayleigh_ritz_centred_input_uses_the_fallback_sign_rule(atp):
    """Columns of U that sum to zero (centred data): the sign comes from the largest entry of b_i."""
    rng = np.random.default_rng(56)
    L, d, r = 120, 48, 12
    X = wl.make_X(L, d, 5.0 * 0.7 ** np.arange(20), 0.0, 950)
    X = X - X.mean(axis=0, keepdims=True)
    U, B = oracle.principal_bases(X, rng.standard_normal((d, r)), 3)
    assert np.abs(U.sum(axis=0)).max() < 1e-12
    Ur, Br, sr = oracle.rayleigh_ritz(U, B)
    Uo, Bo, sig, _ = atp.rayleigh_ritz(to_dev(U[None], "f32"), to_dev(B[None], "f32"), 10)
    torch.cuda.synchronize()
    eu, eb = rel_fro(to_host(Uo[0]), Ur), rel_fro(to_host(Bo[0]), Br)
    print(f"  centred: U {eu:.2e} B {eb:.2e}", flush=True)
    assert eu <= 3e-4 and eb <= 3e-4


def test_new_entry_points_degenerate_sizes(atp):
    """r = 1 and tiny shapes through the Alg.1 extractor, the Rayleigh–Ritz step and the first-order attention."""
    rng = np.random.default_rng(202)
    # Alg.1, one component, matrix smaller than any tile
    X = rng.standard_normal((1, 5, 4))
    V0 = rng.standard_normal((4, 1)).astype(np.float32)
    U, B, info = atp.alternating_bases(to_dev(X, "f32"), 1, 2, to_dev(V0, "f32"))
    Uo, Bo = oracle.alternating_rank1(X[0], V0.astype(np.float64), 2)
    assert int(info[0]) == 0
    assert rel_fro(to_host(U[0]), Uo) <= 1e-5 and rel_fro(to_host(B[0]), Bo) <= 1e-5
    # Rayleigh–Ritz with r = 1 (no rotation at all: only the sign rule) and r = 2 (a single rotation)
    for r in (1, 2):
        Xr = wl.make_X(40, 12, np.array([3.0, 1.0, 0.2]), 0.0, 77)
        Ur, Br = oracle.principal_bases(Xr, rng.standard_normal((12, r)), 2)
        Ur = -Ur; Br = -Br                                 # force the sign rule to act
        Uc, Bc, sig, diag = atp.rayleigh_ritz(to_dev(Ur[None], "f32"), to_dev(Br[None], "f32"), 4)
        U2, B2, s2 = oracle.rayleigh_ritz(Ur, Br)
        assert rel_fro(to_host(Uc[0]), U2) <= 1e-5 and rel_fro(to_host(Bc[0]), B2) <= 1e-5
        assert np.abs(sig[0].cpu().numpy() - s2).max() <= 1e-5 * s2.max()
    # first-order attention with a single principal key
    L, dq = 70, 128
    Q = wl.round_to_bf16(rng.standard_normal((1, L, dq)))
    K = wl.round_to_bf16(0.2 * np.abs(rng.standard_normal((1, 1, dq))))
    V = wl.round_to_bf16(rng.standard_normal((1, 1, dq)))
    Uq = wl.round_to_bf16(np.full((1, L, 1), 1.0 / np.sqrt(L)))
    out = atp.attention_linearised(to_dev(Q, "bf16"), to_dev(K, "bf16"), to_dev(V, "bf16"), to_dev(Uq, "bf16"), 2, scale=0.01)
    torch.cuda.synchronize()
    ref = oracle.linearised_attention(Q[0], K[0], V[0], Uq[0], 2, scale=0.01)
    assert rel_fro(to_host(out[0]), ref) <= 1e-2


ROPE_CASES = [
    # batch, L, r, dq, heads
    (1, 128, 32, 64, 1),
    (2, 300, 100, 256, 2),
    (1, 257, 72, 384, 3),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", ROPE_CASES)
def test_rope_and_principal_keys(atp, dtype, case):
    """Rotary position encoding of a key matrix and the principal keys of the rotated keys,
    K' = Uᵀ·RoPE(U·K'_0), step by step and chained, against the oracle."""
    batch, L, r, dq, heads = case
    print(f"rope {dtype} {case}", flush=True)
    rng = np.random.default_rng(91)
    U = np.stack([np.linalg.qr(rng.standard_normal((L, r)))[0] for _ in range(batch)])
    U = wl.round_to_dtype(U, dtype)
    Kp0 = wl.round_to_dtype(rnd((batch, r, dq), 92), dtype)
    Ud, Kd = to_dev(U, dtype), to_dev(Kp0, dtype)
    K = atp.lowrank_linear(Ud, Kd)                       # K = U·K'_0, per-sequence right operand
    Kr = atp.rope(K, heads, base=10000.0, pos0=3)
    Kp = atp.project_onto_bases(Ud, Kr)
    torch.cuda.synchronize()
    T = tol(dtype)
    for b in range(batch):
        Kh = to_host(K[b])
        e1 = rel_fro(to_host(Kr[b]), oracle.rope(Kh, heads, 10000.0, 3))
        e2 = rel_fro(to_host(Kp[b]), oracle.project_onto_bases(U[b], to_host(Kr[b])))
        e3 = rel_fro(to_host(Kp[b]), oracle.rope_principal_keys(U[b], Kp0[b], heads, 10000.0, 3))
        print(f"  [{b}] rope {e1:.2e} projection {e2:.2e} chained {e3:.2e}", flush=True)
        assert e1 <= T and e2 <= T and e3 <= 2 * T
    # in place gives the same bits
    K2 = K.clone()
    atp.rope(K2, heads, base=10000.0, pos0=3, out=K2)
    torch.cuda.synchronize()
    assert torch.equal(K2, Kr)


# ------------------------------------------------------------------ residual, Norm and chaining on factored pairs
NORM_CASES = [(2, 200, 136, 24, 40), (1, 128, 64, 32, 32), (3, 70, 260, 9, 5), (2, 512, 768, 128, 128)]   # batch, L, d, r1, r2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("center", [False, True])
@pytest.mark.parametrize("case", NORM_CASES)
def test_concat_and_norm_factored(atp, dtype, center, case):
    """First residual H = U1·C1 + U2·C2 as a concatenated pair, and the row-wise normalisation carried through
    the factors, against the oracle on identical (rounded) inputs; the factored result is also multiplied out
    and compared with the dense normalisation of H."""
    batch, L, d, r1, r2 = case
    print(f"norm factored {case} {dtype} center={center}", flush=True)
    U1, C1 = wl.round_to_dtype(rnd((batch, L, r1), 41, L ** -0.5), dtype), wl.round_to_dtype(rnd((batch, r1, d), 42, 3.0), dtype)
    U2, C2 = wl.round_to_dtype(rnd((batch, L, r2), 43, L ** -0.5), dtype), wl.round_to_dtype(rnd((batch, r2, d), 44, 1.0), dtype)
    if center:
        C1 = wl.round_to_dtype(C1 + 0.7, dtype)          # rows with a clear mean
    g = (1.0 + 0.2 * np.sin(np.arange(d))).astype(np.float32)
    P, C = atp.concat_factors(to_dev(U1, dtype), to_dev(C1, dtype), to_dev(U2, dtype), to_dev(C2, dtype))
    Pn, Cn = atp.norm_factored(P, C, to_dev(g, "f32"), 1e-6, center)
    torch.cuda.synchronize()
    for b in range(batch):
        Po, Co = oracle.concat_factors(U1[b], C1[b], U2[b], C2[b])
        assert np.array_equal(to_host(P[b]), Po) and np.array_equal(to_host(C[b]), Co)       # copies: exact
        Pno, Cno = oracle.norm_factored(Po, Co, g, 1e-6, center)
        ep, ec = rel_fro(to_host(Pn[b]), Pno), rel_fro(to_host(Cn[b]), Cno)
        dense = rel_fro(to_host(Pn[b]) @ to_host(Cn[b]), Pno @ Cno)
        print(f"  [{b}] rel Pn {ep:.2e} Cn {ec:.2e} multiplied out {dense:.2e}", flush=True)
        assert ep <= tol(dtype) and ec <= tol(dtype) and dense <= 2 * tol(dtype)


def test_two_blocks_chained_fp32(atp):
    """Two ATP blocks with both residuals and the Norm in factored form, the second extracting the principal
    components of the first one's output Y (small fp32 shape), against oracle.atp_block chained the same way.
    Every side uses its own bases (same start block and sign convention)."""
    # two heads of width 32 and r = 24 < 32: the attention output has rank up to 48 > r, so its extraction is well posed
    L, d, f, r, H, iters = 192, 64, 96, 24, 2, 2
    X = wl.round_to_dtype(wl.make_X(L, d, 8.0 * 0.85 ** np.arange(48), 1e-2, 1234)[None], "f32")
    Wn = [wl.round_to_dtype(wl.make_weight(d, d, 300 + i), "f32") for i in range(4)]
    Wg, Wu, Wd = (wl.round_to_dtype(w, "f32") for w in (wl.make_weight(d, f, 310), wl.make_weight(d, f, 311), wl.make_weight(f, d, 312)))
    g = np.linspace(0.8, 1.2, d).astype(np.float32)
    Om = wl.make_omega(d, r, 1234)
    dev = lambda a: to_dev(np.ascontiguousarray(a), "f32")
    Wgu = dev(np.concatenate([Wg, Wu], axis=1))

    def gpu_block(Xd):
        U, B, info, _ = atp.principal_bases(Xd, r, iters, dev(Om))
        Qp, Kp, Vp = (atp.lowrank_linear(B, dev(W)) for W in Wn[:3])
        O = atp.attention(atp.lowrank_linear(U, Qp), Kp, Vp, H)
        Uo, Bo, info_o, _ = atp.principal_bases(O, r, iters, dev(Om))
        A = atp.lowrank_linear(Bo, dev(Wn[3]))
        P, C = atp.concat_factors(U, B, Uo, A)
        Pn, Cn = atp.norm_factored(P, C, dev(g), 1e-6, False)
        F = atp.lowrank_linear(atp.lowrank_linear(Cn, Wgu, atp.ATP_W_KN, atp.ATP_EPI_SWIGLU), dev(Wd))
        Py, Cy = atp.concat_factors(P, C, Pn, F)
        Y = atp.lowrank_linear(Py, Cy)                 # dense output for the next block (per-sequence weight [C; F])
        torch.cuda.synchronize()
        assert int(info[0]) == 0 and int(info_o[0]) == 0
        return Y

    Y1 = gpu_block(dev(X))
    Y2 = gpu_block(Y1)
    o1 = oracle.atp_block(X[0].astype(np.float64), Om, iters, Wn[0], Wn[1], Wn[2], Wn[3], H, g, Wg, Wu, Wd, 1e-6)
    o2 = oracle.atp_block(o1["Y"], Om, iters, Wn[0], Wn[1], Wn[2], Wn[3], H, g, Wg, Wu, Wd, 1e-6)
    e1, e2 = rel_fro(to_host(Y1[0]), o1["Y"]), rel_fro(to_host(Y2[0]), o2["Y"])
    print(f"  chained blocks (fp32): rel. Frobenius error of Y after block 1 {e1:.2e}, after block 2 {e2:.2e}", flush=True)
    # fp32 tolerance of the path, also after four extractions in a row (measured 6e-7 and 1.3e-6)
    assert e1 <= 1e-4 and e2 <= 1e-4


def test_single_launch_factorisation_gives_up_cleanly(atp):
    """Failure handling of the single-launch factorisation, forced from the host: with a spin limit of one poll
    every wait inside the kernel gives up at once, every workgroup still exits, and the call reports info = -1
    for each sequence instead of hanging.  With the default limit restored the same call certifies its result."""
    rng = np.random.default_rng(77)
    batch, L, d, r = 2, 512, 384, 192                     # three block columns: spine and bulk workgroups both wait
    X = wl.round_to_bf16(rng.standard_normal((batch, L, d)))
    Xd, Om = to_dev(X, "bf16"), to_dev(wl.make_omega(d, r, 3), "f32")
    U0, B0, info0, _ = atp.principal_bases(Xd, r, 1, Om, want_master=True)
    torch.cuda.synchronize()
    assert (info0.cpu().numpy() == 0).all()
    try:
        atp.set_factor_spin_limit(1)
        _, _, info, _ = atp.principal_bases(Xd, r, 1, Om, want_master=True)
        torch.cuda.synchronize()
        print(f"  info with a spin limit of one poll: {info.cpu().numpy()}", flush=True)
        assert (info.cpu().numpy() == -1).all()
    finally:
        atp.set_factor_spin_limit(0)
    U1, B1, info1, _ = atp.principal_bases(Xd, r, 1, Om, want_master=True)
    torch.cuda.synchronize()
    assert (info1.cpu().numpy() == 0).all()
    assert torch.equal(U0, U1) and torch.equal(B0, B1)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_non_finite_input_is_flagged_and_stays_in_its_sequence(atp, dtype):
    """A NaN or an infinity in one sequence: the call returns, that sequence's info is non-zero, and the other
    sequence of the batch is bit-identical to what it gives alone (sequences share no arithmetic)."""
    rng = np.random.default_rng(5)
    L, d, r = 384, 256, 128
    X = wl.round_to_dtype(rng.standard_normal((2, L, d)), dtype)
    Om = to_dev(wl.make_omega(d, r, 11), "f32")
    U_ok, B_ok, info_ok, _ = atp.principal_bases(to_dev(X[1:2], dtype), r, 2, Om)
    torch.cuda.synchronize()
    assert int(info_ok[0]) == 0
    for bad in (np.nan, np.inf):
        Xb = X.copy()
        Xb[0, 7, 9] = bad
        U, B, info, _ = atp.principal_bases(to_dev(Xb, dtype), r, 2, Om)
        torch.cuda.synchronize()
        info = info.cpu().numpy()
        print(f"  {dtype}, X[0,7,9] = {bad}: info = {info}", flush=True)
        assert info[0] != 0 and info[1] == 0
        assert torch.equal(U[1], U_ok[0]) and torch.equal(B[1], B_ok[0])
