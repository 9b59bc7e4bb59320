"""Host-side tests of the C ABI (no GPU needed): the shared library loads, exports every entry
point that include/atp.h declares, and rejects bad arguments before any GPU work."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2403_02352_amd", "libatp.so")
HEADER = os.path.join(ROOT, "include", "atp.h")

OK, INVALID, BAD_RANK, WORKSPACE, UNSUPPORTED, DEVICE = range(6)
F32, BF16 = 0, 1


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
    L = C.CDLL(LIB)
    i64, sz, vp, i32 = C.c_int64, C.c_size_t, C.c_void_p, C.c_int
    L.atp_status_string.restype = C.c_char_p
    L.atp_status_string.argtypes = [i32]
    L.atp_principal_bases_workspace.restype = sz
    L.atp_principal_bases_workspace.argtypes = [i64, i64, i64, i64, i32, i32]
    L.atp_principal_bases.restype = i32
    L.atp_principal_bases.argtypes = [vp, i64, i64, i64, i64, i32, vp, C.c_uint64, vp, vp, vp, vp, vp, sz, i32, vp]
    L.atp_lowrank_linear_workspace.restype = sz
    L.atp_lowrank_linear_workspace.argtypes = [i64, i64, i64, i64, i64, i32, i32]
    L.atp_lowrank_linear.restype = i32
    L.atp_lowrank_linear.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, vp, sz, i32, vp]
    L.atp_attention_workspace.restype = sz
    L.atp_attention_workspace.argtypes = [i64, i64, i64, i64, i32, i32]
    L.atp_attention.restype = i32
    L.atp_attention.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i32, C.c_float, vp, sz, i32, vp]
    L.atp_attention_linearised_workspace.restype = sz
    L.atp_attention_linearised_workspace.argtypes = [i64, i64, i64, i64, i32, i32]
    L.atp_attention_linearised.restype = i32
    L.atp_attention_linearised.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, C.c_float, i32, vp, sz, i32, vp]
    L.atp_alternating_bases_workspace.restype = sz
    L.atp_alternating_bases_workspace.argtypes = [i64, i64, i64, i64, i32]
    L.atp_alternating_bases.restype = i32
    L.atp_alternating_bases.argtypes = [vp, i64, i64, i64, i64, i32, vp, C.c_uint64, vp, vp, vp, vp, sz, i32, vp]
    L.atp_rayleigh_ritz_workspace.restype = sz
    L.atp_rayleigh_ritz_workspace.argtypes = [i64, i64, i64, i64, i32]
    L.atp_rayleigh_ritz.restype = i32
    L.atp_rayleigh_ritz.argtypes = [vp, vp, i64, i64, i64, i64, i32, vp, vp, vp, vp, vp, sz, i32, vp]
    L.atp_rope.restype = i32
    L.atp_rope.argtypes = [vp, vp, i64, i64, i64, i32, C.c_float, i64, i32, vp]
    L.atp_project_onto_bases_workspace.restype = sz
    L.atp_project_onto_bases_workspace.argtypes = [i64, i64, i64, i64, i32]
    L.atp_project_onto_bases.restype = i32
    L.atp_project_onto_bases.argtypes = [vp, vp, vp, i64, i64, i64, i64, vp, sz, i32, vp]
    L.atp_profile_read.restype = i32
    L.atp_profile_read.argtypes = [i32, vp, vp, vp, vp]
    L.atp_attention_static.restype = i32
    L.atp_attention_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i32, C.c_float, i32, vp]
    L.atp_concat_factors.restype = i32
    L.atp_concat_factors.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, vp]
    L.atp_norm_factored_workspace.restype = sz
    L.atp_norm_factored_workspace.argtypes = [i64, i64, i64, i64, i32]
    L.atp_norm_factored.restype = i32
    L.atp_norm_factored.argtypes = [vp, vp, vp, C.c_float, i32, vp, vp, i64, i64, i64, i64, vp, sz, i32, vp]
    L.atp_set_factor_mode.restype = None
    L.atp_set_factor_mode.argtypes = [i32]
    return L


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(atp_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported(lib):
    names = declared_functions()
    assert {"atp_principal_bases", "atp_lowrank_linear", "atp_attention", "atp_principal_bases_workspace",
            "atp_lowrank_linear_workspace", "atp_attention_workspace", "atp_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in atp.h but not exported"


def test_status_strings(lib):
    seen = {lib.atp_status_string(i) for i in range(6)}
    assert len(seen) == 6 and all(seen)
    assert b"rank" in lib.atp_status_string(BAD_RANK)


# fake device pointers: never dereferenced on the host; validation happens before any GPU call
P = 0x10000


def bases(lib, X=P, batch=1, L=128, d=64, r=32, iters=2, Om=P, U=P, B=P, ws=P, ws_bytes=None, t=F32):
    need = lib.atp_principal_bases_workspace(batch, L, d, r, iters, t)
    if ws_bytes is None:
        ws_bytes = need
    return lib.atp_principal_bases(X, batch, L, d, r, iters, Om, 0, U, B, None, None, ws, ws_bytes, t, None)


def test_principal_bases_argument_checks(lib):
    assert bases(lib, X=None) == INVALID
    assert bases(lib, U=None) == INVALID
    assert bases(lib, B=None) == INVALID
    assert bases(lib, batch=0) == INVALID
    assert bases(lib, L=0) == INVALID
    assert bases(lib, iters=-1) == INVALID
    assert bases(lib, t=7) == INVALID
    assert bases(lib, X=P + 4) == INVALID                      # misaligned
    assert bases(lib, r=0) == BAD_RANK
    assert bases(lib, r=65) == BAD_RANK                        # r > min(L, d) = 64
    assert bases(lib, L=40, d=64, r=41) == BAD_RANK
    assert bases(lib, ws=None) == WORKSPACE
    assert bases(lib, ws_bytes=1024) == WORKSPACE


def test_workspace_queries(lib):
    a = lib.atp_principal_bases_workspace(1, 128, 64, 32, 2, F32)
    b = lib.atp_principal_bases_workspace(2, 128, 64, 32, 2, F32)
    c = lib.atp_principal_bases_workspace(1, 256, 64, 32, 2, F32)
    assert 0 < a < b and a < c
    assert lib.atp_principal_bases_workspace(0, 128, 64, 32, 2, F32) == 0
    # (bf16, [k, n] weights) needs room for the transposed copy; every other combination needs none
    assert lib.atp_lowrank_linear_workspace(2, 64, 32, 48, 0, 0, BF16) >= 32 * 48 * 2
    assert lib.atp_lowrank_linear_workspace(2, 64, 32, 48, 32 * 48, 0, BF16) >= 2 * 32 * 48 * 2
    assert lib.atp_lowrank_linear_workspace(2, 64, 32, 48, 0, 1, BF16) == 0
    assert lib.atp_lowrank_linear_workspace(2, 64, 32, 48, 0, 0, F32) == 0
    assert lib.atp_attention_workspace(1, 128, 100, 256, 2, BF16) >= 256 * 128 * 2   # r padded to 128
    assert lib.atp_attention_workspace(1, 128, 100, 256, 2, F32) == 0


def test_lowrank_linear_argument_checks(lib):
    def call(Bp=P, W=P, out=P, batch=1, m=8, k=16, n=8, stride=0, layout=1, epi=0, ws=None, wsb=0, t=F32):
        return lib.atp_lowrank_linear(Bp, W, out, batch, m, k, n, stride, layout, epi, ws, wsb, t, None)
    assert call(Bp=None) == INVALID
    assert call(W=None) == INVALID
    assert call(out=None) == INVALID
    assert call(m=0) == INVALID
    assert call(layout=2) == INVALID
    assert call(epi=5) == INVALID
    assert call(n=7, epi=1) == INVALID                         # SwiGLU needs an even n
    assert call(stride=-1) == INVALID
    assert call(t=BF16, layout=0) == WORKSPACE                 # transposed copy needs a workspace


def test_attention_argument_checks(lib):
    def call(Q=P, K=P, V=P, O=P, batch=1, L=16, r=8, dq=128, heads=1, ws=P, wsb=1 << 20, t=BF16):
        return lib.atp_attention(Q, K, V, O, batch, L, r, dq, heads, 0.0, ws, wsb, t, None)
    assert call(Q=None) == INVALID
    assert call(r=0) == INVALID
    assert call(dq=130, heads=4) == INVALID                    # dq % heads != 0
    assert call(dq=96, heads=1) == UNSUPPORTED                 # bf16 kernel: head width 64 or 128
    assert call(dq=512, heads=1, t=F32) == UNSUPPORTED         # fp32 kernel: head width <= 256
    assert call(ws=None) == WORKSPACE
    assert call(wsb=16) == WORKSPACE


def test_linearised_attention_and_alternating_argument_checks(lib):
    def lin(Q=P, K=P, V=P, U=P, O=P, batch=1, L=16, r=8, dq=128, heads=1, norm=0, ws=P, wsb=1 << 20, t=BF16):
        return lib.atp_attention_linearised(Q, K, V, U, O, batch, L, r, dq, heads, 0.0, norm, ws, wsb, t, None)
    assert lin(U=None) == INVALID
    assert lin(norm=7) == INVALID
    assert lin(dq=96) == UNSUPPORTED
    assert lin(wsb=16) == WORKSPACE
    assert lib.atp_attention_linearised_workspace(2, 100, 40, 128, 1, F32) > 0   # column sums need it on both paths

    def alt(X=P, U=P, B=P, batch=1, L=64, d=64, r=8, sweeps=2, ws=P, wsb=1 << 30, t=F32):
        return lib.atp_alternating_bases(X, batch, L, d, r, sweeps, None, 0, U, B, None, ws, wsb, t, None)
    assert alt(X=None) == INVALID
    assert alt(sweeps=0) == INVALID
    assert alt(r=65) == BAD_RANK
    assert alt(d=8192, L=8192) == UNSUPPORTED                   # one row pass covers at most 4096 columns
    assert alt(d=66, L=128) == UNSUPPORTED                      # 16-byte row pieces
    assert alt(wsb=1024) == WORKSPACE
    assert lib.atp_alternating_bases_workspace(1, 64, 64, 8, F32) >= 64 * 64 * 4

    P2 = 0x20000
    def rr(U=P, B=P, Uo=P2, Bo=P2, sig=P, batch=1, L=64, d=64, r=8, sweeps=10, ws=P, wsb=1 << 30, t=F32):
        return lib.atp_rayleigh_ritz(U, B, batch, L, d, r, sweeps, Uo, Bo, sig, None, ws, wsb, t, None)
    assert rr(U=None) == INVALID
    assert rr(Uo=P) == INVALID                                   # outputs must not alias the inputs
    assert rr(sweeps=0) == INVALID
    assert rr(r=65) == BAD_RANK
    assert rr(wsb=64) == WORKSPACE

    assert lib.atp_rope(None, P, 1, 8, 128, 2, 10000.0, 0, BF16, None) == INVALID
    assert lib.atp_rope(P, P, 1, 8, 130, 4, 10000.0, 0, BF16, None) == INVALID      # dq % heads != 0
    assert lib.atp_rope(P, P, 1, 8, 6, 2, 10000.0, 0, BF16, None) == INVALID        # odd head width
    assert lib.atp_rope(P, P, 1, 8, 128, 2, 1.0, 0, BF16, None) == INVALID          # base must exceed 1
    assert lib.atp_project_onto_bases(P, None, P, 1, 64, 8, 128, P, 1 << 30, BF16, None) == INVALID
    assert lib.atp_project_onto_bases(P, P, P, 1, 64, 8, 128, P, 16, BF16, None) == WORKSPACE
    assert lib.atp_project_onto_bases_workspace(1, 64, 8, 128, F32) == 0


def test_profile_read_rejects_bad_class(lib):
    assert lib.atp_profile_read(-1, None, None, None, None) == INVALID
    assert lib.atp_profile_read(99, None, None, None, None) == INVALID


def test_static_attention_rejects_what_does_not_fit_its_built_in_scratch(lib):
    """The entry point that allocates nothing checks its arguments like atp_attention and refuses inputs whose
    re-laid-out values exceed the built-in buffer (32 MiB), all before any GPU work."""
    def call(Q=P, K=P, V=P, O=P, batch=1, L=16, r=8, dq=128, heads=1, t=BF16):
        return lib.atp_attention_static(Q, K, V, O, batch, L, r, dq, heads, 0.0, t, None)
    SCRATCH_LIMIT = 6
    assert lib.atp_status_string(SCRATCH_LIMIT) not in (None, b"")
    assert call(Q=None) == INVALID
    assert call(r=0) == INVALID
    assert call(dq=130, heads=4) == INVALID
    assert call(dq=96, heads=1) == UNSUPPORTED
    assert call(t=7) == INVALID
    assert call(batch=4, L=4096, r=1088, dq=4096, heads=32) == SCRATCH_LIMIT      # 4*4096*1088*2 bytes > 32 MiB
    assert call(batch=8, L=4096, r=1024, dq=4096, heads=32) == SCRATCH_LIMIT


def test_factored_residual_and_norm_argument_checks(lib):
    def cat(U1=P, C1=P, U2=P, C2=P, Po=P, Co=P, batch=1, L=64, d=32, r1=8, r2=8, t=F32):
        return lib.atp_concat_factors(U1, C1, U2, C2, Po, Co, batch, L, d, r1, r2, t, None)
    assert cat(U1=None) == INVALID
    assert cat(Co=None) == INVALID
    assert cat(r2=0) == INVALID
    assert cat(t=5) == INVALID
    assert cat(U2=0x1008) == INVALID                            # not 16-byte aligned
    assert cat(L=70000) == UNSUPPORTED

    def norm(Pi=P, Ci=P, g=P, eps=1e-6, center=0, Pn=P, Cn=P, batch=1, L=64, d=32, m=16, ws=P, wsb=1 << 24, t=F32):
        return lib.atp_norm_factored(Pi, Ci, g, eps, center, Pn, Cn, batch, L, d, m, ws, wsb, t, None)
    assert norm(g=None) == INVALID
    assert norm(eps=-1.0) == INVALID
    assert norm(m=0) == INVALID
    assert norm(t=9) == INVALID
    assert norm(ws=None) == WORKSPACE
    need = lib.atp_norm_factored_workspace(1, 64, 32, 16, F32)
    assert need > 0 and norm(wsb=need - 1) == WORKSPACE
    assert lib.atp_norm_factored_workspace(0, 64, 32, 16, F32) == 0


def test_factor_mode_setter_clamps(lib):
    for v in (-3, 0, 1, 2, 99):
        lib.atp_set_factor_mode(v)      # host-side setter: any value is accepted and clamped to 0..2
    lib.atp_set_factor_mode(1)
