"""ctypes binding of libatp.so.  Names mirror the C entry points."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

ATP_F32, ATP_BF16 = 0, 1
ATP_W_KN, ATP_W_NK = 0, 1
ATP_EPI_NONE, ATP_EPI_SWIGLU = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libatp.so")


class AtpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib.atp_status_string(status).decode()} (status {status})")


def _load() -> C.CDLL:
    p = lib_path()
    if not os.path.exists(p):
        raise ImportError(
            f"{p} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'); "
            "there is no fallback path")
    L = C.CDLL(p)
    i64, sz, vp, i32 = C.c_int64, C.c_size_t, C.c_void_p, C.c_int
    L.atp_status_string.restype = C.c_char_p
    L.atp_status_string.argtypes = [i32]
    L.atp_version.restype = C.c_char_p
    L.atp_version.argtypes = []
    L.atp_set_qr_passes.restype = None
    L.atp_set_qr_passes.argtypes = [i32, i32, i32]
    L.atp_set_overlap.restype = None
    L.atp_set_overlap.argtypes = [i32]
    L.atp_set_conditioning_gram.restype = None
    L.atp_set_conditioning_gram.argtypes = [i32]
    L.atp_set_factor_mode.restype = None
    L.atp_set_factor_mode.argtypes = [i32]
    L.atp_set_factor_spin_limit.restype = None
    L.atp_set_factor_spin_limit.argtypes = [i32]
    L.atp_principal_bases_workspace.restype = sz
    L.atp_principal_bases_workspace.argtypes = [i64, i64, i64, i64, i32, i32]
    L.atp_principal_bases.restype = i32
    L.atp_principal_bases.argtypes = [vp, i64, i64, i64, i64, i32, vp, C.c_uint64, vp, vp, vp, vp, vp, sz, i32, vp]
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
    L.atp_concat_factors.restype = i32
    L.atp_concat_factors.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, vp]
    L.atp_norm_factored_workspace.restype = sz
    L.atp_norm_factored_workspace.argtypes = [i64, i64, i64, i64, i32]
    L.atp_norm_factored.restype = i32
    L.atp_norm_factored.argtypes = [vp, vp, vp, C.c_float, i32, vp, vp, i64, i64, i64, i64, vp, sz, i32, vp]
    L.atp_lowrank_linear_workspace.restype = sz
    L.atp_lowrank_linear_workspace.argtypes = [i64, i64, i64, i64, i64, i32, i32]
    L.atp_lowrank_linear.restype = i32
    L.atp_lowrank_linear.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, vp, sz, i32, vp]
    L.atp_attention_workspace.restype = sz
    L.atp_attention_workspace.argtypes = [i64, i64, i64, i64, i32, i32]
    L.atp_attention.restype = i32
    L.atp_attention.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i32, C.c_float, vp, sz, i32, vp]
    L.atp_attention_static.restype = i32
    L.atp_attention_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i32, C.c_float, i32, vp]
    L.atp_init.restype = i32
    L.atp_init.argtypes = []
    L.atp_attention_linearised_workspace.restype = sz
    L.atp_attention_linearised_workspace.argtypes = [i64, i64, i64, i64, i32, i32]
    L.atp_attention_linearised.restype = i32
    L.atp_attention_linearised.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, C.c_float, i32, vp, sz, i32, vp]
    L.atp_profile_enable.restype = None
    L.atp_profile_enable.argtypes = [C.c_uint]
    L.atp_profile_reset.restype = None
    L.atp_profile_reset.argtypes = []
    L.atp_profile_read.restype = i32
    L.atp_profile_read.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                   C.POINTER(C.c_double)]
    return L


lib = _load()

KERNEL_CLASSES = ["gemm_bf16", "gemm_bf16_small", "gemm_swiglu", "gemm_split_gram", "gemm_split_apply", "attention",
                  "cholesky", "stream", "gemm_simt"]


def profile_enable(classes) -> None:
    """classes: iterable of names from KERNEL_CLASSES (empty = off)."""
    mask = 0
    for c in classes:
        mask |= 1 << KERNEL_CLASSES.index(c)
    lib.atp_profile_enable(mask)


def profile_reset() -> None:
    lib.atp_profile_reset()


def profile_read(cls: str) -> dict:
    ms, n, fl, by = C.c_double(), C.c_int64(), C.c_double(), C.c_double()
    st = lib.atp_profile_read(KERNEL_CLASSES.index(cls), C.byref(ms), C.byref(n), C.byref(fl), C.byref(by))
    if st != 0:
        raise AtpError(st, "atp_profile_read")
    return {"ms": ms.value, "launches": n.value, "flops": fl.value, "bytes": by.value}

_DT = {torch.float32: ATP_F32, torch.bfloat16: ATP_BF16}


def _dt(t: torch.Tensor) -> int:
    if t.dtype not in _DT:
        raise TypeError(f"unsupported dtype {t.dtype}")
    return _DT[t.dtype]


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(*ts):
    for t in ts:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("tensors must live on the GPU")
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")


def _ws(nbytes: int, like: torch.Tensor, ws: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    if ws is not None:
        return ws
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=like.device)


def version() -> str:
    return lib.atp_version().decode()


def set_qr_passes(first: int, middle: int, last: int) -> None:
    lib.atp_set_qr_passes(first, middle, last)


def set_overlap(on: bool) -> None:
    lib.atp_set_overlap(1 if on else 0)


def set_conditioning_gram(level: int) -> None:
    lib.atp_set_conditioning_gram(int(level))


def set_factor_mode(mode) -> None:
    """0 / False: one launch per block column; 1 / True: single launch when the whole batch fits it (default);
    2: single-launch groups one after the other for any batch."""
    lib.atp_set_factor_mode(int(mode))


def set_factor_spin_limit(polls: int) -> None:
    """Polls before a wait of the single-launch factorisation gives up (info = -1); < 1 restores the default."""
    lib.atp_set_factor_spin_limit(int(polls))


def principal_bases_workspace(batch, L, d, r, iters, dtype) -> int:
    return lib.atp_principal_bases_workspace(batch, L, d, r, iters, _DT[dtype])


def principal_bases(X: torch.Tensor, r: int, iters: int, Omega: Optional[torch.Tensor] = None, seed: int = 0,
                    want_master: bool = False, workspace: Optional[torch.Tensor] = None, out=None):
    """X [batch, L, d] -> (U_r [batch, L, r], B_r [batch, r, d], info [batch], U_master or None)."""
    _check(X, Omega, workspace)
    batch, L, d = X.shape
    if out is None:
        U = torch.empty((batch, L, r), dtype=X.dtype, device=X.device)
        B = torch.empty((batch, r, d), dtype=X.dtype, device=X.device)
        info = torch.empty((batch,), dtype=torch.int32, device=X.device)
        Um = torch.empty((batch, L, r), dtype=torch.float32, device=X.device) if want_master else None
    else:
        U, B, info, Um = out
    if Omega is not None and (Omega.dtype != torch.float32 or tuple(Omega.shape) != (d, r)):
        raise ValueError("Omega must be float32 [d, r]")
    need = principal_bases_workspace(batch, L, d, r, iters, X.dtype)
    ws = _ws(need, X, workspace)
    st = lib.atp_principal_bases(_ptr(X), batch, L, d, r, iters, _ptr(Omega), seed, _ptr(U), _ptr(B), _ptr(Um),
                                 _ptr(info), _ptr(ws), 0 if ws is None else ws.numel(), _dt(X), _stream())
    if st != 0:
        raise AtpError(st, "atp_principal_bases")
    return U, B, info, Um


def alternating_bases_workspace(batch, L, d, r, dtype) -> int:
    return lib.atp_alternating_bases_workspace(batch, L, d, r, _DT[dtype])


def alternating_bases(X: torch.Tensor, r: int, sweeps: int = 2, V0: Optional[torch.Tensor] = None, seed: int = 0,
                      workspace: Optional[torch.Tensor] = None):
    """Alg.1: X [batch, L, d] -> (U_r [batch, L, r], B_r [batch, r, d], info [batch])."""
    _check(X, V0, workspace)
    batch, L, d = X.shape
    if V0 is not None and (V0.dtype != torch.float32 or tuple(V0.shape) != (d, r)):
        raise ValueError("V0 must be float32 [d, r]")
    U = torch.empty((batch, L, r), dtype=X.dtype, device=X.device)
    B = torch.empty((batch, r, d), dtype=X.dtype, device=X.device)
    info = torch.empty((batch,), dtype=torch.int32, device=X.device)
    ws = _ws(alternating_bases_workspace(batch, L, d, r, X.dtype), X, workspace)
    st = lib.atp_alternating_bases(_ptr(X), batch, L, d, r, sweeps, _ptr(V0), seed, _ptr(U), _ptr(B), _ptr(info),
                                   _ptr(ws), 0 if ws is None else ws.numel(), _dt(X), _stream())
    if st != 0:
        raise AtpError(st, "atp_alternating_bases")
    return U, B, info


def rayleigh_ritz_workspace(batch, L, d, r, dtype) -> int:
    return lib.atp_rayleigh_ritz_workspace(batch, L, d, r, _DT[dtype])


def rayleigh_ritz(U: torch.Tensor, B: torch.Tensor, sweeps: int = 10, workspace: Optional[torch.Tensor] = None):
    """(U_r [batch, L, r], B_r [batch, r, d]) -> (U_out, B_out, sigma [batch, r], diagnostics [batch, 4])."""
    _check(U, B, workspace)
    batch, L, r = U.shape
    d = B.shape[2]
    if tuple(B.shape) != (batch, r, d) or B.dtype != U.dtype:
        raise ValueError("B shape / dtype mismatch")
    Uo, Bo = torch.empty_like(U), torch.empty_like(B)
    sigma = torch.empty((batch, r), dtype=torch.float32, device=U.device)
    diag = torch.empty((batch, 4), dtype=torch.float32, device=U.device)
    ws = _ws(rayleigh_ritz_workspace(batch, L, d, r, U.dtype), U, workspace)
    st = lib.atp_rayleigh_ritz(_ptr(U), _ptr(B), batch, L, d, r, sweeps, _ptr(Uo), _ptr(Bo), _ptr(sigma), _ptr(diag),
                               _ptr(ws), 0 if ws is None else ws.numel(), _dt(U), _stream())
    if st != 0:
        raise AtpError(st, "atp_rayleigh_ritz")
    return Uo, Bo, sigma, diag


def rope(Y: torch.Tensor, heads: int, base: float = 10000.0, pos0: int = 0, out: Optional[torch.Tensor] = None):
    """Rotary position encoding of the rows of Y [batch, L, dq] (half-split pairs per head)."""
    _check(Y, out)
    batch, L, dq = Y.shape
    if out is None:
        out = torch.empty_like(Y)
    st = lib.atp_rope(_ptr(Y), _ptr(out), batch, L, dq, heads, float(base), pos0, _dt(Y), _stream())
    if st != 0:
        raise AtpError(st, "atp_rope")
    return out


def project_onto_bases(U: torch.Tensor, Y: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                       out: Optional[torch.Tensor] = None):
    """U [batch, L, r], Y [batch, L, dq] -> Uᵀ·Y [batch, r, dq]."""
    _check(U, Y, workspace, out)
    batch, L, r = U.shape
    dq = Y.shape[2]
    if tuple(Y.shape) != (batch, L, dq) or Y.dtype != U.dtype:
        raise ValueError("Y shape / dtype mismatch")
    if out is None:
        out = torch.empty((batch, r, dq), dtype=U.dtype, device=U.device)
    ws = _ws(lib.atp_project_onto_bases_workspace(batch, L, r, dq, _dt(U)), U, workspace)
    st = lib.atp_project_onto_bases(_ptr(U), _ptr(Y), _ptr(out), batch, L, r, dq, _ptr(ws), 0 if ws is None else ws.numel(),
                                    _dt(U), _stream())
    if st != 0:
        raise AtpError(st, "atp_project_onto_bases")
    return out


def concat_factors(U1: torch.Tensor, C1: torch.Tensor, U2: torch.Tensor, C2: torch.Tensor):
    """(U1 [batch, L, r1], C1 [batch, r1, d]), (U2, C2) -> P = [U1 | U2], C = [C1; C2]: P·C = U1·C1 + U2·C2."""
    _check(U1, C1, U2, C2)
    batch, L, r1 = U1.shape
    r2, d = U2.shape[2], C1.shape[2]
    if tuple(C1.shape) != (batch, r1, d) or tuple(U2.shape) != (batch, L, r2) or tuple(C2.shape) != (batch, r2, d) \
            or len({U1.dtype, C1.dtype, U2.dtype, C2.dtype}) != 1:
        raise ValueError("factor shapes / dtypes do not match")
    P = torch.empty((batch, L, r1 + r2), dtype=U1.dtype, device=U1.device)
    Cc = torch.empty((batch, r1 + r2, d), dtype=U1.dtype, device=U1.device)
    st = lib.atp_concat_factors(_ptr(U1), _ptr(C1), _ptr(U2), _ptr(C2), _ptr(P), _ptr(Cc), batch, L, d, r1, r2, _dt(U1), _stream())
    if st != 0:
        raise AtpError(st, "atp_concat_factors")
    return P, Cc


def norm_factored(P: torch.Tensor, Cf: torch.Tensor, gain: torch.Tensor, eps: float = 1e-6, center: bool = False,
                  workspace: Optional[torch.Tensor] = None):
    """Row-wise normalisation of H = P·C carried through the factors: returns (Pn, Cn) with Pn·Cn = Norm(H)."""
    _check(P, Cf, gain, workspace)
    batch, L, m = P.shape
    d = Cf.shape[2]
    if tuple(Cf.shape) != (batch, m, d) or Cf.dtype != P.dtype or gain.dtype != torch.float32 or tuple(gain.shape) != (d,):
        raise ValueError("shape / dtype mismatch (gain must be float32 [d])")
    Pn, Cn = torch.empty_like(P), torch.empty_like(Cf)
    ws = _ws(lib.atp_norm_factored_workspace(batch, L, d, m, _dt(P)), P, workspace)
    st = lib.atp_norm_factored(_ptr(P), _ptr(Cf), _ptr(gain), float(eps), 1 if center else 0, _ptr(Pn), _ptr(Cn), batch, L, d, m,
                               _ptr(ws), 0 if ws is None else ws.numel(), _dt(P), _stream())
    if st != 0:
        raise AtpError(st, "atp_norm_factored")
    return Pn, Cn


def lowrank_linear_workspace(batch, m, k, n, w_stride, w_layout, dtype) -> int:
    return lib.atp_lowrank_linear_workspace(batch, m, k, n, w_stride, w_layout, _DT[dtype])


def lowrank_linear(B: torch.Tensor, W: torch.Tensor, w_layout: int = ATP_W_KN, epilogue: int = ATP_EPI_NONE,
                   workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """B [batch, m, k] times W ([k, n] / [n, k], or per-sequence [batch, ...]) -> [batch, m, n(/2)]."""
    _check(B, W, workspace, out)
    batch, m, k = B.shape
    per_seq = W.dim() == 3
    wk, wn = (W.shape[-2], W.shape[-1]) if w_layout == ATP_W_KN else (W.shape[-1], W.shape[-2])
    if wk != k or W.dtype != B.dtype or (per_seq and W.shape[0] != batch):
        raise ValueError("weight shape / dtype mismatch")
    n = wn
    w_stride = k * n if per_seq else 0
    nout = n // 2 if epilogue == ATP_EPI_SWIGLU else n
    if out is None:
        out = torch.empty((batch, m, nout), dtype=B.dtype, device=B.device)
    need = lowrank_linear_workspace(batch, m, k, n, w_stride, w_layout, B.dtype)
    ws = _ws(need, B, workspace)
    st = lib.atp_lowrank_linear(_ptr(B), _ptr(W), _ptr(out), batch, m, k, n, w_stride, w_layout, epilogue,
                                _ptr(ws), 0 if ws is None else ws.numel(), _dt(B), _stream())
    if st != 0:
        raise AtpError(st, "atp_lowrank_linear")
    return out


def attention_workspace(batch, L, r, dq, heads, dtype) -> int:
    return lib.atp_attention_workspace(batch, L, r, dq, heads, _DT[dtype])


def attention(Q: torch.Tensor, K_r: torch.Tensor, V_r: torch.Tensor, heads: int, scale: float = 0.0,
              workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Q [batch, L, dq], K_r/V_r [batch, r, dq] -> O [batch, L, dq]."""
    _check(Q, K_r, V_r, workspace, out)
    batch, L, dq = Q.shape
    r = K_r.shape[1]
    if tuple(K_r.shape) != (batch, r, dq) or tuple(V_r.shape) != (batch, r, dq) or K_r.dtype != Q.dtype \
            or V_r.dtype != Q.dtype:
        raise ValueError("K_r / V_r shape or dtype mismatch")
    if out is None:
        out = torch.empty_like(Q)
    need = attention_workspace(batch, L, r, dq, heads, Q.dtype)
    ws = _ws(need, Q, workspace)
    st = lib.atp_attention(_ptr(Q), _ptr(K_r), _ptr(V_r), _ptr(out), batch, L, r, dq, heads, float(scale),
                           _ptr(ws), 0 if ws is None else ws.numel(), _dt(Q), _stream())
    if st != 0:
        raise AtpError(st, "atp_attention")
    return out


STATIC_SCRATCH_BYTES = 32 << 20


def init() -> None:
    """Optional one-time set-up on the current device (see atp_init)."""
    st = lib.atp_init()
    if st != 0:
        raise AtpError(st, "atp_init")


def attention_static(Q: torch.Tensor, K_r: torch.Tensor, V_r: torch.Tensor, heads: int, scale: float = 0.0,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """atp_attention with the library's built-in scratch buffer; `out` must be given by callers that may not allocate."""
    _check(Q, K_r, V_r, out)
    batch, L, dq = Q.shape
    r = K_r.shape[1]
    if tuple(K_r.shape) != (batch, r, dq) or tuple(V_r.shape) != (batch, r, dq) or K_r.dtype != Q.dtype \
            or V_r.dtype != Q.dtype:
        raise ValueError("K_r / V_r shape or dtype mismatch")
    if out is None:
        out = torch.empty_like(Q)
    st = lib.atp_attention_static(_ptr(Q), _ptr(K_r), _ptr(V_r), _ptr(out), batch, L, r, dq, heads, float(scale),
                                  _dt(Q), _stream())
    if st != 0:
        raise AtpError(st, "atp_attention_static")
    return out


ATP_NORM_TAYLOR, ATP_NORM_ROWSUM = 0, 1


def attention_linearised_workspace(batch, L, r, dq, heads, dtype) -> int:
    return lib.atp_attention_linearised_workspace(batch, L, r, dq, heads, _DT[dtype])


def attention_linearised(Q: torch.Tensor, K_r: torch.Tensor, V_r: torch.Tensor, U_r: torch.Tensor, heads: int,
                         scale: float = 0.0, norm: int = ATP_NORM_TAYLOR, workspace: Optional[torch.Tensor] = None,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """First-order attention (Eq.8): Q [batch, L, dq], K_r/V_r [batch, r, dq], U_r [batch, L, r] -> O."""
    _check(Q, K_r, V_r, U_r, workspace, out)
    batch, L, dq = Q.shape
    r = K_r.shape[1]
    if tuple(K_r.shape) != (batch, r, dq) or tuple(V_r.shape) != (batch, r, dq) or tuple(U_r.shape) != (batch, L, r) \
            or K_r.dtype != Q.dtype or V_r.dtype != Q.dtype or U_r.dtype != Q.dtype:
        raise ValueError("K_r / V_r / U_r shape or dtype mismatch")
    if out is None:
        out = torch.empty_like(Q)
    need = attention_linearised_workspace(batch, L, r, dq, heads, Q.dtype)
    ws = _ws(need, Q, workspace)
    st = lib.atp_attention_linearised(_ptr(Q), _ptr(K_r), _ptr(V_r), _ptr(U_r), _ptr(out), batch, L, r, dq, heads,
                                      float(scale), norm, _ptr(ws), 0 if ws is None else ws.numel(), _dt(Q), _stream())
    if st != 0:
        raise AtpError(st, "atp_attention_linearised")
    return out


class AtpLayer:
    """Call sequence of one ATP block (Fig.3) on preallocated buffers: marshalling only.

    extraction -> q/k/v projections of the r bases (Eq.6) -> Q = U·Q' -> attention over the r
    principal keys/values; optionally: second extraction on the attention output, output
    projection and SwiGLU feed-forward on the bases (result factored as (U_o, F)).
    Weights are given packed as [out, in] (ATP_W_NK).

    Sequences are independent, so the batch can be cut into `streams` equal chunks, each issued on
    a HIP stream of its own (default priority) with its own workspace: the latency-bound
    factorisation chain of one chunk then runs beside the GEMMs of the others.  The caller's
    current stream is forked at the start of forward() and joined at its end.
    """

    def __init__(self, batch, L, d, heads, r, iters, dtype, Wq, Wk, Wv, Wo=None, Wgu=None, Wdown=None,
                 Omega=None, device="cuda", streams=1, attention_kind="softmax", scale=0.0, keep_master=False):
        if streams < 1 or batch % streams:
            raise ValueError("streams must divide batch")
        self.batch, self.L, self.d, self.heads, self.r, self.iters = batch, L, d, heads, r, iters
        self.dtype = dtype
        self.Wq, self.Wk, self.Wv, self.Wo, self.Wgu, self.Wdown = Wq, Wk, Wv, Wo, Wgu, Wdown
        self.Omega = Omega
        if attention_kind not in ("softmax", "linearised"):
            raise ValueError("attention_kind must be 'softmax' or 'linearised'")
        self.attention_kind, self.scale = attention_kind, scale
        dev = torch.device(device)
        e = lambda *s: torch.empty(s, dtype=dtype, device=dev)
        self.U, self.B = e(batch, L, r), e(batch, r, d)
        self.info = torch.empty((batch,), dtype=torch.int32, device=dev)
        # fp32 copy of U before rounding to the storage type (optional output of atp_principal_bases)
        self.Um = torch.empty((batch, L, r), dtype=torch.float32, device=dev) if keep_master else None
        self.Qp, self.Kp, self.Vp = e(batch, r, d), e(batch, r, d), e(batch, r, d)
        self.Q, self.O = e(batch, L, d), e(batch, L, d)
        cb = batch // streams
        nws = max(principal_bases_workspace(cb, L, d, r, iters, dtype),
                  lowrank_linear_workspace(cb, L, r, d, r * d, ATP_W_KN, dtype),
                  attention_linearised_workspace(cb, L, r, d, heads, dtype), 256)
        self.wss = [torch.empty(nws, dtype=torch.uint8, device=dev) for _ in range(streams)]
        self.ws = self.wss[0]
        if Wo is not None:
            self.Uo, self.Bo, self.A = e(batch, L, r), e(batch, r, d), e(batch, r, d)
            self.info_o = torch.empty((batch,), dtype=torch.int32, device=dev)
        if Wgu is not None:
            f = Wgu.shape[0] // 2
            self.G, self.F = e(batch, r, f), e(batch, r, d)
        self.nstreams = streams
        self.side = [torch.cuda.Stream(device=dev) for _ in range(streams)] if streams > 1 else []
        self.chunks = [slice(i * cb, (i + 1) * cb) for i in range(streams)]

    def _stages(self, X, c, ws):
        """The calls of one chunk (batch slice c), in order, as closures."""
        v = lambda t: t[c]
        yield lambda: principal_bases(v(X), self.r, self.iters, self.Omega, workspace=ws,
                                      out=(v(self.U), v(self.B), v(self.info), None if self.Um is None else v(self.Um)))
        yield lambda: lowrank_linear(v(self.B), self.Wq, ATP_W_NK, workspace=ws, out=v(self.Qp))
        yield lambda: lowrank_linear(v(self.B), self.Wk, ATP_W_NK, workspace=ws, out=v(self.Kp))
        yield lambda: lowrank_linear(v(self.B), self.Wv, ATP_W_NK, workspace=ws, out=v(self.Vp))
        yield lambda: lowrank_linear(v(self.U), v(self.Qp), ATP_W_KN, workspace=ws, out=v(self.Q))
        if self.attention_kind == "softmax":
            yield lambda: attention(v(self.Q), v(self.Kp), v(self.Vp), self.heads, scale=self.scale, workspace=ws,
                                    out=v(self.O))
        else:   # first-order attention of Eq.8
            yield lambda: attention_linearised(v(self.Q), v(self.Kp), v(self.Vp), v(self.U), self.heads, scale=self.scale,
                                               workspace=ws, out=v(self.O))
        if self.Wo is None:
            return
        yield lambda: principal_bases(v(self.O), self.r, self.iters, self.Omega, workspace=ws,
                                      out=(v(self.Uo), v(self.Bo), v(self.info_o), None))
        yield lambda: lowrank_linear(v(self.Bo), self.Wo, ATP_W_NK, workspace=ws, out=v(self.A))
        if self.Wgu is None:
            return
        yield lambda: lowrank_linear(v(self.A), self.Wgu, ATP_W_NK, ATP_EPI_SWIGLU, workspace=ws, out=v(self.G))
        yield lambda: lowrank_linear(v(self.G), self.Wdown, ATP_W_NK, workspace=ws, out=v(self.F))

    def forward(self, X):
        if self.nstreams == 1:
            for call in self._stages(X, slice(0, self.batch), self.ws):
                call()
        else:
            main = torch.cuda.current_stream()
            plans = [list(self._stages(X, c, ws)) for c, ws in zip(self.chunks, self.wss)]
            for s in self.side:
                s.wait_stream(main)
            # issue stage by stage, round-robin over the chunks, so every stream has work queued early
            for k in range(len(plans[0])):
                for s, plan in zip(self.side, plans):
                    with torch.cuda.stream(s):
                        plan[k]()
            for s in self.side:
                main.wait_stream(s)
        if self.Wo is None:
            return self.O
        if self.Wgu is None:
            return self.Uo, self.A
        return self.Uo, self.F
