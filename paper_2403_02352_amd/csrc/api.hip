// C ABI of the ATP library: argument checks, workspace carve-up and the host-side
// sequencing of kernels.  Nothing here allocates or synchronises.
#include "../../include/atp.h"
#include "common.h"

#include <algorithm>
#include <vector>

using namespace atp;

namespace {

// ---- event timing ------------------------------------------------------------------
struct ProfRec { int cls; hipEvent_t a, b; double flops, bytes; };
unsigned g_prof_mask = 0;
std::vector<ProfRec> g_recs;
std::vector<hipEvent_t> g_pool;

hipEvent_t prof_event() {
    if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

struct ProfScope {
    hipStream_t st; bool on = false; ProfRec rec;
    ProfScope(hipStream_t s, int cls, double flops, double bytes) : st(s) {
        if (g_prof_mask & (1u << cls)) {
            on = true;
            rec.cls = cls; rec.flops = flops; rec.bytes = bytes;
            rec.a = prof_event(); rec.b = prof_event();
            (void)hipEventRecord(rec.a, st);
        }
    }
    ~ProfScope() {
        if (on) { (void)hipEventRecord(rec.b, st); g_recs.push_back(rec); }
    }
};

int g_passes_first = 3, g_passes_middle = 2, g_passes_last = 3;

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }
inline size_t esize(atp_dtype t) { return t == ATP_BF16 ? 2 : 4; }
inline OperandType optype(atp_dtype t) { return t == ATP_BF16 ? OP_BF16 : OP_F32; }

struct Carver {
    uint8_t* base;
    size_t off = 0;
    explicit Carver(void* p) : base(reinterpret_cast<uint8_t*>(p)) {}
    void* take(size_t bytes) {
        void* r = base ? base + off : nullptr;
        off += align_up(bytes);
        return r;
    }
};

// Workspace layout of atp_principal_bases (shared by the query and the call).
struct BasesWs {
    void* XT;        // [batch, d, L]  type t
    float* Om;       // [d, r]   generated start block (only when Omega == NULL)
    float* OmT;      // [r, d]
    float* ZL[2];    // [batch, L, r]
    float* ZLT[2];   // [batch, r, L]
    float* ZD[2];    // [batch, d, r]
    float* ZDT[2];   // [batch, r, d]
    void* UT;        // [batch, r, L]  type t: transposed twin of the returned U_r
    float* S;        // [batch, r, r]
    float* Lf;       // [batch, r, r]
    float* Linv;     // [batch, r, r]
    float* dinv;     // [batch, r]
    int32_t* info;   // [batch]
    size_t total;
};

BasesWs carve_bases(void* ws, int64_t batch, int64_t L, int64_t d, int64_t r, atp_dtype t) {
    Carver c(ws);
    BasesWs w;
    const size_t es = esize(t);
    w.XT = c.take((size_t)batch * d * L * es);
    w.Om = (float*)c.take((size_t)d * r * 4);
    w.OmT = (float*)c.take((size_t)d * r * 4);
    for (int i = 0; i < 2; ++i) {
        w.ZL[i] = (float*)c.take((size_t)batch * L * r * 4);
        w.ZLT[i] = (float*)c.take((size_t)batch * L * r * 4);
        w.ZD[i] = (float*)c.take((size_t)batch * d * r * 4);
        w.ZDT[i] = (float*)c.take((size_t)batch * d * r * 4);
    }
    w.UT = c.take((size_t)batch * r * L * es);
    w.S = (float*)c.take((size_t)batch * r * r * 4);
    w.Lf = (float*)c.take((size_t)batch * r * r * 4);
    w.Linv = (float*)c.take((size_t)batch * r * r * 4);
    w.dinv = (float*)c.take((size_t)batch * r * 4);
    w.info = (int32_t*)c.take((size_t)batch * 4);
    w.total = c.off;
    return w;
}

#define ATP_HIP(expr)                               \
    do {                                            \
        hipError_t e__ = (expr);                    \
        if (e__ != hipSuccess) return ATP_ERR_DEVICE; \
    } while (0)

// C = A · Bᵀ on the backend the storage type calls for: bf16 path -> MFMA (fp32 operands are
// rounded, or split hi/lo when nsplit == 3), fp32 path or unaligned shapes -> fp32 FMA kernel.
hipError_t nt_product(hipStream_t st, bool mfma, OperandType ta, OperandType tb, int nsplit, const GemmArgs& g) {
    const double work = (double)g.batch * g.M * g.N * g.K;
    double flops = 2.0 * work * (g.swiglu ? 2.0 : 1.0);
    if (g.symmetric || g.b_lower) flops *= 0.5;  // algorithmic count: symmetric / triangular operand
    const double out_b = (g.C32 ? 4 : 0) + (g.C16 ? 2 : 0) + (g.CT32 ? 4 : 0) + (g.CT16 ? 2 : 0);
    const double bytes = (double)g.batch * g.M * g.K * (ta == OP_F32 ? 4 : 2) +
                         (double)(g.sB ? g.batch : 1) * g.N * (g.swiglu ? 2 : 1) * g.K * (tb == OP_F32 ? 4 : 2) +
                         (double)g.batch * g.M * g.N * out_b;
    if (mfma && gemm_nt_mfma_ok(ta, tb, g)) {
        int cls;
        if (nsplit == 3) cls = g.symmetric ? ATP_K_GEMM_SPLIT_GRAM : ATP_K_GEMM_SPLIT_APPLY;
        else if (ta != tb) cls = ATP_K_GEMM_MIXED;
        else if (g.swiglu) cls = ATP_K_GEMM_SWIGLU;
        else cls = gemm_nt_mfma_big(g) ? ATP_K_GEMM_BF16 : ATP_K_GEMM_BF16_SMALL;
        ProfScope ps(st, cls, flops, bytes);
        return gemm_nt_mfma(st, ta, tb, nsplit, g);
    }
    ProfScope ps(st, ATP_K_GEMM_SIMT, flops, bytes);
    SimtArgs s;
    s.A = g.A; s.B = g.B;
    s.a_rs = g.lda; s.a_cs = 1; s.b_rs = g.ldb; s.b_cs = 1;
    s.sA = g.sA; s.sB = g.sB;
    s.M = g.M; s.N = g.N; s.K = g.K; s.batch = g.batch;
    s.C32 = g.C32; s.C16 = g.C16; s.ldc = g.ldc; s.sC = g.sC;
    s.CT32 = g.CT32; s.CT16 = g.CT16; s.ldct = g.ldct; s.sCT = g.sCT;
    s.swiglu = g.swiglu;
    return gemm_simt(st, ta, tb, s);
}

struct QrOut {  // where the last pass writes
    float* C32 = nullptr;
    bf16_t* C16 = nullptr;
    float* CT32 = nullptr;
    bf16_t* CT16 = nullptr;
};

// Orthonormalise the columns of Z (n×r, fp32, with transposed twin ZT) by `passes` rounds of
// (Gram, Jacobi scaling + shift, Cholesky, scaled triangular inverse, apply).  Every round
// multiplies from the right by an upper-triangular matrix with positive diagonal, so the result
// is the Q factor of the positive-diagonal QR of Z.  Buffers ping-pong between slot `cur` and 1-cur.
atp_status cholesky_qr(hipStream_t st, bool mfma, int passes, float shift, float* Z[2], float* ZT[2], int& cur, int n,
                       int r, int batch, BasesWs& w, int32_t* info, const QrOut* final_out) {
    for (int p = 0; p < passes; ++p) {
        const bool last = (p == passes - 1);
        GemmArgs g;
        g.A = ZT[cur]; g.B = ZT[cur];
        g.lda = n; g.ldb = n; g.sA = (int64_t)r * n; g.sB = (int64_t)r * n;
        g.M = r; g.N = r; g.K = n; g.batch = batch;
        g.C32 = w.S; g.ldc = r; g.sC = (int64_t)r * r;
        g.symmetric = 1;
        ATP_HIP(nt_product(st, mfma, OP_F32, OP_F32, 3, g));
        {
            ProfScope ps(st, ATP_K_CHOLESKY, (double)batch * r * r * r / 3.0, (double)batch * r * r * 8.0);
            ATP_HIP(gram_scale_shift(st, w.S, w.dinv, r, last ? 0.f : shift, batch));
            ATP_HIP(cholesky_lower(st, w.S, w.Lf, r, info, last ? 1e-3f : 0.f, batch));
        }
        {
            ProfScope ps(st, ATP_K_TRI_INVERSE, (double)batch * r * r * r / 3.0, (double)batch * r * r * 8.0);
            ATP_HIP(tri_inverse_scaled(st, w.Lf, w.dinv, w.Linv, r, batch));
        }
        GemmArgs a;
        a.A = Z[cur]; a.B = w.Linv;
        a.lda = r; a.ldb = r; a.sA = (int64_t)n * r; a.sB = (int64_t)r * r;
        a.M = n; a.N = r; a.K = r; a.batch = batch;
        a.ldc = r; a.sC = (int64_t)n * r; a.ldct = n; a.sCT = (int64_t)n * r;
        a.b_lower = 1;
        if (last && final_out) {
            a.C32 = final_out->C32; a.C16 = final_out->C16;
            a.CT32 = final_out->CT32; a.CT16 = final_out->CT16;
        } else {
            a.C32 = Z[1 - cur]; a.CT32 = ZT[1 - cur];
        }
        ATP_HIP(nt_product(st, mfma, OP_F32, OP_F32, 3, a));
        cur = 1 - cur;
    }
    return ATP_OK;
}

}  // namespace

extern "C" {

const char* atp_status_string(atp_status s) {
    switch (s) {
        case ATP_OK: return "ok";
        case ATP_ERR_INVALID_ARG: return "invalid argument";
        case ATP_ERR_BAD_RANK: return "rank r must satisfy 1 <= r <= min(L, d)";
        case ATP_ERR_WORKSPACE: return "workspace missing or too small";
        case ATP_ERR_UNSUPPORTED: return "unsupported shape";
        case ATP_ERR_DEVICE: return "HIP error";
    }
    return "unknown status";
}

const char* atp_version(void) { return "atp-gfx950 0.1"; }

void atp_profile_enable(unsigned class_mask) { g_prof_mask = class_mask; }

void atp_profile_reset(void) {
    for (auto& r : g_recs) { g_pool.push_back(r.a); g_pool.push_back(r.b); }
    g_recs.clear();
}

atp_status atp_profile_read(int kernel_class, double* total_ms, int64_t* launches, double* flops, double* bytes) {
    if (kernel_class < 0 || kernel_class >= ATP_K_COUNT) return ATP_ERR_INVALID_ARG;
    double ms = 0, fl = 0, by = 0;
    int64_t n = 0;
    for (auto& r : g_recs) {
        if (r.cls != kernel_class) continue;
        if (hipEventSynchronize(r.b) != hipSuccess) return ATP_ERR_DEVICE;
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) return ATP_ERR_DEVICE;
        ms += t; fl += r.flops; by += r.bytes; ++n;
    }
    if (total_ms) *total_ms = ms;
    if (launches) *launches = n;
    if (flops) *flops = fl;
    if (bytes) *bytes = by;
    return ATP_OK;
}

void atp_set_qr_passes(int first, int middle, int last) {
    g_passes_first = std::min(4, std::max(1, first));
    g_passes_middle = std::min(4, std::max(1, middle));
    g_passes_last = std::min(4, std::max(1, last));
}

size_t atp_principal_bases_workspace(int64_t batch, int64_t L, int64_t d, int64_t r, int iters, atp_dtype t) {
    (void)iters;
    if (batch < 1 || L < 1 || d < 1 || r < 1 || (t != ATP_F32 && t != ATP_BF16)) return 0;
    return carve_bases(nullptr, batch, L, d, r, t).total;
}

atp_status atp_principal_bases(const void* X, int64_t batch, int64_t L, int64_t d, int64_t r, int iters,
                               const float* Omega, uint64_t seed, void* U_r, void* B_r, float* U_master,
                               int32_t* info, void* workspace, size_t workspace_bytes, atp_dtype t,
                               void* hip_stream) {
    if (!X || !U_r || !B_r || batch < 1 || L < 1 || d < 1 || iters < 0) return ATP_ERR_INVALID_ARG;
    if (t != ATP_F32 && t != ATP_BF16) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || L > (1 << 30) || d > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (r < 1 || r > std::min(L, d)) return ATP_ERR_BAD_RANK;
    if (!aligned16(X) || !aligned16(U_r) || !aligned16(B_r) || !aligned16(Omega) || !aligned16(U_master) ||
        !aligned16(workspace) || (((uintptr_t)info) & 3))
        return ATP_ERR_INVALID_ARG;
    const size_t need = atp_principal_bases_workspace(batch, L, d, r, iters, t);
    if (!workspace || workspace_bytes < need) return ATP_ERR_WORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    BasesWs w = carve_bases(workspace, batch, L, d, r, t);
    const bool mfma = (t == ATP_BF16);
    const OperandType tx = optype(t);
    const int iL = (int)L, id = (int)d, ir = (int)r, ib = (int)batch;
    const float shift = mfma ? 1e-4f : 1e-5f;
    int32_t* inf = info ? info : w.info;
    ATP_HIP(fill_zero_i32(st, inf, batch));

    // operand twins: Xᵀ and Ωᵀ
    {
        ProfScope ps(st, ATP_K_STREAM, 0.0, 2.0 * (double)batch * L * d * esize(t));
        ATP_HIP(transpose_batched(st, X, w.XT, iL, id, L, L * d, L * d, ib, (int)esize(t), 0));
    }
    const float* Om = Omega;
    if (!Om) {
        ATP_HIP(fill_gaussian(st, w.Om, d * r, seed));
        Om = w.Om;
    }
    ATP_HIP(transpose_batched(st, Om, w.OmT, id, ir, d, 0, 0, 1, 4, 0));

    // Z = X·Ω
    int curL = 0, curD = 0;
    {
        GemmArgs g;
        g.A = X; g.B = w.OmT; g.lda = d; g.ldb = d; g.sA = L * d; g.sB = 0;
        g.M = iL; g.N = ir; g.K = id; g.batch = ib;
        g.C32 = w.ZL[0]; g.ldc = r; g.sC = L * r;
        g.CT32 = w.ZLT[0]; g.ldct = L; g.sCT = L * r;
        ATP_HIP(nt_product(st, mfma, tx, OP_F32, 1, g));
    }
    QrOut fin;
    if (t == ATP_BF16) {
        fin.C16 = (bf16_t*)U_r; fin.C32 = U_master; fin.CT16 = (bf16_t*)w.UT;
    } else {
        fin.C32 = (float*)U_r; fin.CT32 = (float*)w.UT;
    }
    atp_status s = cholesky_qr(st, mfma, iters == 0 ? g_passes_last : g_passes_first, shift, w.ZL, w.ZLT, curL, iL, ir,
                               ib, w, inf, iters == 0 ? &fin : nullptr);
    if (s != ATP_OK) return s;

    for (int it = 0; it < iters; ++it) {
        // W = Xᵀ·U
        GemmArgs g;
        g.A = w.XT; g.B = w.ZLT[curL]; g.lda = L; g.ldb = L; g.sA = L * d; g.sB = L * r;
        g.M = id; g.N = ir; g.K = iL; g.batch = ib;
        g.C32 = w.ZD[0]; g.ldc = r; g.sC = d * r;
        g.CT32 = w.ZDT[0]; g.ldct = d; g.sCT = d * r;
        curD = 0;
        ATP_HIP(nt_product(st, mfma, tx, OP_F32, 1, g));
        s = cholesky_qr(st, mfma, g_passes_middle, shift, w.ZD, w.ZDT, curD, id, ir, ib, w, inf, nullptr);
        if (s != ATP_OK) return s;
        // Z = X·V
        GemmArgs h;
        h.A = X; h.B = w.ZDT[curD]; h.lda = d; h.ldb = d; h.sA = L * d; h.sB = d * r;
        h.M = iL; h.N = ir; h.K = id; h.batch = ib;
        h.C32 = w.ZL[0]; h.ldc = r; h.sC = L * r;
        h.CT32 = w.ZLT[0]; h.ldct = L; h.sCT = L * r;
        curL = 0;
        ATP_HIP(nt_product(st, mfma, tx, OP_F32, 1, h));
        const bool lastit = (it == iters - 1);
        s = cholesky_qr(st, mfma, lastit ? g_passes_last : g_passes_middle, shift, w.ZL, w.ZLT, curL, iL, ir, ib, w, inf,
                        lastit ? &fin : nullptr);
        if (s != ATP_OK) return s;
    }
    if (t == ATP_F32 && U_master)
        ATP_HIP(hipMemcpyAsync(U_master, U_r, (size_t)batch * L * r * 4, hipMemcpyDeviceToDevice, st));

    // B_r = U_rᵀ·X with the returned (rounded) U_r
    {
        GemmArgs g;
        g.A = w.UT; g.B = w.XT; g.lda = L; g.ldb = L; g.sA = r * L; g.sB = d * L;
        g.M = ir; g.N = id; g.K = iL; g.batch = ib;
        g.ldc = d; g.sC = r * d;
        if (t == ATP_BF16) g.C16 = (bf16_t*)B_r; else g.C32 = (float*)B_r;
        ATP_HIP(nt_product(st, mfma, tx, tx, 1, g));
    }
    return ATP_OK;
}

size_t atp_lowrank_linear_workspace(int64_t batch, int64_t m, int64_t k, int64_t n, int64_t w_stride,
                                    atp_wlayout w_layout, atp_dtype t) {
    (void)m;
    if (batch < 1 || k < 1 || n < 1) return 0;
    if (t == ATP_BF16 && w_layout == ATP_W_KN) return align_up((size_t)(w_stride ? batch : 1) * k * n * 2);
    return 0;
}

atp_status atp_lowrank_linear(const void* B, const void* W, void* out, int64_t batch, int64_t m, int64_t k,
                              int64_t n, int64_t w_stride, atp_wlayout w_layout, atp_epilogue epilogue,
                              void* workspace, size_t workspace_bytes, atp_dtype t, void* hip_stream) {
    if (!B || !W || !out || batch < 1 || m < 1 || k < 1 || n < 1 || w_stride < 0) return ATP_ERR_INVALID_ARG;
    if (t != ATP_F32 && t != ATP_BF16) return ATP_ERR_INVALID_ARG;
    if (w_layout != ATP_W_KN && w_layout != ATP_W_NK) return ATP_ERR_INVALID_ARG;
    if (epilogue != ATP_EPI_NONE && epilogue != ATP_EPI_SWIGLU) return ATP_ERR_INVALID_ARG;
    if (epilogue == ATP_EPI_SWIGLU && (n & 1)) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || m > (1 << 30) || k > (1 << 30) || n > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (!aligned16(B) || !aligned16(W) || !aligned16(out) || !aligned16(workspace)) return ATP_ERR_INVALID_ARG;
    const size_t need = atp_lowrank_linear_workspace(batch, m, k, n, w_stride, w_layout, t);
    if (need && (!workspace || workspace_bytes < need)) return ATP_ERR_WORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const bool swiglu = (epilogue == ATP_EPI_SWIGLU);
    const int64_t nout = swiglu ? n / 2 : n;
    const OperandType tx = optype(t);

    if (t == ATP_F32) {
        SimtArgs s;
        s.A = B; s.B = W;
        s.a_rs = k; s.a_cs = 1;
        if (w_layout == ATP_W_KN) { s.b_rs = 1; s.b_cs = n; } else { s.b_rs = k; s.b_cs = 1; }
        s.sA = m * k; s.sB = w_stride;
        s.M = (int)m; s.N = (int)nout; s.K = (int)k; s.batch = (int)batch;
        s.C32 = (float*)out; s.ldc = nout; s.sC = m * nout;
        s.swiglu = swiglu;
        ATP_HIP(gemm_simt(st, OP_F32, OP_F32, s));
        return ATP_OK;
    }
    const void* Wnk = W;
    int64_t sW = w_stride;
    if (w_layout == ATP_W_KN) {
        const int nb = w_stride ? (int)batch : 1;
        ProfScope ps(st, ATP_K_STREAM, 0.0, 4.0 * (double)nb * k * n);
        ATP_HIP(transpose_batched(st, W, workspace, (int)k, (int)n, k, w_stride, k * n, nb, 2, 0));
        Wnk = workspace;
        sW = w_stride ? k * n : 0;
    }
    GemmArgs g;
    g.A = B; g.B = Wnk; g.lda = k; g.ldb = k; g.sA = m * k; g.sB = sW;
    g.M = (int)m; g.N = (int)nout; g.K = (int)k; g.batch = (int)batch;
    g.C16 = (bf16_t*)out; g.ldc = nout; g.sC = m * nout;
    g.swiglu = swiglu;
    ATP_HIP(nt_product(st, true, tx, tx, 1, g));
    return ATP_OK;
}

size_t atp_attention_workspace(int64_t batch, int64_t L, int64_t r, int64_t dq, int heads, atp_dtype t) {
    (void)L; (void)heads;
    if (batch < 1 || r < 1 || dq < 1) return 0;
    if (t != ATP_BF16) return 0;
    const int64_t rp = (r + 63) / 64 * 64;
    return align_up((size_t)batch * dq * rp * 2);
}

atp_status atp_attention(const void* Q, const void* K_r, const void* V_r, void* O, int64_t batch, int64_t L,
                         int64_t r, int64_t dq, int heads, float scale, void* workspace, size_t workspace_bytes,
                         atp_dtype t, void* hip_stream) {
    if (!Q || !K_r || !V_r || !O || batch < 1 || L < 1 || r < 1 || dq < 1 || heads < 1) return ATP_ERR_INVALID_ARG;
    if (t != ATP_F32 && t != ATP_BF16) return ATP_ERR_INVALID_ARG;
    if (dq % heads) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || heads > 65535 || L > (1 << 30) || r > (1 << 30) || dq > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K_r) || !aligned16(V_r) || !aligned16(O) || !aligned16(workspace))
        return ATP_ERR_INVALID_ARG;
    const int64_t dh = dq / heads;
    if (t == ATP_BF16 && dh != 64 && dh != 128) return ATP_ERR_UNSUPPORTED;
    if (t == ATP_F32 && dh > 256) return ATP_ERR_UNSUPPORTED;
    const size_t need = atp_attention_workspace(batch, L, r, dq, heads, t);
    if (need && (!workspace || workspace_bytes < need)) return ATP_ERR_WORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    AttnArgs a;
    a.Q = Q; a.K = K_r; a.V = V_r; a.O = O;
    a.batch = (int)batch; a.L = (int)L; a.nk = (int)r; a.dq = (int)dq; a.heads = heads;
    a.scale = (scale > 0.f) ? scale : 1.0f / sqrtf((float)dh);
    if (t == ATP_F32) {
        ATP_HIP(attention_f32(st, a));
        return ATP_OK;
    }
    const int64_t rp = (r + 63) / 64 * 64;
    // values re-laid out as [dq][r_pad] (zero padded) so a lane reads 8 consecutive keys of one feature
    {
        ProfScope ps(st, ATP_K_STREAM, 0.0, 4.0 * (double)batch * r * dq);
        ATP_HIP(transpose_batched(st, V_r, workspace, (int)r, (int)dq, rp, r * dq, dq * rp, (int)batch, 2, 1));
    }
    a.Vt = workspace;
    a.nk_pad = (int)rp;
    {
        ProfScope ps(st, ATP_K_ATTENTION, 4.0 * (double)batch * L * r * dq,
                     2.0 * (double)batch * (2.0 * L * dq + 2.0 * r * dq));
        ATP_HIP(attention_bf16(st, a));
    }
    return ATP_OK;
}

}  // extern "C"
