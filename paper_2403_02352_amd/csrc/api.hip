// C ABI of the ATP library: argument checks, workspace carve-up and the host-side
// sequencing of kernels.  Nothing here allocates or synchronises.
#include "../../include/atp.h"
#include "common.h"

#include <algorithm>
#include <cstring>
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

int g_passes_first = 2, g_passes_middle = 1, g_passes_last = 2;
int g_overlap = 0;
int g_cond_gram_single = 0;   // 1 / 2: Gram matrix of (intermediate / all) shifted rounds from the hi planes only
int g_factor_mode = 1;   // 0: one launch per block column; 1: single launch when it takes the whole batch; 2: single-launch groups

// Side stream on which the column blocks of Z·R^-1 (and of the product that consumes them) run
// while the factorisation is still working on later block columns.  Created on first use, default
// priority; the events only order work between the caller's stream and this one.
constexpr int SIDE_EVENTS = 64;
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t ev[SIDE_EVENTS] = {};
    int next = 0;
    bool ok = false;
};
SideStream g_side;

bool side_ready() {
    if (g_side.ok) return true;
    if (hipStreamCreateWithFlags(&g_side.stream, hipStreamNonBlocking) != hipSuccess) return false;
    for (int i = 0; i < SIDE_EVENTS; ++i)
        if (hipEventCreateWithFlags(&g_side.ev[i], hipEventDisableTiming) != hipSuccess) return false;
    g_side.ok = true;
    return true;
}
hipEvent_t side_event() {
    hipEvent_t e = g_side.ev[g_side.next];
    g_side.next = (g_side.next + 1) % SIDE_EVENTS;
    return e;
}

// Scratch of atp_attention_static: the per-head re-laid-out values.  One copy per GPU, held until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// device address is resolved once per device and kept in g_static_scratch.
constexpr size_t STATIC_SCRATCH_BYTES = ATP_STATIC_SCRATCH_BYTES;
constexpr int MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
void* g_static_scratch[MAX_DEVICES] = {};

// device address of this GPU's copy of `scratch` (nullptr on failure)
void* static_scratch_ptr() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    if (g_static_scratch[dev]) return g_static_scratch[dev];
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_static_scratch[dev] = ptr;
    return ptr;
}

// Enum-typed arguments come from C callers and may hold any int: read the value without loading it as
// the enum type (which is undefined for values outside the enumerators), then range-check it.
template <class E>
inline int raw_enum(const E& e) {
    static_assert(sizeof(E) == sizeof(int), "C enums are int-sized in this ABI");
    int v;
    std::memcpy(&v, &e, sizeof v);
    return v;
}
inline bool bad_dtype(const atp_dtype& t) { const int v = raw_enum(t); return v != ATP_F32 && v != ATP_BF16; }

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }
inline size_t esize(atp_dtype t) { return t == ATP_BF16 ? 2 : 4; }

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
constexpr int KSPLIT_MAX = 8;
constexpr int NUM_CU = 256;  // compute units of an MI355X
struct BasesWs {
    void* XT;        // [batch, d, L]  type t
    float* Om;       // [d, r]   generated start block (only when Omega == NULL)
    float* OmT;      // [r, d]   fp32
    bf16_t* OmT16;   // [r, d]   bf16 (bf16 path)
    float* ZL[2];    // [batch, L, r]
    float* ZLT[2];   // [batch, r, L]
    float* ZD[2];    // [batch, d, r]
    float* ZDT[2];   // [batch, r, d]
    void* TL;        // [batch, r, L]  type t: transposed twin of the current U (finally of the returned U_r)
    void* TD;        // [batch, r, d]  type t: transposed twin of the current V
    float* Spart;    // [KSPLIT_MAX, batch, r, r] split-K partial Gram matrices
    float* S;        // [batch, r, r]
    float* Lf;       // [batch, r, r]
    float* Y;        // [batch, r, r]
    float* Linv;     // [batch, r, r]
    float* dinv;     // [batch, r]
    int32_t* info;   // [batch]
    unsigned* flags; // hand-over flags of the single-launch factorisation
    size_t total;
};

BasesWs carve_bases(void* ws, int64_t batch, int64_t L, int64_t d, int64_t r, atp_dtype t) {
    Carver c(ws);
    BasesWs w;
    const size_t es = esize(t);
    w.XT = c.take((size_t)batch * d * L * es);
    w.Om = (float*)c.take((size_t)d * r * 4);
    w.OmT = (float*)c.take((size_t)d * r * 4);
    w.OmT16 = (bf16_t*)c.take((size_t)d * r * 2);
    for (int i = 0; i < 2; ++i) {
        w.ZL[i] = (float*)c.take((size_t)batch * L * r * 4);
        w.ZLT[i] = (float*)c.take((size_t)batch * L * r * 4);
        w.ZD[i] = (float*)c.take((size_t)batch * d * r * 4);
        w.ZDT[i] = (float*)c.take((size_t)batch * d * r * 4);
    }
    w.TL = c.take((size_t)batch * r * L * es);
    w.TD = c.take((size_t)batch * r * d * es);
    w.Spart = (float*)c.take((size_t)KSPLIT_MAX * batch * r * r * 4);
    w.S = (float*)c.take((size_t)batch * r * r * 4);
    w.Lf = (float*)c.take((size_t)batch * r * r * 4);
    w.Y = (float*)c.take((size_t)batch * r * r * 4);
    w.Linv = (float*)c.take((size_t)batch * r * r * 4);
    w.dinv = (float*)c.take((size_t)batch * r * 4);
    w.info = (int32_t*)c.take((size_t)batch * 4);
    w.flags = (unsigned*)c.take(factor_dataflow_flag_bytes((int)batch));
    w.total = c.off;
    return w;
}

#define ATP_HIP(expr)                               \
    do {                                            \
        hipError_t e__ = (expr);                    \
        if (e__ != hipSuccess) return ATP_ERR_DEVICE; \
    } while (0)

// C = A · Bᵀ on the backend the storage type calls for: bf16 path -> MFMA kernel (operands bf16,
// optionally hi+lo planes), fp32 path or shapes the MFMA kernel does not cover -> fp32 FMA kernel.
hipError_t nt_product(hipStream_t st, bool mfma, const GemmArgs& g) {
    const bool split = g.A_lo != nullptr;
    const bool gram = g.symmetric != 0;   // the Gram matrix of the orthonormalisation, from one or both planes
    const double work = (double)g.batch * g.M * g.N * g.K;
    double flops = 2.0 * work * (g.swiglu ? 2.0 : 1.0);
    if (g.symmetric || g.b_lower) flops *= 0.5;  // algorithmic count: symmetric / triangular operand
    const double eb = mfma ? (split ? 4 : 2) : 4;
    const double out_b = (g.C32 ? 4 : 0) + (g.C16 ? 2 : 0) + (g.C16lo ? 2 : 0) + (g.CT32 ? 4 : 0) + (g.CT16 ? 2 : 0) +
                         (g.CT16lo ? 2 : 0);
    const double bytes = (double)g.batch * g.M * g.K * eb +
                         (double)(g.sB ? g.batch : 1) * g.N * (g.swiglu ? 2 : 1) * g.K * eb +
                         (double)g.batch * g.M * g.N * out_b * (g.ksplit > 1 ? g.ksplit : 1);
    if (mfma && gemm_nt_mfma_ok(g)) {
        int cls;
        if (split || gram) cls = g.symmetric ? ATP_K_GEMM_SPLIT_GRAM : ATP_K_GEMM_SPLIT_APPLY;
        else if (g.swiglu) cls = ATP_K_GEMM_SWIGLU;
        else cls = gemm_nt_mfma_big(g) ? ATP_K_GEMM_BF16 : ATP_K_GEMM_BF16_SMALL;
        ProfScope ps(st, cls, flops, bytes);
        return gemm_nt_mfma(st, g);
    }
    if (g.ksplit > 1) return hipErrorInvalidValue;  // callers only split K on the MFMA path
    ProfScope ps(st, ATP_K_GEMM_SIMT, flops, bytes);
    SimtArgs s;
    s.A = g.A; s.A_lo = g.A_lo; s.B = g.B; s.B_lo = g.B_lo;
    s.a_rs = g.lda; s.a_cs = 1; s.b_rs = g.ldb; s.b_cs = 1;
    s.sA = g.sA; s.sB = g.sB;
    s.M = g.M; s.N = g.N; s.K = g.K; s.batch = g.batch;
    s.C32 = g.C32; s.C16 = g.C16; s.C16lo = g.C16lo; s.ldc = g.ldc; s.sC = g.sC;
    s.CT32 = g.CT32; s.CT16 = g.CT16; s.CT16lo = g.CT16lo; s.ldct = g.ldct; s.sCT = g.sCT;
    s.swiglu = g.swiglu;
    const OperandType t = mfma ? OP_BF16 : OP_F32;
    return gemm_simt(st, t, t, s);
}

// A working matrix of the orthonormalisation: fp32 on the fp32 path, a hi+lo pair of bf16 planes
// (plane = batch*rows*cols elements) on the bf16 path.  Both fit 4 bytes per element.
struct Work {
    void* base = nullptr;
    int64_t elems = 0;
    float* f32() const { return reinterpret_cast<float*>(base); }
    bf16_t* hi() const { return reinterpret_cast<bf16_t*>(base); }
    bf16_t* lo() const { return reinterpret_cast<bf16_t*>(base) + elems; }
};
inline void set_A(GemmArgs& g, bool mfma, const Work& w) { g.A = w.base; g.A_lo = mfma ? w.lo() : nullptr; }
inline void set_B(GemmArgs& g, bool mfma, const Work& w) { g.B = w.base; g.B_lo = mfma ? w.lo() : nullptr; }
inline void set_C(GemmArgs& g, bool mfma, const Work& c, const Work& ct) {
    if (mfma) { g.C16 = c.hi(); g.C16lo = c.lo(); g.CT16 = ct.hi(); g.CT16lo = ct.lo(); }
    else { g.C32 = c.f32(); g.CT32 = ct.f32(); }
}

struct QrOut {  // where the last pass writes
    float* C32 = nullptr;
    bf16_t* C16 = nullptr;
    float* CT32 = nullptr;
    bf16_t* CT16 = nullptr;
};

// Column block [off, off+width) of a product (bf16 path: all operands are bf16 planes).
GemmArgs slice_n(GemmArgs g, int off, int width) {
    g.B = reinterpret_cast<const bf16_t*>(g.B) + (int64_t)off * g.ldb;
    if (g.B_lo) g.B_lo = reinterpret_cast<const bf16_t*>(g.B_lo) + (int64_t)off * g.ldb;
    g.N = width;
    if (g.C32) g.C32 += off;
    if (g.C16) g.C16 += off;
    if (g.C16lo) g.C16lo += off;
    if (g.CT32) g.CT32 += (int64_t)off * g.ldct;
    if (g.CT16) g.CT16 += (int64_t)off * g.ldct;
    if (g.CT16lo) g.CT16lo += (int64_t)off * g.ldct;
    return g;
}
// Row block [off, off+width) of a product.
GemmArgs slice_m(GemmArgs g, int off, int width) {
    g.A = reinterpret_cast<const bf16_t*>(g.A) + (int64_t)off * g.lda;
    if (g.A_lo) g.A_lo = reinterpret_cast<const bf16_t*>(g.A_lo) + (int64_t)off * g.lda;
    g.M = width;
    if (g.C32) g.C32 += (int64_t)off * g.ldc;
    if (g.C16) g.C16 += (int64_t)off * g.ldc;
    if (g.C16lo) g.C16lo += (int64_t)off * g.ldc;
    if (g.CT32) g.CT32 += off;
    if (g.CT16) g.CT16 += off;
    if (g.CT16lo) g.CT16lo += off;
    return g;
}

// The product that consumes the orthonormalised matrix Q right after a round: Q's column block k
// is the block k of its N dimension (FOLLOW_N: B operand = Qᵀ twin) or of its M dimension
// (FOLLOW_M: A operand = Qᵀ twin).
enum FollowSlice { FOLLOW_NONE = 0, FOLLOW_N = 1, FOLLOW_M = 2 };
struct Follow {
    GemmArgs g;
    FollowSlice slice = FOLLOW_NONE;
    bool done = false;  // set when the round has issued it (in pieces)
};

// Host-side state of one pipelined round: after the factorisation has finished the block columns
// of a 256-wide block of R^-1, the matching column block of Z·R^-1 and of the follow-up product
// are issued on the side stream.
constexpr int PIECE = 256;
struct PipeCtx {
    hipStream_t st;
    GemmArgs apply;
    Follow* follow;
    int r;
    hipError_t err = hipSuccess;
};
hipError_t pipe_after(void* vctx, int j) {
    PipeCtx& c = *reinterpret_cast<PipeCtx*>(vctx);
    if ((j + 1) % (PIECE / 64) != 0) return hipSuccess;
    const int off = (j + 1) * 64 - PIECE;
    hipEvent_t e = side_event();
    hipError_t err = hipEventRecord(e, c.st);
    if (err != hipSuccess) return err;
    err = hipStreamWaitEvent(g_side.stream, e, 0);
    if (err != hipSuccess) return err;
    GemmArgs a = slice_n(c.apply, off, PIECE);
    a.n_origin = off;
    a.K = std::min(c.r, off + PIECE);
    err = nt_product(g_side.stream, true, a);
    if (err != hipSuccess) return err;
    if (c.follow && c.follow->slice != FOLLOW_NONE) {
        const GemmArgs f = (c.follow->slice == FOLLOW_N) ? slice_n(c.follow->g, off, PIECE) : slice_m(c.follow->g, off, PIECE);
        err = nt_product(g_side.stream, true, f);
    }
    return err;
}

// Orthonormalise the columns of Z (n×r, fp32, with transposed twin ZT) by `passes` rounds of
// (Gram, Jacobi scaling + shift, Cholesky with inverse, apply).  Every round multiplies from the
// right by an upper-triangular matrix with positive diagonal, so the result is the Q factor of
// the positive-diagonal QR of Z.  Buffers ping-pong between slot `cur` and 1-cur; the last round
// writes to `out` when given.
//
// Intermediate orthonormalisations (final_qr == false) only have to keep the iterate well
// conditioned: all their rounds are shifted, which cannot break down, and the result has a
// condition number of a few units.  The final one ends with an unshifted round whose pivots certify
// the orthonormality of U_r (info).
//
// `follow` (may be null) is the product that consumes the result.  When the round can be pipelined
// (bf16 path, r a multiple of 256) the last round issues it itself, block by block behind the
// factorisation, and sets follow->done; otherwise the caller issues it.
atp_status cholesky_qr(hipStream_t st, bool mfma, bool final_qr, bool middle, int passes, float shift, Work Z[2], Work ZT[2],
                       int& cur, int n, int r, int batch, BasesWs& w, int32_t* info, const QrOut* out,
                       Follow* follow = nullptr) {
    Work linv;
    linv.base = w.Linv; linv.elems = (int64_t)batch * r * r;
    for (int p = 0; p < passes; ++p) {
        const bool last = (p == passes - 1);
        const bool certify = last && final_qr;
        GemmArgs g;
        set_A(g, mfma, ZT[cur]); set_B(g, mfma, ZT[cur]);
        g.lda = n; g.ldb = n; g.sA = (int64_t)r * n; g.sB = (int64_t)r * n;
        g.M = r; g.N = r; g.K = n; g.batch = batch;
        g.C32 = w.Spart; g.ldc = r; g.sC = (int64_t)r * r;
        g.symmetric = 1;
        if (mfma && !certify && (g_cond_gram_single >= 2 || (g_cond_gram_single == 1 && middle))) {
            // A shifted round only has to condition the iterate: R may be the Cholesky factor of the Gram
            // matrix of the hi planes alone (a 2^-9 relative perturbation of Z).  It is still an exact
            // triangular factor, and Z·R^-1 below is formed from both planes, so the subspace and the
            // triangular relation to Z are untouched; one MFMA product instead of three.
            GemmArgs h = g;
            h.A_lo = nullptr; h.B_lo = nullptr;
            if (gemm_nt_mfma_ok(h)) g = h;
        }
        int nparts = 1;
        if (mfma && gemm_nt_mfma_ok(g)) {
            // the Gram matrix has few output tiles and a long K: split K so that the launch fills the
            // chip.  Cost model in units of one 32-deep k-tile per workgroup: rounds of workgroups
            // (one per compute unit) × (k-tiles per slice + the epilogue, worth about 8 k-tiles).
            const int64_t ntri = (int64_t)((r + 255) / 256) * ((r + 255) / 256 + 1) / 2 * batch;
            const int kt = std::max(1, n / 32);
            const int np_max = std::max(1, std::min(KSPLIT_MAX, n / 256));
            double best = 0.0;
            for (int np = 1; np <= np_max; ++np) {
                const double rounds = (double)((ntri * np + NUM_CU - 1) / NUM_CU);
                const double cost = rounds * ((double)kt / np + 8.0);
                if (np == 1 || cost < best) { best = cost; nparts = np; }
            }
            g.ksplit = nparts;
            g.sKsplit = (int64_t)batch * r * r;
        } else {
            g.symmetric = 0;
        }
        // the product Z·R^-1 below (set up here because the initialisation depends on its kernel)
        GemmArgs a;
        set_A(a, mfma, Z[cur]); set_B(a, mfma, linv);
        a.lda = r; a.ldb = r; a.sA = (int64_t)n * r; a.sB = (int64_t)r * r;
        a.M = n; a.N = r; a.K = r; a.batch = batch;
        a.ldc = r; a.sC = (int64_t)n * r; a.ldct = n; a.sCT = (int64_t)n * r;
        a.b_lower = 1;
        const bool apply_mfma = mfma && gemm_nt_mfma_ok(a);
        const int zero_all = !apply_mfma;
        if (last && out) {
            a.C32 = out->C32; a.C16 = out->C16;
            a.CT32 = out->CT32; a.CT16 = out->CT16;
        } else {
            set_C(a, mfma, Z[1 - cur], ZT[1 - cur]);
        }
        // pipelined round: blocks of Z·R^-1 (and of the follow-up product) run on the side stream
        // behind the factorisation
        const bool pipe = g_overlap && apply_mfma && (r % PIECE == 0) && (r >= 2 * PIECE) && side_ready();
        Follow* fol = (last && follow && follow->slice != FOLLOW_NONE && gemm_nt_mfma_ok(follow->g)) ? follow : nullptr;
        PipeCtx pc;
        pc.st = st; pc.apply = a; pc.follow = fol; pc.r = r;
        ATP_HIP(nt_product(st, mfma, g));
        {
            ProfScope ps(st, ATP_K_CHOLESKY, (double)batch * r * r * r * (2.0 / 3.0), (double)batch * r * r * 16.0);
            const bool dataflow = g_factor_mode >= 1 && !pipe && factor_dataflow_ok(r, batch, g_factor_mode == 1);
            ATP_HIP(gram_prepare(st, w.Spart, nparts, (int64_t)batch * r * r, w.S, w.dinv, w.Y, mfma ? nullptr : w.Linv,
                                 mfma ? linv.hi() : nullptr, mfma ? linv.lo() : nullptr, r, certify ? 0.f : shift, zero_all, batch,
                                 dataflow ? w.flags : nullptr));
            if (dataflow)
                ATP_HIP(factor_inverse_dataflow(st, w.S, w.Lf, w.Y, w.dinv, mfma ? nullptr : w.Linv, mfma ? linv.hi() : nullptr,
                                                mfma ? linv.lo() : nullptr, w.flags, r, info, certify ? 1e-3f : 2e-6f, batch));
            else
                ATP_HIP(factor_inverse(st, w.S, w.Lf, w.Y, w.dinv, mfma ? nullptr : w.Linv, mfma ? linv.hi() : nullptr,
                                       mfma ? linv.lo() : nullptr, r, info, certify ? 1e-3f : 2e-6f, batch,
                                       pipe ? pipe_after : nullptr, &pc));
        }
        if (pipe) {
            hipEvent_t e = side_event();
            ATP_HIP(hipEventRecord(e, g_side.stream));
            ATP_HIP(hipStreamWaitEvent(st, e, 0));
            if (fol) fol->done = true;
        } else {
            ATP_HIP(nt_product(st, mfma, a));
        }
        cur = 1 - cur;
    }
    return ATP_OK;
}

}  // namespace

extern "C" {

const char* atp_status_string(atp_status s) {
    switch (raw_enum(s)) {
        case ATP_OK: return "ok";
        case ATP_ERR_INVALID_ARG: return "invalid argument";
        case ATP_ERR_BAD_RANK: return "rank r must satisfy 1 <= r <= min(L, d)";
        case ATP_ERR_WORKSPACE: return "workspace missing or too small";
        case ATP_ERR_UNSUPPORTED: return "unsupported shape";
        case ATP_ERR_DEVICE: return "HIP error";
        case ATP_ERR_SCRATCH_LIMIT: return "input larger than the library's built-in scratch buffer";
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

void atp_set_overlap(int on) { g_overlap = on ? 1 : 0; }

void atp_set_factor_mode(int mode) { g_factor_mode = mode < 0 ? 0 : (mode > 2 ? 2 : mode); }

void atp_set_factor_spin_limit(int polls) { factor_dataflow_set_spin_limit(polls); }

void atp_set_conditioning_gram(int single_product) { g_cond_gram_single = single_product < 0 ? 0 : (single_product > 2 ? 2 : single_product); }

atp_status atp_init(void) {
    if (!static_scratch_ptr()) return ATP_ERR_DEVICE;
    if (!side_ready()) return ATP_ERR_DEVICE;
    return ATP_OK;
}

void atp_set_qr_passes(int first, int middle, int last) {
    g_passes_first = std::min(4, std::max(1, first));
    g_passes_middle = std::min(4, std::max(1, middle));
    g_passes_last = std::min(4, std::max(1, last));
}

size_t atp_principal_bases_workspace(int64_t batch, int64_t L, int64_t d, int64_t r, int iters, atp_dtype t) {
    (void)iters;
    if (batch < 1 || L < 1 || d < 1 || r < 1 || bad_dtype(t)) return 0;
    return carve_bases(nullptr, batch, L, d, r, t).total;
}

atp_status atp_principal_bases(const void* X, int64_t batch, int64_t L, int64_t d, int64_t r, int iters,
                               const float* Omega, uint64_t seed, void* U_r, void* B_r, float* U_master,
                               int32_t* info, void* workspace, size_t workspace_bytes, atp_dtype t,
                               void* hip_stream) {
    if (!X || !U_r || !B_r || batch < 1 || L < 1 || d < 1 || iters < 0) return ATP_ERR_INVALID_ARG;
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
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
    if (mfma) ATP_HIP(cast_f32_to_bf16(st, w.OmT, w.OmT16, d * r));

    // Z = X·Ω
    int curL = 0, curD = 0;
    Work ZL[2], ZLT[2], ZD[2], ZDT[2];
    for (int i = 0; i < 2; ++i) {
        ZL[i].base = w.ZL[i]; ZLT[i].base = w.ZLT[i]; ZL[i].elems = ZLT[i].elems = batch * L * r;
        ZD[i].base = w.ZD[i]; ZDT[i].base = w.ZDT[i]; ZD[i].elems = ZDT[i].elems = batch * d * r;
    }
    {
        GemmArgs g;
        g.A = X; g.B = mfma ? (const void*)w.OmT16 : (const void*)w.OmT;
        g.lda = d; g.ldb = d; g.sA = L * d; g.sB = 0;
        g.M = iL; g.N = ir; g.K = id; g.batch = ib;
        g.ldc = r; g.sC = L * r; g.ldct = L; g.sCT = L * r;
        set_C(g, mfma, ZL[0], ZLT[0]);
        ATP_HIP(nt_product(st, mfma, g));
    }
    // the last round of every orthonormalisation writes only what its consumer reads: the
    // transposed twin in the storage type (B operand of the next product), and for the final one
    // the outputs U_r / U_master
    QrOut fin, midL, midD;
    if (t == ATP_BF16) {
        fin.C16 = (bf16_t*)U_r; fin.C32 = U_master; fin.CT16 = (bf16_t*)w.TL;
        midL.CT16 = (bf16_t*)w.TL;
        midD.CT16 = (bf16_t*)w.TD;
    } else {
        fin.C32 = (float*)U_r; fin.CT32 = (float*)w.TL;
        midL.CT32 = (float*)w.TL;
        midD.CT32 = (float*)w.TD;
    }
    // the three products that consume an orthonormalised iterate
    auto prod_w = [&]() {  // W = Xᵀ·U      (d×r)
        GemmArgs g;
        g.A = w.XT; g.B = w.TL; g.lda = L; g.ldb = L; g.sA = L * d; g.sB = L * r;
        g.M = id; g.N = ir; g.K = iL; g.batch = ib;
        g.ldc = r; g.sC = d * r; g.ldct = d; g.sCT = d * r;
        set_C(g, mfma, ZD[0], ZDT[0]);
        return g;
    };
    auto prod_z = [&]() {  // Z = X·V       (L×r)
        GemmArgs h;
        h.A = X; h.B = w.TD; h.lda = d; h.ldb = d; h.sA = L * d; h.sB = d * r;
        h.M = iL; h.N = ir; h.K = id; h.batch = ib;
        h.ldc = r; h.sC = L * r; h.ldct = L; h.sCT = L * r;
        set_C(h, mfma, ZL[0], ZLT[0]);
        return h;
    };
    auto prod_b = [&]() {  // B_r = U_rᵀ·X  (r×d) with the returned (rounded) U_r
        GemmArgs g;
        g.A = w.TL; g.B = w.XT; g.lda = L; g.ldb = L; g.sA = r * L; g.sB = d * L;
        g.M = ir; g.N = id; g.K = iL; g.batch = ib;
        g.ldc = d; g.sC = r * d;
        if (t == ATP_BF16) g.C16 = (bf16_t*)B_r; else g.C32 = (float*)B_r;
        return g;
    };
    // an orthonormalisation followed by the product that consumes it (issued here unless the
    // orthonormalisation has already issued it block by block)
    auto qr_then = [&](bool final_qr, bool middle, int passes, Work* Zw, Work* ZTw, int& cur, int n, const QrOut* out, GemmArgs next,
                       FollowSlice how) -> atp_status {
        Follow f;
        f.g = next;
        f.slice = how;
        const atp_status s = cholesky_qr(st, mfma, final_qr, middle, passes, shift, Zw, ZTw, cur, n, ir, ib, w, inf, out, &f);
        if (s != ATP_OK) return s;
        if (final_qr && t == ATP_F32 && U_master)
            ATP_HIP(hipMemcpyAsync(U_master, U_r, (size_t)batch * L * r * 4, hipMemcpyDeviceToDevice, st));
        if (!f.done) ATP_HIP(nt_product(st, mfma, next));
        return ATP_OK;
    };

    atp_status s;
    if (iters == 0) {
        s = qr_then(true, false, g_passes_last, ZL, ZLT, curL, iL, &fin, prod_b(), FOLLOW_M);
        if (s != ATP_OK) return s;
    } else {
        s = qr_then(false, false, g_passes_first, ZL, ZLT, curL, iL, &midL, prod_w(), FOLLOW_N);
        if (s != ATP_OK) return s;
    }
    for (int it = 0; it < iters; ++it) {
        curD = 0;
        s = qr_then(false, true, g_passes_middle, ZD, ZDT, curD, id, &midD, prod_z(), FOLLOW_N);
        if (s != ATP_OK) return s;
        curL = 0;
        const bool lastit = (it == iters - 1);
        if (lastit) s = qr_then(true, false, g_passes_last, ZL, ZLT, curL, iL, &fin, prod_b(), FOLLOW_M);
        else s = qr_then(false, true, g_passes_middle, ZL, ZLT, curL, iL, &midL, prod_w(), FOLLOW_N);
        if (s != ATP_OK) return s;
    }
    return ATP_OK;
}

size_t atp_alternating_bases_workspace(int64_t batch, int64_t L, int64_t d, int64_t r, atp_dtype t) {
    (void)t;
    if (batch < 1 || L < 1 || d < 1 || r < 1) return 0;
    return alternating_workspace((int)batch, (int)L, (int)d) + align_up((size_t)d * r * 4) + align_up((size_t)batch * 4);
}

atp_status atp_alternating_bases(const void* X, int64_t batch, int64_t L, int64_t d, int64_t r, int sweeps,
                                 const float* V0, uint64_t seed, void* U_r, void* B_r, int32_t* info, void* workspace,
                                 size_t workspace_bytes, atp_dtype t, void* hip_stream) {
    if (!X || !U_r || !B_r || batch < 1 || L < 1 || d < 1 || sweeps < 1) return ATP_ERR_INVALID_ARG;
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || L > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (r < 1 || r > std::min(L, d)) return ATP_ERR_BAD_RANK;
    if (d > 4096 || (d & 3)) return ATP_ERR_UNSUPPORTED;
    if (!aligned16(X) || !aligned16(U_r) || !aligned16(B_r) || !aligned16(V0) || !aligned16(workspace) ||
        (((uintptr_t)info) & 3))
        return ATP_ERR_INVALID_ARG;
    const size_t need = atp_alternating_bases_workspace(batch, L, d, r, t);
    if (!workspace || workspace_bytes < need) return ATP_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    uint8_t* ws = reinterpret_cast<uint8_t*>(workspace);
    const size_t core = alternating_workspace((int)batch, (int)L, (int)d);
    float* v0buf = reinterpret_cast<float*>(ws + core);
    int32_t* infbuf = reinterpret_cast<int32_t*>(ws + core + align_up((size_t)d * r * 4));
    const float* V = V0;
    if (!V) {
        ATP_HIP(fill_gaussian(st, v0buf, d * r, seed));
        V = v0buf;
    }
    int32_t* inf = info ? info : infbuf;
    ATP_HIP(fill_zero_i32(st, inf, batch));
    ProfScope ps(st, ATP_K_STREAM, 0.0, (double)batch * L * d * 4.0 * (sweeps + 1.0) * r);
    ATP_HIP(alternating_bases(st, X, (int)batch, (int)L, (int)d, (int)r, sweeps, V, U_r, B_r, inf, workspace,
                              (int)esize(t)));
    return ATP_OK;
}

size_t atp_rayleigh_ritz_workspace(int64_t batch, int64_t L, int64_t d, int64_t r, atp_dtype t) {
    (void)L; (void)d; (void)t;
    if (batch < 1 || r < 1) return 0;
    const int64_t rp = (r + 63) / 64 * 64;
    return 5 * align_up((size_t)batch * r * r * 4) + align_up((size_t)batch * rp * 4) + 2 * align_up((size_t)batch * r * 4);
}

atp_status atp_rayleigh_ritz(const void* U_r, const void* B_r, int64_t batch, int64_t L, int64_t d, int64_t r,
                             int sweeps, void* U_out, void* B_out, float* sigma, float* diagnostics, void* workspace,
                             size_t workspace_bytes, atp_dtype t, void* hip_stream) {
    if (!U_r || !B_r || !U_out || !B_out || !sigma || batch < 1 || L < 1 || d < 1 || sweeps < 1) return ATP_ERR_INVALID_ARG;
    if (U_out == U_r || B_out == B_r) return ATP_ERR_INVALID_ARG;
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || L > (1 << 30) || d > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (r < 1 || r > std::min(L, d)) return ATP_ERR_BAD_RANK;
    if (r > 4096) return ATP_ERR_UNSUPPORTED;
    if (!aligned16(U_r) || !aligned16(B_r) || !aligned16(U_out) || !aligned16(B_out) || !aligned16(workspace) ||
        (((uintptr_t)sigma) & 3) || (((uintptr_t)diagnostics) & 3))
        return ATP_ERR_INVALID_ARG;
    const size_t need = atp_rayleigh_ritz_workspace(batch, L, d, r, t);
    if (!workspace || workspace_bytes < need) return ATP_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const int ib = (int)batch, iL = (int)L, id = (int)d, ir = (int)r;
    const int64_t rp = (r + 63) / 64 * 64;
    Carver c(workspace);
    float* T0 = (float*)c.take((size_t)batch * r * r * 4);
    float* T1 = (float*)c.take((size_t)batch * r * r * 4);
    float* R0 = (float*)c.take((size_t)batch * r * r * 4);
    float* R1 = (float*)c.take((size_t)batch * r * r * 4);
    float* RsT = (float*)c.take((size_t)batch * r * r * 4);
    float* cs = (float*)c.take((size_t)batch * rp * 4);
    int* rank = (int*)c.take((size_t)batch * r * 4);
    int* zsum = (int*)c.take((size_t)batch * r * 4);
    const OperandType ot = (t == ATP_BF16) ? OP_BF16 : OP_F32;
    // T = B·Bᵀ (fp32 accumulation of exact products)
    {
        SimtArgs g;
        g.A = B_r; g.B = B_r; g.a_rs = d; g.a_cs = 1; g.b_rs = d; g.b_cs = 1; g.sA = r * d; g.sB = r * d;
        g.M = ir; g.N = ir; g.K = id; g.batch = ib;
        g.C32 = T0; g.ldc = r; g.sC = r * r;
        ProfScope ps(st, ATP_K_GEMM_SIMT, 2.0 * batch * r * r * d, (double)batch * r * d * esize(t));
        ATP_HIP(gemm_simt(st, ot, ot, g));
    }
    float *Tf = nullptr, *Rf = nullptr;
    ATP_HIP(ritz_jacobi(st, T0, T1, R0, R1, ir, ib, sweeps, &Tf, &Rf));
    ATP_HIP(column_sums(st, U_r, cs, iL, ir, rp, ib, (int)esize(t)));
    const float zero_tol = (t == ATP_BF16 ? 2e-4f : 1e-5f) * sqrtf((float)L);
    ATP_HIP(ritz_order(st, Tf, Rf, cs, rp, rank, RsT, sigma, zsum, ir, ib, zero_tol));
    {   // U_out = U_r·Rs
        SimtArgs g;
        g.A = U_r; g.B = RsT; g.a_rs = r; g.a_cs = 1; g.b_rs = r; g.b_cs = 1; g.sA = L * r; g.sB = r * r;
        g.M = iL; g.N = ir; g.K = ir; g.batch = ib;
        if (t == ATP_BF16) g.C16 = (bf16_t*)U_out; else g.C32 = (float*)U_out;
        g.ldc = r; g.sC = L * r;
        ProfScope ps(st, ATP_K_GEMM_SIMT, 2.0 * batch * L * r * r, (double)batch * L * r * esize(t) * 2);
        ATP_HIP(gemm_simt(st, ot, OP_F32, g));
    }
    {   // B_out = Rsᵀ·B_r
        SimtArgs g;
        g.A = RsT; g.B = B_r; g.a_rs = r; g.a_cs = 1; g.b_rs = 1; g.b_cs = d; g.sA = r * r; g.sB = r * d;
        g.M = ir; g.N = id; g.K = ir; g.batch = ib;
        if (t == ATP_BF16) g.C16 = (bf16_t*)B_out; else g.C32 = (float*)B_out;
        g.ldc = d; g.sC = r * d;
        ProfScope ps(st, ATP_K_GEMM_SIMT, 2.0 * batch * r * r * d, (double)batch * r * d * esize(t) * 2);
        ATP_HIP(gemm_simt(st, OP_F32, ot, g));
    }
    ATP_HIP(ritz_fallback_sign(st, U_out, B_out, zsum, iL, id, ir, ib, (int)esize(t)));
    if (diagnostics) ATP_HIP(ritz_diagnostics(st, Tf, sigma, ir, ib, diagnostics));
    return ATP_OK;
}

atp_status atp_rope(const void* Y, void* out, int64_t batch, int64_t L, int64_t dq, int heads, float base, int64_t pos0,
                    atp_dtype t, void* hip_stream) {
    if (!Y || !out || batch < 1 || L < 1 || dq < 1 || heads < 1 || !(base > 1.f) || pos0 < 0) return ATP_ERR_INVALID_ARG;
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
    if (dq % heads || ((dq / heads) & 1)) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || L > (1 << 30) || dq > (1 << 30) || pos0 > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (!aligned16(Y) || !aligned16(out)) return ATP_ERR_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    ProfScope ps(st, ATP_K_STREAM, 0.0, 2.0 * (double)batch * L * dq * esize(t));
    ATP_HIP(rope_rows(st, Y, out, (int)batch, (int)L, (int)dq, (int)(dq / heads), base, (int)pos0, (int)esize(t)));
    return ATP_OK;
}

size_t atp_project_onto_bases_workspace(int64_t batch, int64_t L, int64_t r, int64_t dq, atp_dtype t) {
    if (batch < 1 || L < 1 || r < 1 || dq < 1) return 0;
    if (t != ATP_BF16) return 0;
    return align_up((size_t)batch * r * L * 2) + align_up((size_t)batch * dq * L * 2);
}

atp_status atp_project_onto_bases(const void* U_r, const void* Y, void* out, int64_t batch, int64_t L, int64_t r,
                                  int64_t dq, void* workspace, size_t workspace_bytes, atp_dtype t, void* hip_stream) {
    if (!U_r || !Y || !out || batch < 1 || L < 1 || r < 1 || dq < 1) return ATP_ERR_INVALID_ARG;
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || L > (1 << 30) || r > (1 << 30) || dq > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (!aligned16(U_r) || !aligned16(Y) || !aligned16(out) || !aligned16(workspace)) return ATP_ERR_INVALID_ARG;
    const size_t need = atp_project_onto_bases_workspace(batch, L, r, dq, t);
    if (need && (!workspace || workspace_bytes < need)) return ATP_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    if (t == ATP_F32) {   // strided fp32 kernel: A(m,k) = U[k][m], B(n,k) = Y[k][n]
        SimtArgs s;
        s.A = U_r; s.B = Y; s.a_rs = 1; s.a_cs = r; s.b_rs = 1; s.b_cs = dq; s.sA = L * r; s.sB = L * dq;
        s.M = (int)r; s.N = (int)dq; s.K = (int)L; s.batch = (int)batch;
        s.C32 = (float*)out; s.ldc = dq; s.sC = r * dq;
        ProfScope ps(st, ATP_K_GEMM_SIMT, 2.0 * batch * r * dq * L, 4.0 * batch * (L * r + L * dq + r * dq));
        ATP_HIP(gemm_simt(st, OP_F32, OP_F32, s));
        return ATP_OK;
    }
    Carver c(workspace);
    void* UT = c.take((size_t)batch * r * L * 2);
    void* YT = c.take((size_t)batch * dq * L * 2);
    {
        ProfScope ps(st, ATP_K_STREAM, 0.0, 4.0 * (double)batch * L * (r + dq));
        ATP_HIP(transpose_batched(st, U_r, UT, (int)L, (int)r, L, L * r, r * L, (int)batch, 2, 0));
        ATP_HIP(transpose_batched(st, Y, YT, (int)L, (int)dq, L, L * dq, dq * L, (int)batch, 2, 0));
    }
    GemmArgs g;
    g.A = UT; g.B = YT; g.lda = L; g.ldb = L; g.sA = r * L; g.sB = dq * L;
    g.M = (int)r; g.N = (int)dq; g.K = (int)L; g.batch = (int)batch;
    g.C16 = (bf16_t*)out; g.ldc = dq; g.sC = r * dq;
    ATP_HIP(nt_product(st, true, g));
    return ATP_OK;
}


atp_status atp_concat_factors(const void* U1, const void* C1, const void* U2, const void* C2, void* P, void* C, int64_t batch,
                              int64_t L, int64_t d, int64_t r1, int64_t r2, atp_dtype t, void* hip_stream) {
    if (!U1 || !C1 || !U2 || !C2 || !P || !C || batch < 1 || L < 1 || d < 1 || r1 < 1 || r2 < 1) return ATP_ERR_INVALID_ARG;
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || L > 65535 || r1 + r2 > 65535 || d > (1 << 30)) return ATP_ERR_UNSUPPORTED;
    if (!aligned16(U1) || !aligned16(C1) || !aligned16(U2) || !aligned16(C2) || !aligned16(P) || !aligned16(C)) return ATP_ERR_INVALID_ARG;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const int es = (int)esize(t);
    const int64_t m = r1 + r2;
    uint8_t* Pb = reinterpret_cast<uint8_t*>(P);
    uint8_t* Cb = reinterpret_cast<uint8_t*>(C);
    ProfScope ps(st, ATP_K_STREAM, 0.0, 2.0 * (double)batch * (L + d) * m * es);
    ATP_HIP(copy_block(st, U1, Pb, (int)L, (int)r1, r1, m, L * r1, L * m, (int)batch, es));
    ATP_HIP(copy_block(st, U2, Pb + (size_t)r1 * es, (int)L, (int)r2, r2, m, L * r2, L * m, (int)batch, es));
    ATP_HIP(copy_block(st, C1, Cb, (int)r1, (int)d, d, d, r1 * d, m * d, (int)batch, es));
    ATP_HIP(copy_block(st, C2, Cb + (size_t)r1 * d * es, (int)r2, (int)d, d, d, r2 * d, m * d, (int)batch, es));
    return ATP_OK;
}

size_t atp_norm_factored_workspace(int64_t batch, int64_t L, int64_t d, int64_t m, atp_dtype t) {
    if (batch < 1 || L < 1 || d < 1 || m < 1 || bad_dtype(t)) return 0;
    return align_up((size_t)batch * m * d * esize(t)) + align_up((size_t)batch * m * m * 4) + align_up((size_t)batch * m * m * 2) +
           align_up((size_t)batch * L * m * 4);
}

atp_status atp_norm_factored(const void* P, const void* C, const float* gain, float eps, int center, void* Pn, void* Cn,
                             int64_t batch, int64_t L, int64_t d, int64_t m, void* workspace, size_t workspace_bytes,
                             atp_dtype t, void* hip_stream) {
    if (!P || !C || !gain || !Pn || !Cn || batch < 1 || L < 1 || d < 1 || m < 1 || !(eps >= 0.f)) return ATP_ERR_INVALID_ARG;
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || L > (1 << 30) || d > (1 << 30) || m > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (batch * L > 0x7fffffffll || batch * m > 0x7fffffffll) return ATP_ERR_UNSUPPORTED;
    if (!aligned16(P) || !aligned16(C) || !aligned16(Pn) || !aligned16(Cn) || !aligned16(workspace) || (((uintptr_t)gain) & 3))
        return ATP_ERR_INVALID_ARG;
    const size_t need = atp_norm_factored_workspace(batch, L, d, m, t);
    if (!workspace || workspace_bytes < need) return ATP_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const bool mfma = (t == ATP_BF16);
    const int es = (int)esize(t);
    Carver c(workspace);
    void* Cc = c.take((size_t)batch * m * d * es);
    float* M32 = (float*)c.take((size_t)batch * m * m * 4);
    bf16_t* M16 = (bf16_t*)c.take((size_t)batch * m * m * 2);
    float* PM = (float*)c.take((size_t)batch * L * m * 4);
    {
        ProfScope ps(st, ATP_K_STREAM, 0.0, 3.0 * (double)batch * m * d * es);
        ATP_HIP(norm_coeff(st, C, gain, Cc, Cn, batch * m, (int)d, center ? 1 : 0, es));
    }
    {   // M = Cc·Ccᵀ: the Gram matrix of the (centred) coefficient rows
        GemmArgs g;
        g.A = Cc; g.B = Cc; g.lda = d; g.ldb = d; g.sA = m * d; g.sB = m * d;
        g.M = (int)m; g.N = (int)m; g.K = (int)d; g.batch = (int)batch;
        g.C32 = M32; g.ldc = m; g.sC = m * m;
        ATP_HIP(nt_product(st, mfma, g));
    }
    const void* Mop = M32;
    if (mfma) {
        ATP_HIP(cast_f32_to_bf16(st, M32, M16, batch * m * m));
        Mop = M16;
    }
    {   // PM = P·M (M is symmetric, so it is its own K-contiguous operand)
        GemmArgs g;
        g.A = P; g.B = Mop; g.lda = m; g.ldb = m; g.sA = L * m; g.sB = m * m;
        g.M = (int)L; g.N = (int)m; g.K = (int)m; g.batch = (int)batch;
        g.C32 = PM; g.ldc = m; g.sC = L * m;
        ATP_HIP(nt_product(st, mfma, g));
    }
    {
        ProfScope ps(st, ATP_K_STREAM, 0.0, (double)batch * L * m * (2.0 * es + 4.0));
        ATP_HIP(norm_basis(st, P, PM, Pn, batch * L, (int)m, (int)d, eps, es));
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
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
    if (raw_enum(w_layout) != ATP_W_KN && raw_enum(w_layout) != ATP_W_NK) return ATP_ERR_INVALID_ARG;
    if (raw_enum(epilogue) != ATP_EPI_NONE && raw_enum(epilogue) != ATP_EPI_SWIGLU) return ATP_ERR_INVALID_ARG;
    if (epilogue == ATP_EPI_SWIGLU && (n & 1)) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || m > (1 << 30) || k > (1 << 30) || n > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (!aligned16(B) || !aligned16(W) || !aligned16(out) || !aligned16(workspace)) return ATP_ERR_INVALID_ARG;
    const size_t need = atp_lowrank_linear_workspace(batch, m, k, n, w_stride, w_layout, t);
    if (need && (!workspace || workspace_bytes < need)) return ATP_ERR_WORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const bool swiglu = (epilogue == ATP_EPI_SWIGLU);
    const int64_t nout = swiglu ? n / 2 : n;

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
    if (sW == 0 && batch > 1 && batch * m < (1ll << 30)) {
        // shared weights: the batch is one tall matrix [batch·m, k]; as a single product every pass over a
        // block of W serves the rows of all sequences
        GemmArgs f = g;
        f.M = (int)(batch * m); f.batch = 1; f.sA = 0; f.sC = 0;
        if (gemm_nt_mfma_ok(f)) g = f;
    }
    ATP_HIP(nt_product(st, true, g));
    return ATP_OK;
}

size_t atp_attention_workspace(int64_t batch, int64_t L, int64_t r, int64_t dq, int heads, atp_dtype t) {
    (void)L; (void)heads;
    if (batch < 1 || r < 1 || dq < 1) return 0;
    if (t != ATP_BF16) return 0;
    const int64_t rp = (r + 63) / 64 * 64;
    return align_up((size_t)batch * dq * rp * 2);
}

size_t atp_attention_linearised_workspace(int64_t batch, int64_t L, int64_t r, int64_t dq, int heads, atp_dtype t) {
    if (batch < 1 || r < 1 || dq < 1) return 0;
    const int64_t rp = (r + 63) / 64 * 64;
    return atp_attention_workspace(batch, L, r, dq, heads, t) + align_up((size_t)batch * rp * 4);
}

namespace {
// shared body of the two attention entry points; U_r == nullptr selects softmax attention
atp_status attention_call(const void* Q, const void* K_r, const void* V_r, const void* U_r, void* O, int64_t batch,
                          int64_t L, int64_t r, int64_t dq, int heads, float scale, int norm, void* workspace,
                          size_t workspace_bytes, atp_dtype t, void* hip_stream, bool linearised,
                          bool static_scratch = false) {
    if (!Q || !K_r || !V_r || !O || batch < 1 || L < 1 || r < 1 || dq < 1 || heads < 1) return ATP_ERR_INVALID_ARG;
    if (linearised && (!U_r || (norm != ATP_NORM_TAYLOR && norm != ATP_NORM_ROWSUM))) return ATP_ERR_INVALID_ARG;
    if (bad_dtype(t)) return ATP_ERR_INVALID_ARG;
    if (dq % heads) return ATP_ERR_INVALID_ARG;
    if (batch > 65535 || heads > 65535 || L > (1 << 30) || r > (1 << 30) || dq > (1 << 30)) return ATP_ERR_INVALID_ARG;
    if (!aligned16(Q) || !aligned16(K_r) || !aligned16(V_r) || !aligned16(O) || !aligned16(U_r) || !aligned16(workspace))
        return ATP_ERR_INVALID_ARG;
    const int64_t dh = dq / heads;
    if (t == ATP_BF16 && dh != 64 && dh != 128) return ATP_ERR_UNSUPPORTED;
    if (t == ATP_BF16 && r * dq >= (1ll << 30)) return ATP_ERR_UNSUPPORTED;   // 32-bit byte offsets within one K'/V' item
    if (t == ATP_F32 && dh > 256) return ATP_ERR_UNSUPPORTED;
    const size_t need = linearised ? atp_attention_linearised_workspace(batch, L, r, dq, heads, t)
                                   : atp_attention_workspace(batch, L, r, dq, heads, t);
    if (static_scratch) {
        // the library's own buffer takes the place of the workspace argument
        if (need > STATIC_SCRATCH_BYTES) return ATP_ERR_SCRATCH_LIMIT;
        workspace = need ? static_scratch_ptr() : nullptr;
        if (need && !workspace) return ATP_ERR_DEVICE;
        workspace_bytes = STATIC_SCRATCH_BYTES;
    }
    if (need && (!workspace || workspace_bytes < need)) return ATP_ERR_WORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const int64_t rp = (r + 63) / 64 * 64;
    AttnArgs a;
    a.Q = Q; a.K = K_r; a.V = V_r; a.O = O;
    a.batch = (int)batch; a.L = (int)L; a.nk = (int)r; a.nk_pad = (int)rp; a.dq = (int)dq; a.heads = heads;
    a.scale = (scale > 0.f) ? scale : 1.0f / sqrtf((float)dh);
    Carver c(workspace);
    void* vt = (t == ATP_BF16) ? c.take((size_t)batch * dq * rp * 2) : nullptr;
    if (linearised) {
        float* cs = (float*)c.take((size_t)batch * rp * 4);
        ProfScope ps(st, ATP_K_STREAM, 0.0, (double)batch * L * r * esize(t));
        ATP_HIP(column_sums(st, U_r, cs, (int)L, (int)r, rp, (int)batch, (int)esize(t)));
        a.linearised = 1; a.colsum = cs; a.norm_rowsum = (norm == ATP_NORM_ROWSUM); a.n_tokens = (float)L;
    }
    if (t == ATP_F32) {
        ATP_HIP(attention_f32(st, a));
        return ATP_OK;
    }
    // values re-laid out as [dq][r_pad] (zero padded) so a lane reads 8 consecutive keys of one feature
    {
        ProfScope ps(st, ATP_K_STREAM, 0.0, 4.0 * (double)batch * r * dq);
        ATP_HIP(transpose_batched(st, V_r, vt, (int)r, (int)dq, rp, r * dq, dq * rp, (int)batch, 2, 1));
    }
    a.Vt = vt;
    {
        ProfScope ps(st, ATP_K_ATTENTION, 4.0 * (double)batch * L * r * dq,
                     2.0 * (double)batch * (2.0 * L * dq + 2.0 * r * dq));
        ATP_HIP(attention_bf16(st, a));
    }
    return ATP_OK;
}
}  // namespace

atp_status atp_attention(const void* Q, const void* K_r, const void* V_r, void* O, int64_t batch, int64_t L,
                         int64_t r, int64_t dq, int heads, float scale, void* workspace, size_t workspace_bytes,
                         atp_dtype t, void* hip_stream) {
    return attention_call(Q, K_r, V_r, nullptr, O, batch, L, r, dq, heads, scale, 0, workspace, workspace_bytes, t,
                          hip_stream, false);
}

atp_status atp_attention_static(const void* Q, const void* K_r, const void* V_r, void* O, int64_t batch, int64_t L,
                                int64_t r, int64_t dq, int heads, float scale, atp_dtype t, void* hip_stream) {
    return attention_call(Q, K_r, V_r, nullptr, O, batch, L, r, dq, heads, scale, 0, nullptr, 0, t, hip_stream, false,
                          true);
}

atp_status atp_attention_linearised(const void* Q, const void* K_r, const void* V_r, const void* U_r, void* O,
                                    int64_t batch, int64_t L, int64_t r, int64_t dq, int heads, float scale,
                                    atp_lin_norm norm, void* workspace, size_t workspace_bytes, atp_dtype t,
                                    void* hip_stream) {
    return attention_call(Q, K_r, V_r, U_r, O, batch, L, r, dq, heads, scale, (int)norm, workspace, workspace_bytes, t,
                          hip_stream, true);
}

}  // extern "C"
