// Shared declarations of the ATP HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace atp {

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// two floats -> packed pair of bfloat16 (lo in bits 0..15), round to nearest even: one
// v_cvt_pk_bf16_f32 on gfx950
__device__ __forceinline__ uint32_t pack_bf2(float a, float b) {
    const f32x2 v = {a, b};
    union { bf16x2 h; uint32_t u; } c;
    c.h = __builtin_convertvector(v, bf16x2);
    return c.u;
}
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(pack_bf2(f, 0.f) & 0xffffu); }
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

// 16-byte-per-lane asynchronous copy global -> LDS written as inline assembly: the compiler neither
// tracks it nor adds waits of its own for it (with the builtin it inserts a full vmcnt(0) drain at
// the head of a loop whose body reads a stage that was filled one trip earlier).  The global address
// is a wave-uniform base (SGPR pair) plus a 32-bit byte offset per lane, the LDS address `lds` a
// wave-uniform byte address (lane q lands at lds + 16·q): three instructions per copy and no vector
// address arithmetic in the loop.
// M0 is written by the copy and is named in the clobber list so that the compiler never assumes a value
// of its own survives the statement (the compiler warns about any reserved register there; silenced).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void copy16_untracked(const void* base, unsigned off_bytes, unsigned lds) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off_bytes), "s"(base), "s"(lds) : "memory", "m0");
}
#pragma clang diagnostic pop

// ---------------------------------------------------------------------------
// C = A · Bᵀ  with both operands K-contiguous ("NT" product), batched.
//   A[M,K] (lda), B[N,K] (ldb); fp32 accumulate.
// MFMA path: operands are bf16.  A value that needs more than bf16 precision is held as a
// hi + lo pair of bf16 planes (hi = bf16(x), lo = bf16(x - hi), ≈16 mantissa bits); when both
// operands carry a lo plane the product is formed from three MFMA products (hi·hi, hi·lo,
// lo·hi, ≈2^-17 relative error).
// Any subset of the outputs may be requested (null = skip):
//   C32 / C16 (+C16lo) : C[M,N] row-major (ldc);  CT32 / CT16 (+CT16lo) : Cᵀ[N,M] (ldct).
// SWIGLU epilogue: B has 2·Nh rows (gate rows then up rows); the output has Nh
// columns: SiLU(A·gateᵀ) ⊙ (A·upᵀ).  N below is Nh in that case.
// ---------------------------------------------------------------------------
struct GemmArgs {
    const void* A = nullptr;
    const void* A_lo = nullptr;
    const void* B = nullptr;
    const void* B_lo = nullptr;
    int64_t lda = 0, ldb = 0, sA = 0, sB = 0;  // leading dims, batch strides (elements)
    int M = 0, N = 0, K = 0, batch = 1;
    float* C32 = nullptr;
    bf16_t* C16 = nullptr;
    bf16_t* C16lo = nullptr;
    int64_t ldc = 0, sC = 0;
    float* CT32 = nullptr;
    bf16_t* CT16 = nullptr;
    bf16_t* CT16lo = nullptr;
    int64_t ldct = 0, sCT = 0;
    int swiglu = 0;
    // K range limit per output tile for triangular B (B[n][k] = 0 for k > n): 1 = on.  When B is a
    // row block of the triangular matrix, n_origin is the index of its first row.
    int b_lower = 0;
    int n_origin = 0;
    // symmetric output (A == B): only tiles with tileN <= tileM are computed and written; the
    // strictly upper tiles of the output are left untouched
    int symmetric = 0;
    // split-K: slice z of the K range writes a partial product to C32 + z*sKsplit (C32 only)
    int ksplit = 0;
    int64_t sKsplit = 0;
};

enum OperandType { OP_BF16 = 0, OP_F32 = 1 };

// MFMA path (bf16 operands, optional lo planes).  Requirements: K % 64 == 0 (K % 32 == 0 with lo
// planes), lda/ldb/sA/sB % 8 == 0, pointers 16-byte aligned.
hipError_t gemm_nt_mfma(hipStream_t st, const GemmArgs& g);
bool gemm_nt_mfma_ok(const GemmArgs& g);
bool gemm_nt_mfma_big(const GemmArgs& g);  // true when the 256×256 tile configuration is chosen

// Generic SIMT fp32-FMA path with element strides (any layout, any size).  ta/tb give the
// element type of A/B; bf16 operands may carry a lo plane (same strides) that is added on load.
struct SimtArgs {
    const void* A = nullptr;
    const void* A_lo = nullptr;
    const void* B = nullptr;
    const void* B_lo = nullptr;
    int64_t a_rs = 0, a_cs = 0, b_rs = 0, b_cs = 0;  // A(m,k) = A[m*a_rs + k*a_cs]; B(n,k) = B[n*b_rs + k*b_cs]
    int64_t sA = 0, sB = 0;
    int M = 0, N = 0, K = 0, batch = 1;
    float* C32 = nullptr;
    bf16_t* C16 = nullptr;
    bf16_t* C16lo = nullptr;
    int64_t ldc = 0, sC = 0;
    float* CT32 = nullptr;
    bf16_t* CT16 = nullptr;
    bf16_t* CT16lo = nullptr;
    int64_t ldct = 0, sCT = 0;
    int swiglu = 0;
};
hipError_t gemm_simt(hipStream_t st, OperandType ta, OperandType tb, const SimtArgs& g);

// ---------------------------------------------------------------------------
// streaming passes
// ---------------------------------------------------------------------------
// out[b][c][r] = in[b][r][c]   (rows×cols -> cols×rows), elem_bytes 2 or 4; out row length ld_out
hipError_t transpose_batched(hipStream_t st, const void* in, void* out, int rows, int cols,
                             int64_t ld_out, int64_t s_in, int64_t s_out, int batch, int elem_bytes,
                             int zero_pad_cols);
// Omega generator: out[d*r] fp32 N(0,1), counter-based
hipError_t fill_gaussian(hipStream_t st, float* out, int64_t n, uint64_t seed);
hipError_t fill_zero_i32(hipStream_t st, int32_t* p, int64_t n);
hipError_t cast_f32_to_bf16(hipStream_t st, const float* in, bf16_t* out, int64_t n);
// rotary position encoding of the rows of in [batch][L][dq] (heads of width dh, half-split pairs); in == out allowed
hipError_t rope_rows(hipStream_t st, const void* in, void* out, int batch, int L, int dq, int dh, float base, int pos0,
                     int elem_bytes);

// rows×cols block of every batch item copied into another matrix (leading dimensions / batch strides in elements)
hipError_t copy_block(hipStream_t st, const void* in, void* out, int rows, int cols, int64_t ld_in, int64_t ld_out,
                      int64_t s_in, int64_t s_out, int batch, int elem_bytes);
// row-wise normalisation of a factored matrix H = P·C: coefficient side (Cc = C - row mean if center; Cn = Cc·diag(gain))
// and basis side (Pn[i] = P[i] / sqrt(p_i·M·p_iᵀ/d + eps), with PM = P·M, M = Cc·Ccᵀ, given in fp32)
hipError_t norm_coeff(hipStream_t st, const void* C, const float* gain, void* Cc, void* Cn, int64_t rows, int d, int center,
                      int elem_bytes);
hipError_t norm_basis(hipStream_t st, const void* P, const float* PM, void* Pn, int64_t rows, int m, int d, float eps,
                      int elem_bytes);

// ---------------------------------------------------------------------------
// r×r pieces of the CholeskyQR (fp32, batched)
// ---------------------------------------------------------------------------
// Sum `nparts` partial Gram matrices (stride `pstride` elements; only their lower 64×64-tile
// triangle is read), scale to unit diagonal (dinv_j = 1/sqrt(S_jj), 1 if S_jj is not positive and
// finite), add `shift` to the diagonal; also sets Y = I on its upper tile triangle and zeroes the
// part of Binv that factor_inverse leaves unwritten (all of its strict upper tile triangle when
// zero_all is set, else only inside the 256-wide diagonal blocks).
hipError_t gram_prepare(hipStream_t st, const float* Spart, int nparts, int64_t pstride, float* S, float* dinv,
                        float* Y, float* Binv, bf16_t* Bh, bf16_t* Bl, int r, float shift, int zero_all, int batch,
                        unsigned* flags = nullptr);
// Cholesky S = L·Lᵀ (S is overwritten with intermediate trailing blocks, L goes to Lf) and Binv[n][k] = (L^-1)[n][k]·dinv[k] (lower triangular).
// info[b] receives the first column (1-based) whose pivot is below `flag_below` (kept if already
// non-zero); pivots that are not positive are replaced by a tiny positive value: no NaN appears.
// Binv is written as fp32 (Binv) and/or as a hi/lo pair of bf16 planes (Bh, Bl); null = skip.
// `after` (may be null) is called on the host after the launch of every 64-wide block column j
// (0-based): rows 0 .. 64(j+1)-1 of Binv are final once that launch has run.
hipError_t factor_inverse(hipStream_t st, float* S, float* Lf, float* Y, const float* dinv, float* Binv, bf16_t* Bh,
                          bf16_t* Bl, int r, int32_t* info, float flag_below, int batch,
                          hipError_t (*after)(void* ctx, int j) = nullptr, void* ctx = nullptr);

// The same factorisation as ONE launch per group of items: co-resident workgroups keep their tiles in
// registers and hand finished panel tiles to each other through global memory and per-tile flags
// (`flags`: factor_dataflow_flag_bytes(batch) bytes, cleared by gram_prepare when passed there).
// Covers r <= 2048 when a group of workgroups fits the chip (factor_dataflow_ok); needs every
// workgroup of a launch resident at the same time, so it must not share the GPU with another such
// launch.  Lf and Y receive the panel tiles (scratch).  info = -1 if a wait inside the kernel gave up.
// factor_dataflow_ok: the shape is covered; with whole_batch, also that all items fit ONE launch (items
// beyond that run as further launches one after the other, which costs more than the launch-per-block-column
// factorisation, whose launches take all items at once).
bool factor_dataflow_ok(int r, int batch, bool whole_batch);
size_t factor_dataflow_flag_bytes(int batch);
// polls after which a wait inside the kernel gives up (< 1: the default, far beyond any healthy wait)
void factor_dataflow_set_spin_limit(int polls);
hipError_t factor_inverse_dataflow(hipStream_t st, float* S, float* Lf, float* Y, const float* dinv, float* Binv,
                                   bf16_t* Bh, bf16_t* Bl, unsigned* flags, int r, int32_t* info, float flag_below,
                                   int batch);

// ---------------------------------------------------------------------------
// attention over n_k keys (n_k = r principal keys, or L for the dense comparator)
// ---------------------------------------------------------------------------
struct AttnArgs {
    const void* Q = nullptr;   // [batch, L, dq]
    const void* K = nullptr;   // [batch, nk, dq]
    const void* V = nullptr;   // [batch, nk, dq]  (f32 path)
    const void* Vt = nullptr;  // [batch, dq, nk_pad] (bf16 path: per-head transposed values, zero padded)
    void* O = nullptr;         // [batch, L, dq]
    int batch = 1, L = 0, nk = 0, nk_pad = 0, dq = 0, heads = 1;
    float scale = 0.f;
    // first-order (linearised) variant, Eq.8: weights 1·U + scale·q·K'ᵀ instead of exp(·)
    int linearised = 0;
    const float* colsum = nullptr;  // [batch, nk_pad] column sums of U (1·U), zero padded
    int norm_rowsum = 0;            // 0: divide by n_tokens + scale·(q·K'ᵀ)·(1·U)ᵀ; 1: by the row sum of the map
    float n_tokens = 0.f;           // rows of U
};
hipError_t attention_bf16(hipStream_t st, const AttnArgs& a);  // d_h in {64,128}
hipError_t attention_f32(hipStream_t st, const AttnArgs& a);   // d_h <= 256
// out[b][j] = sum_i U[b][i][j] (fp32), j < r; out rows have length ld_out >= r, the rest is zeroed
hipError_t column_sums(hipStream_t st, const void* U, float* out, int L, int r, int64_t ld_out, int batch, int elem_bytes);

// ---------------------------------------------------------------------------
// alternating rank-1 extraction (Alg.1): d <= 4096, d % 4 == 0
// ---------------------------------------------------------------------------
size_t alternating_workspace(int batch, int L, int d);
hipError_t alternating_bases(hipStream_t st, const void* X, int batch, int L, int d, int r, int sweeps, const float* V0,
                             void* U, void* B, int32_t* info, void* workspace, int elem_bytes);

// ---------------------------------------------------------------------------
// Rayleigh–Ritz canonicalisation (cyclic Jacobi on T = B·Bᵀ) and diagnostics
// ---------------------------------------------------------------------------
hipError_t ritz_jacobi(hipStream_t st, float* T0, float* T1, float* R0, float* R1, int r, int batch, int sweeps,
                       float** T_final, float** R_final);
hipError_t ritz_order(hipStream_t st, const float* T, const float* R, const float* colsum, int64_t ld_cs, int* rank,
                      float* RsT, float* sigma, int* zero_sum, int r, int batch, float zero_tol);
hipError_t ritz_fallback_sign(hipStream_t st, void* U, void* B, const int* zero_sum, int L, int d, int r, int batch,
                              int elem_bytes);
hipError_t ritz_diagnostics(hipStream_t st, const float* T, const float* sigma, int r, int batch, float* diag);

}  // namespace atp
