// r×r pieces of the CholeskyQR orthonormalisation (fp32, batched over sequences).
// The orthonormal factor they lead to is the U of Eq.5 (UᵀU = I, text after Eq.8).
//
//  1. gram_prepare: sum the split-K partial Gram matrices, Jacobi-scale them to unit diagonal
//     (S' = D·S·D, D = diag(S)^-1/2), add the shift, and initialise the work matrices.
//  2. factor_inverse: blocked right-looking Cholesky of S' = L·Lᵀ carried out on the augmented
//     matrix [S'; I], which yields [L; L^-T] at once: the triangular inverse needs no second
//     sweep.  One launch per 64-wide block column j: the tiles of block column j first apply the
//     rank-64 update of panel j-1 and are then eliminated against the diagonal tile (recomputed
//     redundantly by each of them, so a launch has no internal dependencies).  The trailing tiles
//     are updated lazily: on odd j only block column j+1 (the next panel) is brought up to date, on
//     even j every trailing tile applies the two panels it lacks (j-2 and j-1) in one visit, which
//     halves the passes over the trailing matrix.  The inverse comes out as Binv[n][k] = (L^-1)[n][k]·D[k], the
//     B operand of the product Z·R^-1 that the GEMM kernel then applies to the tall matrix.
//  3. factor_inverse_dataflow: the same factorisation as ONE launch of co-resident workgroups that keep
//     their tiles in registers and hand finished panel tiles to each other through global memory (second
//     half of this file); the form used whenever the whole batch fits one launch.
#include "common.h"

#include <utility>

namespace atp {
namespace {

constexpr int NB = 64;  // block size of the factorisation

// development aid: with ATP_DF_TRACE defined (never in the library build) item 0 records time stamps
#ifdef ATP_DF_TRACE
__device__ long long g_df_trace[1024];
#define DF_STAMP(idx) do { if (blockIdx.y == 0 && threadIdx.x == 0) g_df_trace[idx] = wall_clock64(); } while (0)
#define DF_CYC(idx) do { if (blockIdx.y == 0 && blockIdx.x == 1 && threadIdx.x == 0) g_df_trace[idx] = __builtin_readcyclecounter(); } while (0)
#else
#define DF_STAMP(idx) do { } while (0)
#define DF_CYC(idx) do { } while (0)
#endif

// ---------------------------------------------------------------------------
// dinv[j] = 1/sqrt(sum_p Spart[p][j][j])   (1 if the diagonal entry is not positive and finite)
// Also clears the item's hand-over flags of the single-launch factorisation (flags may be null) and arms
// its exchange slots (wx: the first wx_fill_words words of every item's wx_stride_words are set to the
// "not written yet" pattern).
__global__ void diag_rsqrt_kernel(const float* __restrict__ Sp, int nparts, int64_t pstride, float* __restrict__ dinv,
                                  int r, unsigned* __restrict__ flags, int flag_words, uint4* __restrict__ wx,
                                  int wx_stride_words, int wx_fill_words) {
    const int b = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (flags) {
        for (int e = j; e < flag_words; e += gridDim.x * blockDim.x) flags[(int64_t)b * flag_words + e] = 0u;
        const uint4 unset = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
        for (int e = j; e < wx_fill_words / 4; e += gridDim.x * blockDim.x) wx[(int64_t)b * (wx_stride_words / 4) + e] = unset;
    }
    if (j >= r) return;
    float s = 0.f;
    for (int p = 0; p < nparts; ++p) s += Sp[(int64_t)p * pstride + (int64_t)b * r * r + (int64_t)j * r + j];
    const bool ok = (s > 0.f) && (s < 3.0e38f);
    dinv[(int64_t)b * r + j] = ok ? 1.0f / sqrtf(s) : 1.0f;
}

// Initialises the work matrices of one factorisation, touching only what the factorisation and the
// product Z·R^-1 read afterwards (64×64 tile granularity, ti = i/64, tj = j/64):
//   S'[i][j] = (sum_p Spart[p][i][j])·dinv[i]·dinv[j] (+ shift on the diagonal)   for tj <= ti
//              (the Gram kernel fills the lower 256×256 tiles of the partial sums only);
//   Y = I on the tiles with tj >= ti (the factorisation builds L^-T there);
//   Binv = 0 where the factorisation never writes but the product reads: tj > ti, and, unless
//   zero_all is set, only inside the 256-wide diagonal block (the MFMA product stops its K loop at
//   the end of the diagonal block of a triangular operand).
__global__ void prepare_kernel(const float* __restrict__ Sp, int nparts, int64_t pstride, float* __restrict__ S,
                               const float* __restrict__ dinv, float* __restrict__ Y, float* __restrict__ Binv,
                               bf16_t* __restrict__ Bh, bf16_t* __restrict__ Bl, int r, float shift, int zero_all) {
    const int b = blockIdx.z;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int i = blockIdx.y;
    if (j >= r) return;
    const int ti = i >> 6, tj = j >> 6;
    const int64_t o = (int64_t)b * r * r + (int64_t)i * r + j;
    if (tj <= ti) {
        float s = 0.f;
        for (int p = 0; p < nparts; ++p) s += Sp[(int64_t)p * pstride + o];
        const float* db = dinv + (int64_t)b * r;
        const float v = s * db[i] * db[j];
        S[o] = (i == j) ? v + shift : v;
    }
    if (tj >= ti) Y[o] = (i == j) ? 1.f : 0.f;
    if (tj > ti && (zero_all || (i >> 8) == (j >> 8))) {
        if (Binv) Binv[o] = 0.f;
        if (Bh) { Bh[o] = 0; Bl[o] = 0; }
    }
}

// Same for r a multiple of 4: a thread handles four consecutive columns (they lie in one 64-wide tile)
// with 16-byte accesses.
__global__ void prepare4_kernel(const float* __restrict__ Sp, int nparts, int64_t pstride, float* __restrict__ S,
                                const float* __restrict__ dinv, float* __restrict__ Y, float* __restrict__ Binv,
                                bf16_t* __restrict__ Bh, bf16_t* __restrict__ Bl, int r, float shift, int zero_all) {
    const int b = blockIdx.z;
    const int j = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    const int i = blockIdx.y;
    if (j >= r) return;
    const int ti = i >> 6, tj = j >> 6;
    const int64_t o = (int64_t)b * r * r + (int64_t)i * r + j;
    if (tj <= ti) {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < nparts; ++p) s += *reinterpret_cast<const f32x4*>(Sp + (int64_t)p * pstride + o);
        const float* db = dinv + (int64_t)b * r;
        const float di = db[i];
        const f32x4 dj = *reinterpret_cast<const f32x4*>(db + j);
        f32x4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[q] = s[q] * di * dj[q];
            if (i == j + q) v[q] += shift;
        }
        *reinterpret_cast<f32x4*>(S + o) = v;
    }
    if (tj >= ti) {
        f32x4 e;
#pragma unroll
        for (int q = 0; q < 4; ++q) e[q] = (i == j + q) ? 1.f : 0.f;
        *reinterpret_cast<f32x4*>(Y + o) = e;
    }
    if (tj > ti && (zero_all || (i >> 8) == (j >> 8))) {
        if (Binv) *reinterpret_cast<f32x4*>(Binv + o) = f32x4{0.f, 0.f, 0.f, 0.f};
        if (Bh) {
            *reinterpret_cast<uint2*>(Bh + o) = make_uint2(0u, 0u);
            *reinterpret_cast<uint2*>(Bl + o) = make_uint2(0u, 0u);
        }
    }
}

// Joint right-looking elimination of the two 64×64 tiles, four columns per step (the block index
// is a compile-time constant so that the half tile row each thread keeps in registers is indexed
// statically).   reg[t] = T_sel[a][2t + half].
//   exchange 1: the raw values of the 4 block columns of every row (both tiles);
//   every thread then factors the 4×4 pivot block redundantly and reduces its own row:
//     x_k = current value of T[a][4B+k] after columns 4B .. 4B+k-1 are eliminated, f_k = x_k / piv_k;
//   exchange 2: the x_k of the diagonal tile's rows;
//   trailing columns cc > 4B+3:  T[a][cc] -= sum_k f_k(a) · x_k(cc).
// Columns stay unscaled until they are final (L[a][c] = x_c(a) / sqrt(piv_c)).
// A pivot at or below PIVOT_DROP (the scaled Gram matrix has unit diagonal; rounding noise of its entries is
// ~1e-5) means the column has no energy left beyond noise: the column is dropped (its multipliers and its
// column of L / row of L^-1 are zero) instead of being divided by, so nothing can grow without bound and
// every output stays finite.  Such a pivot is always below the level that sets `info`.
constexpr float PIVOT_DROP = 1e-6f;
__device__ __forceinline__ float drop_rcp(float piv) { return piv > PIVOT_DROP ? __builtin_amdgcn_rcpf(piv) : 0.f; }
__device__ __forceinline__ float drop_rsq(float piv) { return piv > PIVOT_DROP ? __builtin_amdgcn_rsqf(piv) : 0.f; }

struct ElimLds {
    float4 raw[2][2][NB];  // [buffer][tile][row]
    float4 xs[2][NB];      // [buffer][row of the diagonal tile]
};

template <int B>
__device__ __forceinline__ void elim_block(float (&reg)[32], ElimLds& L, int sel, int half, int a, float flag_below,
                                           int& bad_col) {
    constexpr int buf = B & 1;
    {
        float* w = reinterpret_cast<float*>(&L.raw[buf][sel][a]);
        w[half] = reg[2 * B];
        w[half + 2] = reg[2 * B + 1];
    }
    __syncthreads();
    const float4 p0 = L.raw[buf][0][4 * B + 0], p1 = L.raw[buf][0][4 * B + 1];
    const float4 p2 = L.raw[buf][0][4 * B + 2], p3 = L.raw[buf][0][4 * B + 3];
    const float4 R = L.raw[buf][sel][a];
    // pivot block: xp[i][k] = x_k of pivot row i (lower triangle), piv_k = xp[k][k]
    const float piv0r = p0.x;
    const float i0 = drop_rcp(piv0r);
    const float x10 = p1.x, x20 = p2.x, x30 = p3.x;
    const float piv1r = fmaf(-x10 * i0, x10, p1.y);
    const float i1 = drop_rcp(piv1r);
    const float x21 = fmaf(-x20 * i0, x10, p2.y);
    const float x31 = fmaf(-x30 * i0, x10, p3.y);
    const float piv2r = fmaf(-x21 * i1, x21, fmaf(-x20 * i0, x20, p2.z));
    const float i2 = drop_rcp(piv2r);
    const float x32 = fmaf(-x31 * i1, x21, fmaf(-x30 * i0, x20, p3.z));
    const float piv3r = fmaf(-x32 * i2, x32, fmaf(-x31 * i1, x31, fmaf(-x30 * i0, x30, p3.w)));
    const float i3 = drop_rcp(piv3r);
    if (bad_col < 0) {
        if (!(piv0r >= flag_below)) bad_col = 4 * B;
        else if (!(piv1r >= flag_below)) bad_col = 4 * B + 1;
        else if (!(piv2r >= flag_below)) bad_col = 4 * B + 2;
        else if (!(piv3r >= flag_below)) bad_col = 4 * B + 3;
    }
    // own row
    const float x0 = R.x, f0 = x0 * i0;
    const float x1 = fmaf(-f0, x10, R.y), f1 = x1 * i1;
    const float x2 = fmaf(-f1, x21, fmaf(-f0, x20, R.z)), f2 = x2 * i2;
    const float x3 = fmaf(-f2, x32, fmaf(-f1, x31, fmaf(-f0, x30, R.w))), f3 = x3 * i3;
    if (sel == 0 && half == 0) L.xs[buf][a] = make_float4(x0, x1, x2, x3);
    // final (scaled) values of the block columns owned by this thread
    reg[2 * B] = (half ? x1 * drop_rsq(piv1r) : x0 * drop_rsq(piv0r));
    reg[2 * B + 1] = (half ? x3 * drop_rsq(piv3r) : x2 * drop_rsq(piv2r));
    __syncthreads();
#pragma unroll
    for (int t = 2 * B + 2; t < 32; ++t) {
        const float4 d = L.xs[buf][2 * t + half];
        reg[t] = fmaf(-f3, d.w, fmaf(-f2, d.z, fmaf(-f1, d.y, fmaf(-f0, d.x, reg[t]))));
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the steps apart: no hoarding of values in registers
}


// ---------------------------------------------------------------------------
// W = L^-T of one 64×64 symmetric positive definite tile T = L·Lᵀ, for the single-launch
// factorisation (L itself is not needed there).  Same elimination of [T; I], four columns per step,
// arranged for latency:
//  * a thread is (row a, wave w); wave w owns the 4-column blocks B with B % 4 == w (16 registers);
//  * row a of T is dead once block a/4 has been eliminated, and row a of the identity part is born in
//    that step: the same registers hold the T row first and the row of W afterwards, so every thread has
//    exactly one live row per step and the trailing update is half as long;
//  * the raw values of the next block are written by their owner wave right after it has updated them,
//    ahead of the rest of its trailing update.
// T comes in as LDS tile `Tt` (pitch NB+1); W leaves in `Wt` (upper triangular, zeros below).
// ---------------------------------------------------------------------------
struct Elim2Lds {
    float4 raw[2][NB];  // [buffer][row]: the four block columns of the row each thread currently holds
    float4 xs[2][NB];   // [buffer][row of T]: reduced values of the rows below the pivot block
};

// one owned block (local index M) of the trailing update of step B
template <int B, int M>
__device__ __forceinline__ void elim2_update(float (&reg)[16], Elim2Lds& L, int a, int w, bool pivrow, float f0, float f1,
                                             float f2, float f3) {
    constexpr int buf = B & 1;
    const int c0 = 4 * (4 * M + w);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float4 d = L.xs[buf][c0 + j];
        const float base = pivrow ? 0.f : reg[4 * M + j];    // a newborn identity row starts from zero
        reg[4 * M + j] = fmaf(-f3, d.w, fmaf(-f2, d.z, fmaf(-f1, d.y, fmaf(-f0, d.x, base))));
    }
    if (4 * M + w == B + 1) L.raw[buf ^ 1][a] = make_float4(reg[4 * M], reg[4 * M + 1], reg[4 * M + 2], reg[4 * M + 3]);
}

__device__ __forceinline__ void df_st16(float* p, f32x4 v);

// `slot` (may be null): exchange slot of W, four groups of 16 columns, group q at slot + 1024·q as [row][16].
// The four blocks of a group are final after step 4q+3, one in each wave: every thread sends its 16 bytes
// then, so the workgroup that consumes W works through it behind this elimination, group by group.
// `publish` (may be null): a hand-over flag whose tile stores were issued before the elimination began; they
// have completed by the second step: every wave confirms that there (a wait that costs nothing by then),
// and after that step's barrier one thread raises the flag, so the caller need not stall for its stores.
template <int B>
__device__ __forceinline__ void elim2_block(float (&reg)[16], Elim2Lds& L, int a, int w, float flag_below, int& bad_col,
                                            float* slot, unsigned* publish) {
    constexpr int buf = B & 1;
    constexpr int mB = B / 4, wB = B % 4;
    if constexpr (B == 1) {
        if (publish) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();   // raw[buf] of block B is complete (written during the previous step)
    if constexpr (B == 1) {
        if (publish && a == 0 && w == 0) __hip_atomic_store(publish, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const float4 p0 = L.raw[buf][4 * B + 0], p1 = L.raw[buf][4 * B + 1];
    const float4 p2 = L.raw[buf][4 * B + 2], p3 = L.raw[buf][4 * B + 3];
    float4 R = L.raw[buf][a];
    const int ja = a - 4 * B;                 // 0..3: this thread's row is a pivot row and turns into its identity row
    const bool pivrow = (ja >= 0 && ja < 4);
    if (pivrow) R = make_float4(ja == 0 ? 1.f : 0.f, ja == 1 ? 1.f : 0.f, ja == 2 ? 1.f : 0.f, ja == 3 ? 1.f : 0.f);
    const float piv0r = p0.x;
    const float i0 = drop_rcp(piv0r);
    const float x10 = p1.x, x20 = p2.x, x30 = p3.x;
    const float g10 = x10 * i0, g20 = x20 * i0, g30 = x30 * i0;
    const float piv1r = fmaf(-g10, x10, p1.y);
    const float i1 = drop_rcp(piv1r);
    const float x21 = fmaf(-g20, x10, p2.y);
    const float x31 = fmaf(-g30, x10, p3.y);
    const float g21 = x21 * i1, g31 = x31 * i1;
    const float piv2r = fmaf(-g21, x21, fmaf(-g20, x20, p2.z));
    const float i2 = drop_rcp(piv2r);
    const float x32 = fmaf(-g31, x21, fmaf(-g30, x20, p3.z));
    const float piv3r = fmaf(-x32 * i2, x32, fmaf(-g31, x31, fmaf(-g30, x30, p3.w)));
    const float i3 = drop_rcp(piv3r);
    const float x0 = R.x, f0 = x0 * i0;
    const float x1 = fmaf(-f0, x10, R.y), f1 = x1 * i1;
    const float x2 = fmaf(-f1, x21, fmaf(-f0, x20, R.z)), f2 = x2 * i2;
    const float x3 = fmaf(-f2, x32, fmaf(-f1, x31, fmaf(-f0, x30, R.w))), f3 = x3 * i3;
    // xs[row] is read only by the wave that owns the block column `row` lies in (the trailing update of wave w
    // reads xs of the rows 4·blk .. 4·blk+3 of its own blocks blk): written by that same wave, it needs no block
    // barrier; a wave's LDS accesses complete in order
    if (w == ((a >> 2) & 3) && a >= 4 * B + 4) L.xs[buf][a] = make_float4(x0, x1, x2, x3);
    if (bad_col < 0 && !(fminf(fminf(piv0r, piv1r), fminf(piv2r, piv3r)) >= flag_below)) {
        if (!(piv0r >= flag_below)) bad_col = 4 * B;
        else if (!(piv1r >= flag_below)) bad_col = 4 * B + 1;
        else if (!(piv2r >= flag_below)) bad_col = 4 * B + 2;
        else bad_col = 4 * B + 3;
    }
    if (w == wB) {   // final values of block B of the live row (rows of W; rows of L are not kept)
        reg[4 * mB + 0] = x0 * drop_rsq(piv0r);
        reg[4 * mB + 1] = x1 * drop_rsq(piv1r);
        reg[4 * mB + 2] = x2 * drop_rsq(piv2r);
        reg[4 * mB + 3] = x3 * drop_rsq(piv3r);
    }
    // pending blocks of wave w: local block mB only for the waves behind the owner of block B, the later
    // ones for every wave; block B + 1 comes first in this order and its raw values are written at once
    if (w > wB) elim2_update<B, mB>(reg, L, a, w, pivrow, f0, f1, f2, f3);
    if constexpr (mB + 1 < 4) elim2_update<B, (mB + 1 < 4 ? mB + 1 : 3)>(reg, L, a, w, pivrow, f0, f1, f2, f3);
    if constexpr (mB + 2 < 4) elim2_update<B, (mB + 2 < 4 ? mB + 2 : 3)>(reg, L, a, w, pivrow, f0, f1, f2, f3);
    if constexpr (mB + 3 < 4) elim2_update<B, (mB + 3 < 4 ? mB + 3 : 3)>(reg, L, a, w, pivrow, f0, f1, f2, f3);
    if constexpr (wB == 3) {
        if (slot) {   // blocks 4·mB .. 4·mB+3 are final in waves 0..3; a row below its block is still a dead T row there
            const bool dead = 4 * mB + w < (a >> 2);
            const f32x4 v = {dead ? 0.f : reg[4 * mB], dead ? 0.f : reg[4 * mB + 1], dead ? 0.f : reg[4 * mB + 2],
                             dead ? 0.f : reg[4 * mB + 3]};
            df_st16(slot + 1024 * mB + 16 * a + 4 * w, v);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int... Bs>
__device__ __forceinline__ void elim2_all(std::integer_sequence<int, Bs...>, float (&reg)[16], Elim2Lds& L, int a, int w,
                                          float flag_below, int& bad_col, float* slot, unsigned* publish) {
    (elim2_block<Bs>(reg, L, a, w, flag_below, bad_col, slot, publish), ...);
}

// all 256 threads; Tt and Wt may not alias; ends with a block barrier
__device__ __forceinline__ void diag_inverse_factor(const float (*Tt)[NB + 1], float (*Wt)[NB + 1], Elim2Lds& L, int tid,
                                                    float flag_below, int& bad_col, float* slot = nullptr,
                                                    unsigned* publish = nullptr) {
    const int a = tid & 63, w = tid >> 6;
    float reg[16];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j) reg[4 * m + j] = Tt[a][4 * (4 * m + w) + j];
    if (w == 0) L.raw[0][a] = make_float4(reg[0], reg[1], reg[2], reg[3]);
    elim2_all(std::make_integer_sequence<int, NB / 4>{}, reg, L, a, w, flag_below, bad_col, slot, publish);
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = 4 * (4 * m + w) + j;
            Wt[a][c] = (4 * m + w < (a >> 2)) ? 0.f : reg[4 * m + j];   // blocks left of the diagonal still hold the dead T row
        }
    __syncthreads();
}

template <int... Bs>
__device__ __forceinline__ void elim_all(std::integer_sequence<int, Bs...>, float (&reg)[32], ElimLds& L, int sel,
                                         int half, int a, float flag_below, int& bad_col) {
    (elim_block<Bs>(reg, L, sel, half, a, flag_below, bad_col), ...);
}

// ---------------------------------------------------------------------------
// One block column of the augmented factorisation (see the header of this file).
// Tile kinds handled by a workgroup (tile = 64×64, k = its block column):
//   S-kind (i, k), i >= k >= j : tile of S'; panel operand A = L(i, j-1)
//   Y-kind (c, k), c <= k, k >= j : tile of Y (= L^-T when final); panel operand A = Y(c, j-1)
// update (j >= 1, not for the fresh identity tile Y(j, j)):  T -= A · L(k, j-1)ᵀ
// k > j : store T back.   k == j : eliminate the 64 columns of T together with the diagonal
// tile Tjj = S'(j, j) - L(j, j-1)·L(j, j-1)ᵀ and store the result as L(i, j) / Y(c, j) + Binv.
// ---------------------------------------------------------------------------
constexpr int LP = NB + 4;  // padded row length of the MFMA operand tiles (16-byte aligned rows)

// 64×64 tile -> LDS (row-major, padded), optionally negated; rows/cols past r read as zero
__device__ __forceinline__ void tile_to_lds(float (*dst)[LP], const float* __restrict__ src, int r, int row0, int col0,
                                            float sign, bool enable, int tid) {
    const bool vec = ((r & 3) == 0);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = (tid >> 4) + 16 * q, c4 = (tid & 15) * 4;
        const int gr = row0 + row, gc = col0 + c4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (enable && gr < r) {
            const float* ptr = src + (int64_t)gr * r + gc;
            if (vec && gc + 3 < r) {
                v = *reinterpret_cast<const float4*>(ptr);
            } else {
                if (gc + 0 < r) v.x = ptr[0];
                if (gc + 1 < r) v.y = ptr[1];
                if (gc + 2 < r) v.z = ptr[2];
                if (gc + 3 < r) v.w = ptr[3];
            }
        }
        *reinterpret_cast<float4*>(&dst[row][c4]) = make_float4(sign * v.x, sign * v.y, sign * v.z, sign * v.w);
    }
}

__global__ void __launch_bounds__(256, 2) factor_step_kernel(float* S, float* Lf, float* Y, const float* __restrict__ dinv,
                                                             float* Binv, bf16_t* Bh, bf16_t* Bl, int r, int nblk, int j,
                                                             int32_t* info, float flag_below) {
    // MFMA operands (-A and L(k, j-1), row-major) during the update; the tiles T and Tjj afterwards
    __shared__ __align__(16) float lds_a[NB * LP];
    __shared__ __align__(16) float lds_b[NB * LP];
    __shared__ __align__(16) ElimLds elds;
    float (*Am)[LP] = reinterpret_cast<float (*)[LP]>(lds_a);
    float (*Bm)[LP] = reinterpret_cast<float (*)[LP]>(lds_b);
    float (*As)[NB + 1] = reinterpret_cast<float (*)[NB + 1]>(lds_a);
    float (*Bs)[NB + 1] = reinterpret_cast<float (*)[NB + 1]>(lds_b);

    const int b = blockIdx.y;
    const int m = nblk - j;
    int id = blockIdx.x;
    // ---- decode the tile ----------------------------------------------------------------------
    bool ykind, panel;
    int rb, kb;  // row block (i or c) and column block k
    if (id < m) { ykind = false; panel = true; rb = j + id; kb = j; }
    else if (id < m + j + 1) { ykind = true; panel = true; rb = id - m; kb = j; }
    else if (j & 1) {
        // odd block column: only the tiles of the next block column are brought up to date
        id -= m + j + 1;
        panel = false;
        kb = j + 1;
        if (id < m - 1) { ykind = false; rb = j + 1 + id; }
        else { ykind = true; rb = id - (m - 1); }   // c in 0..j-1
    } else {
        id -= m + j + 1;
        panel = false;
        const int nt1 = m * (m - 1) / 2;  // S-kind trailing tiles (i, k), j < k <= i
        if (id < nt1) {
            ykind = false;
            // row-wise enumeration of the triangle: rows ii = 0..m-2 (i = j+1+ii) hold ii+1 tiles
            int ii = (int)((sqrtf(8.f * id + 1.f) - 1.f) * 0.5f);
            while ((ii + 1) * (ii + 2) / 2 <= id) ++ii;
            while (ii * (ii + 1) / 2 > id) --ii;
            rb = j + 1 + ii;
            kb = j + 1 + (id - ii * (ii + 1) / 2);
        } else {
            id -= nt1;
            ykind = true;
            rb = id / (m - 1);            // c in 0..j-1
            kb = j + 1 + id % (m - 1);
        }
    }
    const int64_t boff = (int64_t)b * r * r;
    float* Sb = S + boff;
    float* Lb = Lf + boff;
    float* Yb = Y + boff;
    float* own = ykind ? Yb : Sb;
    const int r0 = rb * NB, c0 = kb * NB;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wr = wave >> 1, wc = wave & 1;   // 32×32 quadrant of the tile owned by this wave

    // Tiles of block column j (and j+1 on odd j) lack panel j-1 only; the other trailing tiles are
    // visited on even j only and lack panels j-2 and j-1.
    const int npanels = (j == 0) ? 0 : ((panel || (j & 1)) ? 1 : 2);
    auto stage_panel = [&](int q) {
        const int pb = j - npanels + q;            // panel block column
        const bool update = !(ykind && rb > pb);   // row rb of Y is still the identity row before block column rb
        tile_to_lds(Am, ykind ? Yb : Lb, r, r0, pb * NB, -1.f, update, tid);
        tile_to_lds(Bm, Lb, r, c0, pb * NB, 1.f, true, tid);
    };
    // the operands of the first pending update are requested first: they are needed first
    if (npanels) stage_panel(0);
    // ---- accumulators start from the own tile (and the diagonal tile) in MFMA C layout ---------------
    // C layout: element v of lane -> row 8*(v/4) + 4*lh + v%4, column l32 (within the quadrant);
    // out-of-range entries pad with the identity
    f32x16 acc, accj;
    {
        const int gc = c0 + 32 * wc + l32;
        const int rq = 32 * wr + 4 * lh;   // first row of this lane within the tile
        if (r0 + NB <= r && c0 + NB <= r) {
            // tile completely inside the matrix (the diagonal tile then is too): plain strided loads
            const float* po = own + (int64_t)(r0 + rq) * r + gc;
            const float* pj = Sb + (int64_t)(c0 + rq) * r + gc;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t o = (int64_t)(8 * (v >> 2) + (v & 3)) * r;
                acc[v] = po[o];
                accj[v] = panel ? pj[o] : 0.f;
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rq + 8 * (v >> 2) + (v & 3);
                const int gr = r0 + row, gj = c0 + row;
                acc[v] = (gr < r && gc < r) ? own[(int64_t)gr * r + gc] : ((gr == gc) ? 1.f : 0.f);
                accj[v] = 0.f;
                if (panel) accj[v] = (gj < r && gc < r) ? Sb[(int64_t)gj * r + gc] : ((gj == gc) ? 1.f : 0.f);
            }
        }
    }
    // ---- pending rank-64 updates on the matrix cores (fp32 MFMA): T -= A(·, p) · L(k, p)ᵀ ------------
    for (int q = 0; q < npanels; ++q) {
        if (q > 0) {
            __syncthreads();
            stage_panel(q);
        }
        __syncthreads();
#pragma unroll
        for (int g = 0; g < NB / 8; ++g) {
            // lanes of half lh take k = 8g + 4*lh .. +3: one 16-byte read per operand feeds 4 MFMAs
            const float4 a4 = *reinterpret_cast<const float4*>(&Am[32 * wr + l32][8 * g + 4 * lh]);
            const float4 b4 = *reinterpret_cast<const float4*>(&Bm[32 * wc + l32][8 * g + 4 * lh]);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, b4.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, b4.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, b4.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, b4.w, acc, 0, 0, 0);
            if (panel) {
                const float4 c4 = *reinterpret_cast<const float4*>(&Bm[32 * wr + l32][8 * g + 4 * lh]);
                accj = __builtin_amdgcn_mfma_f32_32x32x2f32(-c4.x, b4.x, accj, 0, 0, 0);
                accj = __builtin_amdgcn_mfma_f32_32x32x2f32(-c4.y, b4.y, accj, 0, 0, 0);
                accj = __builtin_amdgcn_mfma_f32_32x32x2f32(-c4.z, b4.z, accj, 0, 0, 0);
                accj = __builtin_amdgcn_mfma_f32_32x32x2f32(-c4.w, b4.w, accj, 0, 0, 0);
            }
        }
    }
    if (npanels) __syncthreads();
    if (!panel) {
        const int gc = c0 + 32 * wc + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int gr = r0 + 32 * wr + 8 * (v >> 2) + 4 * lh + (v & 3);
            if (gr < r && gc < r) own[(int64_t)gr * r + gc] = acc[v];
        }
        return;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = 32 * wr + 8 * (v >> 2) + 4 * lh + (v & 3), col = 32 * wc + l32;
        As[row][col] = acc[v];
        Bs[row][col] = accj[v];
    }
    __syncthreads();

    // ---- joint elimination of the 64 columns; every thread keeps half a tile row in registers --
    const int sel = tid >> 7;         // 0: diagonal tile, 1: own tile
    const int a = tid & 63;           // row
    const int half = (tid >> 6) & 1;  // column parity owned (uniform per wave)
    float reg[32];
#pragma unroll
    for (int t = 0; t < 32; ++t) reg[t] = sel ? As[a][2 * t + half] : Bs[a][2 * t + half];
    int bad_col = -1;                          // first column whose pivot is below the flag level
    elim_all(std::make_integer_sequence<int, NB / 4>{}, reg, elds, sel, half, a, flag_below, bad_col);
    if (!ykind && rb == j && tid == 0 && info && bad_col >= 0 && (c0 + bad_col) < r && info[b] == 0)
        info[b] = c0 + bad_col + 1;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 32; ++t) {
        if (sel) As[a][2 * t + half] = reg[t];
        else Bs[a][2 * t + half] = reg[t];
    }
    __syncthreads();
    // ---- store ---------------------------------------------------------------------------------------
    if (!ykind) {
        const bool diag = (rb == j);
        if ((r & 3) == 0) {   // 16-byte row pieces
            for (int e = tid; e < NB * NB / 4; e += 256) {
                const int row = e >> 4, col = (e & 15) * 4;
                const int gr = r0 + row, gc = c0 + col;
                if (gr < r && gc < r) {
                    f32x4 v;
#pragma unroll
                    for (int q = 0; q < 4; ++q) v[q] = diag ? ((row >= col + q) ? Bs[row][col + q] : 0.f) : As[row][col + q];
                    *reinterpret_cast<f32x4*>(Lb + (int64_t)gr * r + gc) = v;
                }
            }
        } else {
            for (int e = tid; e < NB * NB; e += 256) {
                const int row = e >> 6, col = e & 63;
                const int gr = r0 + row, gc = c0 + col;
                if (gr < r && gc < r) {
                    float v = diag ? ((row >= col) ? Bs[row][col] : 0.f) : As[row][col];
                    Lb[(int64_t)gr * r + gc] = v;
                }
            }
        }
    } else {
        const float* db = dinv + (int64_t)b * r;
        if ((r & 3) == 0) {
            for (int e = tid; e < NB * NB / 4; e += 256) {
                const int row = e >> 4, col = (e & 15) * 4;
                const int gr = r0 + row, gc = c0 + col;
                if (gr < r && gc < r) {
                    f32x4 v;
#pragma unroll
                    for (int q = 0; q < 4; ++q) v[q] = As[row][col + q];
                    *reinterpret_cast<f32x4*>(Yb + (int64_t)gr * r + gc) = v;
                }
            }
        } else {
            for (int e = tid; e < NB * NB; e += 256) {
                const int row = e >> 6, col = e & 63;
                const int gr = r0 + row, gc = c0 + col;
                if (gr < r && gc < r) Yb[(int64_t)gr * r + gc] = As[row][col];
            }
        }
        if (Bh && !Binv && (r & 7) == 0) {
            // hi/lo planes of R^-1 (transposed tile): 8 consecutive rows of one column are 8 consecutive
            // bf16 of a Binv row: one 16-byte store per plane
            for (int e = tid; e < NB * NB / 8; e += 256) {
                const int col = e >> 3, row8 = (e & 7) * 8;
                const int gr = r0 + row8, gc = c0 + col;
                if (gr < r && gc < r) {   // r is a multiple of 8: the 8 rows are in range together
                    float v[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) v[q] = As[row8 + q][col] * db[gr + q];
                    uint4 h, l;
                    uint32_t* hp = reinterpret_cast<uint32_t*>(&h);
                    uint32_t* lp = reinterpret_cast<uint32_t*>(&l);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t hh = pack_bf2(v[2 * q], v[2 * q + 1]);
                        hp[q] = hh;
                        lp[q] = pack_bf2(v[2 * q] - bf2f((bf16_t)(hh & 0xffffu)), v[2 * q + 1] - bf2f((bf16_t)(hh >> 16)));
                    }
                    const int64_t o = boff + (int64_t)gc * r + gr;
                    *reinterpret_cast<uint4*>(Bh + o) = h;
                    *reinterpret_cast<uint4*>(Bl + o) = l;
                }
            }
        } else {
            for (int e = tid; e < NB * NB; e += 256) {
                const int col = e >> 6, row = e & 63;   // row fastest: consecutive addresses in Binv
                const int gr = r0 + row, gc = c0 + col;
                if (gr < r && gc < r) {
                    const float v = As[row][col] * db[gr];
                    const int64_t o = boff + (int64_t)gc * r + gr;
                    if (Binv) Binv[o] = v;
                    if (Bh) {
                        const bf16_t h = f2bf(v);
                        Bh[o] = h;
                        Bl[o] = f2bf(v - bf2f(h));
                    }
                }
            }
        }
    }
}


// ---------------------------------------------------------------------------
// Single-launch factorisation: the same augmented block factorisation as above, carried out by one
// grid of co-resident workgroups that hand tiles to each other through global memory and per-tile
// flags instead of kernel boundaries.  Every 64×64 tile lives in the accumulator registers of the
// workgroup that owns it for the whole factorisation; only finished panel tiles travel.
//
// Stacked tile rows: S-rows i (tiles S'(i,k), k <= i) and Y-rows c (tiles Y(c,k), k >= c, Y = L^-T).
//   T(rho,k) = init - sum_{p<k} P(rho,p)·L(k,p)ᵀ ,   P(rho,k) = T(rho,k)·W_k ,   W_k = L_kk^-T
// (init = S'(i,k) for S-rows, 0 for Y-rows; the sum starts at p = c for Y-row c with P(c,c) = W_c).
// Roles inside one item's group of workgroups:
//   spine workgroup i (one per block row) owns S'(i,i-1) and S'(i,i): applies the panels p <= i-2 as
//     they appear, then, once W_{i-1} is published, forms L(i,i-1), the Schur complement of the diagonal
//     tile, factorises it together with an identity tile (which yields W_i) and publishes W_i;
//   bulk workgroups own the remaining tiles, dealt round-robin in order of block column so that a
//     workgroup's slots are sorted by urgency.  Step q: finalise the slots of block column q (product
//     with W_q), publish them, then apply panel q to every later slot.
// Every workgroup walks the steps in the same global order (step, block column), so the oldest
// unfinished task is always at the head of its owner's queue: no cycle of waits, provided the whole
// grid is resident (the host bounds the grid by the number of compute units).  Waits are bounded: a
// workgroup that spins too long raises the item's abort word, sets info = -1 and exits; every other
// wait of that item then ends as well.
// ---------------------------------------------------------------------------
constexpr int DF_SPIN_LIMIT = 1 << 22;   // polls of ~0.1-0.3 µs each: well beyond any healthy wait
constexpr int DF_MAX_NBLK = 32;
constexpr int DF_FLAG_WORDS = 2 * DF_MAX_NBLK * DF_MAX_NBLK + 64;   // per item; the last 64 words hold the abort word
// Exchange slots: W_i travels from spine workgroup i to spine workgroup i+1, the one hand-over on the
// critical path of the factorisation, without a flag and in four pieces.  The slot (a dense 64×64 tile per
// block row, stored as four groups of 16 columns) is armed with a bit pattern no finite number has (all ones:
// a NaN) before the launch; the producer stores a group as soon as its columns are final (columns of
// W = L^-T become final from left to right as the elimination proceeds), the consumer loads a group until
// none of its words shows the pattern any more and at once forms the matching 16 columns of
// L(i+1,i) = T(i+1,i)·W_i and their share of the update of its diagonal tile.  When the last group arrives
// only a quarter of that work is left.  A torn or partly arrived group only looks unfinished.
constexpr unsigned DF_UNSET = 0xFFFFFFFFu;
constexpr int DF_SLOT_WORDS = NB * NB;
constexpr int DF_WX_WORDS = DF_MAX_NBLK * DF_SLOT_WORDS;            // per item

struct DfArgs {
    float* S; float* Lf; float* Y; const float* dinv;
    float* Binv; bf16_t* Bh; bf16_t* Bl;
    unsigned* flags;
    float* wx;              // exchange slots, DF_WX_WORDS per item
    int32_t* info;
    int r, nblk, item0, nbulk;
    int spin_limit;         // polls before a wait gives up
    float flag_below;
};


// Panel tiles travel between workgroups of one running kernel, possibly on different XCDs (each has
// an L2 of its own).  They are written and read with agent-scope ("sc1") accesses, which are coherent
// across the device by themselves: no cache-wide write-back or invalidate is needed, and ordering is
// plain completion order (s_waitcnt before the flag is raised; the flag is polled with relaxed loads).
// The loads are issued through inline assembly, both tiles of an update in flight before one wait.
// eight 16-byte loads in flight, then one wait, in ONE statement: the compiler never sees a register
// whose load is still outstanding
__device__ __forceinline__ void df_ld16x8(const float* const (&p)[8], f32x4 (&v)[8]) {
    asm volatile(
        "global_load_dwordx4 %0, %8, off sc1\n\t"
        "global_load_dwordx4 %1, %9, off sc1\n\t"
        "global_load_dwordx4 %2, %10, off sc1\n\t"
        "global_load_dwordx4 %3, %11, off sc1\n\t"
        "global_load_dwordx4 %4, %12, off sc1\n\t"
        "global_load_dwordx4 %5, %13, off sc1\n\t"
        "global_load_dwordx4 %6, %14, off sc1\n\t"
        "global_load_dwordx4 %7, %15, off sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
        : "v"(p[0]), "v"(p[1]), "v"(p[2]), "v"(p[3]), "v"(p[4]), "v"(p[5]), "v"(p[6]), "v"(p[7])
        : "memory");
}
// A store of more than 8 bytes reads its data registers for two more cycles after it has issued; the
// compiler pads its own stores but cannot see into this statement, so the padding is part of it (without it
// the next instruction may overwrite the data registers: seen as an LDS address stored in place of a value).
__device__ __forceinline__ void df_st16(float* p, f32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void df_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

constexpr int WCP = 20;   // row pitch of a 64×16 column group of W in LDS (16-byte aligned rows, the four k-slices of a read fall into different banks)

__device__ __forceinline__ bool df_written(const f32x4& v) {
    return __float_as_uint(v[0]) != DF_UNSET && __float_as_uint(v[1]) != DF_UNSET && __float_as_uint(v[2]) != DF_UNSET &&
           __float_as_uint(v[3]) != DF_UNSET;
}

// Whole workgroup: load one 64×16 group of an exchange slot until every word of it has been written, then leave
// it in `dst`.  false = gave up (spin limit or the item's abort word).  Ends with a block barrier.
// (Taking every group that is complete at the time of a poll, four loads and a reduction per group, measured
// slower: 225 against 204 µs per factorisation; the plain poll reacts faster.)
__device__ __forceinline__ bool df_poll_group(float (*dst)[WCP], const float* group, unsigned* abort_w, int spin_limit,
                                              int tid) {
    const float* p = group + tid * 4;
    f32x4 v;
    for (int spins = 0;; ++spins) {
        asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
        int give_up = 0;
        if (tid == 0 && (spins > spin_limit / 8 ||
                         ((spins & 63) == 63 && __hip_atomic_load(abort_w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))))
            give_up = 1;
        // two reductions: these calls return "some / every thread passed non-zero", not a combination of the values
        if (__syncthreads_or(give_up)) return false;
        if (__syncthreads_and(df_written(v) ? 1 : 0)) break;
    }
    *reinterpret_cast<f32x4*>(&dst[tid >> 2][(tid & 3) * 4]) = v;
    __syncthreads();
    return true;
}

// Column group q of L = T·W for the wave's 16 rows (wave w: rows 16w..16w+15), 16×16×4 fp32 MFMA.
// T row-major [row][k] (pitch LP), Wg = rows k of the group's 16 columns.  W is upper triangular: k < 16(q+1).
// Lane (l16, kq): the MFMA step (g, e) contracts k = 16g + 4kq + e in lane group kq.
// The result goes to Lm[row][16q + col] (pitch LP).
__device__ __forceinline__ void df_l_group(float (*Lm)[LP], const float (*Tm)[LP], const float (*Wg)[WCP], int q, int w,
                                           int l16, int kq) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int g = 0; g <= q; ++g) {
        const float4 a4 = *reinterpret_cast<const float4*>(&Tm[16 * w + l16][16 * g + 4 * kq]);
        const int k0 = 16 * g + 4 * kq;
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, Wg[k0 + 0][l16], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, Wg[k0 + 1][l16], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, Wg[k0 + 2][l16], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, Wg[k0 + 3][l16], acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) Lm[16 * w + 4 * kq + v][16 * q + l16] = acc[v];
}

// acc[j] += L[16w.., group q]·L[16j.., group q]ᵀ for the 16×16 tiles j <= w of the wave's tile row (the lower
// triangle is all the elimination of the diagonal tile reads)
__device__ __forceinline__ void df_syrk_group(f32x4 (&acc)[4], const float (*Lm)[LP], int q, int w, int l16, int kq) {
    const float4 a4 = *reinterpret_cast<const float4*>(&Lm[16 * w + l16][16 * q + 4 * kq]);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (j > w) continue;
        const float4 b4 = *reinterpret_cast<const float4*>(&Lm[16 * j + l16][16 * q + 4 * kq]);
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, b4.x, acc[j], 0, 0, 0);
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, b4.y, acc[j], 0, 0, 0);
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, b4.z, acc[j], 0, 0, 0);
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, b4.w, acc[j], 0, 0, 0);
    }
}

// Two 64×64 tiles (rows ra0.., columns ca0.. of Ma and rows rb0.., columns cb0.. of Mb) -> LDS, row-major
// with pitch LP; the first is multiplied by sa.  Entries outside the r×r matrix read as zero.
__device__ __forceinline__ void df_tiles_to_lds(float (*da)[LP], const float* Ma, int ra0, int ca0, float sa, float (*dbm)[LP],
                                                const float* Mb, int rb0, int cb0, bool two, int r, int tid) {
    if ((r & 3) == 0) {
        f32x4 v[8];
        const float* ptr[8];
        bool ok[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const bool second = q >= 4;
            const int row = (tid >> 4) + 16 * (q & 3), c4 = (tid & 15) * 4;
            const int gr = (second ? rb0 : ra0) + row, gc = (second ? cb0 : ca0) + c4;
            ok[q] = (gr < r) && (gc < r) && (two || !second);
            ptr[q] = (second ? Mb : Ma) + (ok[q] ? (int64_t)gr * r + gc : 0);   // out of range: a valid address, value dropped
        }
        df_ld16x8(ptr, v);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const bool second = q >= 4;
            if (second && !two) continue;
            const int row = (tid >> 4) + 16 * (q & 3), c4 = (tid & 15) * 4;
            const float sg = second ? 1.f : sa;
            f32x4 o = {0.f, 0.f, 0.f, 0.f};
            if (ok[q]) o = v[q] * sg;
            *reinterpret_cast<f32x4*>(second ? &dbm[row][c4] : &da[row][c4]) = o;
        }
    } else {
        for (int e = tid; e < 2 * NB * NB; e += 256) {
            const bool second = e >= NB * NB;
            if (second && !two) break;
            const int row = (e >> 6) & 63, col = e & 63;
            const int gr = (second ? rb0 : ra0) + row, gc = (second ? cb0 : ca0) + col;
            float x = 0.f;
            if (gr < r && gc < r)
                x = __hip_atomic_load((second ? Mb : Ma) + (int64_t)gr * r + gc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (second) dbm[row][col] = x; else da[row][col] = sa * x;
        }
    }
}

// one thread: wait until both flags are up (f2 may equal f1); the two loads of a poll are in flight together
__device__ __forceinline__ bool df_poll(unsigned* f1, unsigned* f2, unsigned* abort_w, int spin_limit) {
    for (int spins = 0;; ++spins) {
        const unsigned v1 = __hip_atomic_load(f1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned v2 = __hip_atomic_load(f2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (v1 && v2) return true;
        if (spins > spin_limit) return false;
        if ((spins & 255) == 255 && __hip_atomic_load(abort_w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return false;
        __builtin_amdgcn_s_sleep(1);
    }
}

// acc += Am[32wr + ·][:] · (bsign · Bm[32wc + ·][:])ᵀ   (64-deep, operands row-major [row][k] in LDS)
__device__ __forceinline__ void df_mma(f32x16& acc, const float (*Am)[LP], const float (*Bm)[LP], int wr, int wc, int l32,
                                       int lh, float bsign) {
#pragma unroll
    for (int g = 0; g < NB / 8; ++g) {
        const float4 a4 = *reinterpret_cast<const float4*>(&Am[32 * wr + l32][8 * g + 4 * lh]);
        const float4 b4 = *reinterpret_cast<const float4*>(&Bm[32 * wc + l32][8 * g + 4 * lh]);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, bsign * b4.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, bsign * b4.y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, bsign * b4.z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, bsign * b4.w, acc, 0, 0, 0);
    }
}

// returns Am · W with W row-major [k][n] in LDS (the finalising product T·W_k)
__device__ __forceinline__ f32x16 df_times_w(const float (*Am)[LP], const float (*Wm)[LP], int wr, int wc, int l32, int lh) {
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int g = 0; g < NB / 8; ++g) {
        const float4 a4 = *reinterpret_cast<const float4*>(&Am[32 * wr + l32][8 * g + 4 * lh]);
        const int k0 = 8 * g + 4 * lh, n = 32 * wc + l32;
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, Wm[k0 + 0][n], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, Wm[k0 + 1][n], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, Wm[k0 + 2][n], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, Wm[k0 + 3][n], acc, 0, 0, 0);
    }
    return acc;
}

// accumulator (MFMA C layout: element v of a lane -> row 8*(v/4) + 4*lh + v%4, column l32 of the wave's
// 32×32 quadrant) -> LDS tile, row-major with pitch P
template <int P>
__device__ __forceinline__ void df_acc_to_lds(float (*dst)[P], const f32x16& acc, int wr, int wc, int l32, int lh) {
#pragma unroll
    for (int v = 0; v < 16; ++v) dst[32 * wr + 8 * (v >> 2) + 4 * lh + (v & 3)][32 * wc + l32] = acc[v];
}

// 64×64 tile of a global r×r matrix -> accumulator; out-of-range entries read as `diag_pad` on the
// global diagonal and 0 elsewhere
__device__ __forceinline__ f32x16 df_load_acc(const float* __restrict__ M, int r, int r0, int c0, int wr, int wc, int l32,
                                              int lh, float diag_pad) {
    f32x16 acc;
    const int gc = c0 + 32 * wc + l32;
    const int rq = 32 * wr + 4 * lh;
    if (r0 + NB <= r && c0 + NB <= r) {
        const float* po = M + (int64_t)(r0 + rq) * r + gc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = po[(int64_t)(8 * (v >> 2) + (v & 3)) * r];
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int gr = r0 + rq + 8 * (v >> 2) + (v & 3);
            acc[v] = (gr < r && gc < r) ? M[(int64_t)gr * r + gc] : ((gr == gc) ? diag_pad : 0.f);
        }
    }
    return acc;
}

// LDS tile (row-major, pitch P) -> global r×r matrix with agent-scope stores (a panel tile other workgroups
// will read), 16-byte row pieces where the shape allows
template <int P>
__device__ __forceinline__ void df_store_tile(float* __restrict__ M, const float (*src)[P], int r, int r0, int c0, int tid) {
    if ((r & 3) == 0) {
        for (int e = tid; e < NB * NB / 4; e += 256) {
            const int row = e >> 4, col = (e & 15) * 4;
            const int gr = r0 + row, gc = c0 + col;
            if (gr < r && gc < r) {
                f32x4 v;
#pragma unroll
                for (int q = 0; q < 4; ++q) v[q] = src[row][col + q];
                df_st16(M + (int64_t)gr * r + gc, v);
            }
        }
    } else {
        for (int e = tid; e < NB * NB; e += 256) {
            const int row = e >> 6, col = e & 63;
            const int gr = r0 + row, gc = c0 + col;
            if (gr < r && gc < r) __hip_atomic_store(M + (int64_t)gr * r + gc, src[row][col], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Finished Y tile (rows r0.., columns c0.. of Y = L^-T, row-major with pitch P in LDS) -> its transposed
// place in Binv[n][k] = Y[k][n]·dinv[k], as fp32 and/or as hi/lo bf16 planes
template <int P>
__device__ __forceinline__ void df_store_binv(const float (*src)[P], const float* __restrict__ db, float* Binv, bf16_t* Bh,
                                              bf16_t* Bl, int64_t boff, int r, int r0, int c0, int tid) {
    if (Bh && !Binv && (r & 7) == 0) {
        for (int e = tid; e < NB * NB / 8; e += 256) {
            const int col = e >> 3, row8 = (e & 7) * 8;
            const int gr = r0 + row8, gc = c0 + col;
            if (gr < r && gc < r) {
                float v[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = src[row8 + q][col] * db[gr + q];
                uint4 h, l;
                uint32_t* hp = reinterpret_cast<uint32_t*>(&h);
                uint32_t* lp = reinterpret_cast<uint32_t*>(&l);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t hh = pack_bf2(v[2 * q], v[2 * q + 1]);
                    hp[q] = hh;
                    lp[q] = pack_bf2(v[2 * q] - bf2f((bf16_t)(hh & 0xffffu)), v[2 * q + 1] - bf2f((bf16_t)(hh >> 16)));
                }
                const int64_t o = boff + (int64_t)gc * r + gr;
                *reinterpret_cast<uint4*>(Bh + o) = h;
                *reinterpret_cast<uint4*>(Bl + o) = l;
            }
        }
    } else {
        for (int e = tid; e < NB * NB; e += 256) {
            const int col = e >> 6, row = e & 63;
            const int gr = r0 + row, gc = c0 + col;
            if (gr < r && gc < r) {
                const float v = src[row][col] * db[gr];
                const int64_t o = boff + (int64_t)gc * r + gr;
                if (Binv) Binv[o] = v;
                if (Bh) {
                    const bf16_t h = f2bf(v);
                    Bh[o] = h;
                    Bl[o] = f2bf(v - bf2f(h));
                }
            }
        }
    }
}

template <int NT>
__global__ void __launch_bounds__(256, 1) factor_dataflow_kernel(DfArgs a) {
    __shared__ __align__(16) float lds_a[NB * LP];
    __shared__ __align__(16) float lds_b[NB * LP];
    __shared__ __align__(16) Elim2Lds elds;
    __shared__ __align__(16) float lds_l[NB * LP];     // the product with W as it is formed, group by group
    __shared__ __align__(16) float lds_w[NB * WCP];    // the column group of W in hand
    __shared__ int s_ok;
    float (*Am)[LP] = reinterpret_cast<float (*)[LP]>(lds_a);
    float (*Bm)[LP] = reinterpret_cast<float (*)[LP]>(lds_b);
    float (*As)[NB + 1] = reinterpret_cast<float (*)[NB + 1]>(lds_a);
    float (*Bs)[NB + 1] = reinterpret_cast<float (*)[NB + 1]>(lds_b);
    float (*Am2)[LP] = reinterpret_cast<float (*)[LP]>(lds_l);
    float (*Wg)[WCP] = reinterpret_cast<float (*)[WCP]>(lds_w);

    const int b = a.item0 + blockIdx.y;
    const int r = a.r, nb = a.nblk;
    const int64_t boff = (int64_t)b * r * r;
    float* Sb = a.S + boff;
    float* Lb = a.Lf + boff;
    float* Yb = a.Y + boff;
    const float* db = a.dinv + (int64_t)b * r;
    unsigned* fl = a.flags + (int64_t)b * DF_FLAG_WORDS;
    unsigned* abort_w = fl + 2 * DF_MAX_NBLK * DF_MAX_NBLK;
    float* wxb = a.wx + (int64_t)b * DF_WX_WORDS;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wr = wave >> 1, wc = wave & 1;
    const int l16 = lane & 15, kq = lane >> 4;

    // flag of the finished panel tile in stacked row `row` (S-rows 0..nb-1, Y-rows nb..2nb-1), block column p
    auto flag_of = [&](int row, int p) { return fl + row * nb + p; };
    // whole workgroup waits for up to two flags; false = give up (abort raised)
    auto wg_wait = [&](unsigned* f1, unsigned* f2) -> bool {
        if (tid == 0) {
            const bool ok = df_poll(f1, f2 ? f2 : f1, abort_w, a.spin_limit);
            if (!ok) {
                __hip_atomic_store(abort_w, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (a.info) a.info[b] = -1;
            }
            s_ok = ok ? 1 : 0;
        }
        __syncthreads();
        const int ok = s_ok;
        __syncthreads();      // s_ok may be rewritten from here on
        return ok != 0;
    };
    // publish: every wave's stores of the tile have completed, then one thread raises the flag
    auto wg_publish = [&](unsigned* f) {
        df_stores_done();
        __syncthreads();
        if (tid == 0) __hip_atomic_store(f, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };

    // a wait on an exchange slot gave up: raise the item's abort word and flag the result
    auto give_up = [&]() {
        if (tid == 0) {
            __hip_atomic_store(abort_w, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (a.info) a.info[b] = -1;
        }
    };

    const int g = blockIdx.x;
    if (g < nb) {
        // ------------------------------------------------------------------ spine of block row i
        const int i = g;
        const int r0 = i * NB;
        DF_STAMP(i * 8 + 0);
        f32x16 acc_d = df_load_acc(Sb, r, r0, r0, wr, wc, l32, lh, 1.f);
        f32x16 acc_s;
        if (i > 0) acc_s = df_load_acc(Sb, r, r0, r0 - NB, wr, wc, l32, lh, 0.f);
        for (int p = 0; p + 2 <= i; ++p) {
            if (!wg_wait(flag_of(i, p), flag_of(i - 1, p))) return;
            df_tiles_to_lds(Am, Lb, r0, p * NB, -1.f, Bm, Lb, r0 - NB, p * NB, true, r, tid);   // -L(i,p), L(i-1,p)
            __syncthreads();
            df_mma(acc_s, Am, Bm, wr, wc, l32, lh, 1.f);
            df_mma(acc_d, Am, Am, wr, wc, l32, lh, -1.f);
            __syncthreads();
        }
        DF_STAMP(i * 8 + 1);
        float (*Lm)[LP] = Am2;
        unsigned* pending = nullptr;   // flag of L(i,i-1), raised from inside the elimination
        // T_ii with the panels p <= i-2 applied (T in Bs); the panel i-1 follows below, group by group
        df_acc_to_lds<NB + 1>(Bs, acc_d, wr, wc, l32, lh);
        if (i > 0) {
            df_acc_to_lds<LP>(Am, acc_s, wr, wc, l32, lh);   // T(i,i-1)
            f32x4 accp[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) accp[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            const float* slot = wxb + (int64_t)(i - 1) * DF_SLOT_WORDS;
            for (int q = 0; q < 4; ++q) {
                if (!df_poll_group(Wg, slot + 1024 * q, abort_w, a.spin_limit, tid)) {   // 16 columns of W_{i-1}
                    give_up();
                    return;
                }
                if (q == 3) DF_STAMP(i * 8 + 2);
                df_l_group(Lm, Am, Wg, q, wave, l16, kq);          // 16 columns of L(i,i-1)
                __syncthreads();
                if (q == 3) df_store_tile<LP>(Lb, Lm, r, r0, r0 - NB, tid);   // stores in flight under what follows
                df_syrk_group(accp, Lm, q, wave, l16, kq);
            }
            // T_ii -= L(i,i-1)·L(i,i-1)ᵀ on the lower 16×16 tiles
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (j > wave) continue;
#pragma unroll
                for (int v = 0; v < 4; ++v) Bs[16 * wave + 4 * kq + v][16 * j + l16] -= accp[j][v];
            }
            pending = flag_of(i, i - 1);
            DF_STAMP(i * 8 + 3);
        }
        __syncthreads();
        DF_STAMP(i * 8 + 4);
        // W_i = L_ii^-T of the Schur complement T_ii (T in Bs, W in As)
        {
            int bad_col = -1;
            diag_inverse_factor(Bs, As, elds, tid, a.flag_below, bad_col, wxb + (int64_t)i * DF_SLOT_WORDS, pending);
            if (tid == 0 && a.info && bad_col >= 0 && (r0 + bad_col) < r) atomicCAS(a.info + b, 0, r0 + bad_col + 1);
        }
        DF_STAMP(i * 8 + 5);
        df_store_tile<NB + 1>(Yb, As, r, r0, r0, tid);
        wg_publish(flag_of(nb + i, i));
        DF_STAMP(i * 8 + 6);
        df_store_binv<NB + 1>(As, db, a.Binv, a.Bh, a.Bl, boff, r, r0, r0, tid);
        DF_STAMP(i * 8 + 7);
        return;
    }

    // ---------------------------------------------------------------------- bulk workgroup w
    const int w = g - nb;
    const int ntiles = (nb - 1) * (nb - 1);
    const int per = nb - 2;
    f32x16 acc[NT];
    int kcol[NT], rrow[NT];   // block column; stacked row (S-row i, or nb + c for Y-row c); kcol < 0: empty slot
#pragma unroll
    for (int s = 0; s < NT; ++s) {
        const int t = s * a.nbulk + w;
        kcol[s] = -1; rrow[s] = 0;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[s][v] = 0.f;
        if (t < ntiles) {
            int k, idx;
            if (per > 0 && t < (nb - 1) * per) { k = t / per; idx = t - k * per; }
            else { k = nb - 1; idx = t - (nb - 1) * per; }
            const int nS = max(nb - k - 2, 0);
            kcol[s] = k;
            if (idx < nS) {
                rrow[s] = k + 2 + idx;
                acc[s] = df_load_acc(Sb, r, rrow[s] * NB, k * NB, wr, wc, l32, lh, 0.f);
            } else {
                rrow[s] = nb + (idx - nS);
            }
        }
    }
    for (int q = 0; q < nb; ++q) {
        if (w == 0) DF_STAMP(512 + q * 4 + 0);
        // finalise the slots of block column q:  P = T·W_q
        // The first slot of the column takes W_q from the exchange slot, group by group behind the elimination
        // that produces it, and leaves the whole of W_q in Bm for any further slot of the column.
        bool have_w = false;
#pragma unroll
        for (int s = 0; s < NT; ++s) {
            if (kcol[s] != q) continue;
            const bool ykind = rrow[s] >= nb;
            const int r0 = (ykind ? rrow[s] - nb : rrow[s]) * NB;
            df_acc_to_lds<LP>(Am, acc[s], wr, wc, l32, lh);
            if (!have_w) {
                const float* slot = wxb + (int64_t)q * DF_SLOT_WORDS;
                for (int g = 0; g < 4; ++g) {
                    if (!df_poll_group(Wg, slot + 1024 * g, abort_w, a.spin_limit, tid)) {
                        give_up();
                        return;
                    }
                    *reinterpret_cast<f32x4*>(&Bm[tid >> 2][16 * g + (tid & 3) * 4]) =
                        *reinterpret_cast<const f32x4*>(&Wg[tid >> 2][(tid & 3) * 4]);
                    df_l_group(Am2, Am, Wg, g, wave, l16, kq);
                }
                have_w = true;
                __syncthreads();
            } else {
                __syncthreads();
                const f32x16 pr = df_times_w(Am, Bm, wr, wc, l32, lh);
                df_acc_to_lds<LP>(Am2, pr, wr, wc, l32, lh);
                __syncthreads();
            }
            df_store_tile<LP>(ykind ? Yb : Lb, Am2, r, r0, q * NB, tid);
            wg_publish(flag_of(rrow[s], q));
            if (ykind) df_store_binv<LP>(Am2, db, a.Binv, a.Bh, a.Bl, boff, r, r0, q * NB, tid);
            __syncthreads();
        }
        if (w == 0) DF_STAMP(512 + q * 4 + 1);
        // apply panel q to the later slots
#pragma unroll
        for (int s = 0; s < NT; ++s) {
            if (kcol[s] <= q) continue;                    // empty, finished, or just finalised
            const bool ykind = rrow[s] >= nb;
            if (ykind && rrow[s] - nb > q) continue;       // Y-row c starts at panel c
            if (!wg_wait(flag_of(rrow[s], q), flag_of(kcol[s], q))) return;
            const int r0 = (ykind ? rrow[s] - nb : rrow[s]) * NB;
            df_tiles_to_lds(Am, ykind ? Yb : Lb, r0, q * NB, -1.f, Bm, Lb, kcol[s] * NB, q * NB, true, r, tid);
            __syncthreads();
            df_mma(acc[s], Am, Bm, wr, wc, l32, lh, 1.f);
            __syncthreads();
        }
        if (w == 0) DF_STAMP(512 + q * 4 + 2);
    }
}

}  // namespace


namespace {
int g_df_spin_limit = DF_SPIN_LIMIT;
// compute units of the current device (the single-launch factorisation runs one workgroup on each and needs them
// all resident at once); 256 on an MI355X, asked once so that a partitioned or smaller device is sized correctly
int compute_units() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
        (void)hipGetLastError();
    }
    return n;
}
// workgroups per item of the single-launch factorisation, 0 = shape not covered
int dataflow_group(int nblk, int items, int& nt) {
    const int ntiles = (nblk - 1) * (nblk - 1);
    if (nblk < 1 || nblk > DF_MAX_NBLK || items < 1) return 0;
    int room = compute_units() / items - nblk;   // bulk workgroups that fit beside the spine (one workgroup per compute unit)
    const int enough = (ntiles + 4) / 5;     // five tiles per bulk workgroup keep up with the spine; more workgroups only idle
    if (room > enough) room = enough;
    if (ntiles == 0) { nt = 1; return nblk; }
    if (room < 1) return 0;
    const int nbulk = room < ntiles ? room : ntiles;
    nt = (ntiles + nbulk - 1) / nbulk;
    if (nt > 6) return 0;
    return nblk + nbulk;
}
}  // namespace

bool factor_dataflow_ok(int r, int batch, bool whole_batch) {
    const int nblk = (r + NB - 1) / NB;
    int nt;
    if (batch < 1) return false;
    // the whole batch in one launch, or at least one item per launch
    return dataflow_group(nblk, whole_batch ? batch : 1, nt) != 0;
}

// per item: the flag words, then (after the flags of all items) the exchange slots
void factor_dataflow_set_spin_limit(int polls) { g_df_spin_limit = polls >= 1 ? polls : DF_SPIN_LIMIT; }

size_t factor_dataflow_flag_bytes(int batch) { return (size_t)batch * (DF_FLAG_WORDS + DF_WX_WORDS) * sizeof(unsigned); }

hipError_t factor_inverse_dataflow(hipStream_t st, float* S, float* Lf, float* Y, const float* dinv, float* Binv,
                                   bf16_t* Bh, bf16_t* Bl, unsigned* flags, int r, int32_t* info, float flag_below,
                                   int batch) {
    const int nblk = (r + NB - 1) / NB;
    // as many items per launch as keep every workgroup of the launch resident at once
    int per_launch = batch, nt = 0, G = 0;
    while (per_launch >= 1 && (G = dataflow_group(nblk, per_launch, nt)) == 0) --per_launch;
    if (per_launch < 1) return hipErrorInvalidValue;
    for (int item0 = 0; item0 < batch; item0 += per_launch) {
        const int n = (batch - item0 < per_launch) ? batch - item0 : per_launch;
        DfArgs a;
        a.S = S; a.Lf = Lf; a.Y = Y; a.dinv = dinv; a.Binv = Binv; a.Bh = Bh; a.Bl = Bl; a.flags = flags; a.info = info;
        a.wx = reinterpret_cast<float*>(flags + (size_t)batch * DF_FLAG_WORDS);
        a.spin_limit = g_df_spin_limit;
        a.r = r; a.nblk = nblk; a.item0 = item0; a.nbulk = G - nblk > 0 ? G - nblk : 1; a.flag_below = flag_below;
        const dim3 grid(G, n), block(256);
        switch (nt) {
            case 1: hipLaunchKernelGGL(factor_dataflow_kernel<1>, grid, block, 0, st, a); break;
            case 2: hipLaunchKernelGGL(factor_dataflow_kernel<2>, grid, block, 0, st, a); break;
            case 3: hipLaunchKernelGGL(factor_dataflow_kernel<3>, grid, block, 0, st, a); break;
            case 4: hipLaunchKernelGGL(factor_dataflow_kernel<4>, grid, block, 0, st, a); break;
            case 5: hipLaunchKernelGGL(factor_dataflow_kernel<5>, grid, block, 0, st, a); break;
            default: hipLaunchKernelGGL(factor_dataflow_kernel<6>, grid, block, 0, st, a); break;
        }
    }
    return hipGetLastError();
}

hipError_t gram_prepare(hipStream_t st, const float* Spart, int nparts, int64_t pstride, float* S, float* dinv,
                        float* Y, float* Binv, bf16_t* Bh, bf16_t* Bl, int r, float shift, int zero_all, int batch,
                        unsigned* flags) {
    const int nblk = (r + NB - 1) / NB;
    hipLaunchKernelGGL(diag_rsqrt_kernel, dim3((r + 255) / 256, batch), dim3(256), 0, st, Spart, nparts, pstride,
                       dinv, r, flags, DF_FLAG_WORDS, flags ? reinterpret_cast<uint4*>(flags + (size_t)batch * DF_FLAG_WORDS) : nullptr,
                       DF_WX_WORDS, (nblk <= DF_MAX_NBLK ? nblk : 0) * DF_SLOT_WORDS);
    if ((r & 3) == 0)
        hipLaunchKernelGGL(prepare4_kernel, dim3((r / 4 + 255) / 256, r, batch), dim3(256), 0, st, Spart, nparts, pstride, S,
                           dinv, Y, Binv, Bh, Bl, r, shift, zero_all);
    else
        hipLaunchKernelGGL(prepare_kernel, dim3((r + 255) / 256, r, batch), dim3(256), 0, st, Spart, nparts, pstride, S,
                           dinv, Y, Binv, Bh, Bl, r, shift, zero_all);
    return hipGetLastError();
}

hipError_t factor_inverse(hipStream_t st, float* S, float* Lf, float* Y, const float* dinv, float* Binv, bf16_t* Bh,
                          bf16_t* Bl, int r, int32_t* info, float flag_below, int batch,
                          hipError_t (*after)(void* ctx, int j), void* ctx) {
    const int nblk = (r + NB - 1) / NB;
    for (int j = 0; j < nblk; ++j) {
        const int m = nblk - j;
        int tiles = m + j + 1;                                   // block column j of S and of Y
        if (j & 1) tiles += (m - 1) + ((m > 1) ? j : 0);        // odd j: the tiles of block column j+1
        else if (j >= 2) tiles += m * (m - 1) / 2 + j * (m - 1);  // even j: every trailing tile
        hipLaunchKernelGGL(factor_step_kernel, dim3(tiles, batch), dim3(256), 0, st, S, Lf, Y, dinv, Binv, Bh, Bl, r, nblk,
                           j, info, flag_below);
        if (after) {
            const hipError_t e = after(ctx, j);
            if (e != hipSuccess) return e;
        }
    }
    return hipGetLastError();
}

}  // namespace atp
