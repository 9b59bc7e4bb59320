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
#include "common.h"

#include <utility>

namespace atp {
namespace {

constexpr int NB = 64;  // block size of the factorisation

// ---------------------------------------------------------------------------
// dinv[j] = 1/sqrt(sum_p Spart[p][j][j])   (1 if the diagonal entry is not positive and finite)
__global__ void diag_rsqrt_kernel(const float* __restrict__ Sp, int nparts, int64_t pstride, float* __restrict__ dinv,
                                  int r) {
    const int b = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
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
    const float piv0 = fmaxf(piv0r, 1e-7f), i0 = __builtin_amdgcn_rcpf(piv0);
    const float x10 = p1.x, x20 = p2.x, x30 = p3.x;
    const float piv1r = fmaf(-x10 * i0, x10, p1.y);
    const float piv1 = fmaxf(piv1r, 1e-7f), i1 = __builtin_amdgcn_rcpf(piv1);
    const float x21 = fmaf(-x20 * i0, x10, p2.y);
    const float x31 = fmaf(-x30 * i0, x10, p3.y);
    const float piv2r = fmaf(-x21 * i1, x21, fmaf(-x20 * i0, x20, p2.z));
    const float piv2 = fmaxf(piv2r, 1e-7f), i2 = __builtin_amdgcn_rcpf(piv2);
    const float x32 = fmaf(-x31 * i1, x21, fmaf(-x30 * i0, x20, p3.z));
    const float piv3r = fmaf(-x32 * i2, x32, fmaf(-x31 * i1, x31, fmaf(-x30 * i0, x30, p3.w)));
    const float piv3 = fmaxf(piv3r, 1e-7f), i3 = __builtin_amdgcn_rcpf(piv3);
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
    reg[2 * B] = (half ? x1 * __builtin_amdgcn_rsqf(piv1) : x0 * __builtin_amdgcn_rsqf(piv0));
    reg[2 * B + 1] = (half ? x3 * __builtin_amdgcn_rsqf(piv3) : x2 * __builtin_amdgcn_rsqf(piv2));
    __syncthreads();
#pragma unroll
    for (int t = 2 * B + 2; t < 32; ++t) {
        const float4 d = L.xs[buf][2 * t + half];
        reg[t] = fmaf(-f3, d.w, fmaf(-f2, d.z, fmaf(-f1, d.y, fmaf(-f0, d.x, reg[t]))));
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the steps apart: no hoarding of values in registers
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

}  // namespace

hipError_t gram_prepare(hipStream_t st, const float* Spart, int nparts, int64_t pstride, float* S, float* dinv,
                        float* Y, float* Binv, bf16_t* Bh, bf16_t* Bl, int r, float shift, int zero_all, int batch) {
    hipLaunchKernelGGL(diag_rsqrt_kernel, dim3((r + 255) / 256, batch), dim3(256), 0, st, Spart, nparts, pstride,
                       dinv, r);
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
