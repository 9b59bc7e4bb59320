// r×r pieces of the CholeskyQR orthonormalisation (fp32, batched over sequences):
// Jacobi scaling + shift of the Gram matrix, blocked lower Cholesky, and the
// scaled inverse of the triangular factor that the GEMM kernel then applies to
// the tall matrix (Z ← Z·R⁻¹).  The orthonormal factor they produce is the U of
// Eq.5 (UᵀU = I, text after Eq.8).
#include "common.h"

namespace atp {
namespace {

constexpr int NB = 64;  // block size of the factorisation

// ---------------------------------------------------------------------------
__global__ void diag_rsqrt_kernel(const float* __restrict__ S, float* __restrict__ dinv, int r) {
    const int b = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= r) return;
    const float s = S[(int64_t)b * r * r + (int64_t)j * r + j];
    const bool ok = (s > 0.f) && (s < 3.0e38f);
    dinv[(int64_t)b * r + j] = ok ? 1.0f / sqrtf(s) : 1.0f;
}

__global__ void scale_shift_kernel(float* __restrict__ S, const float* __restrict__ dinv, int r, float shift) {
    const int b = blockIdx.z;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int i = blockIdx.y;
    if (j >= r) return;
    float* Sb = S + (int64_t)b * r * r;
    const float* db = dinv + (int64_t)b * r;
    const float v = Sb[(int64_t)i * r + j] * db[i] * db[j];
    Sb[(int64_t)i * r + j] = (i == j) ? v + shift : v;
}

// ---------------------------------------------------------------------------
// One block column of the left-looking blocked Cholesky.  Workgroup (i, b) owns
// row block i >= j of batch item b: it forms T_ij = S_ij - sum_k L_ik L_jkᵀ and
// (redundantly) T_jj, then eliminates the 64 columns of both tiles together,
// so no second launch is needed for the triangular solve.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) chol_step_kernel(const float* __restrict__ S, float* Lo, int r, int j,
                                                        int32_t* info, float flag_below) {
    __shared__ float Tj[NB][NB + 1];
    __shared__ float Ti[NB][NB + 1];
    __shared__ float Pi[32][NB + 1];
    __shared__ float Pj[32][NB + 1];
    __shared__ float piv_s[NB];

    const int b = blockIdx.y;
    const int i = j + blockIdx.x;
    const float* Sb = S + (int64_t)b * r * r;   // scaled Gram matrix, never written here
    float* Lb = Lo + (int64_t)b * r * r;         // factor: columns < j*NB come from earlier launches
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int ri0 = i * NB, rj0 = j * NB;

    float acc_i[4][4] = {}, acc_j[4][4] = {};
    for (int k0 = 0; k0 < rj0; k0 += 32) {
        for (int e = tid; e < NB * 32; e += 256) {
            const int row = e >> 5, kk = e & 31;
            const int gi = ri0 + row, gj = rj0 + row;
            Pi[kk][row] = (gi < r) ? Lb[(int64_t)gi * r + k0 + kk] : 0.f;
            Pj[kk][row] = (gj < r) ? Lb[(int64_t)gj * r + k0 + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int kk = 0; kk < 32; ++kk) {
            float ai[4], aj[4], bj[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                ai[a] = Pi[kk][ty * 4 + a];
                aj[a] = Pj[kk][ty * 4 + a];
                bj[a] = Pj[kk][tx * 4 + a];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    acc_i[a][c] = fmaf(ai[a], bj[c], acc_i[a][c]);
                    acc_j[a][c] = fmaf(aj[a], bj[c], acc_j[a][c]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int row = ty * 4 + a, col = tx * 4 + c;
            const int gc = rj0 + col, gi = ri0 + row, gj = rj0 + row;
            const float si = (gi < r && gc < r) ? Sb[(int64_t)gi * r + gc] : ((gi == gc) ? 1.f : 0.f);
            const float sj = (gj < r && gc < r) ? Sb[(int64_t)gj * r + gc] : ((gj == gc) ? 1.f : 0.f);
            Ti[row][col] = si - acc_i[a][c];
            Tj[row][col] = sj - acc_j[a][c];
        }
    __syncthreads();

    // right-looking elimination of the 64 columns; column c stays unscaled until the end
    const int sel = tid >> 7;          // 0: diagonal tile, 1: own tile
    const int a = tid & 63;            // row
    const int half = (tid >> 6) & 1;   // column parity
    float(*T)[NB + 1] = sel ? Ti : Tj;
    for (int c = 0; c < NB; ++c) {
        float piv = Tj[c][c];
        if (!(piv >= flag_below)) {
            if (i == j && tid == 0 && info && (rj0 + c) < r && info[b] == 0) info[b] = rj0 + c + 1;
            if (!(piv > 1e-7f)) piv = 1e-7f;
        }
        if (tid == 0) piv_s[c] = piv;
        const float f = T[a][c] / piv;
        for (int cc = c + 1 + half; cc < NB; cc += 2) T[a][cc] = fmaf(-f, Tj[cc][c], T[a][cc]);
        __syncthreads();
    }
    // scale columns, write back
    for (int e = tid; e < NB * NB; e += 256) {
        const int row = e >> 6, col = e & 63;
        const float rs = 1.0f / sqrtf(piv_s[col]);
        const int gc = rj0 + col;
        if (i == j) {
            const int gr = rj0 + row;
            if (gr < r && gc < r) {
                float v = 0.f;
                if (row > col) v = Tj[row][col] * rs;
                else if (row == col) v = piv_s[col] * rs;
                Lb[(int64_t)gr * r + gc] = v;
            }
        } else {
            const int gr = ri0 + row;
            if (gr < r && gc < r) Lb[(int64_t)gr * r + gc] = Ti[row][col] * rs;
        }
    }
}

// zero the strictly upper block triangle (blocks with column block > row block)
__global__ void zero_upper_blocks_kernel(float* __restrict__ S, int r) {
    const int b = blockIdx.z;
    const int row = blockIdx.y;
    const int col = blockIdx.x * blockDim.x + threadIdx.x;
    if (col >= r) return;
    if (col / NB > row / NB) S[(int64_t)b * r * r + (int64_t)row * r + col] = 0.f;
}

// ---------------------------------------------------------------------------
// Scaled inverse of the lower factor: X = L^-1 · diag(dinv).  Columns of X are
// independent; workgroup (jc, b) owns CW consecutive columns and walks down the
// row blocks: X_ij = -L_ii^-1 · sum_{k<i} L_ik X_kj, by forward substitution.
// ---------------------------------------------------------------------------
constexpr int CW = 16;

__global__ void __launch_bounds__(256) tri_inv_kernel(const float* __restrict__ Lm, const float* __restrict__ dinv,
                                                      float* X, int r) {
    __shared__ float Ls[NB][NB + 1];
    __shared__ float Ts[NB][CW + 1];
    __shared__ float Pa[32][NB + 1];
    __shared__ float Pb[32][CW + 1];

    const int b = blockIdx.y;
    const int c0 = blockIdx.x * CW;   // first column owned
    const int jb = c0 / NB;           // block row where the columns start
    const float* Lb = Lm + (int64_t)b * r * r;
    float* Xb = X + (int64_t)b * r * r;
    const float* db = dinv + (int64_t)b * r;
    const int nblk = (r + NB - 1) / NB;
    const int tid = threadIdx.x;
    const int col = tid & 15, rq = tid >> 4;  // GEMM: rows rq*4..rq*4+3, column col

    // blocks above the diagonal block are zero
    for (int e = tid; e < jb * NB * CW; e += 256) {
        const int row = e / CW, cc = e % CW;
        if (c0 + cc < r) Xb[(int64_t)row * r + c0 + cc] = 0.f;
    }

    for (int i = jb; i < nblk; ++i) {
        const int ri0 = i * NB;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        if (i > jb) {
            __threadfence();
            __syncthreads();  // X rows written in earlier iterations are visible
            for (int k0 = jb * NB; k0 < ri0; k0 += 32) {
                for (int e = tid; e < NB * 32; e += 256) {
                    const int row = e >> 5, kk = e & 31;
                    const int gr = ri0 + row;
                    Pa[kk][row] = (gr < r) ? Lb[(int64_t)gr * r + k0 + kk] : 0.f;
                }
                for (int e = tid; e < 32 * CW; e += 256) {
                    const int kk = e / CW, cc = e % CW;
                    Pb[kk][cc] = (c0 + cc < r) ? Xb[(int64_t)(k0 + kk) * r + c0 + cc] : 0.f;
                }
                __syncthreads();
#pragma unroll 8
                for (int kk = 0; kk < 32; ++kk) {
                    const float bv = Pb[kk][col];
#pragma unroll
                    for (int a = 0; a < 4; ++a) acc[a] = fmaf(Pa[kk][rq * 4 + a], bv, acc[a]);
                }
                __syncthreads();
            }
        }
        // right-hand side
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int row = rq * 4 + a;
            float v = -acc[a];
            if (i == jb) v = (ri0 + row == c0 + col && c0 + col < r) ? db[c0 + col] : 0.f;
            Ts[row][col] = v;
        }
        for (int e = tid; e < NB * NB; e += 256) {
            const int row = e >> 6, cc = e & 63;
            const int gr = ri0 + row, gc = ri0 + cc;
            Ls[row][cc] = (gr < r && gc < r) ? Lb[(int64_t)gr * r + gc] : ((row == cc) ? 1.f : 0.f);
        }
        __syncthreads();
        // forward substitution, row c stays unscaled until the end
        const int part = tid >> 4;  // 16 row phases
        for (int c = 0; c < NB; ++c) {
            const float f = Ts[c][col] / Ls[c][c];
            for (int a = c + 1 + part; a < NB; a += 16) Ts[a][col] = fmaf(-Ls[a][c], f, Ts[a][col]);
            __syncthreads();
        }
        for (int e = tid; e < NB * CW; e += 256) {
            const int row = e / CW, cc = e % CW;
            const int gr = ri0 + row;
            if (gr < r && c0 + cc < r) Xb[(int64_t)gr * r + c0 + cc] = Ts[row][cc] / Ls[row][row];
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t gram_scale_shift(hipStream_t st, float* S, float* dinv, int r, float shift, int batch) {
    hipLaunchKernelGGL(diag_rsqrt_kernel, dim3((r + 255) / 256, batch), dim3(256), 0, st, S, dinv, r);
    hipLaunchKernelGGL(scale_shift_kernel, dim3((r + 255) / 256, r, batch), dim3(256), 0, st, S, dinv, r, shift);
    return hipGetLastError();
}

hipError_t cholesky_lower(hipStream_t st, const float* S, float* Lo, int r, int32_t* info, float flag_below,
                          int batch) {
    const int nblk = (r + NB - 1) / NB;
    for (int j = 0; j < nblk; ++j)
        hipLaunchKernelGGL(chol_step_kernel, dim3(nblk - j, batch), dim3(256), 0, st, S, Lo, r, j, info, flag_below);
    hipLaunchKernelGGL(zero_upper_blocks_kernel, dim3((r + 255) / 256, r, batch), dim3(256), 0, st, Lo, r);
    return hipGetLastError();
}

hipError_t tri_inverse_scaled(hipStream_t st, const float* Lm, const float* dinv, float* Binv, int r, int batch) {
    hipLaunchKernelGGL(tri_inv_kernel, dim3((r + CW - 1) / CW, batch), dim3(256), 0, st, Lm, dinv, Binv, r);
    return hipGetLastError();
}

}  // namespace atp
