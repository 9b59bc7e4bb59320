// Rayleigh–Ritz canonicalisation of a basis pair (U_r, B_r) (Eq.9: the rows of X' are σ_i·v_iᵀ in
// descending order): eigen-decomposition T = B_r·B_rᵀ = R·Λ·Rᵀ by the cyclic two-sided Jacobi method
// (fp32), then U_r ← U_r·R, B_r ← Rᵀ·B_r with the columns ordered by descending eigenvalue and signed
// so that 1ᵀ·u_i ≥ 0.  Also the diagnostics the paper uses to choose r: captured energy (Fig.5) and
// the SVD-entropy low-rankness ⌈2^μ⌉ (Eq.4) of the estimated singular values.
//
// Jacobi: one launch per round of n/2 disjoint rotations (round-robin pairing, n-1 rounds per
// sweep).  A workgroup owns one index pair (p, q): it rotates rows p, q of T (and of Rᵀ, whose rows
// are the eigenvector estimates) and applies the column rotations of every other pair to its two
// rows; the angles of all pairs come from the previous buffer (ping-pong), so a round has no
// internal dependencies.
#include "common.h"

#include <algorithm>

namespace atp {
namespace {

// partner of index x in round k of the round-robin schedule over n (even) indices
__device__ __forceinline__ int rr_partner(int x, int k, int n) {
    const int m = n - 1;
    if (x == m) return k;
    if (x == k) return m;
    int y = 2 * k - x;
    y %= m;
    if (y < 0) y += m;
    return y;
}

// rotation that annihilates T[p][q]: c, s with J = [[c, s], [-s, c]] on (p, q); identity when the pair
// reaches past r (padding index) or the entry is already zero
__device__ __forceinline__ void jacobi_cs(const float* __restrict__ T, int n_ld, int r, int p, int q, float& c, float& s) {
    c = 1.f; s = 0.f;
    if (p >= r || q >= r) return;
    const float apq = T[(int64_t)p * n_ld + q];
    if (apq == 0.f) return;
    const float app = T[(int64_t)p * n_ld + p], aqq = T[(int64_t)q * n_ld + q];
    const float tau = (aqq - app) / (2.f * apq);
    const float t = (tau >= 0.f ? 1.f : -1.f) / (fabsf(tau) + sqrtf(1.f + tau * tau));
    c = 1.0f / sqrtf(1.f + t * t);
    s = t * c;
}

// One round.  Tin/Tout [batch][r][r], Rin/Rout [batch][r][r] (rows = eigenvector estimates).
__global__ void __launch_bounds__(256) jacobi_round_kernel(const float* __restrict__ Tin, float* __restrict__ Tout,
                                                           const float* __restrict__ Rin, float* __restrict__ Rout, int r,
                                                           int n, int k) {
    extern __shared__ float lds[];   // a[n], b[n]: rows p, q after the row rotation
    float* ra = lds;
    float* rb = lds + n;
    const int b = blockIdx.y;
    const float* T = Tin + (int64_t)b * r * r;
    const float* R = Rin + (int64_t)b * r * r;
    float* To = Tout + (int64_t)b * r * r;
    float* Ro = Rout + (int64_t)b * r * r;
    // pair of this workgroup: x = blockIdx.x runs over the "first" members
    const int m = n - 1;
    int p, q;
    {
        const int i = blockIdx.x;  // 0 .. n/2-1
        int x, y;
        if (i == 0) { x = m; y = k; }
        else { x = (k + i) % m; y = (k - i + m) % m; }
        p = min(x, y); q = max(x, y);
    }
    float c, s;
    jacobi_cs(T, r, r, p, q, c, s);
    const bool live_p = p < r, live_q = q < r;
    for (int j = threadIdx.x; j < n; j += 256) {
        const float tp = (live_p && j < r) ? T[(int64_t)p * r + j] : 0.f;
        const float tq = (live_q && j < r) ? T[(int64_t)q * r + j] : 0.f;
        ra[j] = c * tp - s * tq;
        rb[j] = s * tp + c * tq;
        if (j < r) {   // eigenvector rows: Rᵀ ← Jᵀ·Rᵀ
            const float rp = live_p ? R[(int64_t)p * r + j] : 0.f;
            const float rq = live_q ? R[(int64_t)q * r + j] : 0.f;
            if (live_p) Ro[(int64_t)p * r + j] = c * rp - s * rq;
            if (live_q) Ro[(int64_t)q * r + j] = s * rp + c * rq;
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < r; j += 256) {
        const int jp = rr_partner(j, k, n);
        const int pj = min(j, jp), qj = max(j, jp);
        float cj, sj;
        jacobi_cs(T, r, r, pj, qj, cj, sj);
        float op, oq;
        if (j == pj) { op = cj * ra[pj] - sj * ra[qj]; oq = cj * rb[pj] - sj * rb[qj]; }
        else { op = sj * ra[pj] + cj * ra[qj]; oq = sj * rb[pj] + cj * rb[qj]; }
        if (live_p) To[(int64_t)p * r + j] = op;
        if (live_q) To[(int64_t)q * r + j] = oq;
    }
}

__global__ void __launch_bounds__(256) ritz_identity_kernel(float* __restrict__ R, int r) {
    const int b = blockIdx.z, i = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    if (j < r) R[((int64_t)b * r + i) * r + j] = (i == j) ? 1.f : 0.f;
}

// rank of eigenvalue i in descending order (ties: lower index first); lam = diag(T)
__global__ void __launch_bounds__(256) ritz_rank_kernel(const float* __restrict__ T, int r, int* __restrict__ rank) {
    const int b = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i >= r) return;
    const float* Tb = T + (int64_t)b * r * r;
    const float li = Tb[(int64_t)i * r + i];
    int cnt = 0;
    for (int j = 0; j < r; ++j) {
        const float lj = Tb[(int64_t)j * r + j];
        cnt += (lj > li || (lj == li && j < i)) ? 1 : 0;
    }
    rank[(int64_t)b * r + i] = cnt;
}

// One workgroup (64 threads) per eigenvector i: sign from 1ᵀ·u_i = (1ᵀU)·R[:, i]; writes row rank_i of
// RsT (= signed eigenvector), sigma[rank_i] and the "sum is numerically zero" flag.
__global__ void __launch_bounds__(64) ritz_order_kernel(const float* __restrict__ T, const float* __restrict__ R,
                                                        const float* __restrict__ colsum, int64_t ld_cs,
                                                        const int* __restrict__ rank, float* __restrict__ RsT,
                                                        float* __restrict__ sigma, int* __restrict__ zero_sum, int r,
                                                        float zero_tol) {
    const int b = blockIdx.y, i = blockIdx.x, lane = threadIdx.x;
    const float* row = R + ((int64_t)b * r + i) * r;
    float t = 0.f;
    for (int k = lane; k < r; k += 64) t = fmaf(colsum[(int64_t)b * ld_cs + k], row[k], t);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) t += __shfl_xor(t, off);
    const int dst = rank[(int64_t)b * r + i];
    const bool small = fabsf(t) < zero_tol;
    const float sg = (!small && t < 0.f) ? -1.f : 1.f;
    float* out = RsT + ((int64_t)b * r + dst) * r;
    for (int k = lane; k < r; k += 64) out[k] = sg * row[k];
    if (lane == 0) {
        const float lam = T[((int64_t)b * r + i) * r + i];
        sigma[(int64_t)b * r + dst] = sqrtf(fmaxf(lam, 0.f));
        zero_sum[(int64_t)b * r + dst] = small ? 1 : 0;
    }
}

// Fallback sign rule for components whose 1ᵀ·u_i is numerically zero: make the largest-magnitude
// entry of b_i positive.  One workgroup per flagged component.
template <typename T>
__global__ void __launch_bounds__(256) ritz_fallback_sign_kernel(T* __restrict__ U, T* __restrict__ B,
                                                                 const int* __restrict__ zero_sum, int L, int d, int r) {
    __shared__ float smax[256];
    __shared__ int sidx[256];
    const int b = blockIdx.y, i = blockIdx.x, tid = threadIdx.x;
    if (!zero_sum[(int64_t)b * r + i]) return;
    T* brow = B + ((int64_t)b * r + i) * d;
    float best = -1.f; int bi = 0;
    for (int c = tid; c < d; c += 256) {
        float v;
        if constexpr (sizeof(T) == 2) v = bf2f(brow[c]); else v = brow[c];
        if (fabsf(v) > best) { best = fabsf(v); bi = c; }
    }
    smax[tid] = best; sidx[tid] = bi;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if (tid < s) {
            if (smax[tid + s] > smax[tid] || (smax[tid + s] == smax[tid] && sidx[tid + s] < sidx[tid])) {
                smax[tid] = smax[tid + s]; sidx[tid] = sidx[tid + s];
            }
        }
        __syncthreads();
    }
    float lead;
    if constexpr (sizeof(T) == 2) lead = bf2f(brow[sidx[0]]); else lead = brow[sidx[0]];
    if (!(lead < 0.f)) return;
    __syncthreads();
    for (int c = tid; c < d; c += 256) {
        if constexpr (sizeof(T) == 2) brow[c] = brow[c] ^ 0x8000u; else brow[c] = -brow[c];
    }
    T* ucol = U + (int64_t)b * L * r + i;
    for (int l = tid; l < L; l += 256) {
        if constexpr (sizeof(T) == 2) ucol[(int64_t)l * r] = ucol[(int64_t)l * r] ^ 0x8000u; else ucol[(int64_t)l * r] = -ucol[(int64_t)l * r];
    }
}

// diag[b] = { Σ λ (= ‖B_r‖²_F), max_{i≠j} |T_ij| / max_i λ_i, μ = -log2 Σ (σ_i/Σσ)², ⌈2^μ⌉ }
__global__ void __launch_bounds__(256) ritz_diag_kernel(const float* __restrict__ T, const float* __restrict__ sigma, int r,
                                                        float* __restrict__ diag) {
    __shared__ float sh[4][256];
    const int b = blockIdx.x, tid = threadIdx.x;
    const float* Tb = T + (int64_t)b * r * r;
    float off = 0.f, lmax = 0.f, s1 = 0.f, s2 = 0.f;
    for (int64_t e = tid; e < (int64_t)r * r; e += 256) {
        const int i = (int)(e / r), j = (int)(e % r);
        const float v = Tb[e];
        if (i == j) lmax = fmaxf(lmax, fabsf(v)); else off = fmaxf(off, fabsf(v));
    }
    for (int i = tid; i < r; i += 256) {
        const float s = sigma[(int64_t)b * r + i];
        s1 += s; s2 += s * s;
    }
    sh[0][tid] = off; sh[1][tid] = lmax; sh[2][tid] = s1; sh[3][tid] = s2;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if (tid < s) {
            sh[0][tid] = fmaxf(sh[0][tid], sh[0][tid + s]);
            sh[1][tid] = fmaxf(sh[1][tid], sh[1][tid + s]);
            sh[2][tid] += sh[2][tid + s];
            sh[3][tid] += sh[3][tid + s];
        }
        __syncthreads();
    }
    if (tid == 0) {
        const float sum1 = sh[2][0], sum2 = sh[3][0];
        const float mu = (sum1 > 0.f && sum2 > 0.f) ? -log2f(sum2 / (sum1 * sum1)) : 0.f;
        diag[b * 4 + 0] = sum2;
        diag[b * 4 + 1] = (sh[1][0] > 0.f) ? sh[0][0] / sh[1][0] : 0.f;
        diag[b * 4 + 2] = mu;
        diag[b * 4 + 3] = ceilf(exp2f(mu) - 1e-4f);
    }
}

}  // namespace

hipError_t ritz_jacobi(hipStream_t st, float* T0, float* T1, float* R0, float* R1, int r, int batch, int sweeps,
                       float** T_final, float** R_final) {
    const int n = (r + 1) & ~1;
    hipLaunchKernelGGL(ritz_identity_kernel, dim3((r + 255) / 256, r, batch), dim3(256), 0, st, R0, r);
    float *Ti = T0, *To = T1, *Ri = R0, *Ro = R1;
    if (n >= 2) {
        const size_t lds = (size_t)2 * n * sizeof(float);
        for (int sw = 0; sw < sweeps; ++sw)
            for (int k = 0; k < n - 1; ++k) {
                hipLaunchKernelGGL(jacobi_round_kernel, dim3(n / 2, batch), dim3(256), lds, st, Ti, To, Ri, Ro, r, n, k);
                std::swap(Ti, To);
                std::swap(Ri, Ro);
            }
    }
    *T_final = Ti;
    *R_final = Ri;
    return hipGetLastError();
}

hipError_t ritz_order(hipStream_t st, const float* T, const float* R, const float* colsum, int64_t ld_cs, int* rank,
                      float* RsT, float* sigma, int* zero_sum, int r, int batch, float zero_tol) {
    hipLaunchKernelGGL(ritz_rank_kernel, dim3((r + 255) / 256, batch), dim3(256), 0, st, T, r, rank);
    hipLaunchKernelGGL(ritz_order_kernel, dim3(r, batch), dim3(64), 0, st, T, R, colsum, ld_cs, rank, RsT, sigma, zero_sum, r,
                       zero_tol);
    return hipGetLastError();
}

hipError_t ritz_fallback_sign(hipStream_t st, void* U, void* B, const int* zero_sum, int L, int d, int r, int batch,
                              int elem_bytes) {
    if (elem_bytes == 2)
        hipLaunchKernelGGL(ritz_fallback_sign_kernel<bf16_t>, dim3(r, batch), dim3(256), 0, st, (bf16_t*)U, (bf16_t*)B, zero_sum,
                           L, d, r);
    else
        hipLaunchKernelGGL(ritz_fallback_sign_kernel<float>, dim3(r, batch), dim3(256), 0, st, (float*)U, (float*)B, zero_sum, L,
                           d, r);
    return hipGetLastError();
}

hipError_t ritz_diagnostics(hipStream_t st, const float* T, const float* sigma, int r, int batch, float* diag) {
    hipLaunchKernelGGL(ritz_diag_kernel, dim3(batch), dim3(256), 0, st, T, sigma, r, diag);
    return hipGetLastError();
}

}  // namespace atp
