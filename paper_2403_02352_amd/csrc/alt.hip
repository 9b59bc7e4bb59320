// Alternating rank-1 extraction (Alg.1 of the appendix): for each component i, two alternations
//     u ← X·v / ‖v‖²,   v ← Xᵀ·u / ‖u‖²,
// then the deflation X ← X − u·vᵀ.  Every pass is one sweep over an fp32 working copy of X and is
// HBM-bound; the components are inherently sequential.
//
// One sweep does a whole alternation: a workgroup owns 64 consecutive rows, takes them four at a
// time (a thread keeps 4 rows × 16 columns in registers), forms the four row products with v, turns
// them into u (the scalar 1/‖v‖² is known), and accumulates its share of Xᵀ·u for its 16 columns
// from the same registers.  The per-workgroup column sums and Σu² go to a partial buffer that a
// second, small kernel adds up in a fixed order (run-to-run identical results).  The deflation by
// the previous component is applied on the fly by the first sweep of the next one (the only sweep
// that writes X).
#include "common.h"

#include <algorithm>

namespace atp {
namespace {

constexpr int ROWS_PER_WG = 16;  // many small workgroups: three fit a CU and hide each other's load latency
constexpr int RG = 4;            // rows per register group
constexpr int CB = 64;           // columns per ‖v‖² slot (one wave) and per workgroup of the reduction

// Σ of n floats in a fixed order (every caller gets the same bits)
__device__ __forceinline__ float ordered_sum(const float* p, int n) {
    float s = 0.f;
    for (int i = 0; i < n; ++i) s += p[i];
    return s;
}

// vec [batch][d]: current v;  part_vv [batch][ncb]: ‖v‖² by column block;  prev_u [batch][L],
// prev_v [batch][d]: component to deflate by (deflate != 0);  u_out [batch][L];
// part_v [batch][nwg][d], part_uu [batch][nwg]: this workgroup's share of Xᵀ·u and of ‖u‖².
__global__ void __launch_bounds__(256) alt_sweep_kernel(float* __restrict__ Xw, const float* __restrict__ vec,
                                                        const float* __restrict__ part_vv, int ncb,
                                                        const float* __restrict__ prev_u, const float* __restrict__ prev_v,
                                                        int deflate, float* __restrict__ u_out, float* __restrict__ part_v,
                                                        float* __restrict__ part_uu, int L, int d) {
    __shared__ float red[4][RG];
    __shared__ float ush[RG];
    const int b = blockIdx.y, wg = blockIdx.x, nwg = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* X = Xw + (int64_t)b * L * d;
    const float* v = vec + (int64_t)b * d;
    const float vv = ordered_sum(part_vv + (int64_t)b * ncb, ncb);
    const float inv_vv = (vv > 1e-30f) ? 1.0f / vv : 0.f;
    const float* pu = prev_u + (int64_t)b * L;
    const float* pv = prev_v + (int64_t)b * d;
    float uu = 0.f;
    const int row_base = wg * ROWS_PER_WG;
    // columns of this thread: 4·tid + 1024·k + {0..3}, k < 4 (d <= 4096, a multiple of 4)
    float vacc[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) vacc[k] = 0.f;
    float vreg[16], pvreg[16];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = 4 * tid + 1024 * k;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            vreg[4 * k + e] = (c + e < d) ? v[c + e] : 0.f;
            pvreg[4 * k + e] = (deflate && c + e < d) ? pv[c + e] : 0.f;
        }
    }
    for (int g = 0; g < ROWS_PER_WG / RG; ++g) {
        const int r0 = row_base + g * RG;
        float x[RG][16];
        float dot[RG];
#pragma unroll
        for (int i = 0; i < RG; ++i) {
            const int row = r0 + i;
            const float pui = (deflate && row < L) ? pu[row] : 0.f;
            dot[i] = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int c = 4 * tid + 1024 * k;
                f32x4 xv = {0.f, 0.f, 0.f, 0.f};
                if (row < L && c < d) xv = *reinterpret_cast<const f32x4*>(X + (int64_t)row * d + c);
                if (deflate) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) xv[e] = fmaf(-pui, pvreg[4 * k + e], xv[e]);
                    if (row < L && c < d) *reinterpret_cast<f32x4*>(X + (int64_t)row * d + c) = xv;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x[i][4 * k + e] = xv[e];
                    dot[i] = fmaf(xv[e], vreg[4 * k + e], dot[i]);
                }
            }
        }
        // row products: wave reduction, then the four waves through LDS (fixed order)
#pragma unroll
        for (int i = 0; i < RG; ++i) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) dot[i] += __shfl_xor(dot[i], off);
        }
        if (lane == 0) {
#pragma unroll
            for (int i = 0; i < RG; ++i) red[wave][i] = dot[i];
        }
        __syncthreads();
        if (tid < RG) {
            const float s = ((red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid])) * inv_vv;
            ush[tid] = s;
            const int row = r0 + tid;
            if (row < L) u_out[(int64_t)b * L + row] = s;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < RG; ++i) {
            const float ui = (r0 + i < L) ? ush[i] : 0.f;
            if (tid == 0) uu = fmaf(ui, ui, uu);
#pragma unroll
            for (int k = 0; k < 16; ++k) vacc[k] = fmaf(x[i][k], ui, vacc[k]);
        }
    }
    float* pvout = part_v + ((int64_t)b * nwg + wg) * d;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = 4 * tid + 1024 * k;
        if (c < d) {
            f32x4 o = {vacc[4 * k], vacc[4 * k + 1], vacc[4 * k + 2], vacc[4 * k + 3]};
            *reinterpret_cast<f32x4*>(pvout + c) = o;
        }
    }
    if (tid == 0) part_uu[(int64_t)b * nwg + wg] = uu;
}

// Σ x² over the 64 lanes of a wave (same value in every lane)
__device__ __forceinline__ float wave_sumsq(float x) {
    float s = x * x;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    return s;
}

// 64 columns per workgroup: v = (Σ_wg part_v)/‖u‖², ‖u‖² = Σ_wg part_uu; leaves ‖v‖² of its columns
// in part_vv[cb].  Wave g adds the partials w = g, g+4, ... with four independent running sums, the
// four waves are combined through LDS; the order is fixed.
// When final_comp >= 0 it also emits row final_comp of B (= ‖u‖·v) and keeps ‖u‖² in scal[b].
// A vanishing ‖u‖ (the input has no energy left) gives zeros instead of a division by zero and
// records the component in info.
template <typename T>
__global__ void __launch_bounds__(256) alt_reduce_kernel(const float* __restrict__ part_v, const float* __restrict__ part_uu,
                                                         int nwg, float* __restrict__ vec, float* __restrict__ part_vv,
                                                         float* __restrict__ scal, int d, int final_comp,
                                                         T* __restrict__ B, int r, int32_t* __restrict__ info) {
    __shared__ float sh[4][CB];
    const int b = blockIdx.y, cb = blockIdx.x, ncb = gridDim.x, tid = threadIdx.x;
    const int cx = tid & 63, g = tid >> 6;
    const int c = cb * CB + cx;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    if (c < d) {
        const float* p = part_v + (int64_t)b * nwg * d + c;
        int w = g;
        for (; w + 12 < nwg; w += 16) {
            a0 += p[(int64_t)w * d];
            a1 += p[(int64_t)(w + 4) * d];
            a2 += p[(int64_t)(w + 8) * d];
            a3 += p[(int64_t)(w + 12) * d];
        }
        for (; w < nwg; w += 4) a0 += p[(int64_t)w * d];
    }
    sh[g][cx] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (g != 0) return;
    const float uu = ordered_sum(part_uu + (int64_t)b * nwg, nwg);
    const bool dead = !(uu > 1e-30f);
    const float inv_uu = dead ? 0.f : 1.0f / uu;
    float s = ((sh[0][cx] + sh[1][cx]) + (sh[2][cx] + sh[3][cx])) * inv_uu;
    if (c < d) {
        vec[(int64_t)b * d + c] = s;
        if (final_comp >= 0) {
            const float o = s * sqrtf(uu);
            if constexpr (sizeof(T) == 2) B[((int64_t)b * r + final_comp) * d + c] = f2bf(o);
            else B[((int64_t)b * r + final_comp) * d + c] = o;
        }
    } else {
        s = 0.f;
    }
    const float vv = wave_sumsq(s);
    if (cx == 0) {
        part_vv[(int64_t)b * ncb + cb] = vv;
        if (cb == 0) {
            scal[b] = uu;
            if (final_comp >= 0 && dead && info && info[b] == 0) info[b] = final_comp + 1;
        }
    }
}

// After component `comp`: U[b][row][comp] = u[row]/‖u‖; (u, v) become the pair to deflate by; v is
// replaced by column comp+1 of the start block V0 [d][r] (fp32, shared by the batch) and its ‖·‖²
// goes to part_vv.  comp = -1 only loads the first start vector.
template <typename T>
__global__ void __launch_bounds__(256) alt_emit_kernel(const float* __restrict__ u, float* __restrict__ vec,
                                                       const float* __restrict__ scal, float* __restrict__ prev_u,
                                                       float* __restrict__ prev_v, T* __restrict__ U,
                                                       const float* __restrict__ V0, float* __restrict__ part_vv, int ncb,
                                                       int L, int d, int r, int comp) {
    const int b = blockIdx.y, blk = blockIdx.x;
    const int i = blk * 256 + threadIdx.x;
    if (comp >= 0 && i < L) {
        const float uu = scal[b];
        const float inv_n = (uu > 1e-30f) ? 1.0f / sqrtf(uu) : 0.f;
        const float x = u[(int64_t)b * L + i];
        prev_u[(int64_t)b * L + i] = x;
        const float o = x * inv_n;
        if constexpr (sizeof(T) == 2) U[((int64_t)b * L + i) * r + comp] = f2bf(o);
        else U[((int64_t)b * L + i) * r + comp] = o;
    }
    const int slot = blk * 4 + (threadIdx.x >> 6);   // 64 columns per ‖v‖² slot, one wave each
    if (slot < ncb) {                                 // uniform per wave
        float nv = 0.f;
        if (i < d) {
            if (comp >= 0) prev_v[(int64_t)b * d + i] = vec[(int64_t)b * d + i];
            if (comp + 1 < r) {
                nv = V0[(int64_t)i * r + comp + 1];
                vec[(int64_t)b * d + i] = nv;
            }
        }
        const float vv = wave_sumsq(nv);
        if ((threadIdx.x & 63) == 0) part_vv[(int64_t)b * ncb + slot] = vv;
    }
}

template <typename T>
__global__ void __launch_bounds__(256) alt_widen_kernel(const T* __restrict__ in, float* __restrict__ out, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) {
        if constexpr (sizeof(T) == 2) out[i] = bf2f(in[i]);
        else out[i] = in[i];
    }
}

}  // namespace

size_t alternating_workspace(int batch, int L, int d) {
    const size_t nwg = (L + ROWS_PER_WG - 1) / ROWS_PER_WG;
    const size_t ncb = (d + CB - 1) / CB;
    auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
    return al((size_t)batch * L * d * 4) + al((size_t)batch * d * 4) * 2 + al((size_t)batch * L * 4) * 2 +
           al((size_t)batch * 4) + al((size_t)batch * ncb * 4) + al((size_t)batch * nwg * d * 4) + al((size_t)batch * nwg * 4);
}

hipError_t alternating_bases(hipStream_t st, const void* X, int batch, int L, int d, int r, int sweeps, const float* V0,
                             void* U, void* B, int32_t* info, void* workspace, int elem_bytes) {
    if (d > 4096 || (d & 3)) return hipErrorInvalidValue;
    const int nwg = (L + ROWS_PER_WG - 1) / ROWS_PER_WG;
    const int ncb = (d + CB - 1) / CB;
    if (nwg > 65535 * 16) return hipErrorInvalidValue;
    auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
    uint8_t* p = reinterpret_cast<uint8_t*>(workspace);
    float* Xw = (float*)p; p += al((size_t)batch * L * d * 4);
    float* vec = (float*)p; p += al((size_t)batch * d * 4);
    float* prev_v = (float*)p; p += al((size_t)batch * d * 4);
    float* u = (float*)p; p += al((size_t)batch * L * 4);
    float* prev_u = (float*)p; p += al((size_t)batch * L * 4);
    float* scal = (float*)p; p += al((size_t)batch * 4);
    float* part_vv = (float*)p; p += al((size_t)batch * ncb * 4);
    float* part_v = (float*)p; p += al((size_t)batch * nwg * d * 4);
    float* part_uu = (float*)p;
    const int64_t n = (int64_t)batch * L * d;
    if (elem_bytes == 2)
        hipLaunchKernelGGL(alt_widen_kernel<bf16_t>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const bf16_t*)X, Xw, n);
    else
        hipLaunchKernelGGL(alt_widen_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const float*)X, Xw, n);
    const dim3 gs(nwg, batch), gr(ncb, batch);
    const dim3 ge((std::max(L, d) + 255) / 256, batch);
    auto emit = [&](int comp) {
        if (elem_bytes == 2)
            hipLaunchKernelGGL(alt_emit_kernel<bf16_t>, ge, dim3(256), 0, st, u, vec, scal, prev_u, prev_v, (bf16_t*)U, V0,
                               part_vv, ncb, L, d, r, comp);
        else
            hipLaunchKernelGGL(alt_emit_kernel<float>, ge, dim3(256), 0, st, u, vec, scal, prev_u, prev_v, (float*)U, V0,
                               part_vv, ncb, L, d, r, comp);
    };
    emit(-1);   // first start vector
    for (int i = 0; i < r; ++i) {
        for (int j = 0; j < sweeps; ++j) {
            const int deflate = (i > 0 && j == 0) ? 1 : 0;
            hipLaunchKernelGGL(alt_sweep_kernel, gs, dim3(256), 0, st, Xw, vec, part_vv, ncb, prev_u, prev_v, deflate, u,
                               part_v, part_uu, L, d);
            const int fin = (j == sweeps - 1) ? i : -1;
            if (elem_bytes == 2)
                hipLaunchKernelGGL(alt_reduce_kernel<bf16_t>, gr, dim3(256), 0, st, part_v, part_uu, nwg, vec, part_vv, scal,
                                   d, fin, (bf16_t*)B, r, info);
            else
                hipLaunchKernelGGL(alt_reduce_kernel<float>, gr, dim3(256), 0, st, part_v, part_uu, nwg, vec, part_vv, scal, d,
                                   fin, (float*)B, r, info);
        }
        emit(i);
    }
    return hipGetLastError();
}

}  // namespace atp
