// HBM-bound streaming passes: batched transposes (operand twins for the
// K-contiguous GEMM kernel, per-head value re-layout for the attention kernel),
// casts, fills and the counter-based Gaussian generator of the start block.
#include "common.h"

namespace atp {
namespace {

constexpr int TT = 64;  // transpose tile

// out[b][c][r] = in[b][r][c]; out rows have length ld_out (>= rows); when zero_pad is set the
// columns rows..ld_out-1 of out are written with zeros.
template <typename T>
__global__ void __launch_bounds__(256) transpose_kernel(const T* __restrict__ in, T* __restrict__ out, int rows,
                                                        int cols, int64_t ld_out, int64_t s_in, int64_t s_out,
                                                        int zero_pad) {
    __shared__ T tile[TT][TT + 2];
    const int b = blockIdx.z;
    const T* src = in + (int64_t)b * s_in;
    T* dst = out + (int64_t)b * s_out;
    const int r0 = blockIdx.y * TT, c0 = blockIdx.x * TT;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 × 4
    for (int i = ty; i < TT; i += 4) {
        const int r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < rows && c < cols) ? src[(int64_t)r * cols + c] : (T)0;
    }
    __syncthreads();
    const int out_cols = zero_pad ? (int)ld_out : rows;
    for (int i = ty; i < TT; i += 4) {
        const int c = c0 + i, r = r0 + tx;
        if (c < cols && r < out_cols) dst[(int64_t)c * ld_out + r] = tile[tx][i];
    }
}

// Same operation for 2-byte elements when every extent is a multiple of 8: global traffic moves as
// 16-byte pieces (8 elements) on both sides, the 64×64 tile turns in LDS.
__global__ void __launch_bounds__(256) transpose_u16x8_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ out,
                                                              int rows, int cols, int64_t ld_out, int64_t s_in,
                                                              int64_t s_out, int zero_pad) {
    __shared__ __align__(16) uint16_t tile[TT][TT + 2];
    const int b = blockIdx.z;
    const uint16_t* src = in + (int64_t)b * s_in;
    uint16_t* dst = out + (int64_t)b * s_out;
    const int r0 = blockIdx.y * TT, c0 = blockIdx.x * TT;
    for (int v = threadIdx.x; v < TT * 8; v += 256) {
        const int i = v >> 3, q = v & 7;
        const int r = r0 + i, c = c0 + 8 * q;
        uint4 x = make_uint4(0u, 0u, 0u, 0u);
        if (r < rows && c < cols) x = *reinterpret_cast<const uint4*>(src + (int64_t)r * cols + c);
        uint32_t* d = reinterpret_cast<uint32_t*>(&tile[i][8 * q]);
        d[0] = x.x; d[1] = x.y; d[2] = x.z; d[3] = x.w;
    }
    __syncthreads();
    const int out_cols = zero_pad ? (int)ld_out : rows;
    for (int v = threadIdx.x; v < TT * 8; v += 256) {
        const int i = v >> 3, q = v & 7;
        const int c = c0 + i, r = r0 + 8 * q;
        if (c < cols && r < out_cols) {
            uint4 x;
            x.x = (uint32_t)tile[8 * q + 0][i] | ((uint32_t)tile[8 * q + 1][i] << 16);
            x.y = (uint32_t)tile[8 * q + 2][i] | ((uint32_t)tile[8 * q + 3][i] << 16);
            x.z = (uint32_t)tile[8 * q + 4][i] | ((uint32_t)tile[8 * q + 5][i] << 16);
            x.w = (uint32_t)tile[8 * q + 6][i] | ((uint32_t)tile[8 * q + 7][i] << 16);
            *reinterpret_cast<uint4*>(dst + (int64_t)c * ld_out + r) = x;
        }
    }
}

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

// Element i is a function of (seed, i) only: 64 hashed bits -> two uniforms -> Box–Muller.
__global__ void gaussian_kernel(float* out, int64_t n, uint64_t seed) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint64_t h = mix64(mix64(seed) + 0x9e3779b97f4a7c15ull * (uint64_t)(i + 1));
    const float u1 = ((float)(uint32_t)(h >> 40) + 0.5f) * (1.0f / 16777216.0f);        // 24 bits, (0,1)
    const float u2 = ((float)(uint32_t)((h >> 16) & 0xffffffu) + 0.5f) * (1.0f / 16777216.0f);
    out[i] = sqrtf(-2.0f * logf(u1)) * cosf(6.28318530717958647692f * u2);
}

__global__ void zero_i32_kernel(int32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ void cast_kernel(const float* __restrict__ in, bf16_t* __restrict__ out, int64_t n) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i + 3 < n) {
        const float4 v = *reinterpret_cast<const float4*>(in + i);
        uint2 o;
        o.x = pack_bf2(v.x, v.y);
        o.y = pack_bf2(v.z, v.w);
        *reinterpret_cast<uint2*>(out + i) = o;
    } else {
        for (int64_t j = i; j < n; ++j) out[j] = f2bf(in[j]);
    }
}

// Rotary position encoding, half-split pairing: within a head of width dh, coordinate j < dh/2 of
// row i is paired with j + dh/2 and the pair is rotated by (pos0 + i)·base^(-2j/dh).
template <typename T>
__global__ void __launch_bounds__(256) rope_kernel(const T* __restrict__ in, T* __restrict__ out, int L, int dq, int dh,
                                                   float log2_base, int pos0) {
    const int b = blockIdx.y;
    const int half = dh >> 1;
    const int pb = (dq / 2 + 255) / 256;            // workgroups per row
    const int i = blockIdx.x / pb;
    const int p = (blockIdx.x % pb) * 256 + threadIdx.x;   // pair index within the row
    if (p >= dq / 2) return;
    const int h = p / half, j = p % half;
    const int64_t o = ((int64_t)b * L + i) * dq + h * dh + j;
    const float freq = exp2f(-2.0f * (float)j / (float)dh * log2_base);
    float sn, cs;
    sincosf((float)(pos0 + i) * freq, &sn, &cs);
    float x, y;
    if constexpr (sizeof(T) == 2) { x = bf2f(in[o]); y = bf2f(in[o + half]); } else { x = in[o]; y = in[o + half]; }
    const float ox = x * cs - y * sn, oy = x * sn + y * cs;
    if constexpr (sizeof(T) == 2) { out[o] = f2bf(ox); out[o + half] = f2bf(oy); } else { out[o] = ox; out[o + half] = oy; }
}


// out[b][i][c_off + j] = in[b][i][j]: rows×cols block copied into a wider (or taller) matrix; 2- or 4-byte elements
template <typename T>
__global__ void __launch_bounds__(256) copy_block_kernel(const T* __restrict__ in, T* __restrict__ out, int rows, int cols,
                                                         int64_t ld_in, int64_t ld_out, int64_t s_in, int64_t s_out) {
    const int b = blockIdx.z, i = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (i >= rows || j >= cols) return;
    out[(int64_t)b * s_out + (int64_t)i * ld_out + j] = in[(int64_t)b * s_in + (int64_t)i * ld_in + j];
}

// Row-wise normalisation carried through a factored matrix H = P·C (one workgroup per row).
// Coefficient side: Cc[j][:] = C[j][:] - mean_j (mean removed only when `center`), Cn = Cc · diag(gain).
template <typename T>
__global__ void __launch_bounds__(256) norm_coeff_kernel(const T* __restrict__ C, const float* __restrict__ gain,
                                                         T* __restrict__ Cc, T* __restrict__ Cn, int d, int center) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const T* src = C + row * d;
    float mean = 0.f;
    if (center) {
        float s = 0.f;
        for (int j = threadIdx.x; j < d; j += 256) {
            if constexpr (sizeof(T) == 2) s += bf2f(src[j]); else s += src[j];
        }
        for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
        __syncthreads();
        mean = (red[0] + red[1] + red[2] + red[3]) / (float)d;
    }
    for (int j = threadIdx.x; j < d; j += 256) {
        float x;
        if constexpr (sizeof(T) == 2) x = bf2f(src[j]); else x = src[j];
        x -= mean;
        if constexpr (sizeof(T) == 2) { Cc[row * d + j] = f2bf(x); Cn[row * d + j] = f2bf(x * gain[j]); }
        else { Cc[row * d + j] = x; Cn[row * d + j] = x * gain[j]; }
    }
}

// Basis side: var_i = (1/d)·p_i·M·p_iᵀ with T = P·M given; Pn[i][:] = P[i][:] / sqrt(var_i + eps).
template <typename T>
__global__ void __launch_bounds__(256) norm_basis_kernel(const T* __restrict__ P, const float* __restrict__ PM,
                                                         T* __restrict__ Pn, int m, float inv_d, float eps) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const T* p = P + row * m;
    const float* t = PM + row * m;
    float s = 0.f;
    for (int j = threadIdx.x; j < m; j += 256) {
        float x;
        if constexpr (sizeof(T) == 2) x = bf2f(p[j]); else x = p[j];
        s += x * t[j];
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    const float var = fmaxf((red[0] + red[1] + red[2] + red[3]) * inv_d, 0.f);
    const float sc = 1.0f / sqrtf(var + eps);
    for (int j = threadIdx.x; j < m; j += 256) {
        if constexpr (sizeof(T) == 2) Pn[row * m + j] = f2bf(bf2f(p[j]) * sc); else Pn[row * m + j] = p[j] * sc;
    }
}

}  // namespace

hipError_t copy_block(hipStream_t st, const void* in, void* out, int rows, int cols, int64_t ld_in, int64_t ld_out,
                      int64_t s_in, int64_t s_out, int batch, int elem_bytes) {
    if (rows <= 0 || cols <= 0 || batch <= 0) return hipSuccess;
    dim3 grid((cols + 255) / 256, rows, batch);
    if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;   // the callers check their sizes against this
    if (elem_bytes == 2)
        hipLaunchKernelGGL(copy_block_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)in, (uint16_t*)out, rows, cols,
                           ld_in, ld_out, s_in, s_out);
    else
        hipLaunchKernelGGL(copy_block_kernel<uint32_t>, grid, dim3(256), 0, st, (const uint32_t*)in, (uint32_t*)out, rows, cols,
                           ld_in, ld_out, s_in, s_out);
    return hipGetLastError();
}

hipError_t norm_coeff(hipStream_t st, const void* C, const float* gain, void* Cc, void* Cn, int64_t rows, int d, int center,
                      int elem_bytes) {
    if (rows <= 0) return hipSuccess;
    if (rows > 0x7fffffff) return hipErrorInvalidValue;
    if (elem_bytes == 2)
        hipLaunchKernelGGL(norm_coeff_kernel<bf16_t>, dim3((unsigned)rows), dim3(256), 0, st, (const bf16_t*)C, gain, (bf16_t*)Cc,
                           (bf16_t*)Cn, d, center);
    else
        hipLaunchKernelGGL(norm_coeff_kernel<float>, dim3((unsigned)rows), dim3(256), 0, st, (const float*)C, gain, (float*)Cc,
                           (float*)Cn, d, center);
    return hipGetLastError();
}

hipError_t norm_basis(hipStream_t st, const void* P, const float* PM, void* Pn, int64_t rows, int m, int d, float eps,
                      int elem_bytes) {
    if (rows <= 0) return hipSuccess;
    if (rows > 0x7fffffff) return hipErrorInvalidValue;
    if (elem_bytes == 2)
        hipLaunchKernelGGL(norm_basis_kernel<bf16_t>, dim3((unsigned)rows), dim3(256), 0, st, (const bf16_t*)P, PM, (bf16_t*)Pn, m,
                           1.0f / (float)d, eps);
    else
        hipLaunchKernelGGL(norm_basis_kernel<float>, dim3((unsigned)rows), dim3(256), 0, st, (const float*)P, PM, (float*)Pn, m,
                           1.0f / (float)d, eps);
    return hipGetLastError();
}

hipError_t rope_rows(hipStream_t st, const void* in, void* out, int batch, int L, int dq, int dh, float base, int pos0,
                     int elem_bytes) {
    const int64_t nx = (int64_t)L * ((dq / 2 + 255) / 256);
    if (nx > 0x7fffffff || batch > 65535) return hipErrorInvalidValue;
    dim3 grid((unsigned)nx, batch);
    const float lb = log2f(base);
    if (elem_bytes == 2)
        hipLaunchKernelGGL(rope_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)in, (bf16_t*)out, L, dq, dh, lb, pos0);
    else
        hipLaunchKernelGGL(rope_kernel<float>, grid, dim3(256), 0, st, (const float*)in, (float*)out, L, dq, dh, lb, pos0);
    return hipGetLastError();
}

hipError_t transpose_batched(hipStream_t st, const void* in, void* out, int rows, int cols, int64_t ld_out,
                             int64_t s_in, int64_t s_out, int batch, int elem_bytes, int zero_pad) {
    if (rows <= 0 || cols <= 0 || batch <= 0) return hipSuccess;
    const int span = zero_pad ? (int)ld_out : rows;
    dim3 grid((cols + TT - 1) / TT, (span + TT - 1) / TT, batch);
    if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;
    const bool vec8 = elem_bytes == 2 && rows % 8 == 0 && cols % 8 == 0 && ld_out % 8 == 0 && s_in % 8 == 0 &&
                      s_out % 8 == 0 && ((((uintptr_t)in) | ((uintptr_t)out)) & 15) == 0;
    if (vec8)
        hipLaunchKernelGGL(transpose_u16x8_kernel, grid, dim3(256), 0, st, (const uint16_t*)in, (uint16_t*)out, rows, cols,
                           ld_out, s_in, s_out, zero_pad);
    else if (elem_bytes == 2)
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)in, (uint16_t*)out,
                           rows, cols, ld_out, s_in, s_out, zero_pad);
    else
        hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, st, (const uint32_t*)in, (uint32_t*)out,
                           rows, cols, ld_out, s_in, s_out, zero_pad);
    return hipGetLastError();
}

hipError_t fill_gaussian(hipStream_t st, float* out, int64_t n, uint64_t seed) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(gaussian_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, out, n, seed);
    return hipGetLastError();
}

hipError_t fill_zero_i32(hipStream_t st, int32_t* p, int64_t n) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n);
    return hipGetLastError();
}

hipError_t cast_f32_to_bf16(hipStream_t st, const float* in, bf16_t* out, int64_t n) {
    if (n <= 0) return hipSuccess;
    const int64_t nt = (n + 3) / 4;
    hipLaunchKernelGGL(cast_kernel, dim3((unsigned)((nt + 255) / 256)), dim3(256), 0, st, in, out, n);
    return hipGetLastError();
}

}  // namespace atp
