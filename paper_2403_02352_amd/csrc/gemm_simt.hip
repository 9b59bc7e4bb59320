// Generic fp32-FMA GEMM with element strides:  C(m,n) = sum_k A(m,k) · B(n,k).
// Serves the ATP_F32 storage path (true fp32 arithmetic, 1e-4 parity) and every
// shape or alignment the MFMA kernel does not cover.  64×64 block tile, 16-deep
// k slices staged k-major in LDS, 4×4 register tile per thread.
#include "common.h"

namespace atp {
namespace {

template <typename T> __device__ __forceinline__ float ldf(const T* p);
template <> __device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ldf<bf16_t>(const bf16_t* p) { return bf2f(*p); }

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }

constexpr int SB = 64, SK = 16;

template <typename TA, typename TB, bool SWIGLU>
__global__ void __launch_bounds__(256) gemm_simt_kernel(SimtArgs p) {
    __shared__ float As[SK][SB + 1];
    __shared__ float Bs[SWIGLU ? 2 : 1][SK][SB + 1];
    const int bz = blockIdx.z;
    const TA* A = reinterpret_cast<const TA*>(p.A) + (int64_t)bz * p.sA;
    const TB* B = reinterpret_cast<const TB*>(p.B) + (int64_t)bz * p.sB;
    const TA* Alo = p.A_lo ? reinterpret_cast<const TA*>(p.A_lo) + (int64_t)bz * p.sA : nullptr;
    const TB* Blo = p.B_lo ? reinterpret_cast<const TB*>(p.B_lo) + (int64_t)bz * p.sB : nullptr;
    const int m0 = blockIdx.y * SB, n0 = blockIdx.x * SB;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {}, acc2[4][4] = {};
    for (int k0 = 0; k0 < p.K; k0 += SK) {
        for (int e = tid; e < SB * SK; e += 256) {
            int row, kk;
            // pick the loop order that walks memory contiguously
            if (p.a_cs == 1) { row = e / SK; kk = e % SK; } else { kk = e / SB; row = e % SB; }
            const int gm = m0 + row, gk = k0 + kk;
            float av = 0.f;
            if (gm < p.M && gk < p.K) {
                const int64_t o = (int64_t)gm * p.a_rs + (int64_t)gk * p.a_cs;
                av = ldf<TA>(A + o);
                if (Alo) av += ldf<TA>(Alo + o);
            }
            As[kk][row] = av;
        }
        for (int e = tid; e < SB * SK; e += 256) {
            int row, kk;
            if (p.b_cs == 1) { row = e / SK; kk = e % SK; } else { kk = e / SB; row = e % SB; }
            const int gn = n0 + row, gk = k0 + kk;
            const bool ok = gn < p.N && gk < p.K;
            float bv = 0.f;
            if (ok) {
                const int64_t o = (int64_t)gn * p.b_rs + (int64_t)gk * p.b_cs;
                bv = ldf<TB>(B + o);
                if (Blo) bv += ldf<TB>(Blo + o);
            }
            Bs[0][kk][row] = bv;
            if constexpr (SWIGLU)
                Bs[1][kk][row] = ok ? ldf<TB>(B + (int64_t)(gn + p.N) * p.b_rs + (int64_t)gk * p.b_cs) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < SK; ++kk) {
            float a[4], b[4], b2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                b[j] = Bs[0][kk][tx * 4 + j];
                if constexpr (SWIGLU) b2[j] = Bs[1][kk][tx * 4 + j];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
                    if constexpr (SWIGLU) acc2[i][j] = fmaf(a[i], b2[j], acc2[i][j]);
                }
        }
        __syncthreads();
    }
    float* C32 = p.C32 ? p.C32 + (int64_t)bz * p.sC : nullptr;
    bf16_t* C16 = p.C16 ? p.C16 + (int64_t)bz * p.sC : nullptr;
    float* CT32 = p.CT32 ? p.CT32 + (int64_t)bz * p.sCT : nullptr;
    bf16_t* CT16 = p.CT16 ? p.CT16 + (int64_t)bz * p.sCT : nullptr;
    bf16_t* C16lo = p.C16lo ? p.C16lo + (int64_t)bz * p.sC : nullptr;
    bf16_t* CT16lo = p.CT16lo ? p.CT16lo + (int64_t)bz * p.sCT : nullptr;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
            if (row < p.M && col < p.N) {
                float o = acc[i][j];
                if constexpr (SWIGLU) o = silu_f(o) * acc2[i][j];
                if (C32) C32[(int64_t)row * p.ldc + col] = o;
                const bf16_t h = f2bf(o);
                const bf16_t l = f2bf(o - bf2f(h));
                if (C16) C16[(int64_t)row * p.ldc + col] = h;
                if (C16lo) C16lo[(int64_t)row * p.ldc + col] = l;
                if (CT32) CT32[(int64_t)col * p.ldct + row] = o;
                if (CT16) CT16[(int64_t)col * p.ldct + row] = h;
                if (CT16lo) CT16lo[(int64_t)col * p.ldct + row] = l;
            }
        }
}

template <typename TA, typename TB>
hipError_t launch_simt(hipStream_t st, const SimtArgs& g) {
    dim3 grid((g.N + SB - 1) / SB, (g.M + SB - 1) / SB, g.batch);
    if (g.swiglu)
        hipLaunchKernelGGL((gemm_simt_kernel<TA, TB, true>), grid, dim3(256), 0, st, g);
    else
        hipLaunchKernelGGL((gemm_simt_kernel<TA, TB, false>), grid, dim3(256), 0, st, g);
    return hipGetLastError();
}

}  // namespace

hipError_t gemm_simt(hipStream_t st, OperandType ta, OperandType tb, const SimtArgs& g) {
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
    if (g.batch > 65535 || (g.M + SB - 1) / SB > 65535) return hipErrorInvalidValue;
    if (ta == OP_F32 && tb == OP_F32) return launch_simt<float, float>(st, g);
    if (ta == OP_BF16 && tb == OP_BF16) return launch_simt<bf16_t, bf16_t>(st, g);
    if (ta == OP_BF16 && tb == OP_F32) return launch_simt<bf16_t, float>(st, g);
    return launch_simt<float, bf16_t>(st, g);
}

}  // namespace atp
