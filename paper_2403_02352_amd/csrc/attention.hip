// Softmax attention of all L queries over n_k keys/values (Fig.2b, Tab.1 row
// "Attention"; Eq.1 with K', V' in place of K, V).  n_k = r on the ATP path,
// n_k = L for the dense comparator.  The L×n_k score matrix lives only in
// registers: scores of a 64-key tile come out of the MFMA unit, the online
// softmax (running row max and row sum) is applied in registers, and the
// probabilities feed the value MFMA directly.
//
// bf16 kernel layout trick: the score tile is computed transposed,
// Sᵀ = K'·Qᵀ, so that every lane owns ONE query column (all 16 accumulator
// registers of a 32×32 MFMA tile belong to the same query).  Row max / row sum
// are then in-lane reductions plus one exchange between the two lane halves,
// and the probabilities are already laid out as the B operand of
// Oᵀ += V'ᵀ·Pᵀ.  Rows of the K' tile are fetched in a permuted order (bits 2 and
// 3 of the row index swapped) so that the 8 consecutive accumulator registers a
// lane feeds to the second MFMA correspond to 8 consecutive keys, i.e. to one
// 16-byte read of the transposed value tile.
#include "common.h"

namespace atp {
namespace {

__device__ __forceinline__ bf16x8 u4_as_bf16x8(const uint4& u) {
    union { uint4 u; bf16x8 b; } c;
    c.u = u;
    return c.b;
}

constexpr int QT = 128;  // queries per workgroup (4 waves × 32)
constexpr int KT = 64;   // keys per tile

template <int DH>
__global__ void __launch_bounds__(256) attn_bf16_kernel(AttnArgs a, float c_log2e) {
    constexpr int CK = DH / 8;   // 16-byte chunks per K-tile row
    constexpr int NKS = DH / 16; // k-steps of the score MFMA
    constexpr int NCT = DH / 32; // 32-row tiles of Oᵀ
    constexpr int LK = (KT * CK) / 256;  // K chunks per thread
    constexpr int LV = (DH * 8) / 256;   // Vᵀ chunks per thread (8 chunks per row of 64 keys)
    __shared__ __align__(16) uint4 sK[KT * CK];
    __shared__ __align__(16) uint4 sV[DH * 8];

    const int b = blockIdx.z, h = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int q = blockIdx.x * QT + wave * 32 + l32;
    const bf16_t* Qp = reinterpret_cast<const bf16_t*>(a.Q) + ((int64_t)b * a.L) * a.dq + h * DH;
    const bf16_t* Kp = reinterpret_cast<const bf16_t*>(a.K) + ((int64_t)b * a.nk) * a.dq + h * DH;
    const bf16_t* Vp = reinterpret_cast<const bf16_t*>(a.Vt) + ((int64_t)b * a.dq + h * DH) * a.nk_pad;

    // query fragments (B operand of the score MFMA): 8 consecutive features per lane and k-step
    bf16x8 qf[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (q < a.L) v = *reinterpret_cast<const uint4*>(Qp + (int64_t)q * a.dq + ks * 16 + lh * 8);
        qf[ks] = u4_as_bf16x8(v);
    }

    f32x16 o[NCT];
#pragma unroll
    for (int i = 0; i < NCT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    uint4 rk[LK], rv[LV];
    auto load_tiles = [&](int kt0) {
#pragma unroll
        for (int i = 0; i < LK; ++i) {
            const int c = tid + i * 256;
            const int row = c / CK, kc = c % CK;
            const int key = kt0 + row;
            rk[i] = (key < a.nk) ? *reinterpret_cast<const uint4*>(Kp + (int64_t)key * a.dq + kc * 8)
                                 : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < LV; ++i) {
            const int c = tid + i * 256;
            const int row = c >> 3, kc = c & 7;
            rv[i] = *reinterpret_cast<const uint4*>(Vp + (int64_t)row * a.nk_pad + kt0 + kc * 8);
        }
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int i = 0; i < LK; ++i) {
            const int c = tid + i * 256;
            const int row = c / CK, kc = c % CK;
            sK[row * CK + (kc ^ (row & 7))] = rk[i];
        }
#pragma unroll
        for (int i = 0; i < LV; ++i) {
            const int c = tid + i * 256;
            const int row = c >> 3, kc = c & 7;
            sV[row * 8 + (kc ^ (row & 7))] = rv[i];
        }
    };

    // S-tile row i holds key perm(i): bits 2 and 3 swapped
    const int prow = (l32 & ~0xC) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);

    const int ntiles = (a.nk + KT - 1) / KT;
    load_tiles(0);
    for (int kt = 0; kt < ntiles; ++kt) {
        const int kt0 = kt * KT;
        store_tiles();
        __syncthreads();
        if (kt + 1 < ntiles) load_tiles(kt0 + KT);

        // ---- scores: Sᵀ[key, query] ------------------------------------------------
        f32x16 s[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[t][v] = 0.f;
            const int row = 32 * t + prow;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const int kc = 2 * ks + lh;
                const bf16x8 kf = u4_as_bf16x8(sK[row * CK + (kc ^ (row & 7))]);
                s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[t], 0, 0, 0);
            }
        }
        // ---- mask ragged tail, running max --------------------------------------
        float mloc = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = kt0 + 32 * t + 16 * (v >> 3) + 8 * lh + (v & 7);
                if (key >= a.nk) s[t][v] = -INFINITY;
                mloc = fmaxf(mloc, s[t][v]);
            }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run, mloc);
        const float alpha = exp2f((m_run - m_new) * c_log2e);
        const float mc = m_new * c_log2e;
        float psum = 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float pv = exp2f(fmaf(s[t][v], c_log2e, -mc));
                s[t][v] = pv;
                psum += pv;
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int i = 0; i < NCT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[i][v] *= alpha;

        // ---- Oᵀ += V'ᵀ · Pᵀ ---------------------------------------------------------
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                uint4 pu;
                pu.x = pack_bf2(s[t][8 * tt + 0], s[t][8 * tt + 1]);
                pu.y = pack_bf2(s[t][8 * tt + 2], s[t][8 * tt + 3]);
                pu.z = pack_bf2(s[t][8 * tt + 4], s[t][8 * tt + 5]);
                pu.w = pack_bf2(s[t][8 * tt + 6], s[t][8 * tt + 7]);
                const bf16x8 pf = u4_as_bf16x8(pu);
                const int kc = 4 * t + 2 * tt + lh;
#pragma unroll
                for (int i = 0; i < NCT; ++i) {
                    const int row = 32 * i + l32;
                    const bf16x8 vf = u4_as_bf16x8(sV[row * 8 + (kc ^ (row & 7))]);
                    o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[i], 0, 0, 0);
                }
            }
        __syncthreads();
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.0f / l_tot;
    if (q < a.L) {
        bf16_t* Op = reinterpret_cast<bf16_t*>(a.O) + ((int64_t)b * a.L + q) * a.dq + h * DH;
#pragma unroll
        for (int i = 0; i < NCT; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int c = 32 * i + 8 * g + 4 * lh;
                uint2 w;
                w.x = pack_bf2(o[i][4 * g + 0] * inv, o[i][4 * g + 1] * inv);
                w.y = pack_bf2(o[i][4 * g + 2] * inv, o[i][4 * g + 3] * inv);
                *reinterpret_cast<uint2*>(Op + c) = w;
            }
    }
}

// ---------------------------------------------------------------------------
// fp32 storage path: one wave per query row, features spread over the lanes,
// scalar online softmax over the keys.  True fp32 arithmetic throughout.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) attn_f32_kernel(AttnArgs a, int dh) {
    const int b = blockIdx.z, h = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = blockIdx.x * 4 + wave;
    if (q >= a.L) return;
    const float* Qp = reinterpret_cast<const float*>(a.Q) + ((int64_t)b * a.L + q) * a.dq + h * dh;
    const float* Kp = reinterpret_cast<const float*>(a.K) + ((int64_t)b * a.nk) * a.dq + h * dh;
    const float* Vp = reinterpret_cast<const float*>(a.V) + ((int64_t)b * a.nk) * a.dq + h * dh;
    float qv[4], ov[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = lane + 64 * i;
        qv[i] = (c < dh) ? Qp[c] * a.scale : 0.f;
        ov[i] = 0.f;
    }
    float m_run = -INFINITY, l_run = 0.f;
    for (int j = 0; j < a.nk; ++j) {
        const float* kr = Kp + (int64_t)j * a.dq;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = lane + 64 * i;
            if (c < dh) s = fmaf(qv[i], kr[c], s);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        const float m_new = fmaxf(m_run, s);
        const float alpha = expf(m_run - m_new);
        const float p = expf(s - m_new);
        l_run = l_run * alpha + p;
        m_run = m_new;
        const float* vr = Vp + (int64_t)j * a.dq;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = lane + 64 * i;
            if (c < dh) ov[i] = fmaf(p, vr[c], ov[i] * alpha);
        }
    }
    float* Op = reinterpret_cast<float*>(a.O) + ((int64_t)b * a.L + q) * a.dq + h * dh;
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = lane + 64 * i;
        if (c < dh) Op[c] = ov[i] * inv;
    }
}

}  // namespace

hipError_t attention_bf16(hipStream_t st, const AttnArgs& a) {
    const int dh = a.dq / a.heads;
    dim3 grid((a.L + QT - 1) / QT, a.heads, a.batch);
    if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;
    const float c = a.scale * 1.4426950408889634f;
    if (dh == 128)
        hipLaunchKernelGGL(attn_bf16_kernel<128>, grid, dim3(256), 0, st, a, c);
    else if (dh == 64)
        hipLaunchKernelGGL(attn_bf16_kernel<64>, grid, dim3(256), 0, st, a, c);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t attention_f32(hipStream_t st, const AttnArgs& a) {
    const int dh = a.dq / a.heads;
    if (dh > 256) return hipErrorInvalidValue;
    dim3 grid((a.L + 3) / 4, a.heads, a.batch);
    if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_f32_kernel, grid, dim3(256), 0, st, a, dh);
    return hipGetLastError();
}

}  // namespace atp
