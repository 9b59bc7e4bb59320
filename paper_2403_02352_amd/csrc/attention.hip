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


// Tiles sit in LDS as plain rows of W 16-byte chunks (W = 16, 8 or 4); position p of row r holds chunk
// p ^ tile_swz<W>(r).  A 16-byte-per-lane LDS read is served 16 lanes at a time (16 × 16 B = all 64
// banks), and the 16 lanes of such a group read the same chunk of 16 consecutive rows (in some
// order): 16/W rows share one 256-byte bank span, so the swizzle counts those spans.
template <int W>
__device__ __forceinline__ int tile_swz(int r) {
    static_assert(W == 16 || W == 8 || W == 4, "row width");
    return W == 16 ? (r & 15) : W == 8 ? ((r >> 1) & 7) : ((r >> 2) & 3);
}

// The key/value tiles travel global -> LDS with asynchronous 16-byte copies (no registers), two
// stages: the copies of tile t+1 fly while tile t is multiplied.  Consecutive lanes of a copy
// fetch consecutive chunks of one row.
// LIN selects the first-order variant (Eq.8): the weight of key j is (1·U)_j + scale·<q, k_j>, no
// exponential and no running maximum; the normaliser is accumulated beside the numerator.
// KT = keys per tile (64, or 32: half the LDS and fewer live registers, so more workgroups per CU).
template <int DH, bool LIN, int KT>
__global__ void __launch_bounds__(256, KT == 32 ? 3 : 2) attn_bf16_kernel(AttnArgs a, float c_log2e) {
    constexpr int CK = DH / 8;            // 16-byte chunks per K-tile row
    constexpr int NKS = DH / 16;          // k-steps of the score MFMA
    constexpr int NCT = DH / 32;          // 32-row tiles of Oᵀ
    constexpr int NT = KT / 32;           // 32-key score tiles per key tile
    constexpr int KRPI = 64 / CK;         // K rows per copy instruction
    constexpr int NKI = KT / KRPI / 4;    // K copy instructions per wave and tile
    constexpr int VC = KT / 8;            // 16-byte chunks per Vᵀ-tile row
    constexpr int VRPI = 64 / VC;         // Vᵀ rows per copy instruction
    constexpr int NVI = DH / VRPI / 4;    // Vᵀ copy instructions per wave and tile
    static_assert(NKI >= 1 && NVI >= 1, "tile too small for four waves");
    __shared__ __align__(16) uint4 sK0[KT * CK];
    __shared__ __align__(16) uint4 sK1[KT * CK];
    __shared__ __align__(16) uint4 sV0[DH * VC];
    __shared__ __align__(16) uint4 sV1[DH * VC];

    // 1-D grid over (batch item, head, query block).  Consecutive workgroup ids go to the 8 XCDs in
    // turn: all query blocks of one (item, head) are given to one XCD, whose L2 then serves the
    // re-reads of that head's keys and values.
    const int nqb = (a.L + QT - 1) / QT, nbh = a.batch * a.heads;
    int bh, qb;
    if ((nbh & 7) == 0) {
        const int slot = blockIdx.x >> 3;
        bh = (blockIdx.x & 7) + 8 * (slot / nqb);
        qb = slot % nqb;
    } else {
        bh = blockIdx.x / nqb;
        qb = blockIdx.x % nqb;
    }
    const int b = bh / a.heads, h = bh % a.heads;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int q = qb * QT + wave * 32 + l32;
    const bf16_t* Qp = reinterpret_cast<const bf16_t*>(a.Q) + ((int64_t)b * a.L) * a.dq + h * DH;
    const bf16_t* Kp = reinterpret_cast<const bf16_t*>(a.K) + ((int64_t)b * a.nk) * a.dq + h * DH;
    const bf16_t* Vp = reinterpret_cast<const bf16_t*>(a.Vt) + ((int64_t)b * a.dq + h * DH) * a.nk_pad;
    const float* csum = LIN ? a.colsum + (int64_t)b * a.nk_pad : nullptr;

    // per-lane pieces of the copy addresses
    int k_row[NKI];
    unsigned k_chunk[NKI], v_off[NVI];   // byte offsets
#pragma unroll
    for (int i = 0; i < NKI; ++i) {
        const int row = (i * 4 + wave) * KRPI + lane / CK;
        k_row[i] = row;
        k_chunk[i] = (unsigned)(((lane % CK) ^ tile_swz<CK>(row)) * 16);
    }
#pragma unroll
    for (int i = 0; i < NVI; ++i) {
        const int row = (i * 4 + wave) * VRPI + lane / VC;
        v_off[i] = (unsigned)(((int64_t)row * a.nk_pad + (((lane % VC) ^ tile_swz<VC>(row)) * 8)) * 2);
    }
    // LDS byte address of this wave's first copy slot in each stage array (scalar registers); every
    // copy is a scalar base plus a 32-bit lane offset, untracked by the compiler: all waits for them
    // are explicit
    const unsigned wave_s = (unsigned)__builtin_amdgcn_readfirstlane(wave) * 1024u;
    const unsigned lK0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void*)sK0) + wave_s;
    const unsigned lK1 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void*)sK1) + wave_s;
    const unsigned lV0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void*)sV0) + wave_s;
    const unsigned lV1 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void*)sV1) + wave_s;
    const unsigned row_bytes = (unsigned)a.dq * 2u;
    auto issue = [&](int kt0, const uint4* sK, const uint4*) {
        const unsigned lk = (sK == sK0) ? lK0 : lK1, lv = (sK == sK0) ? lV0 : lV1;
#pragma unroll
        for (int i = 0; i < NKI; ++i) {
            const int key = min(kt0 + k_row[i], a.nk - 1);  // rows past the end: any valid row, masked below
            copy16_untracked(Kp, (unsigned)key * row_bytes + k_chunk[i], lk + (unsigned)i * 4096u);
        }
#pragma unroll
        for (int i = 0; i < NVI; ++i) copy16_untracked(Vp + kt0, v_off[i], lv + (unsigned)i * 4096u);
    };

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

    // S-tile row i holds key perm(i): bits 2 and 3 swapped
    const int prow = (l32 & ~0xC) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    const int pswz = tile_swz<CK>(prow);

    auto compute = [&](int kt0, const uint4* sK, const uint4* sV) {
        // ---- scores: Sᵀ[key, query] ------------------------------------------------
        f32x16 s[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[t][v] = 0.f;
            const int row = 32 * t + prow;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const bf16x8 kf = u4_as_bf16x8(sK[row * CK + ((2 * ks + lh) ^ pswz)]);
                s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[t], 0, 0, 0);
            }
        }
        if constexpr (LIN) {
            // weights (1·U)_key + scale·s; keys past the end weigh nothing.  The 8 consecutive
            // accumulator registers of a lane are 8 consecutive keys.
            float acc_den = 0.f;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    const int key0 = kt0 + 32 * t + 16 * g + 8 * lh;
                    const f32x4 c0 = *reinterpret_cast<const f32x4*>(csum + key0);
                    const f32x4 c1 = *reinterpret_cast<const f32x4*>(csum + key0 + 4);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float cj = e < 4 ? c0[e] : c1[e - 4];
                        const float sv = s[t][8 * g + e] * c_log2e;   // c_log2e carries the plain scale here
                        const bool live = (key0 + e) < a.nk;
                        const float pv = live ? cj + sv : 0.f;
                        acc_den += a.norm_rowsum ? pv : (live ? sv * cj : 0.f);
                        s[t][8 * g + e] = pv;
                    }
                }
            l_run += acc_den;
        } else {
            if (kt0 + KT > a.nk) {  // only the last tile can be ragged
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = kt0 + 32 * t + 16 * (v >> 3) + 8 * lh + (v & 7);
                        if (key >= a.nk) s[t][v] = -INFINITY;
                    }
            }
            float mloc = -INFINITY;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) mloc = fmaxf(mloc, s[t][v]);
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
            const float m_new = fmaxf(m_run, mloc);
            // the running maximum settles after a few tiles: rescale only when some query of this wave
            // raised it (the factor is exactly 1 otherwise)
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2e);
                l_run *= alpha;
#pragma unroll
                for (int i = 0; i < NCT; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[i][v] *= alpha;
                m_run = m_new;
            }
            const float mc = m_run * c_log2e;
            float psum = 0.f;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(s[t][v], c_log2e, -mc));
                    s[t][v] = pv;
                    psum += pv;
                }
            l_run += psum;
        }

        // ---- Oᵀ += V'ᵀ · Pᵀ ---------------------------------------------------------
#pragma unroll
        for (int t = 0; t < NT; ++t)
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
                    const bf16x8 vf = u4_as_bf16x8(sV[row * VC + (kc ^ tile_swz<VC>(row))]);
                    o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[i], 0, 0, 0);
                }
            }
    };

    const int ntiles = (a.nk + KT - 1) / KT;
    issue(0, sK0, sV0);
    for (int kt = 0; kt < ntiles; kt += 2) {
        // the explicit vmcnt(0) makes this wave's copies of tile kt land before the barrier (the
        // compiler does not count asynchronous LDS copies as something a barrier has to wait for)
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();  // everybody's copies have landed; stage 1 is free
        if (kt + 1 < ntiles) issue((kt + 1) * KT, sK1, sV1);
        compute(kt * KT, sK0, sV0);
        if (kt + 1 < ntiles) {
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            if (kt + 2 < ntiles) issue((kt + 2) * KT, sK0, sV0);
            compute((kt + 1) * KT, sK1, sV1);
        }
    }
    __syncthreads();

    // ---- normalise; the output tile turns in a wave-private LDS tile [32 queries][DH + 8] so that
    //      each query row leaves as 16-byte pieces -------------------------------------------------
    float l_tot = l_run + __shfl_xor(l_run, 32);
    if (LIN && !a.norm_rowsum) l_tot += a.n_tokens;
    const float inv = 1.0f / l_tot;
    // (row pitch DH elements; 16-byte piece p of query row q sits at piece p ^ (q & (DH/8 - 1)))
    static_assert(32 * DH * 2 <= KT * CK * 16 && 32 * DH * 2 <= DH * VC * 16, "output staging: one stage array per wave");
    bf16_t* ob = reinterpret_cast<bf16_t*>(wave == 0 ? sK0 : wave == 1 ? sK1 : wave == 2 ? sV0 : sV1);
#pragma unroll
    for (int i = 0; i < NCT; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint2 w;
            w.x = pack_bf2(o[i][4 * g + 0] * inv, o[i][4 * g + 1] * inv);
            w.y = pack_bf2(o[i][4 * g + 2] * inv, o[i][4 * g + 3] * inv);
            const int piece = (4 * i + g) ^ (l32 & (DH / 8 - 1));   // features 32i + 8g + 4lh .. +3 live in piece 4i + g
            *reinterpret_cast<uint2*>(ob + l32 * DH + piece * 8 + 4 * lh) = w;
        }
    constexpr int CPQ = DH / 8;  // 16-byte pieces per query row
#pragma unroll
    for (int it = 0; it < 32 * CPQ / 64; ++it) {
        const int c = it * 64 + lane, qq = c / CPQ, part = c % CPQ;
        const int qg = qb * QT + wave * 32 + qq;
        const uint4 v = *reinterpret_cast<const uint4*>(ob + qq * DH + (part ^ (qq & (CPQ - 1))) * 8);
        if (qg < a.L)
            *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(a.O) + ((int64_t)b * a.L + qg) * a.dq + h * DH + part * 8) = v;
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
    if (a.linearised) {
        // first-order variant (Eq.8): weight (1·U)_j + scale·<q, k_j>
        const float* csum = a.colsum + (int64_t)b * a.nk_pad;
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
            const float cj = csum[j];
            const float p = cj + s;
            l_run += a.norm_rowsum ? p : s * cj;
            const float* vr = Vp + (int64_t)j * a.dq;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = lane + 64 * i;
                if (c < dh) ov[i] = fmaf(p, vr[c], ov[i]);
            }
        }
        if (!a.norm_rowsum) l_run += a.n_tokens;
        float* Ol = reinterpret_cast<float*>(a.O) + ((int64_t)b * a.L + q) * a.dq + h * dh;
        const float invl = 1.0f / l_run;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = lane + 64 * i;
            if (c < dh) Ol[c] = ov[i] * invl;
        }
        return;
    }
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

// out[b][j] = sum over the L rows of U[b][:, j]; one workgroup per (64 columns, item): thread (ry, cx)
// adds rows ry, ry+4, ... of column cx in a fixed order, then the four partial sums are added in a
// fixed order.  Columns r .. ld_out-1 of out are zeroed.
template <typename T>
__global__ void __launch_bounds__(256) colsum_kernel(const T* __restrict__ U, float* __restrict__ out, int L, int r,
                                                     int64_t ld_out) {
    __shared__ float part[4][64];
    const int b = blockIdx.y;
    const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + cx;
    float s = 0.f;
    if (col < r) {
        const T* p = U + (int64_t)b * L * r + col;
        for (int i = ry; i < L; i += 4) {
            if constexpr (sizeof(T) == 2) s += bf2f(p[(int64_t)i * r]);
            else s += p[(int64_t)i * r];
        }
    }
    part[ry][cx] = s;
    __syncthreads();
    if (ry == 0 && col < ld_out) out[(int64_t)b * ld_out + col] = (col < r) ? ((part[0][cx] + part[1][cx]) + (part[2][cx] + part[3][cx])) : 0.f;
}

}  // namespace

hipError_t column_sums(hipStream_t st, const void* U, float* out, int L, int r, int64_t ld_out, int batch, int elem_bytes) {
    dim3 grid((unsigned)((ld_out + 63) / 64), batch);
    if (grid.y > 65535) return hipErrorInvalidValue;
    if (elem_bytes == 2)
        hipLaunchKernelGGL(colsum_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)U, out, L, r, ld_out);
    else
        hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, st, (const float*)U, out, L, r, ld_out);
    return hipGetLastError();
}

hipError_t attention_bf16(hipStream_t st, const AttnArgs& a) {
    const int dh = a.dq / a.heads;
    const int64_t nwg = (int64_t)((a.L + QT - 1) / QT) * a.heads * a.batch;
    if (nwg > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)nwg);
    const float c = a.linearised ? a.scale : a.scale * 1.4426950408889634f;
    if (dh != 128 && dh != 64) return hipErrorInvalidValue;
#ifndef ATP_ATTN_KT
#define ATP_ATTN_KT 64
#endif
    if (a.linearised) {
        if (dh == 128) hipLaunchKernelGGL((attn_bf16_kernel<128, true, 64>), grid, dim3(256), 0, st, a, c);
        else hipLaunchKernelGGL((attn_bf16_kernel<64, true, 64>), grid, dim3(256), 0, st, a, c);
    } else {
        if (dh == 128) hipLaunchKernelGGL((attn_bf16_kernel<128, false, ATP_ATTN_KT>), grid, dim3(256), 0, st, a, c);
        else hipLaunchKernelGGL((attn_bf16_kernel<64, false, ATP_ATTN_KT>), grid, dim3(256), 0, st, a, c);
    }
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
