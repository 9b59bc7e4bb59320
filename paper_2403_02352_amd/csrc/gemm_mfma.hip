// bf16 MFMA GEMM family for gfx950:  C = A · Bᵀ, both operands K-contiguous.
//
// One kernel template carries every dense contraction of the ATP path that is
// not the fused attention: the power-iteration products X·V and Xᵀ·U, the
// coefficient product B_r = U_rᵀ·X (Eq.5), the projections X'·W (Eq.6, Tab.1
// "Projection"), the query expansion U·Q' (Eq.6), and, with fp32 operands split
// into hi+lo bf16 parts (three MFMA products, ≈2^-17 relative error), the Gram
// matrix ZᵀZ and the triangular apply Z·R⁻¹ of the CholeskyQR.
//
// Tiling: BM×BN×BK block tile staged through LDS (XOR-swizzled 16-byte chunks,
// conflict-free for both the 16-byte writes and the ds_read_b128 fragment
// reads), v_mfma_f32_32x32x16_bf16, 64-lane waves each owning a WM×WN sub-tile.
// Global loads for tile k+1 are issued before the MFMA loop of tile k.
// Workgroup ids are remapped so that consecutive tiles share an XCD (its L2)
// and walk the output in groups of 8 tile-rows.
#include "common.h"

namespace atp {
namespace {

template <int BK>
__device__ __forceinline__ int swz(int row, int kc) {
    if constexpr (BK == 64) return kc ^ (row & 7);
    else return kc ^ ((row >> 1) & 3);
}

template <typename T> struct Raw;
template <> struct Raw<bf16_t> { uint4 v; };
template <> struct Raw<float> { float4 a, b; };

__device__ __forceinline__ void load_raw(Raw<bf16_t>& r, const bf16_t* p, bool ok) {
    r.v = ok ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
}
__device__ __forceinline__ void load_raw(Raw<float>& r, const float* p, bool ok) {
    if (ok) {
        r.a = *reinterpret_cast<const float4*>(p);
        r.b = *reinterpret_cast<const float4*>(p + 4);
    } else {
        r.a = make_float4(0.f, 0.f, 0.f, 0.f);
        r.b = r.a;
    }
}

// split 8 floats into hi (and lo) bf16 planes
template <int NSPLIT>
__device__ __forceinline__ void to_planes(const Raw<float>& r, uint4& hi, uint4& lo) {
    const float x[8] = {r.a.x, r.a.y, r.a.z, r.a.w, r.b.x, r.b.y, r.b.z, r.b.w};
    uint32_t h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bf16_t h0 = f2bf(x[2 * i]), h1 = f2bf(x[2 * i + 1]);
        h[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        if constexpr (NSPLIT > 1) {
            l[i] = pack_bf2(x[2 * i] - bf2f(h0), x[2 * i + 1] - bf2f(h1));
        } else {
            l[i] = 0;
        }
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]);
    lo = make_uint4(l[0], l[1], l[2], l[3]);
}
template <int NSPLIT>
__device__ __forceinline__ void to_planes(const Raw<bf16_t>& r, uint4& hi, uint4& lo) {
    hi = r.v;
    lo = make_uint4(0, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& u) {
    union { uint4 u; bf16x8 b; } c;
    c.u = u;
    return c.b;
}

__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }

template <typename TA, typename TB, int NSPLIT, int BM, int BN, int BK, int WM, int WN, bool SWIGLU>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
gemm_nt_kernel(GemmArgs p, int tilesM, int tilesN) {
    constexpr int NWN = BN / WN;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int CPR = BK / 8;  // 16-byte bf16 chunks per tile row
    constexpr int CA = (BM * CPR) / NT, CB = (BN * CPR) / NT;
    constexpr int NP = (NSPLIT > 1) ? 2 : 1;
    static_assert((BM * CPR) % NT == 0 && (BN * CPR) % NT == 0, "tile/threads mismatch");
    static_assert(!SWIGLU || (TN % 2 == 0), "swiglu needs an even number of column tiles per wave");

    extern __shared__ __align__(16) uint4 smem[];
    uint4* sA = smem;                     // [NP][BM*CPR]
    uint4* sB = smem + NP * BM * CPR;     // [NP][BN*CPR]

    // ---- tile mapping: XCD-aware remap, then grouped walk -------------------
    const int T = tilesM * tilesN;
    int id = blockIdx.x;
    if ((T & 7) == 0) id = (id & 7) * (T >> 3) + (id >> 3);
    constexpr int GROUP = 8;
    const int gsz = GROUP * tilesN;
    const int g = id / gsz;
    const int first_m = g * GROUP;
    const int gm = min(tilesM - first_m, GROUP);
    const int tile_m = first_m + (id % gsz) % gm;
    const int tile_n = (id % gsz) / gm;
    if (p.symmetric && tile_n > tile_m) return;
    const int bz = blockIdx.y;

    const int m0 = tile_m * BM;
    const int n0 = tile_n * (SWIGLU ? BN / 2 : BN);  // first output column of this tile
    const TA* __restrict__ A = reinterpret_cast<const TA*>(p.A) + (int64_t)bz * p.sA;
    const TB* __restrict__ B = reinterpret_cast<const TB*>(p.B) + (int64_t)bz * p.sB;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / NWN, wn = wave % NWN;
    const int l32 = lane & 31, lh = lane >> 5;

    int kend = p.K;
    if (p.b_lower) kend = min(p.K, ((n0 + BN + BK - 1) / BK) * BK);
    const int KT = (kend + BK - 1) / BK;

    // ---- per-thread chunk coordinates --------------------------------------
    int a_row[CA], a_kc[CA];
    const TA* a_ptr[CA];
    bool a_ok[CA];
#pragma unroll
    for (int i = 0; i < CA; ++i) {
        const int c = tid + i * NT;
        a_row[i] = c / CPR;
        a_kc[i] = c % CPR;
        const int gr = m0 + a_row[i];
        a_ok[i] = gr < p.M;
        a_ptr[i] = A + (int64_t)(a_ok[i] ? gr : 0) * p.lda + a_kc[i] * 8;
    }
    int b_row[CB], b_kc[CB];
    const TB* b_ptr[CB];
    bool b_ok[CB];
#pragma unroll
    for (int i = 0; i < CB; ++i) {
        const int c = tid + i * NT;
        b_row[i] = c / CPR;
        b_kc[i] = c % CPR;
        int gr;
        bool ok;
        if constexpr (SWIGLU) {
            // wave-column w holds WN/2 gate columns then the matching WN/2 up columns
            const int w = b_row[i] / WN, within = b_row[i] % WN;
            const int half = within / (WN / 2), jj = within % (WN / 2);
            const int oc = n0 + w * (WN / 2) + jj;
            ok = oc < p.N;
            gr = half * p.N + oc;
        } else {
            gr = n0 + b_row[i];
            ok = gr < p.N;
        }
        b_ok[i] = ok;
        b_ptr[i] = B + (int64_t)(ok ? gr : 0) * p.ldb + b_kc[i] * 8;
    }

    Raw<TA> ra[CA];
    Raw<TB> rb[CB];
    auto load_tile = [&](int kt) {
        const int k0 = kt * BK;
#pragma unroll
        for (int i = 0; i < CA; ++i) load_raw(ra[i], a_ptr[i] + k0, a_ok[i] && (k0 + a_kc[i] * 8 < kend));
#pragma unroll
        for (int i = 0; i < CB; ++i) load_raw(rb[i], b_ptr[i] + k0, b_ok[i] && (k0 + b_kc[i] * 8 < kend));
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            uint4 hi, lo;
            to_planes<NSPLIT>(ra[i], hi, lo);
            const int o = a_row[i] * CPR + swz<BK>(a_row[i], a_kc[i]);
            sA[o] = hi;
            if constexpr (NP > 1) sA[BM * CPR + o] = lo;
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            uint4 hi, lo;
            to_planes<NSPLIT>(rb[i], hi, lo);
            const int o = b_row[i] * CPR + swz<BK>(b_row[i], b_kc[i]);
            sB[o] = hi;
            if constexpr (NP > 1) sB[BN * CPR + o] = lo;
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    load_tile(0);
    for (int kt = 0; kt < KT; ++kt) {
        store_tile();
        __syncthreads();
        if (kt + 1 < KT) load_tile(kt + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int kc = ks * 2 + lh;
            bf16x8 ah[TM], bh[TN];
            bf16x8 al[TM], bl[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm * WM + i * 32 + l32;
                const int o = row * CPR + swz<BK>(row, kc);
                ah[i] = as_bf16x8(sA[o]);
                if constexpr (NP > 1) al[i] = as_bf16x8(sA[BM * CPR + o]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = wn * WN + j * 32 + l32;
                const int o = row * CPR + swz<BK>(row, kc);
                bh[j] = as_bf16x8(sB[o]);
                if constexpr (NP > 1) bl[j] = as_bf16x8(sB[BN * CPR + o]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (NP > 1) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
                    }
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    // ---- epilogue ------------------------------------------------------------
    float* C32 = p.C32 ? p.C32 + (int64_t)bz * p.sC : nullptr;
    bf16_t* C16 = p.C16 ? p.C16 + (int64_t)bz * p.sC : nullptr;
    float* CT32 = p.CT32 ? p.CT32 + (int64_t)bz * p.sCT : nullptr;
    bf16_t* CT16 = p.CT16 ? p.CT16 + (int64_t)bz * p.sCT : nullptr;
    const bool mirror = p.symmetric && (tile_n < tile_m);

    if constexpr (SWIGLU) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN / 2; ++j) {
                const int col = n0 + wn * (WN / 2) + j * 32 + l32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (row < p.M && col < p.N) {
                        const float o = silu(acc[i][j][v]) * acc[i][j + TN / 2][v];
                        if (C32) C32[(int64_t)row * p.ldc + col] = o;
                        if (C16) C16[(int64_t)row * p.ldc + col] = f2bf(o);
                        if (CT32) CT32[(int64_t)col * p.ldct + row] = o;
                        if (CT16) CT16[(int64_t)col * p.ldct + row] = f2bf(o);
                    }
                }
            }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * WN + j * 32 + l32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (row < p.M && col < p.N) {
                        const float o = acc[i][j][v];
                        if (C32) {
                            C32[(int64_t)row * p.ldc + col] = o;
                            if (mirror) C32[(int64_t)col * p.ldc + row] = o;
                        }
                        if (C16) {
                            C16[(int64_t)row * p.ldc + col] = f2bf(o);
                            if (mirror) C16[(int64_t)col * p.ldc + row] = f2bf(o);
                        }
                        if (CT32) CT32[(int64_t)col * p.ldct + row] = o;
                        if (CT16) CT16[(int64_t)col * p.ldct + row] = f2bf(o);
                    }
                }
            }
    }
}

template <typename TA, typename TB, int NSPLIT, int BM, int BN, int BK, int WM, int WN, bool SWIGLU>
hipError_t launch(hipStream_t st, const GemmArgs& g) {
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int NP = (NSPLIT > 1) ? 2 : 1;
    constexpr size_t lds = (size_t)NP * (BM + BN) * BK * 2;
    auto kern = gemm_nt_kernel<TA, TB, NSPLIT, BM, BN, BK, WM, WN, SWIGLU>;
    static bool attr_done = false;  // per instantiation
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int tilesM = (g.M + BM - 1) / BM;
    const int tilesN = (g.N + (SWIGLU ? BN / 2 : BN) - 1) / (SWIGLU ? BN / 2 : BN);
    dim3 grid(tilesM * tilesN, g.batch, 1);
    hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, g, tilesM, tilesN);
    return hipGetLastError();
}

template <typename TA, typename TB, int NSPLIT>
hipError_t dispatch_cfg(hipStream_t st, const GemmArgs& g) {
    constexpr int BKs = (NSPLIT > 1) ? 32 : 64;
    const bool big = gemm_nt_mfma_big(g);
    if (g.swiglu) {
        if (big) return launch<TA, TB, NSPLIT, 256, 256, BKs, 128, 64, true>(st, g);
        return launch<TA, TB, NSPLIT, 128, 128, BKs, 64, 64, true>(st, g);
    }
    if (big) return launch<TA, TB, NSPLIT, 256, 256, BKs, 128, 64, false>(st, g);
    return launch<TA, TB, NSPLIT, 128, 128, BKs, 64, 64, false>(st, g);
}

}  // namespace

bool gemm_nt_mfma_big(const GemmArgs& g) {
    const int bn = g.swiglu ? 128 : 256;  // output columns per 256-wide tile
    const int64_t tiles = (int64_t)((g.M + 255) / 256) * ((g.N + bn - 1) / bn) * g.batch;
    return tiles >= 128 && g.M >= 256 && g.N >= bn;
}

bool gemm_nt_mfma_ok(OperandType ta, OperandType tb, const GemmArgs& g) {
    if (g.K % 8 || g.lda % 8 || g.ldb % 8 || g.sA % 8 || g.sB % 8) return false;
    if (((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15)) return false;
    (void)ta; (void)tb;
    return true;
}

hipError_t gemm_nt_mfma(hipStream_t st, OperandType ta, OperandType tb, int nsplit, const GemmArgs& g) {
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
    if (nsplit == 3) {
        if (ta == OP_F32 && tb == OP_F32) return dispatch_cfg<float, float, 3>(st, g);
        return hipErrorInvalidValue;
    }
    if (ta == OP_BF16 && tb == OP_BF16) return dispatch_cfg<bf16_t, bf16_t, 1>(st, g);
    if (ta == OP_BF16 && tb == OP_F32) return dispatch_cfg<bf16_t, float, 1>(st, g);
    if (ta == OP_F32 && tb == OP_F32) return dispatch_cfg<float, float, 1>(st, g);
    if (ta == OP_F32 && tb == OP_BF16) return dispatch_cfg<float, bf16_t, 1>(st, g);
    return hipErrorInvalidValue;
}

}  // namespace atp
