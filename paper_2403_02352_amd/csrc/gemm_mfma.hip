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

#include <type_traits>

namespace atp {
namespace {

template <int BK>
__device__ __forceinline__ int swz(int row, int kc) {
    if constexpr (BK == 64) return kc ^ (row & 7);
    else return kc ^ ((row >> 1) & 3);
}

template <typename T> struct Raw;
template <> struct Raw<bf16_t> { uint4 v; };
template <> struct Raw<float> { f32x4 a, b; };

__device__ __forceinline__ void load_raw(Raw<bf16_t>& r, const bf16_t* p, bool ok) {
    r.v = ok ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
}
__device__ __forceinline__ void load_raw(Raw<float>& r, const float* p, bool ok) {
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    r.a = ok ? *reinterpret_cast<const f32x4*>(p) : z;
    r.b = ok ? *reinterpret_cast<const f32x4*>(p + 4) : z;
}

// split 8 floats into hi (and lo) bf16 planes
template <int NSPLIT>
__device__ __forceinline__ void split2(float x0, float x1, uint32_t& h, uint32_t& l) {
    const bf16_t h0 = f2bf(x0), h1 = f2bf(x1);
    h = (uint32_t)h0 | ((uint32_t)h1 << 16);
    if constexpr (NSPLIT > 1) l = pack_bf2(x0 - bf2f(h0), x1 - bf2f(h1));
    else l = 0;
}
template <int NSPLIT>
__device__ __forceinline__ void to_planes(const Raw<float>& r, uint4& hi, uint4& lo) {
    split2<NSPLIT>(r.a.x, r.a.y, hi.x, lo.x);
    split2<NSPLIT>(r.a.z, r.a.w, hi.y, lo.y);
    split2<NSPLIT>(r.b.x, r.b.y, hi.z, lo.z);
    split2<NSPLIT>(r.b.z, r.b.w, hi.w, lo.w);
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

// ---------------------------------------------------------------------------
// Epilogue shared by both kernels.  Row-major outputs are stored straight from the
// accumulators (32 lanes cover 32 consecutive columns).  Transposed outputs (and the mirror
// image of a symmetric product) go through a per-wave 32×33 LDS patch so that 32 lanes again
// cover 32 consecutive addresses.
// ---------------------------------------------------------------------------
template <int TM, int TN>
__device__ __forceinline__ void store_outputs(const GemmArgs& p, f32x16 (&acc)[TM][TN], float* stage, int row0,
                                              int col0, int lane, int bz, bool mirror, int64_t c32_off) {
    const int l32 = lane & 31, lh = lane >> 5;
    float* C32 = p.C32 ? p.C32 + (int64_t)bz * p.sC + c32_off : nullptr;
    bf16_t* C16 = p.C16 ? p.C16 + (int64_t)bz * p.sC : nullptr;
    float* CT32 = p.CT32 ? p.CT32 + (int64_t)bz * p.sCT : nullptr;
    bf16_t* CT16 = p.CT16 ? p.CT16 + (int64_t)bz * p.sCT : nullptr;
    int64_t ldct = p.ldct;
    if (mirror) { CT32 = C32; ldct = p.ldc; }
    if (C32) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = col0 + j * 32 + l32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row0 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (row < p.M && col < p.N) C32[(int64_t)row * p.ldc + col] = acc[i][j][v];
                }
            }
    }
    if (C16) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = col0 + j * 32 + l32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row0 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (row < p.M && col < p.N) C16[(int64_t)row * p.ldc + col] = f2bf(acc[i][j][v]);
                }
            }
    }
    if (CT32 || CT16) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                __syncthreads();
#pragma unroll
                for (int v = 0; v < 16; ++v) stage[l32 * 33 + 8 * (v >> 2) + 4 * lh + (v & 3)] = acc[i][j][v];
                __syncthreads();
                const int row = row0 + i * 32 + l32;
#pragma unroll
                for (int cc = 0; cc < 32; cc += 2) {
                    const int c = cc + lh;
                    const int col = col0 + j * 32 + c;
                    const float val = stage[c * 33 + l32];
                    if (row < p.M && col < p.N) {
                        if (CT32) CT32[(int64_t)col * ldct + row] = val;
                        if (CT16) CT16[(int64_t)col * ldct + row] = f2bf(val);
                    }
                }
            }
    }
}

template <int TM, int TN>
__device__ __forceinline__ void store_swiglu(const GemmArgs& p, f32x16 (&acc)[TM][TN], int row0, int col0, int lane,
                                             int bz) {
    const int l32 = lane & 31, lh = lane >> 5;
    float* C32 = p.C32 ? p.C32 + (int64_t)bz * p.sC : nullptr;
    bf16_t* C16 = p.C16 ? p.C16 + (int64_t)bz * p.sC : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN / 2; ++j) {
            const int col = col0 + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (row < p.M && col < p.N) {
                    const float o = silu(acc[i][j][v]) * acc[i][j + TN / 2][v];
                    if (C32) C32[(int64_t)row * p.ldc + col] = o;
                    if (C16) C16[(int64_t)row * p.ldc + col] = f2bf(o);
                }
            }
        }
}

// XCD-aware remap of the linear workgroup id, then a walk in groups of 8 tile rows
__device__ __forceinline__ void tile_coords(int id, int tilesM, int tilesN, int& tile_m, int& tile_n) {
    const int T = tilesM * tilesN;
    if ((T & 7) == 0) id = (id & 7) * (T >> 3) + (id >> 3);
    constexpr int GROUP = 8;
    const int gsz = GROUP * tilesN;
    const int g = id / gsz;
    const int first_m = g * GROUP;
    const int gm = min(tilesM - first_m, GROUP);
    tile_m = first_m + (id % gsz) % gm;
    tile_n = (id % gsz) / gm;
}

// row of the B operand (N×K) that feeds local tile row `b_row`; SWIGLU interleaves, per wave
// column, WN/2 gate rows with the matching WN/2 up rows
template <int WN, bool SWIGLU>
__device__ __forceinline__ int b_global_row(int b_row, int n0, int N, bool& ok) {
    if constexpr (SWIGLU) {
        const int w = b_row / WN, within = b_row % WN;
        const int half = within / (WN / 2), jj = within % (WN / 2);
        const int oc = n0 + w * (WN / 2) + jj;
        ok = oc < N;
        return half * N + oc;
    } else {
        ok = (n0 + b_row) < N;
        return n0 + b_row;
    }
}

// ---------------------------------------------------------------------------
// Register-staged kernel: any operand types (bf16 / fp32, optional hi+lo split), K % 8 == 0.
// grid = (tiles, batch, ksplit); with ksplit > 1 slice z of the K range writes its partial
// product to C32 + z*sKsplit.
// ---------------------------------------------------------------------------
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

    int tile_m, tile_n;
    tile_coords(blockIdx.x, tilesM, tilesN, tile_m, tile_n);
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
    const int KT_all = (kend + BK - 1) / BK;
    // K slice of this workgroup
    const int ks_n = max(p.ksplit, 1);
    const int per = (KT_all + ks_n - 1) / ks_n;
    const int kt_begin = blockIdx.z * per;
    const int kt_end = min(KT_all, kt_begin + per);

    Raw<TA> ra[CA];
    Raw<TB> rb[CB];
    auto load_tile = [&](int kt) {
        const int k0 = kt * BK;
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int c = tid + i * NT;
            const int row = c / CPR, kc = c % CPR;
            const int gr = m0 + row;
            const bool ok = gr < p.M && (k0 + kc * 8 < kend);
            load_raw(ra[i], A + (int64_t)(gr < p.M ? gr : 0) * p.lda + k0 + kc * 8, ok);
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const int c = tid + i * NT;
            const int row = c / CPR, kc = c % CPR;
            bool rok;
            const int gr = b_global_row<WN, SWIGLU>(row, n0, p.N, rok);
            const bool ok = rok && (k0 + kc * 8 < kend);
            load_raw(rb[i], B + (int64_t)(rok ? gr : 0) * p.ldb + k0 + kc * 8, ok);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int c = tid + i * NT;
            const int row = c / CPR, kc = c % CPR;
            uint4 hi, lo;
            to_planes<NSPLIT>(ra[i], hi, lo);
            const int o = row * CPR + swz<BK>(row, kc);
            sA[o] = hi;
            if constexpr (NP > 1) sA[BM * CPR + o] = lo;
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const int c = tid + i * NT;
            const int row = c / CPR, kc = c % CPR;
            uint4 hi, lo;
            to_planes<NSPLIT>(rb[i], hi, lo);
            const int o = row * CPR + swz<BK>(row, kc);
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

    load_tile(kt_begin);  // unconditional: chunks past the K range are zero-filled
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        store_tile();
        __syncthreads();
        if (kt + 1 < kt_end) load_tile(kt + 1);
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

    if constexpr (SWIGLU) {
        store_swiglu<TM, TN>(p, acc, m0 + wm * WM, n0 + wn * (WN / 2), lane, bz);
    } else {
        float* stage = reinterpret_cast<float*>(smem) + wave * (32 * 33);
        store_outputs<TM, TN>(p, acc, stage, m0 + wm * WM, n0 + wn * WN, lane, bz,
                              p.symmetric && (tile_n < tile_m),
                              p.ksplit > 1 ? (int64_t)blockIdx.z * p.sKsplit : 0);
    }
}

// ---------------------------------------------------------------------------
// bf16·bf16 kernel with asynchronous global→LDS copies (no register staging) and two LDS
// stages: the copies of k-tile t+1 are in flight while the MFMAs of k-tile t run, one barrier
// per k-tile.  Requires K % 64 == 0.
//
// One copy instruction moves 64 × 16 bytes: a group of 8 tile rows × 64 k.  Eight consecutive
// lanes fetch the 128 contiguous bytes of one row (lanes that stride across rows instead cost
// 4x the time in the address coalescer) and the 64 lanes land on 1 KB of consecutive LDS, so a
// tile is stored as plain 128-byte rows.  Bank conflicts of the fragment reads (32 lanes = 32
// consecutive rows) are avoided on the GLOBAL side: position s of row r holds 16-byte chunk
// s ^ (r & 7) ^ ((r >> 3) & 1), i.e. lane q of group g fetches chunk (q%8) ^ (q/8) ^ (g&1).
// ---------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

template <int BM, int BN, int WM, int WN, bool SWIGLU>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
gemm_bf16_async_kernel(GemmArgs p, int tilesM, int tilesN) {
    constexpr int BK = 64;
    constexpr int NWN = BN / WN;
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int GA = BM / 8 / NW, GB = BN / 8 / NW;  // 8-row groups copied per wave
    constexpr int STAGE = (BM + BN) * 8;                // uint4 per stage
    static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "tile/waves mismatch");

    // two statically distinct stages: copies into one do not alias fragment reads from the other
    __shared__ __align__(16) uint4 stage0[STAGE];
    __shared__ __align__(16) uint4 stage1[STAGE];

    int tile_m, tile_n;
    tile_coords(blockIdx.x, tilesM, tilesN, tile_m, tile_n);
    const int bz = blockIdx.y;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * (SWIGLU ? BN / 2 : BN);
    const bf16_t* __restrict__ A = reinterpret_cast<const bf16_t*>(p.A) + (int64_t)bz * p.sA;
    const bf16_t* __restrict__ B = reinterpret_cast<const bf16_t*>(p.B) + (int64_t)bz * p.sB;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / NWN, wn = wave % NWN;
    const int l32 = lane & 31, lh = lane >> 5;
    const int KT = p.K / BK;

    // copy i of this wave moves row group g = i*NW + wave; lane q -> row 8g + q/8, position q%8
    const bf16_t* a_src[GA];
    const bf16_t* b_src[GB];
#pragma unroll
    for (int i = 0; i < GA; ++i) {
        const int g = i * NW + wave;
        const int row = 8 * g + (lane >> 3);
        const int kc = (lane & 7) ^ (lane >> 3) ^ (g & 1);
        const int gr = min(m0 + row, p.M - 1);  // rows past M: any valid row, never stored
        a_src[i] = A + (int64_t)gr * p.lda + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < GB; ++i) {
        const int g = i * NW + wave;
        const int row = 8 * g + (lane >> 3);
        const int kc = (lane & 7) ^ (lane >> 3) ^ (g & 1);
        bool rok;
        int gr = b_global_row<WN, SWIGLU>(row, n0, p.N, rok);
        if (!rok) gr = 0;
        b_src[i] = B + (int64_t)gr * p.ldb + kc * 8;
    }
    auto issue = [&](int kt, uint4* sA) {
        uint4* sB = sA + BM * 8;
        const int k0 = kt * BK;
#pragma unroll
        for (int i = 0; i < GA; ++i)
            __builtin_amdgcn_global_load_lds((glb_void*)(a_src[i] + k0), (lds_void*)(sA + (i * NW + wave) * 64), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < GB; ++i)
            __builtin_amdgcn_global_load_lds((glb_void*)(b_src[i] + k0), (lds_void*)(sB + (i * NW + wave) * 64), 16, 0, 0);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment offsets (uint4 units): rows of this lane's fragments differ by multiples of 32, so
    // the swizzle term is one per-lane constant and each k-step needs one precomputed offset
    const int xs = (l32 & 7) ^ ((l32 >> 3) & 1);
    const int rowA = (wm * WM + l32) * 8, rowB = BM * 8 + (wn * WN + l32) * 8;
    int kofs[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) kofs[ks] = (2 * ks + lh) ^ xs;
    auto compute = [&](const uint4* st) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = as_bf16x8(st[rowA + i * 256 + kofs[ks]]);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[j] = as_bf16x8(st[rowB + j * 256 + kofs[ks]]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    };

    issue(0, stage0);
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's copies of tile kt have landed
        __syncthreads();                     // ... and everybody else's; stage1 is free again
        issue(kt + 1, stage1);
        __builtin_amdgcn_sched_barrier(0);   // keep the copies ahead of the MFMA loop
        compute(stage0);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (kt + 2 < KT) issue(kt + 2, stage0);
        __builtin_amdgcn_sched_barrier(0);
        compute(stage1);
    }
    if (kt < KT) {  // odd number of k-tiles: the last one sits in stage0
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        compute(stage0);
    }
    __syncthreads();
    if constexpr (SWIGLU) {
        store_swiglu<TM, TN>(p, acc, m0 + wm * WM, n0 + wn * (WN / 2), lane, bz);
    } else {
        float* stage = reinterpret_cast<float*>(stage0) + wave * (32 * 33);
        store_outputs<TM, TN>(p, acc, stage, m0 + wm * WM, n0 + wn * WN, lane, bz, false, 0);
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
    dim3 grid(tilesM * tilesN, g.batch, g.ksplit > 1 ? g.ksplit : 1);
    hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, g, tilesM, tilesN);
    return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, bool SWIGLU>
hipError_t launch_async(hipStream_t st, const GemmArgs& g) {
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    auto kern = gemm_bf16_async_kernel<BM, BN, WM, WN, SWIGLU>;
    const int tilesM = (g.M + BM - 1) / BM;
    const int tilesN = (g.N + (SWIGLU ? BN / 2 : BN) - 1) / (SWIGLU ? BN / 2 : BN);
    dim3 grid(tilesM * tilesN, g.batch, 1);
    hipLaunchKernelGGL(kern, grid, dim3(NT), 0, st, g, tilesM, tilesN);
    return hipGetLastError();
}

template <typename TA, typename TB, int NSPLIT>
hipError_t dispatch_cfg(hipStream_t st, const GemmArgs& g) {
    constexpr int BKs = (NSPLIT > 1) ? 32 : 64;
    const bool big = gemm_nt_mfma_big(g);
    if (g.swiglu) {
        if constexpr (NSPLIT == 1 && std::is_same<TA, bf16_t>::value && std::is_same<TB, bf16_t>::value) {
            if (big) return launch<TA, TB, NSPLIT, 256, 256, BKs, 128, 64, true>(st, g);
            return launch<TA, TB, NSPLIT, 128, 128, BKs, 64, 64, true>(st, g);
        } else {
            return hipErrorInvalidValue;
        }
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

bool gemm_nt_mfma_async(const GemmArgs& g) {
    return g.K % 64 == 0 && g.K >= 64 && !g.symmetric && !g.b_lower && g.ksplit <= 1 && g.M >= 1;
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
    if (ta == OP_BF16 && tb == OP_BF16) {
        if (gemm_nt_mfma_async(g)) {
            const bool big = gemm_nt_mfma_big(g);
            if (g.swiglu) {
                if (big) return launch_async<256, 256, 128, 64, true>(st, g);
                return launch_async<128, 128, 64, 64, true>(st, g);
            }
            if (big) return launch_async<256, 256, 128, 64, false>(st, g);
            return launch_async<128, 128, 64, 64, false>(st, g);
        }
        return dispatch_cfg<bf16_t, bf16_t, 1>(st, g);
    }
    if (ta == OP_BF16 && tb == OP_F32) return dispatch_cfg<bf16_t, float, 1>(st, g);
    if (ta == OP_F32 && tb == OP_F32) return dispatch_cfg<float, float, 1>(st, g);
    if (ta == OP_F32 && tb == OP_BF16) return dispatch_cfg<float, bf16_t, 1>(st, g);
    return hipErrorInvalidValue;
}

}  // namespace atp
