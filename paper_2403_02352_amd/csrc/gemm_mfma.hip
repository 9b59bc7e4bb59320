// bf16 MFMA GEMM for gfx950:  C = A · Bᵀ, both operands K-contiguous.
//
// One kernel template carries every dense contraction of the ATP path that is not the fused
// attention: the power-iteration products X·V and Xᵀ·U, the coefficient product B_r = U_rᵀ·X
// (Eq.5), the projections X'·W (Eq.6, Tab.1 "Projection"), the query expansion U·Q' (Eq.6), and,
// with operands held as hi+lo pairs of bf16 planes (three MFMA products, ≈2^-17 relative error),
// the Gram matrix ZᵀZ and the triangular apply Z·R⁻¹ of the CholeskyQR.
//
// Pipeline: asynchronous global→LDS copies (no register staging) into two LDS stages; the copies
// of k-tile t+1 are in flight while the MFMAs (v_mfma_f32_32x32x16_bf16) of k-tile t run, one
// barrier per k-tile.  64-lane waves each own a WM×WN sub-tile of the BM×BN block tile.
//
// One copy instruction moves 64 × 16 bytes.  Consecutive lanes fetch consecutive 16-byte chunks
// of one tile row (lanes that stride across rows cost 4x the time in the address coalescer), and
// the 64 lanes land on 1 KB of consecutive LDS, so a tile is stored as plain rows of BK bf16.
// Bank conflicts of the fragment reads (32 lanes = 32 consecutive rows) are avoided on the GLOBAL
// side: position s of row r holds chunk s ^ swz(r).  Rows of one lane's fragments differ by
// multiples of 32, so swz is a per-lane constant and each k-step needs one precomputed offset.
//
// Workgroup ids are remapped so that consecutive tiles share an XCD (its L2) and walk the output
// in groups of 8 tile rows.
#include "common.h"

#include <utility>

namespace atp {
namespace {

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& u) {
    union { uint4 u; bf16x8 b; } c;
    c.u = u;
    return c.b;
}

__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }

// ---------------------------------------------------------------------------
// Epilogue, one 64×64 piece of the wave tile at a time (the piece index is a template parameter,
// so accumulators are only ever indexed statically).  fp32 outputs are stored straight from the
// accumulators (32 lanes cover 32 consecutive columns).  bf16 planes are staged in a wave-private
// LDS tile and leave as 16-byte pieces, 8 lanes per 128-byte row segment; for the transposed
// twin a lane's 4 consecutive rows are 4 consecutive elements of a transposed row.
// ---------------------------------------------------------------------------
constexpr int WPITCH = 72;            // bf16 elements per row of the wave-private staging tile (64 + pad)
constexpr int WBUF = 64 * WPITCH;     // elements per wave

struct EpiPtrs {
    float* C32;
    bf16_t *C16, *C16lo, *CT16, *CT16lo;
    bool vecC, vecT;  // 16-byte stores allowed (extents and leading dimensions multiples of 8, aligned bases)
};

template <int IH, int JH, int TM, int TN>
__device__ __forceinline__ void store_piece(const GemmArgs& p, const EpiPtrs& e, const f32x16 (&acc)[TM][TN],
                                            bf16_t* wbuf, int row0, int col0, int lane) {
    const int l32 = lane & 31, lh = lane >> 5;
    const int prow = row0 + 64 * IH, pcol = col0 + 64 * JH;
    if (e.C32) {
#pragma unroll
        for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = pcol + 32 * j + l32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = prow + 32 * i2 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (row < p.M && col < p.N) e.C32[(int64_t)row * p.ldc + col] = acc[2 * IH + i2][2 * JH + j][v];
                }
            }
    }
#pragma unroll
    for (int pl = 0; pl < 2; ++pl) {
        bf16_t* dst = pl ? e.C16lo : e.C16;
        if (!dst) continue;
#pragma unroll
        for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float a = acc[2 * IH + i2][2 * JH + j][v];
                    const bf16_t h = f2bf(a);
                    wbuf[(32 * i2 + 8 * (v >> 2) + 4 * lh + (v & 3)) * WPITCH + 32 * j + l32] = pl ? f2bf(a - bf2f(h)) : h;
                }
        if (e.vecC) {
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int c = it * 64 + lane, rr = c >> 3, part = c & 7;
                const uint4 q = *reinterpret_cast<const uint4*>(wbuf + rr * WPITCH + part * 8);
                const int row = prow + rr, col = pcol + part * 8;
                if (row < p.M && col < p.N) *reinterpret_cast<uint4*>(dst + (int64_t)row * p.ldc + col) = q;
            }
        } else {
            for (int c = lane; c < 64 * 64; c += 64) {
                const int rr = c >> 6, cc = c & 63;
                const int row = prow + rr, col = pcol + cc;
                if (row < p.M && col < p.N) dst[(int64_t)row * p.ldc + col] = wbuf[rr * WPITCH + cc];
            }
        }
    }
#pragma unroll
    for (int pl = 0; pl < 2; ++pl) {
        bf16_t* dst = pl ? e.CT16lo : e.CT16;
        if (!dst) continue;
#pragma unroll
        for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    bf16_t h[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float a = acc[2 * IH + i2][2 * JH + j][4 * vq + q];
                        h[q] = f2bf(a);
                        if (pl) h[q] = f2bf(a - bf2f(h[q]));
                    }
                    uint2 w;
                    w.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
                    w.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
                    *reinterpret_cast<uint2*>(wbuf + (32 * j + l32) * WPITCH + 32 * i2 + 8 * vq + 4 * lh) = w;
                }
        if (e.vecT) {
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int c = it * 64 + lane, cc = c >> 3, part = c & 7;
                const uint4 q = *reinterpret_cast<const uint4*>(wbuf + cc * WPITCH + part * 8);
                const int col = pcol + cc, row = prow + part * 8;
                if (row < p.M && col < p.N) *reinterpret_cast<uint4*>(dst + (int64_t)col * p.ldct + row) = q;
            }
        } else {
            for (int c = lane; c < 64 * 64; c += 64) {
                const int cc = c >> 6, rr = c & 63;
                const int row = prow + rr, col = pcol + cc;
                if (row < p.M && col < p.N) dst[(int64_t)col * p.ldct + row] = wbuf[cc * WPITCH + rr];
            }
        }
    }
}

template <int TM, int TN, int... Is>
__device__ __forceinline__ void store_pieces(std::integer_sequence<int, Is...>, const GemmArgs& p, const EpiPtrs& e,
                                             const f32x16 (&acc)[TM][TN], bf16_t* wbuf, int row0, int col0, int lane) {
    (store_piece<Is / (TN / 2), Is % (TN / 2), TM, TN>(p, e, acc, wbuf, row0, col0, lane), ...);
}

template <int TM, int TN>
__device__ __forceinline__ void store_outputs(const GemmArgs& p, const f32x16 (&acc)[TM][TN], bf16_t* wbuf, int row0,
                                              int col0, int lane, int bz, int64_t c32_off) {
    static_assert(TM % 2 == 0 && TN % 2 == 0, "wave tiles are made of 64x64 pieces");
    EpiPtrs e;
    e.C32 = p.C32 ? p.C32 + (int64_t)bz * p.sC + c32_off : nullptr;
    e.C16 = p.C16 ? p.C16 + (int64_t)bz * p.sC : nullptr;
    e.C16lo = p.C16lo ? p.C16lo + (int64_t)bz * p.sC : nullptr;
    e.CT16 = p.CT16 ? p.CT16 + (int64_t)bz * p.sCT : nullptr;
    e.CT16lo = p.CT16lo ? p.CT16lo + (int64_t)bz * p.sCT : nullptr;
    e.vecC = (p.N % 8 == 0) && (p.ldc % 8 == 0) && (p.sC % 8 == 0) &&
             ((((uintptr_t)p.C16) | ((uintptr_t)p.C16lo)) & 15) == 0;
    e.vecT = (p.M % 8 == 0) && (p.ldct % 8 == 0) && (p.sCT % 8 == 0) &&
             ((((uintptr_t)p.CT16) | ((uintptr_t)p.CT16lo)) & 15) == 0;
    store_pieces<TM, TN>(std::make_integer_sequence<int, (TM / 2) * (TN / 2)>{}, p, e, acc, wbuf, row0, col0, lane);
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

// Workgroup id -> (batch item, tile).  The hardware hands consecutive workgroup ids to the 8 XCDs in
// turn, so XCD x runs ids x, x+8, ...: give it one contiguous chunk of the (item, tile) list, and
// order the tiles of an item in groups of 8 tile rows × all tile columns (tile row fastest).  The
// 32 workgroups resident on an XCD then form an 8×4 (or 4×8) block of one item and share their
// operand rows through its L2.
__device__ __forceinline__ void tile_coords(int id, int tilesM, int tilesN, int batch, bool longest_first, int& bz,
                                            int& tile_m, int& tile_n) {
    const int T = tilesM * tilesN;
    if (longest_first) {
        // triangular B operand: the K extent grows with tile_n.  Hand out the long tiles first so
        // that workgroups dispatched later (short tiles) fill the gaps
        tile_n = tilesN - 1 - id / (tilesM * batch);
        const int rem = id % (tilesM * batch);
        bz = rem / tilesM;
        tile_m = rem % tilesM;
        return;
    }
    const int all = T * batch;
    if ((all & 7) == 0) id = (id & 7) * (all >> 3) + (id >> 3);
    bz = id / T;
    id -= bz * T;
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


// NP = 1: plain bf16 operands, BK = 64.  NP = 2: hi+lo planes, BK = 32, three products.
template <int BM, int BN, int WM, int WN, int NP, bool SWIGLU>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
gemm_bf16_async_kernel(GemmArgs p, int tilesM, int tilesN) {
    constexpr int BK = 64 / NP;
    constexpr int CPR = BK / 8;          // 16-byte chunks per tile row
    constexpr int RPI = 64 / CPR;        // tile rows moved by one copy instruction
    constexpr int NWN = BN / WN;
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int GA = BM / RPI / NW, GB = BN / RPI / NW;  // copy instructions per wave and plane
    constexpr int PA = BM * CPR, PB = BN * CPR;            // plane sizes (uint4)
    constexpr int STAGE = NP * (PA + PB);
    static_assert((BM / RPI) % NW == 0 && (BN / RPI) % NW == 0, "tile/waves mismatch");
    static_assert(!SWIGLU || NP == 1, "swiglu epilogue only for plain operands");

    // two statically distinct stages: copies into one do not alias fragment reads from the other
    __shared__ __align__(16) uint4 stage0[STAGE];
    __shared__ __align__(16) uint4 stage1[STAGE];

    int tile_m, tile_n, bz, kz;
    const int ks_n = max(p.ksplit, 1);
    if (p.symmetric) {
        // 1-D grid over (batch item, K slice, lower tile).  The tiles of one (item, slice) group share
        // their operand rows: keep a group on one XCD (workgroup id modulo 8) so its L2 serves the reuse
        const int ntri = tilesM * (tilesM + 1) / 2, groups = p.batch * ks_n;
        int g, t;
        if ((groups & 7) == 0) {
            const int slot = blockIdx.x >> 3;
            g = (blockIdx.x & 7) + 8 * (slot / ntri);
            t = slot % ntri;
        } else {
            g = blockIdx.x / ntri;
            t = blockIdx.x % ntri;
        }
        bz = g / ks_n;
        kz = g % ks_n;
        tile_m = (int)((sqrtf(8.f * t + 1.f) - 1.f) * 0.5f);
        while ((tile_m + 1) * (tile_m + 2) / 2 <= t) ++tile_m;
        while (tile_m * (tile_m + 1) / 2 > t) --tile_m;
        tile_n = t - tile_m * (tile_m + 1) / 2;
    } else {
        tile_coords(blockIdx.x, tilesM, tilesN, p.batch, p.b_lower != 0, bz, tile_m, tile_n);
        kz = blockIdx.z;
    }
    const int m0 = tile_m * BM;
    const int n0 = tile_n * (SWIGLU ? BN / 2 : BN);
    const int64_t offA = (int64_t)bz * p.sA, offB = (int64_t)bz * p.sB;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / NWN, wn = wave % NWN;
    const int l32 = lane & 31, lh = lane >> 5;

    int kend = p.K;
    if (p.b_lower) kend = min(p.K, ((p.n_origin + n0 + BN + BK - 1) / BK) * BK);
    const int KT_all = kend / BK;
    const int per = (KT_all + ks_n - 1) / ks_n;
    const int kt_begin = min(KT_all, kz * per);
    const int kt_end = min(KT_all, kt_begin + per);

    // copy i of this wave moves row group g = i*NW + wave: lane q -> row RPI*g + q/CPR, position q%CPR
    unsigned a_off[GA], b_off[GB];  // byte offsets of this lane's chunk at k = 0 within the batch item
#pragma unroll
    for (int i = 0; i < GA; ++i) {
        const int g = i * NW + wave;
        const int row = RPI * g + lane / CPR;
        const int sw = (BK == 64) ? ((row & 7) ^ ((row >> 3) & 1)) : ((row >> 2) & 3);
        const int kc = (lane % CPR) ^ sw;
        const int gr = min(m0 + row, p.M - 1);  // rows past M: any valid row, never stored
        a_off[i] = (unsigned)(((int64_t)gr * p.lda + kc * 8) * 2);
    }
#pragma unroll
    for (int i = 0; i < GB; ++i) {
        const int g = i * NW + wave;
        const int row = RPI * g + lane / CPR;
        const int sw = (BK == 64) ? ((row & 7) ^ ((row >> 3) & 1)) : ((row >> 2) & 3);
        const int kc = (lane % CPR) ^ sw;
        bool rok;
        int gr = b_global_row<WN, SWIGLU>(row, n0, p.N, rok);
        if (!rok) gr = 0;
        b_off[i] = (unsigned)(((int64_t)gr * p.ldb + kc * 8) * 2);
    }
    const bf16_t* Ah = reinterpret_cast<const bf16_t*>(p.A) + offA;
    const bf16_t* Al = reinterpret_cast<const bf16_t*>(p.A_lo) + offA;
    const bf16_t* Bh = reinterpret_cast<const bf16_t*>(p.B) + offB;
    const bf16_t* Bl = reinterpret_cast<const bf16_t*>(p.B_lo) + offB;
    // LDS byte address of this wave's first copy slot in each stage (scalar registers)
    const unsigned wave_s = (unsigned)__builtin_amdgcn_readfirstlane(wave);
    const unsigned lds_stage0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void*)stage0) + wave_s * 1024u;
    const unsigned lds_stage1 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void*)stage1) + wave_s * 1024u;
    // (every wait for these copies is explicit below)
    auto issue = [&](int kt, const uint4* stp) {
        const int k0 = kt * BK;
        const unsigned st = (stp == stage0) ? lds_stage0 : lds_stage1;
#pragma unroll
        for (int i = 0; i < GA; ++i) {
            copy16_untracked(Ah + k0, a_off[i], st + (unsigned)(i * NW * 64) * 16u);
            if constexpr (NP == 2) copy16_untracked(Al + k0, a_off[i], st + (unsigned)(PA + i * NW * 64) * 16u);
        }
#pragma unroll
        for (int i = 0; i < GB; ++i) {
            copy16_untracked(Bh + k0, b_off[i], st + (unsigned)(NP * PA + i * NW * 64) * 16u);
            if constexpr (NP == 2) copy16_untracked(Bl + k0, b_off[i], st + (unsigned)(NP * PA + PB + i * NW * 64) * 16u);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment offsets (uint4 units)
    const int xs = (BK == 64) ? ((l32 & 7) ^ ((l32 >> 3) & 1)) : ((l32 >> 2) & 3);
    const int rowA = (wm * WM + l32) * CPR, rowB = NP * PA + (wn * WN + l32) * CPR;
    int kofs[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) kofs[ks] = (2 * ks + lh) ^ xs;
    constexpr int KS = BK / 16;  // k-steps per tile
    struct Frag { bf16x8 ah[TM], bh[TN], al[TM], bl[TN]; };
    auto read_frags = [&](const uint4* st, int ks, Frag& f) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            f.ah[i] = as_bf16x8(st[rowA + i * 32 * CPR + kofs[ks]]);
            if constexpr (NP == 2) f.al[i] = as_bf16x8(st[PA + rowA + i * 32 * CPR + kofs[ks]]);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            f.bh[j] = as_bf16x8(st[rowB + j * 32 * CPR + kofs[ks]]);
            if constexpr (NP == 2) f.bl[j] = as_bf16x8(st[PB + rowB + j * 32 * CPR + kofs[ks]]);
        }
    };
    auto mfma_step = [&](const Frag& f) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (NP == 2) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.al[i], f.bh[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ah[i], f.bl[j], acc[i][j], 0, 0, 0);
                }
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ah[i], f.bh[j], acc[i][j], 0, 0, 0);
            }
    };

    if constexpr (NP == 1) {
        // Software-pipelined main loop: the fragments of k-step ks+1 are fetched (and fenced ahead of
        // the MFMAs: left to itself the scheduler sinks the fetches to share registers) while the MFMAs
        // of k-step ks run.  The single barrier per k-tile sits before the last k-step, when every
        // fragment of the tile is in registers: it frees this stage for the copies of tile kt+2 and
        // publishes tile kt+1, whose first fragments are fetched under the last MFMAs.
        static_assert(KS % 2 == 0, "fragment buffers alternate per k-step");
        Frag F[2];
        auto tile_body = [&](const uint4* cur, const uint4* oth, int kt) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks == KS - 1) {
                    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's copies of tile kt+1 have landed
                    __syncthreads();                     // ... and everybody else's; nobody reads `cur` any more
                    if (kt + 2 < kt_end) issue(kt + 2, cur);
                    if (kt + 1 < kt_end) read_frags(oth, 0, F[(ks + 1) & 1]);
                } else {
                    read_frags(cur, ks + 1, F[(ks + 1) & 1]);
                }
                __builtin_amdgcn_sched_barrier(0);
                mfma_step(F[ks & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        int kt = kt_begin;
        if (kt_begin < kt_end) {
            issue(kt_begin, stage0);
            if (kt_begin + 1 < kt_end) issue(kt_begin + 1, stage1);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            read_frags(stage0, 0, F[0]);
        }
        for (; kt + 1 < kt_end; kt += 2) {
            tile_body(stage0, stage1, kt);
            tile_body(stage1, stage0, kt + 1);
        }
        if (kt < kt_end) tile_body(stage0, stage1, kt);
    } else {
        // hi+lo planes (three MFMAs per fragment pair): pipelining the fetches measures no gain; a k-step
        // fetches its own fragments
        auto compute = [&](const uint4* st) {
    #pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                Frag f;
                read_frags(st, ks, f);
                mfma_step(f);
            }
        };
        if (kt_begin < kt_end) issue(kt_begin, stage0);
        int kt = kt_begin;
        for (; kt + 1 < kt_end; kt += 2) {
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's copies of tile kt have landed
            __syncthreads();                     // ... and everybody else's; stage1 is free again
            issue(kt + 1, stage1);
            __builtin_amdgcn_sched_barrier(0);   // keep the copies ahead of the MFMA loop
            compute(stage0);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            if (kt + 2 < kt_end) issue(kt + 2, stage0);
            __builtin_amdgcn_sched_barrier(0);
            compute(stage1);
        }
        if (kt < kt_end) {  // odd number of k-tiles: the last one sits in stage0
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            compute(stage0);
        }
    }
    __syncthreads();
    if constexpr (SWIGLU) {
        store_swiglu<TM, TN>(p, acc, m0 + wm * WM, n0 + wn * (WN / 2), lane, bz);
    } else {
        // wave-private staging tiles: first half of the waves in stage0, second half in stage1
        static_assert((NW / 2) * WBUF * 2 <= STAGE * 16, "staging does not fit");
        bf16_t* wbuf = reinterpret_cast<bf16_t*>(wave < NW / 2 ? stage0 : stage1) + (wave % (NW / 2)) * WBUF;
        store_outputs<TM, TN>(p, acc, wbuf, m0 + wm * WM, n0 + wn * WN, lane, bz,
                              p.ksplit > 1 ? (int64_t)kz * p.sKsplit : 0);
    }
}

template <int BM, int BN, int WM, int WN, int NP, bool SWIGLU>
hipError_t launch_async(hipStream_t st, const GemmArgs& g) {
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    auto kern = gemm_bf16_async_kernel<BM, BN, WM, WN, NP, SWIGLU>;
    const int tilesM = (g.M + BM - 1) / BM;
    const int tilesN = (g.N + (SWIGLU ? BN / 2 : BN) - 1) / (SWIGLU ? BN / 2 : BN);
    dim3 grid(tilesM * tilesN * g.batch, 1, g.ksplit > 1 ? g.ksplit : 1);
    if (g.symmetric) grid = dim3(tilesM * (tilesM + 1) / 2 * g.batch * (g.ksplit > 1 ? g.ksplit : 1), 1, 1);
    hipLaunchKernelGGL(kern, grid, dim3(NT), 0, st, g, tilesM, tilesN);
    return hipGetLastError();
}

}  // namespace

bool gemm_nt_mfma_big(const GemmArgs& g) {
    const int bn = g.swiglu ? 128 : 256;  // output columns per 256-wide tile
    const int64_t tiles =
        (int64_t)((g.M + 255) / 256) * ((g.N + bn - 1) / bn) * g.batch * (g.ksplit > 1 ? g.ksplit : 1);
    return tiles >= 128 && g.M >= 256 && g.N >= bn;
}

bool gemm_nt_mfma_ok(const GemmArgs& g) {
    const bool split = g.A_lo != nullptr || g.B_lo != nullptr;
    if (split && (!g.A_lo || !g.B_lo || g.swiglu)) return false;
    const int bk = split ? 32 : 64;
    if (g.K < bk || g.K % bk || g.lda % 8 || g.ldb % 8 || g.sA % 8 || g.sB % 8) return false;
    if (((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15) || ((uintptr_t)g.A_lo & 15) || ((uintptr_t)g.B_lo & 15))
        return false;
    if (g.symmetric && g.M != g.N) return false;
    if (g.CT32) return false;  // fp32 transposed output: only the SIMT kernel writes it
    // copies address an operand as a base plus a 32-bit byte offset within the batch item
    if ((int64_t)g.M * g.lda * 2 >= (1ll << 31) || (int64_t)g.N * (g.swiglu ? 2 : 1) * g.ldb * 2 >= (1ll << 31)) return false;
    if (g.ksplit > 1 && (g.C16 || g.CT16)) return false;
    return true;
}

hipError_t gemm_nt_mfma(hipStream_t st, const GemmArgs& g) {
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
    if (!gemm_nt_mfma_ok(g)) return hipErrorInvalidValue;
    const bool big = gemm_nt_mfma_big(g);
    if (g.A_lo) {
        // triangular apply: 256×128 tiles give two rounds of workgroups whose K extents pair up
        if (big && g.b_lower && !g.symmetric && g.ksplit <= 1) return launch_async<256, 128, 64, 64, 2, false>(st, g);
        if (big) return launch_async<256, 256, 128, 64, 2, false>(st, g);
        return launch_async<128, 128, 64, 64, 2, false>(st, g);
    }
    if (g.swiglu) {
        if (big) return launch_async<256, 256, 128, 64, 1, true>(st, g);
        return launch_async<128, 128, 64, 64, 1, true>(st, g);
    }
    if (big) return launch_async<256, 256, 128, 64, 1, false>(st, g);
    return launch_async<128, 128, 64, 64, 1, false>(st, g);
}

}  // namespace atp
