/*
 * atp.h — C ABI of the MI355X (gfx950) hot path of ATP, "attention on top
 * principal keys".
 *
 * Notation follows the paper: X (L×d) hidden state of one sequence, U (L×r)
 * orthonormal left basis, X' = B_r (r×d) principal components, W (d×d')
 * projection weights, Q', K', V' (r×d') principal queries / keys / values.
 *
 * Conventions shared by every call
 *  - Every matrix pointer is a DEVICE pointer owned by the caller, row-major,
 *    contiguous, 16-byte aligned.  The library allocates no device memory and
 *    frees nothing; scratch memory comes in through the `workspace` argument,
 *    whose minimum size the matching `*_workspace` query returns (host call, no
 *    GPU work).  Two kinds of small HIP objects ARE created lazily, both only
 *    by options that are off by default: HIP events while kernel timing is
 *    enabled (atp_profile_enable), and one extra stream plus 64 events on the
 *    first call after atp_set_overlap(1).  atp_init() creates the latter ahead
 *    of time; call it before capturing a HIP graph that uses the overlap option.
 *    The option setters, atp_init and the timing calls keep process-wide state
 *    and are not thread-safe: call them from one thread, between calls.
 *  - `t` is the storage type of all matrix arguments of that call (ATP_F32 or
 *    ATP_BF16); accumulation is always fp32.  Inputs are never modified,
 *    outputs are fully overwritten.
 *  - All work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *    the null stream) and the call returns without synchronising.
 *  - The return value reports host-side argument checks and launch errors
 *    only; numerical breakdown is reported on the device through `info`.
 *  - Same inputs (and same seed) give bit-identical outputs run to run.
 */
#ifndef ATP_H
#define ATP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ATP_OK = 0,
    ATP_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, misaligned pointer, bad enum */
    ATP_ERR_BAD_RANK = 2,    /* r outside 1 … min(L, d) */
    ATP_ERR_WORKSPACE = 3,   /* workspace missing or smaller than the query says */
    ATP_ERR_UNSUPPORTED = 4, /* shape the kernels do not cover (e.g. head width) */
    ATP_ERR_DEVICE = 5,      /* a HIP call failed (launch error) */
    ATP_ERR_SCRATCH_LIMIT = 6 /* atp_attention_static: input needs more than ATP_STATIC_SCRATCH_BYTES */
} atp_status;

typedef enum { ATP_F32 = 0, ATP_BF16 = 1 } atp_dtype;

/* layout of the weight operand of atp_lowrank_linear */
typedef enum {
    ATP_W_KN = 0, /* W[k][n], the paper's X'·W as written (Eq.6) */
    ATP_W_NK = 1  /* Wᵀ stored as [n][k]: weights packed once at load time */
} atp_wlayout;

typedef enum {
    ATP_EPI_NONE = 0,
    ATP_EPI_SWIGLU = 1 /* out[:, j] = SiLU(acc[:, j]) · acc[:, j + n/2], j < n/2 */
} atp_epilogue;

const char* atp_status_string(atp_status s);

/* Library / build identification (static string). */
const char* atp_version(void);

/* Optional one-time set-up on the current device, outside any stream capture: resolves the device
 * address of the built-in scratch buffer of atp_attention_static and creates the stream and events
 * the overlap option uses.  Every entry point also works without it (the set-up then happens inside
 * the first call that needs it).  Returns ATP_ERR_DEVICE if a HIP call fails. */
atp_status atp_init(void);

/* --------------------------------------------------------------------------
 * atp_principal_bases — top-r principal bases of each L×d input (Eq.5, Eq.9).
 *
 * Computes, for every sequence b of the batch, X_b ≈ U_r · B_r with U_rᵀU_r = I
 * (text after Eq.8) by block orthogonal iteration:
 *     U ← qf(X·Ω);  repeat `iters` times { V ← qf(Xᵀ·U);  U ← qf(X·V) };
 *     B_r = U_rᵀ·X,
 * where qf is the Q factor of the thin QR with positive-diagonal R, computed by
 * rounds of CholeskyQR.  Intermediate orthonormalisations use shifted rounds only
 * (they keep the iterate well conditioned; in exact arithmetic any such
 * triangular normalisation leaves the final U_r unchanged); the last one ends
 * with an unshifted round that makes U_r orthonormal to working accuracy.  In exact arithmetic
 * U_r = qf(X (XᵀX)^iters Ω); the subspace converges to the one spanned by the r
 * leading left singular vectors, the minimiser of Eq.9.
 *
 *  X         [batch, L, d]  in   device, storage type t
 *  Omega     [d, r]         in   device, fp32, start block shared by the batch;
 *                                NULL → generated on the device from `seed`
 *                                with the library's counter-based Gaussian
 *                                generator
 *  U_r       [batch, L, r]  out  device, type t, orthonormal columns
 *  B_r       [batch, r, d]  out  device, type t, = U_rᵀ·X (with the returned U_r)
 *  U_master  [batch, L, r]  out  device, fp32 copy of U_r before rounding to t;
 *                                may be NULL
 *  info      [batch]        out  device int32; 0 = U_r is certified: all pivots
 *                                of the last (unshifted) Cholesky round were
 *                                >= 1e-3 and no shifted round met a pivot at
 *                                noise level.  j > 0 = first column (1-based) where
 *                                that failed: the matrix to orthonormalise was
 *                                numerically rank deficient beyond what the
 *                                shifted rounds repair (e.g. X = 0), and U_r may
 *                                not be orthonormal.  A column whose pivot is at
 *                                noise level (<= 1e-6 of its scaled norm) is
 *                                dropped (zero column) rather than divided by,
 *                                so finite input gives finite output.  -1: a wait inside the
 *                                single-launch factorisation gave up (its workgroups
 *                                were not all resident, see atp_set_factor_mode; or
 *                                the input was not finite).  May be NULL.
 *  workspace                     device, ≥ atp_principal_bases_workspace bytes
 *
 * Errors: ATP_ERR_INVALID_ARG (null X/U_r/B_r, batch/L/d < 1, iters < 0, bad t,
 * misaligned pointer), ATP_ERR_BAD_RANK (r < 1 or r > min(L, d)),
 * ATP_ERR_WORKSPACE, ATP_ERR_DEVICE.
 * -------------------------------------------------------------------------- */
size_t atp_principal_bases_workspace(int64_t batch, int64_t L, int64_t d, int64_t r,
                                     int iters, atp_dtype t);

atp_status atp_principal_bases(const void* X, int64_t batch, int64_t L, int64_t d,
                               int64_t r, int iters, const float* Omega, uint64_t seed,
                               void* U_r, void* B_r, float* U_master, int32_t* info,
                               void* workspace, size_t workspace_bytes, atp_dtype t,
                               void* hip_stream);

/* Number of CholeskyQR passes used for the first orthonormalisation (of X·Ω),
 * for the intermediate ones, and for the last one (which produces U_r).  Each
 * value is clamped to 1 … 4.  Process-wide; defaults 2, 1, 2.  Host call. */
void atp_set_qr_passes(int first, int middle, int last);

/* While the r×r factorisation of an orthonormalisation round is still working on later block
 * columns, the finished 256-column blocks of Z·R⁻¹ and of the product that consumes them
 * (Xᵀ·U, X·V or B_r = U_rᵀ·X) run on a second, library-owned HIP stream (created on first use,
 * default priority; forked from and joined back into the caller's stream with events inside the
 * call, so the call keeps its single-stream semantics).  Results do not depend on the setting.
 * Used on the ATP_BF16 path when r is a multiple of 256 and r >= 512.  Process-wide, default off
 * (measured gain at batch 4, L = d = 4096, r = 1024: 1.2 %; the factorisation slows down almost as
 * much as the products are hidden).  Host call. */
void atp_set_overlap(int on);

/* How the r×r Cholesky factorisation (with inverse) inside every orthonormalisation round runs.
 * 1 (default): as ONE launch whenever r <= 2048 and the whole batch fits the chip (at r = 1024: up
 * to 4 sequences): a grid of co-resident workgroups keeps the 64×64 tiles in registers and passes
 * finished panel tiles through global memory and flags.  Every workgroup of that launch must be
 * resident at the same time, so while this mode is on, calls of atp_principal_bases must not
 * overlap in time with each other on one GPU (different streams or processes); a wait that gives
 * up makes the call return info = -1 for that sequence instead of hanging.  Larger batches take
 * the launch-per-block-column form, whose launches cover all sequences at once.
 * 2: the single-launch form also for larger batches, as several launches one after the other
 * (measured slower than mode 0 from batch 8 on at r = 1024; kept for tests and measurements).
 * 0: one launch per 64-wide block column (no residency requirement; at small batch slower: the
 * chain of launches is latency-bound).  Results of the modes agree to rounding.  Values outside
 * 0..2 are clamped.  Process-wide.  Host call. */
void atp_set_factor_mode(int mode);

/* Number of polls after which a wait inside the single-launch factorisation gives up (the call then
 * reports info = -1 for that sequence and every workgroup of it exits).  The default (any value
 * < 1 restores it) is about 4 million polls, seconds beyond any healthy wait; a tiny value makes
 * every wait give up at once, which is how the tests exercise that path.  Process-wide.  Host call. */
void atp_set_factor_spin_limit(int polls);

/* Gram matrix of the SHIFTED (conditioning-only) CholeskyQR rounds on the ATP_BF16 path.
 * 0 (default): from both bf16 planes of the iterate (three MFMA products), as in the last, unshifted
 * round.  1: the single-round orthonormalisations between the products with X and Xᵀ use the leading
 * plane alone (one product); 2: every shifted round does.  R stays an exact triangular factor and
 * Z·R^-1 is always formed from both planes, so U_r = qf(X (XᵀX)^iters Ω) is unchanged in exact
 * arithmetic, but the rounds condition less well: harmless while σ_1/σ_r of the input is below about
 * 1e4 (orthonormality of U_r within 5e-5 on the benchmark inputs), not beyond (at σ_1/σ_r = 5e4 the
 * fp32 copy of U_r loses orthonormality: 1e-4 -> 2e-3 -> 8e-2 for levels 0, 1, 2).  Process-wide.
 * Host call. */
void atp_set_conditioning_gram(int level);

/* --------------------------------------------------------------------------
 * atp_alternating_bases — the paper's own extractor (Alg.1, appendix "Alternating
 * Optimization"): for component i = 1 … r, starting from the i-th column v of V0,
 *     repeat `sweeps` times { u ← X·v / ‖v‖² ;  v ← Xᵀ·u / ‖u‖² } ;   X ← X − u·vᵀ
 * (Alg.1 fixes sweeps = 2).  Because the last update is v = Xᵀu/‖u‖², the deflation removes the
 * component of X along u, so the u_i come out mutually orthogonal and Σ u_i·v_iᵀ = P_U·X: the result
 * is returned in the same form as atp_principal_bases,
 *     U_r[:, i] = u_i / ‖u_i‖   (orthonormal columns),   B_r[i, :] = ‖u_i‖ · v_iᵀ   (= U_rᵀ·X).
 * The caller's X is not modified (the deflation runs on an fp32 copy in the workspace).  Components
 * are inherently sequential and every sweep is one HBM-bound pass over the L×d copy.
 *
 *  X [batch, L, d] in (type t);  V0 [d, r] fp32 start vectors shared by the batch, NULL → generated
 *  from `seed`;  U_r [batch, L, r], B_r [batch, r, d] out (type t);  info [batch] out, may be NULL:
 *  0, or i+1 for the first component i whose ‖u‖ vanished (no energy left: that column of U_r and
 *  row of B_r are zero).
 * Errors: as atp_principal_bases; ATP_ERR_UNSUPPORTED for d > 4096 or d not a multiple of 4.
 * -------------------------------------------------------------------------- */
size_t atp_alternating_bases_workspace(int64_t batch, int64_t L, int64_t d, int64_t r, atp_dtype t);

atp_status atp_alternating_bases(const void* X, int64_t batch, int64_t L, int64_t d, int64_t r, int sweeps,
                                 const float* V0, uint64_t seed, void* U_r, void* B_r, int32_t* info,
                                 void* workspace, size_t workspace_bytes, atp_dtype t, void* hip_stream);

/* --------------------------------------------------------------------------
 * atp_rayleigh_ritz — turns any orthonormal basis pair (U_r, B_r = U_rᵀX) of a subspace into the
 * singular basis of the rank-r approximation U_r·B_r, the X' = [σ_1 v_1 … σ_r v_r] of Eq.9, and
 * returns the diagnostics the paper derives from the singular values.
 *   T = B_r·B_rᵀ = R·Λ·Rᵀ (cyclic two-sided Jacobi, fp32, `sweeps` sweeps of r-1 rounds; 10 are
 *   enough for r ≤ 2048); columns of R ordered by descending eigenvalue;
 *   U_out = U_r·R,  B_out = Rᵀ·B_r  (so U_out·B_out = U_r·B_r, rows of B_out mutually orthogonal);
 *   sigma_i = sqrt(λ_i) = ‖B_out[i, :]‖;
 *   sign: 1ᵀ·u_i ≥ 0 (the 1·U term of Eq.8); when |1ᵀ·u_i| is below the rounding level of the
 *   storage type (1e-5·√L fp32, 2e-4·√L bf16) the largest-magnitude entry of B_out[i, :] is made
 *   positive instead.
 * T is formed and diagonalised in fp32: eigenvalues are accurate to ≈1e-7·λ_1 and eigenvector i is
 * resolved to ≈1e-7·λ_1/(gap to its neighbours), i.e. directions whose σ is below ≈3e-4·σ_1 come
 * out as an arbitrary orthonormal basis of their span.
 * After this the layer output no longer depends on the start block Ω once the iteration has
 * converged.  diagnostics[b] = { Σλ = ‖B_r‖²_F (captured energy, numerator of Fig.5's ratio),
 * max_{i≠j}|T_ij| / max λ after the last sweep (convergence of the Jacobi method),
 * μ = −log2 Σ_i (σ_i/Σσ)² (Eq.4), ⌈2^μ⌉ (components Eq.4 asks for) }.
 *
 *  U_r [batch, L, r], B_r [batch, r, d] in (type t);  U_out, B_out same shapes, out, must not
 *  alias the inputs;  sigma [batch, r] fp32 out;  diagnostics [batch, 4] fp32 out, may be NULL.
 * Errors: as atp_principal_bases; ATP_ERR_UNSUPPORTED for r > 4096.
 * -------------------------------------------------------------------------- */
size_t atp_rayleigh_ritz_workspace(int64_t batch, int64_t L, int64_t d, int64_t r, atp_dtype t);

atp_status atp_rayleigh_ritz(const void* U_r, const void* B_r, int64_t batch, int64_t L, int64_t d, int64_t r,
                             int sweeps, void* U_out, void* B_out, float* sigma, float* diagnostics,
                             void* workspace, size_t workspace_bytes, atp_dtype t, void* hip_stream);

/* --------------------------------------------------------------------------
 * atp_lowrank_linear — projection of the r principal components instead of the
 * L tokens: Q', K', V' = X'·{W^Q, W^K, W^V} (Eq.6; Tab.1 row "Projection",
 * cost O(r·d·d')).  A plain batched product out_b = B_b · W; with m = L it is
 * also the dense projection X·W of Eq.2 and the query expansion Q = U·Q' of
 * Eq.6 (there W differs per sequence: w_stride = k·n).
 *
 *  B         [batch, m, k]  in   device, type t
 *  W         in   device, type t; [k, n] for ATP_W_KN, [n, k] for ATP_W_NK;
 *                 item b starts at W + b·w_stride elements (0 = shared weights)
 *  out       out  device, type t; [batch, m, n] for ATP_EPI_NONE,
 *                 [batch, m, n/2] for ATP_EPI_SWIGLU (gate columns first, then
 *                 up columns, in W: the gated feed-forward applied to the bases)
 *  workspace      device; needed only for (ATP_BF16, ATP_W_KN): the call
 *                 transposes W there first.  May be NULL when the query
 *                 returns 0.
 *
 * Errors: ATP_ERR_INVALID_ARG (null pointer, size < 1, n odd with SWIGLU, bad
 * enum, misaligned pointer), ATP_ERR_WORKSPACE, ATP_ERR_DEVICE.
 * -------------------------------------------------------------------------- */
size_t atp_lowrank_linear_workspace(int64_t batch, int64_t m, int64_t k, int64_t n,
                                    int64_t w_stride, atp_wlayout w_layout, atp_dtype t);

atp_status atp_lowrank_linear(const void* B, const void* W, void* out, int64_t batch,
                              int64_t m, int64_t k, int64_t n, int64_t w_stride,
                              atp_wlayout w_layout, atp_epilogue epilogue, void* workspace,
                              size_t workspace_bytes, atp_dtype t, void* hip_stream);

/* --------------------------------------------------------------------------
 * atp_attention — softmax attention of all L queries over the r principal keys
 * and values (Fig.2b; Tab.1 row "Attention": Q·K'ᵀ, cost O(r·L·d'), the L×r
 * attention map is never written to memory).  Per sequence b, head h (columns
 * h·d_h … (h+1)·d_h − 1, d_h = dq / heads) and query row i:
 *     s_j = scale · <Q[i, h], K_r[j, h]>,  p = softmax_j(s),  O[i, h] = Σ_j p_j · V_r[j, h]
 * (Eq.1 with K', V' in place of K, V).  No mask, no bias, no dropout.  With
 * r = L, K_r = K and V_r = V it is standard dense self-attention (Eq.1), used as
 * the comparator.
 *
 *  Q    [batch, L, dq] in;  K_r, V_r [batch, r, dq] in;  O [batch, L, dq] out
 *  scale  ≤ 0 → 1/sqrt(d_h)
 *  workspace  device; ATP_BF16 needs it (V_r is re-laid out per head there)
 *
 * Errors: ATP_ERR_INVALID_ARG (null pointer, size < 1, dq % heads ≠ 0,
 * misaligned pointer), ATP_ERR_UNSUPPORTED (ATP_BF16 with d_h not in {64, 128};
 * ATP_F32 with d_h > 256), ATP_ERR_WORKSPACE, ATP_ERR_DEVICE.
 * -------------------------------------------------------------------------- */
size_t atp_attention_workspace(int64_t batch, int64_t L, int64_t r, int64_t dq, int heads,
                               atp_dtype t);

atp_status atp_attention(const void* Q, const void* K_r, const void* V_r, void* O,
                         int64_t batch, int64_t L, int64_t r, int64_t dq, int heads,
                         float scale, void* workspace, size_t workspace_bytes, atp_dtype t,
                         void* hip_stream);

/* --------------------------------------------------------------------------
 * atp_attention_static — atp_attention for callers that cannot allocate or pass scratch memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments and results as atp_attention without `workspace`; the re-laid-out values go to a
 * buffer of ATP_STATIC_SCRATCH_BYTES that is built into the library (one copy per GPU, resident
 * until the process ends; its address on the current device is resolved by atp_init() or by the
 * first call).  Calls no hipMalloc / hipFree or other allocating routine.
 * Limit: batch · dq · ceil64(r) · 2 bytes ≤ ATP_STATIC_SCRATCH_BYTES for ATP_BF16 (ATP_F32 uses no
 * scratch); larger inputs return ATP_ERR_SCRATCH_LIMIT and enqueue nothing.
 * Every call on one GPU uses that GPU's single buffer: two calls that overlap in time on one GPU
 * (different streams or threads) race; serialise them.  Other errors as atp_attention.
 * -------------------------------------------------------------------------- */
#define ATP_STATIC_SCRATCH_BYTES (32u << 20)

atp_status atp_attention_static(const void* Q, const void* K_r, const void* V_r, void* O,
                                int64_t batch, int64_t L, int64_t r, int64_t dq, int heads,
                                float scale, atp_dtype t, void* hip_stream);

/* --------------------------------------------------------------------------
 * atp_attention_linearised — first-order attention over the r principal keys (Eq.8): the
 * exponential of the attention weights is replaced by its first-order Taylor expansion, which for
 * K = U·K', V = U·V' and UᵀU = I turns the unnormalised attention of a query q on all L tokens into
 * A'·V' with the 1×r map
 *     A' = 1·U_r + scale·q·K'ᵀ        (1·U_r = column sums of U_r, shared by the heads).
 * The row-wise normalisation the text after Eq.8 asks for is applied in one of two ways:
 *   ATP_NORM_TAYLOR  divide by the same expansion of the softmax denominator,
 *                    L + scale·(q·K'ᵀ)·(1·U_r)ᵀ   (= Σ over the L tokens of 1 + scale·q·k_j);
 *   ATP_NORM_ROWSUM  divide by the sum of the r entries of A'.
 * With ATP_NORM_TAYLOR the output equals the token-by-token first-order attention on an input of
 * rank r and does not depend on the orthonormal basis chosen.  A query whose denominator is zero
 * gives non-finite output rows (the expansion is only meaningful while |scale·q·k_j| is small).
 *
 *  Q [batch, L, dq] in;  K_r, V_r [batch, r, dq] in;  U_r [batch, L, r] in (type t);
 *  O [batch, L, dq] out;  heads, scale, workspace, stream and errors as for atp_attention
 *  (workspace size from atp_attention_linearised_workspace; needed for both types).
 * -------------------------------------------------------------------------- */
typedef enum { ATP_NORM_TAYLOR = 0, ATP_NORM_ROWSUM = 1 } atp_lin_norm;

size_t atp_attention_linearised_workspace(int64_t batch, int64_t L, int64_t r, int64_t dq, int heads,
                                          atp_dtype t);

atp_status atp_attention_linearised(const void* Q, const void* K_r, const void* V_r, const void* U_r, void* O,
                                    int64_t batch, int64_t L, int64_t r, int64_t dq, int heads, float scale,
                                    atp_lin_norm norm, void* workspace, size_t workspace_bytes, atp_dtype t,
                                    void* hip_stream);

/* --------------------------------------------------------------------------
 * Rotary position encoding with principal keys (Sec. "Combine with Position Encoding"):
 * k_i = x_i·W^K·R_i with R_i the rotary matrix of position i; the r principal keys are then the
 * coordinates of the rotated key matrix in the basis U_r:
 *     K = U_r·K'_0 (atp_lowrank_linear),  K̃ = RoPE(K) (atp_rope),  K' = U_rᵀ·K̃ (atp_project_onto_bases);
 * queries: Q̃ = RoPE(U_r·Q').
 *
 * atp_rope rotates every row i of Y [batch, L, dq] by position pos0 + i.  The paper leaves the
 * layout of R_i open; the half-split pairing of the Llama family is used: within a head of width
 * d_h = dq/heads (even), coordinate j < d_h/2 is paired with j + d_h/2 and the pair (a, b) becomes
 * (a·cos θ − b·sin θ, a·sin θ + b·cos θ), θ = (pos0 + i)·base^(−2j/d_h).  out may equal Y.
 *
 * atp_project_onto_bases: out [batch, r, dq] = U_rᵀ·Y for U_r [batch, L, r], Y [batch, L, dq]
 * (coordinates of the projection of Y on the subspace; with Y = X it is B_r of Eq.5).
 * Errors: ATP_ERR_INVALID_ARG (null/misaligned pointer, size < 1, dq % heads ≠ 0, odd d_h,
 * base ≤ 1, pos0 < 0), ATP_ERR_WORKSPACE (ATP_BF16 projection needs the transposed operands there).
 * -------------------------------------------------------------------------- */
atp_status atp_rope(const void* Y, void* out, int64_t batch, int64_t L, int64_t dq, int heads, float base,
                    int64_t pos0, atp_dtype t, void* hip_stream);

size_t atp_project_onto_bases_workspace(int64_t batch, int64_t L, int64_t r, int64_t dq, atp_dtype t);

atp_status atp_project_onto_bases(const void* U_r, const void* Y, void* out, int64_t batch, int64_t L,
                                  int64_t r, int64_t dq, void* workspace, size_t workspace_bytes,
                                  atp_dtype t, void* hip_stream);

/* --------------------------------------------------------------------------
 * Residual and Norm on factored matrices, for chaining blocks (Fig.3; last paragraph of Sec.4.2: the next
 * block first attains the principal components of this block's output Y).  Fig.3 gives no equations;
 * the reading implemented here keeps every tensor of the residual stream as a pair (basis, coefficients):
 *   first residual   H = U·X' + U_o·A            = P·C,  P = [U | U_o] (L×2r), C = [X'; A] (2r×d)
 *   Norm             Norm(H) = Pn·Cn,  Cn = (C − c̄·1ᵀ)·diag(gain), Pn[i,:] = P[i,:]/sqrt(var_i + eps),
 *                    var_i = mean square of row i of P·(C − c̄·1ᵀ) = p_i·M·p_iᵀ/d, M = (C − c̄·1ᵀ)(C − c̄·1ᵀ)ᵀ;
 *                    c̄ = C·1/d when `center` (LayerNorm without bias), 0 otherwise (RMSNorm)
 *   feed-forward     F = FFN(Cn) row-wise (atp_lowrank_linear with the SWIGLU epilogue, then the down projection)
 *   second residual  Y = H + Pn·F                 = [P | Pn]·[C; F]  (atp_concat_factors, then atp_lowrank_linear
 *                    with the per-sequence weight [C; F] to obtain the dense Y for the next block).
 * H is never formed: the row statistics come from the 2r×2r matrix M.
 *
 * atp_concat_factors: P [batch, L, r1+r2] = [U1 | U2], C [batch, r1+r2, d] = [C1; C2] (all type t).
 * atp_norm_factored:  P [batch, L, m], C [batch, m, d] in; gain [d] fp32, shared by the batch; Pn, Cn out, same
 *                     shapes (may not alias the inputs); eps >= 0.
 * Errors: ATP_ERR_INVALID_ARG (null / misaligned pointer, size < 1, bad t, eps < 0), ATP_ERR_WORKSPACE,
 * ATP_ERR_UNSUPPORTED (atp_concat_factors with L or r1+r2 above 65535).
 * -------------------------------------------------------------------------- */
atp_status atp_concat_factors(const void* U1, const void* C1, const void* U2, const void* C2, void* P, void* C,
                              int64_t batch, int64_t L, int64_t d, int64_t r1, int64_t r2, atp_dtype t,
                              void* hip_stream);

size_t atp_norm_factored_workspace(int64_t batch, int64_t L, int64_t d, int64_t m, atp_dtype t);

atp_status atp_norm_factored(const void* P, const void* C, const float* gain, float eps, int center, void* Pn,
                             void* Cn, int64_t batch, int64_t L, int64_t d, int64_t m, void* workspace,
                             size_t workspace_bytes, atp_dtype t, void* hip_stream);

/* --------------------------------------------------------------------------
 * Kernel timing with HIP events (diagnostic; used by the benchmark to measure
 * per-kernel durations live, on the stream the kernels are launched on).
 * While a class bit is enabled every launch of that class is bracketed by two
 * events.  Host calls; atp_profile_read waits for the recorded events.
 * -------------------------------------------------------------------------- */
typedef enum {
    ATP_K_GEMM_BF16 = 0,        /* bf16·bf16 MFMA GEMM, 256×256 tile                */
    ATP_K_GEMM_BF16_SMALL = 1,  /* same, 128×128 tile                               */
    ATP_K_GEMM_SWIGLU = 2,      /* bf16·bf16 MFMA GEMM with SiLU·mul epilogue       */
    ATP_K_GEMM_SPLIT_GRAM = 3,  /* hi/lo bf16 planes: Gram matrix ZᵀZ               */
    ATP_K_GEMM_SPLIT_APPLY = 4, /* hi/lo bf16 planes: Z·R⁻¹                         */
    ATP_K_ATTENTION = 5,
    ATP_K_CHOLESKY = 6,         /* scaling + all block columns of one factorisation */
    ATP_K_STREAM = 7,           /* transposes, casts, fills, column sums, Alg.1     */
    ATP_K_GEMM_SIMT = 8,        /* fp32-FMA GEMM (fp32 path, odd shapes)            */
    ATP_K_COUNT = 9
} atp_kernel_class;

void atp_profile_enable(unsigned class_mask); /* bit c enables class c; 0 disables */
void atp_profile_reset(void);
/* Sums over the launches recorded since the last reset.  flops / bytes are the
 * ALGORITHMIC counts of those launches.  Returns ATP_ERR_INVALID_ARG for a bad class. */
atp_status atp_profile_read(int kernel_class, double* total_ms, int64_t* launches, double* flops,
                            double* bytes);

#ifdef __cplusplus
}
#endif
#endif /* ATP_H */
