// Host-side paths of the C ABI (argument checks, workspace queries and carve-up arithmetic) exercised
// without a GPU; built together with csrc/api.hip under -fsanitize=address,undefined by
// tests/test_host_sanitizer.py.  Every call below must return before any kernel launch.
#include "../include/atp.h"

#include <cstdio>
#include <cstdlib>
#include <vector>

static int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
    } while (0)

int main() {
    // aligned host memory standing in for device buffers: the checks never dereference them
    std::vector<char> store(4096 + 64);
    char* P = reinterpret_cast<char*>((reinterpret_cast<uintptr_t>(store.data()) + 63) & ~uintptr_t(63));
    char* odd = P + 2;

    for (int s = 0; s <= 7; ++s) EXPECT(atp_status_string((atp_status)s) != nullptr);
    EXPECT(atp_version() != nullptr);

    // workspace queries over a grid of shapes, including the benchmark shapes and ragged / large ones
    const int64_t Ls[] = {1, 7, 128, 512, 4096, 32768, 100003}, ds[] = {1, 52, 64, 768, 4096}, rs[] = {1, 20, 32, 128, 1024, 2048, 4096};
    for (int64_t L : Ls) for (int64_t d : ds) for (int64_t r : rs) for (int t = 0; t < 2; ++t) for (int64_t b : {1, 4, 32}) {
        const size_t w = atp_principal_bases_workspace(b, L, d, r, 2, (atp_dtype)t);
        EXPECT(w > 0 && w % 256 == 0);
        EXPECT(atp_principal_bases_workspace(b + 1, L, d, r, 2, (atp_dtype)t) > w);
        const size_t wa = atp_alternating_bases_workspace(b, L, d, r, (atp_dtype)t);
        const size_t wr = atp_rayleigh_ritz_workspace(b, L, d, r, (atp_dtype)t);
        EXPECT(wa > 0 && wr > 0);
        EXPECT(atp_attention_workspace(b, L, r, d, 1, ATP_F32) == 0);
        EXPECT(atp_attention_linearised_workspace(b, L, r, d, 1, (atp_dtype)t) >= atp_attention_workspace(b, L, r, d, 1, (atp_dtype)t));
        EXPECT(atp_project_onto_bases_workspace(b, L, r, d, ATP_F32) == 0);
        EXPECT(atp_lowrank_linear_workspace(b, r, d, d, 0, ATP_W_NK, (atp_dtype)t) == 0);
        EXPECT(atp_lowrank_linear_workspace(b, r, d, d, d * d, ATP_W_KN, ATP_BF16) >= (size_t)b * d * d * 2);
    }
    EXPECT(atp_principal_bases_workspace(0, 1, 1, 1, 0, ATP_F32) == 0);
    EXPECT(atp_principal_bases_workspace(1, 1, 1, 1, 0, (atp_dtype)5) == 0);

    // argument checks of every entry point (all return on the host)
    const size_t big = size_t(1) << 40;
    EXPECT(atp_principal_bases(nullptr, 1, 128, 64, 32, 2, nullptr, 0, P, P, nullptr, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_principal_bases(P, 1, 128, 64, 65, 2, nullptr, 0, P, P, nullptr, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_BAD_RANK);
    EXPECT(atp_principal_bases(P, 1, 16384, 4096, 8192, 2, nullptr, 0, P, P, nullptr, nullptr, P, big, ATP_BF16, nullptr) == ATP_ERR_BAD_RANK);
    EXPECT(atp_principal_bases(P, 1, 128, 64, 0, 2, nullptr, 0, P, P, nullptr, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_BAD_RANK);
    EXPECT(atp_principal_bases(P, 1, 128, 64, 32, -1, nullptr, 0, P, P, nullptr, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_principal_bases(odd, 1, 128, 64, 32, 2, nullptr, 0, P, P, nullptr, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_principal_bases(P, 1, 128, 64, 32, 2, nullptr, 0, P, P, nullptr, nullptr, P, 16, ATP_F32, nullptr) == ATP_ERR_WORKSPACE);
    EXPECT(atp_principal_bases(P, 1, 128, 64, 32, 2, nullptr, 0, P, P, nullptr, nullptr, nullptr, 0, ATP_F32, nullptr) == ATP_ERR_WORKSPACE);
    EXPECT(atp_principal_bases(P, 70000, 128, 64, 32, 2, nullptr, 0, P, P, nullptr, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_alternating_bases(P, 1, 128, 64, 32, 0, nullptr, 0, P, P, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_alternating_bases(P, 1, 128, 64, 65, 2, nullptr, 0, P, P, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_BAD_RANK);
    EXPECT(atp_alternating_bases(P, 1, 128, 8192, 32, 2, nullptr, 0, P, P, nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_UNSUPPORTED);
    EXPECT(atp_rayleigh_ritz(P, P, 1, 128, 64, 32, 10, P + 64, P + 128, reinterpret_cast<float*>(P), nullptr, P, 16, ATP_F32, nullptr) == ATP_ERR_WORKSPACE);
    EXPECT(atp_rayleigh_ritz(P, P, 1, 128, 64, 32, 10, P, P + 128, reinterpret_cast<float*>(P), nullptr, P, big, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_lowrank_linear(P, P, P, 1, 8, 8, 7, 0, ATP_W_KN, ATP_EPI_SWIGLU, nullptr, 0, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_lowrank_linear(P, P, P, 1, 8, 8, 8, 0, (atp_wlayout)3, ATP_EPI_NONE, nullptr, 0, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_lowrank_linear(P, P, P, 1, 8, 64, 8, 0, ATP_W_KN, ATP_EPI_NONE, nullptr, 0, ATP_BF16, nullptr) == ATP_ERR_WORKSPACE);
    EXPECT(atp_attention(P, P, P, P, 1, 8, 8, 66, 4, 0.f, nullptr, 0, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_attention(P, P, P, P, 1, 8, 8, 96, 1, 0.f, P, big, ATP_BF16, nullptr) == ATP_ERR_UNSUPPORTED);
    EXPECT(atp_attention(P, P, P, P, 1, 8, 8, 64, 1, 0.f, nullptr, 0, ATP_BF16, nullptr) == ATP_ERR_WORKSPACE);
    EXPECT(atp_attention_static(P, P, P, P, 8, 4096, 1024, 4096, 32, 0.f, ATP_BF16, nullptr) == ATP_ERR_SCRATCH_LIMIT);
    EXPECT(atp_attention_static(nullptr, P, P, P, 1, 8, 8, 64, 1, 0.f, ATP_BF16, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_attention_linearised(P, P, P, nullptr, P, 1, 8, 8, 64, 1, 0.f, ATP_NORM_TAYLOR, P, big, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_rope(P, P, 1, 8, 66, 2, 10000.f, 0, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_rope(P, P, 1, 8, 64, 2, 1.0f, 0, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_project_onto_bases(P, P, P, 1, 64, 8, 64, nullptr, 0, ATP_BF16, nullptr) == ATP_ERR_WORKSPACE);
    EXPECT(atp_concat_factors(P, P, P, nullptr, P, P, 1, 8, 8, 2, 2, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_concat_factors(P, P, P, P, P, P, 1, 70000, 8, 2, 2, ATP_F32, nullptr) == ATP_ERR_UNSUPPORTED);
    EXPECT(atp_norm_factored_workspace(2, 100, 64, 48, ATP_BF16) > 0);
    EXPECT(atp_norm_factored(P, P, reinterpret_cast<float*>(P), -1.f, 0, P + 64, P + 128, 1, 8, 8, 4, P, big, ATP_F32, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_norm_factored(P, P, reinterpret_cast<float*>(P), 1e-6f, 0, P + 64, P + 128, 1, 8, 8, 4, P, 16, ATP_F32, nullptr) == ATP_ERR_WORKSPACE);
    double ms; int64_t n;
    EXPECT(atp_profile_read(99, &ms, &n, nullptr, nullptr) == ATP_ERR_INVALID_ARG);
    EXPECT(atp_profile_read(0, &ms, &n, nullptr, nullptr) == ATP_OK && n == 0);
    atp_set_qr_passes(9, 0, 2); atp_set_qr_passes(2, 1, 2);
    atp_set_overlap(0); atp_set_factor_mode(1); atp_set_factor_spin_limit(0); atp_set_conditioning_gram(0);
    std::printf("%s (%d failures)\n", failures ? "FAILED" : "host checks ok", failures);
    return failures ? 1 : 0;
}
