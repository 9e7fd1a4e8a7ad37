// Sanitizer driver for the argument-validation layer of the C ABI (csrc/bed_api.hip built for
// the host only, launchers replaced by tests/sanitize/api_stubs.cpp).  Every entry point is
// called with each class of bad argument (which must be refused with the documented code before
// any launcher is reached) and once with valid arguments (which must reach a launcher exactly
// once); pointer values are made-up device addresses that the layer may compare but never read.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <limits>

#include "bed.h"

extern int g_stub_launches;

static int failures = 0;
#define EXPECT(call, code)                                                            \
    do {                                                                              \
        const int before_ = g_stub_launches;                                          \
        const int st_ = (call);                                                       \
        const int want_ = (code);                                                     \
        const int launches_ = g_stub_launches - before_;                              \
        if (st_ != want_ || launches_ != ((want_ == BED_OK) ? 1 : 0)) {               \
            std::fprintf(stderr, "%s:%d: %s -> %d (%d launches), expected %d\n", __FILE__, __LINE__, #call, st_, \
                         launches_, want_);                                           \
            ++failures;                                                               \
        }                                                                             \
    } while (0)
#define EXPECT_NOOP(call)                                                             \
    do {                                                                              \
        const int before_ = g_stub_launches;                                          \
        const int st_ = (call);                                                       \
        if (st_ != BED_OK || g_stub_launches != before_) {                            \
            std::fprintf(stderr, "%s:%d: %s -> %d, expected a no-op\n", __FILE__, __LINE__, #call, st_); \
            ++failures;                                                               \
        }                                                                             \
    } while (0)

template <typename T>
static T* dev(uintptr_t a) { return reinterpret_cast<T*>(a); }

int main() {
    float* A = dev<float>(0x10000000);
    float* L = dev<float>(0x20000000);
    float* V = dev<float>(0x30000000);
    float* W = dev<float>(0x40000000);
    float* X = dev<float>(0x50000000);
    int* I = dev<int>(0x60000000);
    unsigned* R = dev<unsigned>(0x70000000);
    void* WS = dev<void>(0x80000000);
    const float inf = std::numeric_limits<float>::infinity();
    const float nan = std::nanf("");
    const int big_n = 128, big_batch = 1 << 20;     // sizes whose byte counts exceed 32 bits

    // bed_syevd / bed_syevd_info
    EXPECT(bed_syevd(A, 8, 16, L, V, nullptr), BED_OK);
    EXPECT(bed_syevd(A, 8, 16, L, nullptr, nullptr), BED_OK);
    EXPECT(bed_syevd(A, big_batch, big_n, L, nullptr, nullptr), BED_ERR_ALIAS);   // 64 GiB of A covers L
    EXPECT(bed_syevd(nullptr, 8, 16, L, V, nullptr), BED_ERR_NULL);
    EXPECT(bed_syevd(A, 8, 16, nullptr, V, nullptr), BED_ERR_NULL);
    EXPECT(bed_syevd(A, -1, 16, L, V, nullptr), BED_ERR_BATCH);
    EXPECT(bed_syevd(A, 8, 0, L, V, nullptr), BED_ERR_N);
    EXPECT(bed_syevd(A, 8, 129, L, V, nullptr), BED_ERR_N);
    EXPECT(bed_syevd(dev<float>(0x10000002), 8, 16, L, V, nullptr), BED_ERR_ALIGN);
    EXPECT(bed_syevd(A, 8, 16, L, dev<float>(0x10000010), nullptr), BED_ERR_ALIAS);
    EXPECT(bed_syevd(A, 8, 16, A + 8 * 16 * 16 - 1, V, nullptr), BED_ERR_ALIAS);
    EXPECT(bed_syevd(A, 8, 16, A + 8 * 16 * 16, V, nullptr), BED_OK);             // adjacent, not overlapping
    EXPECT_NOOP(bed_syevd(nullptr, 0, 16, nullptr, nullptr, nullptr));
    EXPECT(bed_syevd_info(A, 8, 16, L, V, I, R, nullptr), BED_OK);
    EXPECT(bed_syevd_info(A, 8, 16, L, V, dev<int>(0x60000001), R, nullptr), BED_ERR_ALIGN);

    EXPECT(bed_syevd_family(A, 8, 16, L, V, I, R, BED_FAMILY_PACKED, nullptr), BED_OK);
    EXPECT(bed_syevd_family(A, 8, 33, L, V, I, R, BED_FAMILY_PACKED, nullptr), BED_ERR_N);
    EXPECT(bed_syevd_family(A, 8, 9, L, V, I, R, BED_FAMILY_LANE, nullptr), BED_ERR_N);
    EXPECT(bed_syevd_family(A, 8, 16, L, V, I, R, 7, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_family(A, 8, 48, L, nullptr, I, R, BED_FAMILY_PAIR, nullptr), BED_ERR_NULL);
    EXPECT(bed_syevd_family(A, 8, 48, L, V, I, R, BED_FAMILY_PAIR, nullptr), BED_OK);
    EXPECT(bed_syevd_family(A, 8, 16, L, V, I, R, -1, nullptr), BED_ERR_ARG);

    EXPECT(bed_syevd_tol(A, 8, 16, L, V, I, R, 1e-5f, 32, nullptr), BED_OK);
    EXPECT(bed_syevd_tol(A, 8, 16, L, V, I, R, 0.f, 0, nullptr), BED_OK);
    EXPECT(bed_syevd_tol(A, 8, 16, L, V, I, R, -1e-5f, 0, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_tol(A, 8, 16, L, V, I, R, nan, 0, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_tol(A, 8, 16, L, V, I, R, inf, 0, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_tol(A, 8, 16, L, V, I, R, 1e-5f, -1, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_tol(A, 8, 0, L, V, I, R, -1.f, 0, nullptr), BED_ERR_N);
    EXPECT(bed_syevd_tol(nullptr, 8, 16, L, V, I, R, 1e-5f, 0, nullptr), BED_ERR_NULL);

    // stage hooks
    EXPECT(bed_tridiag(A, 8, 16, L, W, V, nullptr), BED_OK);
    EXPECT(bed_tridiag(A, 8, 16, L, W, nullptr, nullptr), BED_OK);
    EXPECT(bed_tridiag(A, 8, 16, nullptr, W, V, nullptr), BED_ERR_NULL);
    EXPECT(bed_tridiag(A, 8, 16, L, L, V, nullptr), BED_ERR_ALIAS);
    EXPECT(bed_tridiag_qr(L, W, 8, 16, X, V, I, R, nullptr), BED_OK);
    EXPECT(bed_tridiag_qr(L, nullptr, 8, 16, X, V, I, R, nullptr), BED_ERR_NULL);
    EXPECT(bed_tridiag_qr(L, W, 8, 16, L, V, I, R, nullptr), BED_ERR_ALIAS);
    EXPECT(bed_tridiag_qr_sweeps(L, W, 8, 16, 2, X, dev<float>(0x58000000), V, R, nullptr), BED_OK);
    EXPECT(bed_tridiag_qr_sweeps(L, W, 8, 16, 0, X, dev<float>(0x58000000), V, R, nullptr), BED_ERR_ARG);
    EXPECT(bed_tridiag_qr_sweeps(L, W, 8, 65, 2, X, dev<float>(0x58000000), V, R, nullptr), BED_ERR_N);
    EXPECT(bed_tridiag_qr_sweeps(L, W, 8, 16, 2, X, X, V, R, nullptr), BED_ERR_ALIAS);

    // spectral function
    EXPECT(bed_spd_fn(A, 8, 16, BED_FN_SQRT, 0.f, V, L, I, nullptr), BED_OK);
    EXPECT(bed_spd_fn(A, 8, 16, BED_FN_INV_SQRT, 1e-6f, V, nullptr, nullptr, nullptr), BED_OK);
    EXPECT(bed_spd_fn(A, 8, 16, 2, 0.f, V, L, I, nullptr), BED_ERR_ARG);
    EXPECT(bed_spd_fn(A, 8, 16, BED_FN_INV_SQRT, 0.f, V, L, I, nullptr), BED_ERR_ARG);
    EXPECT(bed_spd_fn(A, 8, 16, BED_FN_SQRT, -1.f, V, L, I, nullptr), BED_ERR_ARG);
    EXPECT(bed_spd_fn(A, 8, 16, BED_FN_SQRT, nan, V, L, I, nullptr), BED_ERR_ARG);
    EXPECT(bed_spd_fn(A, 8, 16, BED_FN_SQRT, inf, V, L, I, nullptr), BED_ERR_ARG);
    EXPECT(bed_spd_fn(A, 8, 16, BED_FN_SQRT, 0.f, A, L, I, nullptr), BED_ERR_ALIAS);
    EXPECT(bed_spd_fn(A, 8, 16, BED_FN_SQRT, 0.f, nullptr, L, I, nullptr), BED_ERR_NULL);

    // gradients
    EXPECT(bed_syevd_backward(L, V, W, X, 8, 16, BED_GRAD_TAYLOR, 9, 0.f, A, nullptr), BED_OK);
    EXPECT(bed_syevd_backward(L, V, nullptr, X, 8, 16, BED_GRAD_EXACT, 0, 1e-6f, A, nullptr), BED_OK);
    EXPECT(bed_syevd_backward(L, V, nullptr, nullptr, 8, 16, BED_GRAD_TAYLOR, 9, 0.f, A, nullptr), BED_ERR_NULL);
    EXPECT(bed_syevd_backward(L, V, W, X, 8, 16, 5, 9, 0.f, A, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_backward(L, V, W, X, 8, 16, BED_GRAD_TAYLOR, 65, 0.f, A, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_backward(L, V, W, X, 8, 16, BED_GRAD_EXACT, 0, nan, A, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_backward(L, V, W, X, 8, 16, BED_GRAD_TAYLOR, 9, 0.f, V, nullptr), BED_ERR_ALIAS);
    EXPECT(bed_spd_fn_backward(L, V, X, 8, 16, BED_FN_SQRT, 0.f, A, nullptr), BED_OK);
    EXPECT(bed_spd_fn_backward(L, V, X, 8, 16, BED_FN_INV_SQRT, 0.f, A, nullptr), BED_ERR_ARG);
    EXPECT(bed_spd_fn_backward(L, V, X, 8, 16, BED_FN_SQRT, 0.f, X, nullptr), BED_ERR_ALIAS);
    EXPECT(bed_spd_fn_backward(L, nullptr, X, 8, 16, BED_FN_SQRT, 0.f, A, nullptr), BED_ERR_NULL);

    // lock-step procedure, both forms
    const size_t need = bed_syevd_lockstep_workspace(8, 16, 16);
    if (need != ((2 * 8 * 16 + 16 + 8) * 4 + 255) / 256 * 256) { std::fprintf(stderr, "workspace size %zu\n", need); ++failures; }
    if (bed_syevd_lockstep_workspace(-1, 16, 16) != 0 || bed_syevd_lockstep_workspace(8, 65, 16) != 0) ++failures;
    EXPECT(bed_syevd_lockstep(A, 8, 16, 1e-5f, 16, 1, L, V, W, I, WS, need, nullptr), BED_OK);
    EXPECT(bed_syevd_lockstep(A, 8, 16, 1e-5f, 16, 1, L, V, W, I, WS, need - 1, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_lockstep(A, 8, 16, 1e-5f, 16, 1, L, V, W, I, nullptr, need, nullptr), BED_ERR_NULL);
    EXPECT(bed_syevd_lockstep(A, 8, 16, -1.f, 16, 1, L, V, W, I, WS, need, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_lockstep(A, 8, 16, 1e-5f, 16, 3, L, V, W, I, WS, need, nullptr), BED_ERR_ARG);
    EXPECT(bed_syevd_lockstep(A, 8, 16, 1e-5f, 16, 1, L, V, W, I, L, need, nullptr), BED_ERR_ALIAS);
    EXPECT(bed_syevd_lockstep(A, 8, 65, 1e-5f, 16, 1, L, V, W, I, WS, need, nullptr), BED_ERR_N);
    EXPECT(bed_syevd_lockstep_static(A, 8, 16, 1e-5f, 16, 0, L, V, W, I, nullptr), BED_OK);
    EXPECT(bed_syevd_lockstep_static(A, 4096, 64, 1e-5f, 64, 1, L, nullptr, nullptr, nullptr, nullptr), BED_ERR_SCRATCH);
    EXPECT(bed_syevd_lockstep_static(nullptr, 8, 16, 1e-5f, 16, 0, L, V, W, I, nullptr), BED_ERR_NULL);
    if (bed_syevd_lockstep_static_capacity() != (1u << 20)) ++failures;

    for (int code = 0; code >= -9; --code)
        if (!bed_status_string(code) || !bed_status_string(code)[0]) ++failures;
    if (bed_version() != BED_VERSION) ++failures;
    if (!bed_kernel_variant(8, 16, 1) || bed_kernel_variant(8, 0, 1)) ++failures;

    std::printf(failures ? "FAILED (%d)\n" : "api sanitizer driver OK\n", failures);
    return failures ? 1 : 0;
}
