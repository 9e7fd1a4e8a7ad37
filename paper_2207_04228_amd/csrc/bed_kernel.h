// Internal interface between the C-ABI layer and the device code.
#ifndef BED_KERNEL_H
#define BED_KERNEL_H

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bed {

// Per-launch kernel timing (bed_timing_* of the C ABI): while a thread has armed its timer, each
// kernel it enqueues through this library is launched with a start and a stop event of its own
// (hipExtLaunchKernel: the events take the dispatch's own begin and end timestamps, with no marker
// packets between the kernels of the stream).
struct LaunchTimer {
    hipEvent_t* start = nullptr;
    hipEvent_t* stop = nullptr;
    int capacity = 0;
    int used = 0;
    bool armed = false;
};
inline LaunchTimer& launch_timer() {
    static thread_local LaunchTimer timer;
    return timer;
}

// Launches `kernel` and returns the status of THIS launch.  (Reading hipGetLastError() after a
// triple-chevron launch would also report, and consume, an error left behind by an unrelated
// earlier HIP call of the calling thread.)
template <typename T>
struct same_type { using type = T; };

template <typename... KArgs>
inline hipError_t enqueue(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream,
                          typename same_type<KArgs>::type... args) {
    void* argv[] = {const_cast<void*>(static_cast<const void*>(&args))...};
    LaunchTimer& t = launch_timer();
    if (t.armed && t.used < t.capacity) {
        const int i = t.used++;
        return hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, 0, stream, t.start[i],
                                  t.stop[i], 0);
    }
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, 0, stream);
}

// Lane-strided copy of `count` consecutive elements between global memory and an on-chip layout
// (every instruction touches 64 consecutive addresses).  CHUNK elements per lane are in flight at
// once: all loads of a chunk (global loads, or the LDS reads that feed global stores) are issued
// before the first value is consumed, instead of one memory round trip per element.
template <int CHUNK, typename Load, typename Store>
__device__ __forceinline__ void chunked_copy(int count, int lane, Load&& load, Store&& store) {
    for (int base = lane; base < count; base += 64 * CHUNK) {
        float t[CHUNK];
#pragma unroll
        for (int k = 0; k < CHUNK; ++k) {
            const int idx = base + 64 * k;
            t[k] = idx < count ? load(idx) : 0.f;
        }
#pragma unroll
        for (int k = 0; k < CHUNK; ++k) {
            const int idx = base + 64 * k;
            if (idx < count) store(idx, t[k]);
        }
    }
}
constexpr int copy_chunk(int elements_per_wavefront) {
    return elements_per_wavefront >= 1024 ? 16 : (elements_per_wavefront <= 64 ? 1 : (elements_per_wavefront + 63) / 64);
}

// 1 / x for x an exact power of two in [2^-125, 2^126] (the pre-scaling factors), bit-exact.
__device__ __forceinline__ float pow2_reciprocal(float x) { return __uint_as_float(0x7F000000u - __float_as_uint(x)); }

enum Stage { kFull = 0, kTridiagOnly = 1, kQrOnly = 2, kSpectral = 3, kQrPartial = 4 };
enum SpectralFn { kFnSqrt = 0, kFnInvSqrt = 1 };

struct KernelArgs {
    const float* A;      // [batch][n][n]            (kFull, kTridiagOnly)
    const float* d_in;   // [batch][n]               (kQrOnly)
    const float* e_in;   // [batch][n]               (kQrOnly)
    float* evals;        // [batch][n]               (kFull, kQrOnly)
    float* evecs;        // [batch][n][n] or P       (when vectors are wanted)
    float* d_out;        // [batch][n]               (kTridiagOnly)
    float* e_out;        // [batch][n]               (kTridiagOnly)
    float* fn_out;       // [batch][n][n]            (kSpectral) V f(lambda) V^T
    float fn_floor;      // eigenvalues are raised to this floor before f is applied (kSpectral)
    int fn;              // SpectralFn (kSpectral)
    uint32_t sweep_cap;  // at most this many sweeps (0: the default cap of 30 n); kQrPartial stops there
    float abs_eps;       // > 0: the paper's absolute deflation threshold on |e_k| (in units of A); 0: the relative test
    int* info;           // [batch] or nullptr
    uint32_t* rotations; // [batch] or nullptr
    unsigned long long* phases;  // [batch][8] cycle counts per phase; read only by the profiling build
    int batch;
    int n;
};

// Gradient kernels (bed_grad.hip).
enum GradMode { kGradExact = 0, kGradTaylor = 1, kGradSqrt = 2, kGradInvSqrt = 3 };

struct GradArgs {
    const float* evals;    // [batch][n]
    const float* evecs;    // [batch][n][n], eigenvectors as columns
    const float* g_evals;  // [batch][n] or nullptr        (kGradExact, kGradTaylor)
    const float* g_mat;    // [batch][n][n] or nullptr: gradient w.r.t. evecs, or w.r.t. the spectral function
    float* g_A;            // [batch][n][n]
    int batch;
    int n;
    int mode;              // GradMode
    int degree;            // kGradTaylor: degree of the truncated series
    float param;           // kGradExact: gap floor; kGradSqrt / kGradInvSqrt: eigenvalue floor
};

hipError_t launch_grad(const GradArgs& args, hipStream_t stream);

// The paper's fixed-budget procedure (bed_lockstep.hip).
struct LockstepArgs {
    const float* A;      // [batch][n][n]
    float* evals;        // [batch][n]
    float* evecs;        // [batch][n][n] or nullptr; holds P, then V between the launches
    float* offdiag;      // [batch][n] or nullptr
    int* reductions;     // [batch] or nullptr
    float* d;            // workspace [batch][n]
    float* e;            // workspace [batch][n]
    int* flags;          // workspace [iterations]: matrices that did not pass the test after iteration i
    int* window;         // workspace [batch]: window size per matrix (per-matrix rule)
    int batch;
    int n;
    int iterations;
    int uniform;         // 1: the window is shared by the batch
    float epsilon;
};

hipError_t launch_lockstep(const LockstepArgs& args, hipStream_t stream);

// Size of the library's built-in scratch memory for the lock-step procedure, and its device
// address on the current device (looked up on the first call per device; allocates nothing).
constexpr size_t kLockstepScratchBytes = 1u << 20;
hipError_t lockstep_scratch(void** ptr);

// Name of the kernel that serves a full decomposition of this batch and n.
const char* kernel_variant(int batch, int n, bool want_v);

// Kernel families (values of bed_family in bed.h).
enum FamilyId { kFamilyAuto = 0, kFamilyWave = 1, kFamilyPacked = 2, kFamilyLane = 3, kFamilyBlock = 4, kFamilyPair = 5, kFamilyPackedRows = 6 };
bool family_serves(int family, int n);

// Enqueue one launch; returns the status of that launch.  `forced`: a family other than
// kFamilyAuto (full decomposition only; the caller has checked family_serves).
hipError_t launch(const KernelArgs& args, int stage, bool want_v, hipStream_t stream, int forced = kFamilyAuto);

}  // namespace bed

#endif
