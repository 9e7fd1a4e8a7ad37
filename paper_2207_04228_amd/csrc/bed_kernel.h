// Internal interface between the C-ABI layer and the device code.
#ifndef BED_KERNEL_H
#define BED_KERNEL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bed {

enum Stage { kFull = 0, kTridiagOnly = 1, kQrOnly = 2, kSpectral = 3 };
enum SpectralFn { kFnSqrt = 0, kFnInvSqrt = 1 };
enum ShiftPolicy { kShiftDouble = 0, kShiftSingle = 1 };

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
    int* info;           // [batch] or nullptr
    uint32_t* rotations; // [batch] or nullptr
    int batch;
    int n;
#ifdef BED_PROFILE
    long long* prof;     // [batch][8] development-only phase timers
#endif
};

// Enqueue one launch; returns hipGetLastError() of the launch.
hipError_t launch(const KernelArgs& args, int stage, int shift, bool want_v, hipStream_t stream);

}  // namespace bed

#endif
