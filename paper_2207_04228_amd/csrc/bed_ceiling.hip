// Measured ceilings of the machine, for the roofline report: a plain fused-multiply-add kernel
// (v_fma_f32, no packed forms: the library is compiled without them) and a plain device copy.
// They exist so that the benchmark can state the solver's rates against what THIS build and
// THIS box reach, beside the datasheet peaks.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bed.h"
#include "bed_kernel.h"

namespace bed {
namespace {

// CHAINS independent dependency chains per lane, `iters` FMAs each: CHAINS = 16 with many
// wavefronts per SIMD is throughput-bound (the vector ALU's rate); CHAINS = 1 with one wavefront
// per SIMD is what a single dependent instruction stream can issue (the regime of a launch of a
// few hundred one-wavefront workgroups).
template <int CHAINS>
__global__ void fma_kernel(float* __restrict__ out, int iters, float a, float b) {
    float x[CHAINS];
#pragma unroll
    for (int j = 0; j < CHAINS; ++j) x[j] = (float)(threadIdx.x + j) * 1.0e-3f;
    // 64 FMAs per chain between two loop branches, so that the loop itself does not count
    for (int i = 0; i < iters; i += 64) {
#pragma unroll
        for (int u = 0; u < 64; ++u) {
#pragma unroll
            for (int j = 0; j < CHAINS; ++j) x[j] = fmaf(x[j], a, b);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < CHAINS; ++j) s += x[j];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n4) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) dst[i] = src[i];
}

}  // namespace
}  // namespace bed

extern "C" {

int bed_ceiling_fma(float* out, int blocks, int threads, int chains, int iters, void* stream) {
    if (!out) return BED_ERR_NULL;
    if (blocks < 1 || threads < 64 || threads > 1024 || (threads & 63) || iters < 64 || (iters & 63)) return BED_ERR_ARG;
    if (chains != 1 && chains != 16) return BED_ERR_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // a and b keep the values bounded (x -> 0.999 x + 0.001) and are not compile-time constants
    hipError_t err = chains == 1
        ? bed::enqueue(bed::fma_kernel<1>, dim3(blocks), dim3(threads), st, out, iters, 0.999f, 1.0e-3f)
        : bed::enqueue(bed::fma_kernel<16>, dim3(blocks), dim3(threads), st, out, iters, 0.999f, 1.0e-3f);
    return err == hipSuccess ? BED_OK : BED_ERR_LAUNCH;
}

int bed_ceiling_copy(const float* src, float* dst, size_t count, int blocks, void* stream) {
    if (!src || !dst) return BED_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return BED_ERR_ALIGN;
    if (count == 0 || (count & 3u) || blocks < 1) return BED_ERR_ARG;
    hipError_t err = bed::enqueue(bed::copy_kernel, dim3(blocks), dim3(256), static_cast<hipStream_t>(stream),
                                  reinterpret_cast<const float4*>(src), reinterpret_cast<float4*>(dst), count / 4);
    return err == hipSuccess ? BED_OK : BED_ERR_LAUNCH;
}

}  // extern "C"
