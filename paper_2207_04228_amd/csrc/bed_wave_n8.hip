// Instantiation of the one-wave-per-matrix kernels for padded size 8.
#include "bed_wave_kernel.hpp"

namespace bed {
hipError_t launch_wave_n8(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    return launch_n<8>(args, stage, want_v, stream);
}
}  // namespace bed
