// Instantiation of the one-wave-per-matrix kernels for padded size 12.
#include "bed_wave_kernel.hpp"

namespace bed {
hipError_t launch_wave_n12(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    return launch_n<12>(args, stage, want_v, stream);
}
}  // namespace bed
