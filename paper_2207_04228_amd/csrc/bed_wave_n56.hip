// Instantiation of the one-wave-per-matrix kernels for padded size 56.
#include "bed_wave_kernel.hpp"

namespace bed {
hipError_t launch_wave_n56(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    return launch_n<56>(args, stage, want_v, stream);
}
}  // namespace bed
