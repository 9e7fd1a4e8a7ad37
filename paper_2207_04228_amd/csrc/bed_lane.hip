// Instantiation of the one-matrix-per-lane kernels (n <= 4 and n <= 8).
#include "bed_lane_kernel.hpp"

namespace bed {
hipError_t launch_lane(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (args.n <= 4) return launch_lane_n<4>(args, stage, want_v, stream);
    return launch_lane_n<8>(args, stage, want_v, stream);
}
}  // namespace bed
