// Instantiation of the several-matrices-per-wavefront kernels: two per wavefront for 16 < n <= 32.
#include "bed_packed_kernel.hpp"

namespace bed {
hipError_t launch_packed32(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (args.n <= 24) return launch_packed_n<32, 24>(args, stage, want_v, stream);
    return launch_packed_n<32, 32>(args, stage, want_v, stream);
}
}  // namespace bed
