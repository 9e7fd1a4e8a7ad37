// Instantiation of the several-matrices-per-wavefront kernels: four per wavefront for n <= 16.
#include "bed_packed_kernel.hpp"

namespace bed {
hipError_t launch_packed32(const KernelArgs& args, int stage, bool want_v, hipStream_t stream);

hipError_t launch_packed(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (args.n <= 4) return launch_packed_n<16, 4>(args, stage, want_v, stream);
    if (args.n <= 8) return launch_packed_n<16, 8>(args, stage, want_v, stream);
    if (args.n <= 12) return launch_packed_n<16, 12>(args, stage, want_v, stream);
    if (args.n <= 16) return launch_packed_n<16, 16>(args, stage, want_v, stream);
    return launch_packed32(args, stage, want_v, stream);
}
}  // namespace bed
