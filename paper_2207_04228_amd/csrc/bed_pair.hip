// Instantiation of the two-wavefronts-per-matrix kernels (32 < n <= 64).
#include "bed_pair_kernel.hpp"

namespace bed {
hipError_t launch_pair(const KernelArgs& args, hipStream_t stream) {
    if (args.n <= 40) return launch_pair_n<40>(args, stream);
    if (args.n <= 48) return launch_pair_n<48>(args, stream);
    if (args.n <= 56) return launch_pair_n<56>(args, stream);
    return launch_pair_n<64>(args, stream);
}
}  // namespace bed
