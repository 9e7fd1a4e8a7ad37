// Four matrices per wavefront, two rows per lane (instantiations for 24 < n <= 32).
#include "bed_packed_rows_kernel.hpp"

namespace bed {
hipError_t launch_packed_rows_32(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (args.n <= 28) return launch_packed_rows_n<28>(args, stage, want_v, stream);
    return launch_packed_rows_n<32>(args, stage, want_v, stream);
}
}  // namespace bed
