// Four matrices per wavefront, two rows per lane, for 16 < n <= 32 (instantiations for n <= 24).
#include "bed_packed_rows_kernel.hpp"

namespace bed {
hipError_t launch_packed_rows_32(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_packed_rows(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (args.n <= 20) return launch_packed_rows_n<20>(args, stage, want_v, stream);
    if (args.n <= 24) return launch_packed_rows_n<24>(args, stage, want_v, stream);
    return launch_packed_rows_32(args, stage, want_v, stream);
}
}  // namespace bed
