// Size dispatch: picks the kernel whose register arrays fit n.
#include "bed_kernel.h"

namespace bed {

hipError_t launch_lane(const KernelArgs&, bool, hipStream_t);
hipError_t launch_wave_n4(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n8(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n12(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n16(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n20(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n24(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n28(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n32(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n40(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n48(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n56(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_wave_n64(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_block(const KernelArgs&, int, bool, hipStream_t);

hipError_t launch(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (args.batch == 0) return hipSuccess;
    const int n = args.n;
    // Tiny matrices in very large batches: one matrix per lane (64 per wavefront).  Below these
    // batch sizes the chip is not full and the one-wavefront-per-matrix kernels, whose
    // per-matrix latency is much lower, finish first (measured crossovers on MI355X).
    if (stage == kFull && ((n <= 4 && args.batch >= 6144) || (n <= 8 && args.batch >= 12288)))
        return launch_lane(args, want_v, stream);
    if (n <= 4) return launch_wave_n4(args, stage, want_v, stream);
    if (n <= 8) return launch_wave_n8(args, stage, want_v, stream);
    if (n <= 12) return launch_wave_n12(args, stage, want_v, stream);
    if (n <= 16) return launch_wave_n16(args, stage, want_v, stream);
    if (n <= 20) return launch_wave_n20(args, stage, want_v, stream);
    if (n <= 24) return launch_wave_n24(args, stage, want_v, stream);
    if (n <= 28) return launch_wave_n28(args, stage, want_v, stream);
    if (n <= 32) return launch_wave_n32(args, stage, want_v, stream);
    if (n <= 40) return launch_wave_n40(args, stage, want_v, stream);
    if (n <= 48) return launch_wave_n48(args, stage, want_v, stream);
    if (n <= 56) return launch_wave_n56(args, stage, want_v, stream);
    if (n <= 64) return launch_wave_n64(args, stage, want_v, stream);
    return launch_block(args, stage, want_v, stream);     // 64 < n <= 128: four wavefronts per matrix
}

}  // namespace bed
