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

namespace {

enum Family { kLaneFamily, kWaveFamily, kBlockFamily };
struct Choice {
    Family family;
    int N;               // register-array size of the instantiation (0 for the block kernel)
    const char* name;
};

// The one place that decides which kernel serves a problem.
Choice choose(int batch, int n, int stage) {
    // Tiny matrices in very large batches: one matrix per lane (64 per wavefront).  Below these
    // batch sizes the chip is not full and the one-wavefront-per-matrix kernels, whose
    // per-matrix latency is much lower, finish first (measured crossovers on MI355X).
    if (stage == kFull && n <= 4 && batch >= 6144) return {kLaneFamily, 4, "lane_kernel<4>"};
    if (stage == kFull && n <= 8 && batch >= 12288) return {kLaneFamily, 8, "lane_kernel<8>"};
    if (n <= 4) return {kWaveFamily, 4, "wave_kernel<4>"};
    if (n <= 8) return {kWaveFamily, 8, "wave_kernel<8>"};
    if (n <= 12) return {kWaveFamily, 12, "wave_kernel<12>"};
    if (n <= 16) return {kWaveFamily, 16, "wave_kernel<16>"};
    if (n <= 20) return {kWaveFamily, 20, "wave_kernel<20>"};
    if (n <= 24) return {kWaveFamily, 24, "wave_kernel<24>"};
    if (n <= 28) return {kWaveFamily, 28, "wave_kernel<28>"};
    if (n <= 32) return {kWaveFamily, 32, "wave_kernel<32>"};
    if (n <= 40) return {kWaveFamily, 40, "wave_kernel<40>"};
    if (n <= 48) return {kWaveFamily, 48, "wave_kernel<48>"};
    if (n <= 56) return {kWaveFamily, 56, "wave_kernel<56>"};
    if (n <= 64) return {kWaveFamily, 64, "wave_kernel<64>"};
    return {kBlockFamily, 0, "block_kernel"};     // 64 < n <= 128: four wavefronts per matrix
}

}  // namespace

const char* kernel_variant(int batch, int n) { return choose(batch, n, kFull).name; }

hipError_t launch(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (args.batch == 0) return hipSuccess;
    const Choice c = choose(args.batch, args.n, stage);
    if (c.family == kLaneFamily) return launch_lane(args, want_v, stream);
    if (c.family == kBlockFamily) return launch_block(args, stage, want_v, stream);
    switch (c.N) {
        case 4: return launch_wave_n4(args, stage, want_v, stream);
        case 8: return launch_wave_n8(args, stage, want_v, stream);
        case 12: return launch_wave_n12(args, stage, want_v, stream);
        case 16: return launch_wave_n16(args, stage, want_v, stream);
        case 20: return launch_wave_n20(args, stage, want_v, stream);
        case 24: return launch_wave_n24(args, stage, want_v, stream);
        case 28: return launch_wave_n28(args, stage, want_v, stream);
        case 32: return launch_wave_n32(args, stage, want_v, stream);
        case 40: return launch_wave_n40(args, stage, want_v, stream);
        case 48: return launch_wave_n48(args, stage, want_v, stream);
        case 56: return launch_wave_n56(args, stage, want_v, stream);
        default: return launch_wave_n64(args, stage, want_v, stream);
    }
}

}  // namespace bed
