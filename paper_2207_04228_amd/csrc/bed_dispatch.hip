// Size dispatch: picks the kernel whose register arrays fit n.
#include "bed_kernel.h"

namespace bed {

hipError_t launch_lane(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_packed(const KernelArgs&, int, bool, hipStream_t);
hipError_t launch_pair(const KernelArgs&, hipStream_t);
hipError_t launch_packed_rows(const KernelArgs&, int, bool, hipStream_t);
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

constexpr int kPackedFromBatch = 2560;
constexpr int kPackedRowsFromBatch = 4096;
constexpr int kPackedRowsValuesFromBatch = 3072;   // eigenvalues only
constexpr int kPairUpToBatch = 512;
constexpr int kLane4FromBatch = 20480;
constexpr int kLane8FromBatch = 32768;

enum Family { kLaneFamily, kPackedFamily, kWaveFamily, kPairFamily, kBlockFamily, kPackedRowsFamily };
struct Choice {
    Family family;
    int N;               // register-array size of the instantiation (0 for the block kernel)
    const char* name;
};

Choice wave_choice(int n);

// The one place that decides which kernel serves a problem.  `forced` (kFamilyAuto unless a test
// or a measurement asks for one family) must be able to serve n: the caller has checked.
Choice choose(int batch, int n, int stage, bool want_v, int forced) {
    if (forced == kFamilyLane) return n <= 4 ? Choice{kLaneFamily, 4, "lane_kernel<4>"} : Choice{kLaneFamily, 8, "lane_kernel<8>"};
    if (forced == kFamilyPacked) {
        if (n <= 4) return {kPackedFamily, 4, "packed_kernel<4>"};
        if (n <= 8) return {kPackedFamily, 8, "packed_kernel<8>"};
        if (n <= 12) return {kPackedFamily, 12, "packed_kernel<12>"};
        if (n <= 16) return {kPackedFamily, 16, "packed_kernel<16>"};
        if (n <= 24) return {kPackedFamily, 24, "packed_kernel<24>"};
        return {kPackedFamily, 32, "packed_kernel<32>"};
    }
    if (forced == kFamilyWave) return wave_choice(n);
    if (forced == kFamilyPair) return {kPairFamily, 0, n <= 40 ? "pair_kernel<40>" : n <= 48 ? "pair_kernel<48>" : n <= 56 ? "pair_kernel<56>" : "pair_kernel<64>"};
    if (forced == kFamilyBlock) return {kBlockFamily, 0, "block_kernel"};
    if (forced == kFamilyPackedRows) {
        if (n <= 20) return {kPackedRowsFamily, 20, "packed_rows_kernel<20>"};
        if (n <= 24) return {kPackedRowsFamily, 24, "packed_rows_kernel<24>"};
        if (n <= 28) return {kPackedRowsFamily, 28, "packed_rows_kernel<28>"};
        return {kPackedRowsFamily, 32, "packed_rows_kernel<32>"};
    }
    // Measured crossovers on MI355X (us per launch, eigenvectors on; wave / packed / lane):
    //   n = 4:  batch 2048: 8.4 / 8.6 / 13.0   4096: 11.5 / 9.1 / 13.7   16384: 27.7 / 13.2 / 14.2   32768: 49 / 21.7 / 14.9
    //   n = 8:  batch 2048: 17.2 / 17.8 / 49.5  4096: 25.3 / 18.0 / 49.4  32768: 127 / 58.1 / 56.6    65536: 231 / 96.9 / 57.6
    //   n = 16: batch 2048: 34.1 / 36.3         3072: 42.6 / 35.4         4096: 51.6 / 35.5           16384: 152 / 76.7
    //   n = 24: batch 2048: 73.4 / 80.4         3072: 93.7 / 97.0         4096: 112 / 100             16384: 356 / 289
    //   n = 32: batch 2048: 115 / 123           3072: 145 / 161           4096: 179 / 163             16384: 571 / 496
    // Below kPackedFromBatch the chip is not full and one wavefront per matrix, whose per-matrix
    // latency is lowest, finishes first.  Then four matrices per wavefront (n <= 16) share the
    // instructions of the scalar recurrence.  For tiny matrices in very large batches one matrix per
    // lane (64 per wavefront) has no redundant work at all, but a latency several times higher.
    // The fused spectral function follows the same choice; the stage hooks stay with one wavefront
    // per matrix.
    const bool whole = (stage == kFull || stage == kSpectral);
    if (whole && n <= 4 && batch >= kLane4FromBatch) return {kLaneFamily, 4, "lane_kernel<4>"};
    if (whole && n <= 8 && batch >= kLane8FromBatch) return {kLaneFamily, 8, "lane_kernel<8>"};
    if (whole && n <= 16 && batch >= kPackedFromBatch) return choose(batch, n, stage, want_v, kFamilyPacked);
    // 16 < n <= 32, from batch 4096 (us per launch, wave / two per wavefront / four per wavefront with
    // two rows per lane:
    //   n = 20: batch 3072: 72.8 / 80.5 / 75.3   4096: 87.5 / 80.6 / 74.7   8192: 146 / 124 / 97    16384: 264 / 220 / 195
    //   n = 24: batch 3072: 93.6 / 97.5 / 96.3   4096: 115 / 101 / 95       8192: 193 / 163 / 129   16384: 355 / 288 / 238
    //   n = 28: batch 3072: 119 / 130 / 125      4096: 145 / 131 / 124      8192: 247 / 232 / 165   16384: 456 / 400 / 309
    //   n = 32: batch 3072: 148 / 162 / 152      4096: 180 / 163 / 152      8192: 309 / 275 / 205   16384: 571 / 488 / 379):
    // four matrices per wavefront, also for the fused spectral function (16384 x 32x32: 529 us with
    // two per wavefront, 388 us with four); two per wavefront remains for forced-family runs
    // (eigenvalues only, n = 32: batch 3072: 125 / 109 / 95   4096: 149 / 108 / 94   16384: 479 / 379 / 230)
    if (whole && n > 16 && n <= 32 && batch >= (want_v ? kPackedRowsFromBatch : kPackedRowsValuesFromBatch))
        return choose(batch, n, stage, want_v, kFamilyPackedRows);
    // 32 < n <= 64 with eigenvectors while the chip is mostly idle: two wavefronts per matrix
    // (us per launch, wave / pair: n = 48: batch 256: 175 / 165, 512: 179 / 168, 768: 179 / 203;
    //  n = 64: batch 256: 285 / 274, 512: 293 / 274, 768: 290 / 327)
    if (stage == kFull && want_v && n > 32 && n <= 64 && batch <= kPairUpToBatch) return choose(batch, n, stage, want_v, kFamilyPair);
    if (n <= 64) return wave_choice(n);
    return {kBlockFamily, 0, "block_kernel"};     // 64 < n <= 128: four wavefronts per matrix
}

Choice wave_choice(int n) {
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
    return {kWaveFamily, 64, "wave_kernel<64>"};
}

}  // namespace

const char* kernel_variant(int batch, int n, bool want_v) { return choose(batch, n, kFull, want_v, kFamilyAuto).name; }

bool family_serves(int family, int n) {
    switch (family) {
        case kFamilyAuto: return n >= 1 && n <= 128;
        case kFamilyWave: return n >= 1 && n <= 64;
        case kFamilyPacked: return n >= 1 && n <= 32;
        case kFamilyLane: return n >= 1 && n <= 8;
        case kFamilyBlock: return n > 64 && n <= 128;
        case kFamilyPair: return n > 32 && n <= 64;
        case kFamilyPackedRows: return n >= 1 && n <= 32;
        default: return false;
    }
}

hipError_t launch(const KernelArgs& args, int stage, bool want_v, hipStream_t stream, int forced) {
    if (args.batch == 0) return hipSuccess;
    const Choice c = choose(args.batch, args.n, stage, want_v, forced);
    if (c.family == kPairFamily) {
        if (!want_v || stage != kFull) return hipErrorInvalidValue;     // the pair kernels always form eigenvectors
        return launch_pair(args, stream);
    }
    if (c.family == kPackedRowsFamily) {
        if (stage != kFull && stage != kSpectral) return hipErrorInvalidValue;     // no stage hooks
        return launch_packed_rows(args, stage, want_v, stream);
    }
    if (c.family == kLaneFamily) return launch_lane(args, stage, want_v, stream);
    if (c.family == kPackedFamily) return launch_packed(args, stage, want_v, stream);
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
