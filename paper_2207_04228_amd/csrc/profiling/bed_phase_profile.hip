// Profiling build of the one-wavefront-per-matrix kernels: the same source compiled with
// BED_PHASE_CLOCKS, so that every wavefront also records the shader-clock cycles it spent in each
// phase (load, tridiagonalisation, iteration boundary, fill, steady-state steps, drain, sort and
// store).  Built into its own small library by paper_2207_04228_amd/phase_profile.py; not part of
// libbed.so and not declared in include/bed.h.  The clock reads (s_memtime plus a wait for it)
// cost a few hundred cycles per outer iteration; the script reports the instrumented launch time
// beside the product's so that the perturbation is on record.
#define BED_PHASE_CLOCKS 1
#include "../bed_pair_kernel.hpp"

// family: 1 = one wavefront per matrix (n = 4, 8, 16, 32, 64), 5 = two wavefronts per matrix (n = 48, 64)
extern "C" int bed_phase_profile(const float* A, int batch, int n, float* evals, float* evecs,
                                 unsigned long long* phases, int family, void* stream) {
    if (!A || !evals || !evecs || !phases || batch < 1) return -1;
    bed::KernelArgs args{};
    args.A = A;
    args.evals = evals;
    args.evecs = evecs;
    args.phases = phases;
    args.batch = batch;
    args.n = n;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t err;
    if (family == 5 && n == 64) err = bed::launch_pair_n<64>(args, st);
    else if (family == 5 && n == 48) err = bed::launch_pair_n<48>(args, st);
    else if (family != 1) return -7;
    else if (n == 4) err = bed::launch_one<4, true, bed::kFull>(args, st);
    else if (n == 8) err = bed::launch_one<8, true, bed::kFull>(args, st);
    else if (n == 16) err = bed::launch_one<16, true, bed::kFull>(args, st);
    else if (n == 32) err = bed::launch_one<32, true, bed::kFull>(args, st);
    else if (n == 48) err = bed::launch_one<48, true, bed::kFull>(args, st);
    else if (n == 64) err = bed::launch_one<64, true, bed::kFull>(args, st);
    else return -3;
    return err == hipSuccess ? 0 : -5;
}
