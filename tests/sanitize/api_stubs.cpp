// Host-only stand-ins for the launchers that the C-ABI layer (csrc/bed_api.hip) calls, so that
// the argument-validation layer can be built without device code and run under
// -fsanitize=address,undefined on a machine without a GPU.  Each stub records that it was
// reached and reports success; nothing is enqueued.
#include "bed_kernel.h"

int g_stub_launches = 0;

namespace bed {
hipError_t launch(const KernelArgs&, int, bool, hipStream_t, int) { ++g_stub_launches; return hipSuccess; }
bool family_serves(int family, int n) {        // the real table lives beside the kernels
    const int limit[] = {128, 64, 32, 8, 128, 64, 32};
    return family >= 0 && family <= 6 && n >= 1 && n <= limit[family];
}
hipError_t launch_grad(const GradArgs&, hipStream_t) { ++g_stub_launches; return hipSuccess; }
hipError_t launch_lockstep(const LockstepArgs&, hipStream_t) { ++g_stub_launches; return hipSuccess; }
hipError_t lockstep_scratch(void** ptr) {
    static float host_stand_in[64];          // never dereferenced by the validation layer
    *ptr = host_stand_in;
    return hipSuccess;
}
const char* kernel_variant(int, int, bool) { return "stub"; }
}  // namespace bed
