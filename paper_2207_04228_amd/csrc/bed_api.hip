// C ABI of libbed.so: argument validation and dispatch.  See include/bed.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bed.h"
#include "bed_kernel.h"

namespace {

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

int check_common(int batch, int n) {
    if (batch < 0) return BED_ERR_BATCH;
    if (n < 1 || n > BED_MAX_N) return BED_ERR_N;
    return BED_OK;
}

int syevd_checked(const float* A, int batch, int n, float* evals, float* evecs, int* info, unsigned* rotations,
                  int family, float epsilon_abs, int sweep_cap, void* stream);

int run(const bed::KernelArgs& args, int stage, bool want_v, void* stream, int family = bed::kFamilyAuto) {
    if (args.batch == 0) return BED_OK;
    hipError_t err = bed::launch(args, stage, want_v, static_cast<hipStream_t>(stream), family);
    return err == hipSuccess ? BED_OK : BED_ERR_LAUNCH;
}

// Both lock-step entry points.  builtin_scratch: the workspace is the library's own scratch
// memory, whose device address is looked up only after every host-side check has passed.
int lockstep_checked(const float* A, int batch, int n, float epsilon, int iterations, int uniform, float* evals,
                     float* evecs, float* offdiag, int* reductions, void* workspace, size_t workspace_bytes,
                     bool builtin_scratch, void* stream) {
    int st = check_common(batch, n);
    if (st != BED_OK) return st;
    if (n > 64) return BED_ERR_N;
    if (iterations < 0 || (uniform != 0 && uniform != 1)) return BED_ERR_ARG;
    if (!(epsilon >= 0.f) || !(epsilon < __builtin_inff())) return BED_ERR_ARG;
    if (batch == 0) return BED_OK;
    if (!A || !evals || (!workspace && !builtin_scratch)) return BED_ERR_NULL;
    if (misaligned(A) || misaligned(evals) || misaligned(evecs) || misaligned(offdiag) || misaligned(reductions) ||
        misaligned(workspace))
        return BED_ERR_ALIGN;
    const size_t need = bed_syevd_lockstep_workspace(batch, n, iterations);
    if (builtin_scratch) {
        if (need > bed::kLockstepScratchBytes) return BED_ERR_SCRATCH;
        if (bed::lockstep_scratch(&workspace) != hipSuccess) return BED_ERR_LAUNCH;
    } else if (workspace_bytes < need) {
        return BED_ERR_ARG;
    }
    const size_t mat = (size_t)batch * n * n * sizeof(float), vec = (size_t)batch * n * sizeof(float);
    const size_t cnt = (size_t)batch * sizeof(int);
    if (overlaps(A, mat, evals, vec) || overlaps(A, mat, evecs, mat) || overlaps(A, mat, offdiag, vec) ||
        overlaps(A, mat, reductions, cnt) || overlaps(A, mat, workspace, need) || overlaps(evals, vec, evecs, mat) ||
        overlaps(evals, vec, offdiag, vec) || overlaps(evals, vec, reductions, cnt) ||
        overlaps(evals, vec, workspace, need) || overlaps(evecs, mat, offdiag, vec) ||
        overlaps(evecs, mat, reductions, cnt) || overlaps(evecs, mat, workspace, need) ||
        overlaps(offdiag, vec, reductions, cnt) || overlaps(offdiag, vec, workspace, need) ||
        overlaps(reductions, cnt, workspace, need))
        return BED_ERR_ALIAS;
    bed::LockstepArgs args{};
    args.A = A;
    args.evals = evals;
    args.evecs = evecs;
    args.offdiag = offdiag;
    args.reductions = reductions;
    float* ws = static_cast<float*>(workspace);
    args.d = ws;
    args.e = ws + (size_t)batch * n;
    args.flags = reinterpret_cast<int*>(ws + 2 * (size_t)batch * n);
    args.window = args.flags + iterations;
    args.batch = batch;
    args.n = n;
    args.iterations = iterations;
    args.uniform = uniform;
    args.epsilon = epsilon;
    return bed::launch_lockstep(args, static_cast<hipStream_t>(stream)) == hipSuccess ? BED_OK : BED_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int bed_syevd_info(const float* A, int batch, int n, float* evals, float* evecs, int* info,
                   unsigned* rotations, void* stream) {
    return bed_syevd_family(A, batch, n, evals, evecs, info, rotations, BED_FAMILY_AUTO, stream);
}

int bed_syevd_family(const float* A, int batch, int n, float* evals, float* evecs, int* info,
                     unsigned* rotations, int family, void* stream) {
    return syevd_checked(A, batch, n, evals, evecs, info, rotations, family, 0.f, 0, stream);
}

int bed_syevd_tol(const float* A, int batch, int n, float* evals, float* evecs, int* info,
                  unsigned* rotations, float epsilon_abs, int sweep_cap, void* stream) {
    if (!(epsilon_abs >= 0.f) || !(epsilon_abs < __builtin_inff()) || sweep_cap < 0) {
        int st = check_common(batch, n);
        return st != BED_OK ? st : BED_ERR_ARG;
    }
    return syevd_checked(A, batch, n, evals, evecs, info, rotations, BED_FAMILY_AUTO, epsilon_abs, sweep_cap, stream);
}

}  // extern "C"

namespace {

int syevd_checked(const float* A, int batch, int n, float* evals, float* evecs, int* info, unsigned* rotations,
                  int family, float epsilon_abs, int sweep_cap, void* stream) {
    int st = check_common(batch, n);
    if (st != BED_OK) return st;
    if (family < BED_FAMILY_AUTO || family > BED_FAMILY_PACKED_ROWS) return BED_ERR_ARG;
    if (family == BED_FAMILY_PAIR && !evecs) return BED_ERR_NULL;
    if (!bed::family_serves(family, n)) return BED_ERR_N;
    if (batch == 0) return BED_OK;
    if (!A || !evals) return BED_ERR_NULL;
    if (misaligned(A) || misaligned(evals) || misaligned(evecs) || misaligned(info) || misaligned(rotations))
        return BED_ERR_ALIGN;
    const size_t mat = (size_t)batch * n * n * sizeof(float), vec = (size_t)batch * n * sizeof(float);
    if (overlaps(A, mat, evals, vec) || overlaps(A, mat, evecs, mat) || overlaps(evals, vec, evecs, mat))
        return BED_ERR_ALIAS;
    bed::KernelArgs args{};
    args.A = A;
    args.evals = evals;
    args.evecs = evecs;
    args.info = info;
    args.rotations = rotations;
    args.batch = batch;
    args.n = n;
    args.abs_eps = epsilon_abs;
    args.sweep_cap = (uint32_t)sweep_cap;
    return run(args, bed::kFull, evecs != nullptr, stream, family);
}

}  // namespace

extern "C" {

int bed_syevd(const float* A, int batch, int n, float* evals, float* evecs, void* stream) {
    return bed_syevd_info(A, batch, n, evals, evecs, nullptr, nullptr, stream);
}

int bed_tridiag(const float* A, int batch, int n, float* d, float* e, float* P, void* stream) {
    int st = check_common(batch, n);
    if (st != BED_OK) return st;
    if (batch == 0) return BED_OK;
    if (!A || !d || !e) return BED_ERR_NULL;
    if (misaligned(A) || misaligned(d) || misaligned(e) || misaligned(P)) return BED_ERR_ALIGN;
    const size_t mat = (size_t)batch * n * n * sizeof(float), vec = (size_t)batch * n * sizeof(float);
    if (overlaps(A, mat, d, vec) || overlaps(A, mat, e, vec) || overlaps(A, mat, P, mat) ||
        overlaps(d, vec, e, vec) || overlaps(d, vec, P, mat) || overlaps(e, vec, P, mat))
        return BED_ERR_ALIAS;
    bed::KernelArgs args{};
    args.A = A;
    args.d_out = d;
    args.e_out = e;
    args.evecs = P;
    args.batch = batch;
    args.n = n;
    return run(args, bed::kTridiagOnly, P != nullptr, stream);
}

int bed_tridiag_qr(const float* d, const float* e, int batch, int n, float* evals, float* evecs,
                   int* info, unsigned* rotations, void* stream) {
    int st = check_common(batch, n);
    if (st != BED_OK) return st;
    if (batch == 0) return BED_OK;
    if (!d || !e || !evals) return BED_ERR_NULL;
    if (misaligned(d) || misaligned(e) || misaligned(evals) || misaligned(evecs) || misaligned(info) ||
        misaligned(rotations))
        return BED_ERR_ALIGN;
    const size_t mat = (size_t)batch * n * n * sizeof(float), vec = (size_t)batch * n * sizeof(float);
    if (overlaps(d, vec, evals, vec) || overlaps(e, vec, evals, vec) || overlaps(d, vec, evecs, mat) ||
        overlaps(e, vec, evecs, mat) || overlaps(evals, vec, evecs, mat))
        return BED_ERR_ALIAS;
    bed::KernelArgs args{};
    args.d_in = d;
    args.e_in = e;
    args.evals = evals;
    args.evecs = evecs;
    args.info = info;
    args.rotations = rotations;
    args.batch = batch;
    args.n = n;
    return run(args, bed::kQrOnly, evecs != nullptr, stream);
}

int bed_tridiag_qr_sweeps(const float* d, const float* e, int batch, int n, int sweeps, float* d_out,
                          float* e_out, float* Q, unsigned* rotations, void* stream) {
    int st = check_common(batch, n);
    if (st != BED_OK) return st;
    if (n > 64) return BED_ERR_N;
    if (sweeps < 1) return BED_ERR_ARG;
    if (batch == 0) return BED_OK;
    if (!d || !e || !d_out || !e_out || !Q) return BED_ERR_NULL;
    if (misaligned(d) || misaligned(e) || misaligned(d_out) || misaligned(e_out) || misaligned(Q) ||
        misaligned(rotations))
        return BED_ERR_ALIGN;
    const size_t mat = (size_t)batch * n * n * sizeof(float), vec = (size_t)batch * n * sizeof(float);
    if (overlaps(d, vec, d_out, vec) || overlaps(d, vec, e_out, vec) || overlaps(e, vec, d_out, vec) ||
        overlaps(e, vec, e_out, vec) || overlaps(d, vec, Q, mat) || overlaps(e, vec, Q, mat) ||
        overlaps(d_out, vec, e_out, vec) || overlaps(d_out, vec, Q, mat) || overlaps(e_out, vec, Q, mat))
        return BED_ERR_ALIAS;
    bed::KernelArgs args{};
    args.d_in = d;
    args.e_in = e;
    args.d_out = d_out;
    args.e_out = e_out;
    args.evecs = Q;
    args.rotations = rotations;
    args.sweep_cap = (uint32_t)sweeps;
    args.batch = batch;
    args.n = n;
    return run(args, bed::kQrPartial, true, stream);
}

int bed_spd_fn(const float* A, int batch, int n, int fn, float floor, float* out, float* evals, int* info,
               void* stream) {
    int st = check_common(batch, n);
    if (st != BED_OK) return st;
    if (fn != BED_FN_SQRT && fn != BED_FN_INV_SQRT) return BED_ERR_ARG;
    if (!(floor >= 0.f) || !(floor < __builtin_inff())) return BED_ERR_ARG;
    if (fn == BED_FN_INV_SQRT && !(floor > 0.f)) return BED_ERR_ARG;
    if (batch == 0) return BED_OK;
    if (!A || !out) return BED_ERR_NULL;
    if (misaligned(A) || misaligned(out) || misaligned(evals) || misaligned(info)) return BED_ERR_ALIGN;
    const size_t mat = (size_t)batch * n * n * sizeof(float), vec = (size_t)batch * n * sizeof(float);
    if (overlaps(A, mat, out, mat) || overlaps(A, mat, evals, vec) || overlaps(out, mat, evals, vec))
        return BED_ERR_ALIAS;
    bed::KernelArgs args{};
    args.A = A;
    args.fn_out = out;
    args.fn = (fn == BED_FN_INV_SQRT) ? bed::kFnInvSqrt : bed::kFnSqrt;
    args.fn_floor = floor;
    args.evals = evals;
    args.info = info;
    args.batch = batch;
    args.n = n;
    return run(args, bed::kSpectral, true, stream);
}

int bed_syevd_backward(const float* evals, const float* evecs, const float* grad_evals, const float* grad_evecs,
                       int batch, int n, int mode, int degree, float gap_floor, float* grad_A, void* stream) {
    int st = check_common(batch, n);
    if (st != BED_OK) return st;
    if (mode != BED_GRAD_EXACT && mode != BED_GRAD_TAYLOR) return BED_ERR_ARG;
    if (mode == BED_GRAD_TAYLOR && (degree < 0 || degree > 64)) return BED_ERR_ARG;
    if (mode == BED_GRAD_EXACT && (!(gap_floor >= 0.f) || !(gap_floor < __builtin_inff()))) return BED_ERR_ARG;
    if (batch == 0) return BED_OK;
    if (!evals || !evecs || !grad_A || (!grad_evals && !grad_evecs)) return BED_ERR_NULL;
    if (misaligned(evals) || misaligned(evecs) || misaligned(grad_evals) || misaligned(grad_evecs) ||
        misaligned(grad_A))
        return BED_ERR_ALIGN;
    const size_t mat = (size_t)batch * n * n * sizeof(float), vec = (size_t)batch * n * sizeof(float);
    if (overlaps(grad_A, mat, evals, vec) || overlaps(grad_A, mat, evecs, mat) ||
        overlaps(grad_A, mat, grad_evals, vec) || overlaps(grad_A, mat, grad_evecs, mat))
        return BED_ERR_ALIAS;
    bed::GradArgs args{};
    args.evals = evals;
    args.evecs = evecs;
    args.g_evals = grad_evals;
    args.g_mat = grad_evecs;
    args.g_A = grad_A;
    args.batch = batch;
    args.n = n;
    args.mode = (mode == BED_GRAD_TAYLOR) ? bed::kGradTaylor : bed::kGradExact;
    args.degree = degree;
    args.param = gap_floor;
    return bed::launch_grad(args, static_cast<hipStream_t>(stream)) == hipSuccess ? BED_OK : BED_ERR_LAUNCH;
}

int bed_spd_fn_backward(const float* evals, const float* evecs, const float* grad_out, int batch, int n, int fn,
                        float floor, float* grad_A, void* stream) {
    int st = check_common(batch, n);
    if (st != BED_OK) return st;
    if (fn != BED_FN_SQRT && fn != BED_FN_INV_SQRT) return BED_ERR_ARG;
    if (!(floor >= 0.f) || !(floor < __builtin_inff())) return BED_ERR_ARG;
    if (fn == BED_FN_INV_SQRT && !(floor > 0.f)) return BED_ERR_ARG;
    if (batch == 0) return BED_OK;
    if (!evals || !evecs || !grad_out || !grad_A) return BED_ERR_NULL;
    if (misaligned(evals) || misaligned(evecs) || misaligned(grad_out) || misaligned(grad_A)) return BED_ERR_ALIGN;
    const size_t mat = (size_t)batch * n * n * sizeof(float), vec = (size_t)batch * n * sizeof(float);
    if (overlaps(grad_A, mat, evals, vec) || overlaps(grad_A, mat, evecs, mat) || overlaps(grad_A, mat, grad_out, mat))
        return BED_ERR_ALIAS;
    bed::GradArgs args{};
    args.evals = evals;
    args.evecs = evecs;
    args.g_mat = grad_out;
    args.g_A = grad_A;
    args.batch = batch;
    args.n = n;
    args.mode = (fn == BED_FN_INV_SQRT) ? bed::kGradInvSqrt : bed::kGradSqrt;
    args.param = floor;
    return bed::launch_grad(args, static_cast<hipStream_t>(stream)) == hipSuccess ? BED_OK : BED_ERR_LAUNCH;
}

size_t bed_syevd_lockstep_workspace(int batch, int n, int iterations) {
    if (batch < 0 || n < 1 || n > 64 || iterations < 0) return 0;
    const size_t words = 2 * (size_t)batch * n + (size_t)iterations + (size_t)batch;
    return (words * 4 + 255) & ~(size_t)255;
}

int bed_syevd_lockstep(const float* A, int batch, int n, float epsilon, int iterations, int uniform, float* evals,
                       float* evecs, float* offdiag, int* reductions, void* workspace, size_t workspace_bytes,
                       void* stream) {
    return lockstep_checked(A, batch, n, epsilon, iterations, uniform, evals, evecs, offdiag, reductions, workspace,
                            workspace_bytes, false, stream);
}

size_t bed_syevd_lockstep_static_capacity(void) { return bed::kLockstepScratchBytes; }

int bed_syevd_lockstep_static(const float* A, int batch, int n, float epsilon, int iterations, int uniform,
                              float* evals, float* evecs, float* offdiag, int* reductions, void* stream) {
    return lockstep_checked(A, batch, n, epsilon, iterations, uniform, evals, evecs, offdiag, reductions, nullptr, 0,
                            true, stream);
}

const char* bed_kernel_variant(int batch, int n, int want_vectors) {
    if (batch < 0 || n < 1 || n > BED_MAX_N) return nullptr;
    return bed::kernel_variant(batch, n, want_vectors != 0);
}

const char* bed_status_string(int status) {
    switch (status) {
        case BED_OK: return "BED_OK";
        case BED_ERR_NULL: return "BED_ERR_NULL: a required pointer is NULL";
        case BED_ERR_BATCH: return "BED_ERR_BATCH: batch must be >= 0";
        case BED_ERR_N: return "BED_ERR_N: n must be in 1..128 (1..64 for bed_tridiag_qr_sweeps)";
        case BED_ERR_ALIGN: return "BED_ERR_ALIGN: pointers must be 4-byte aligned";
        case BED_ERR_LAUNCH: return "BED_ERR_LAUNCH: kernel launch failed";
        case BED_ERR_ALIAS: return "BED_ERR_ALIAS: buffers overlap";
        case BED_ERR_ARG: return "BED_ERR_ARG: argument out of range";
        case BED_ERR_SCRATCH: return "BED_ERR_SCRATCH: the problem does not fit the library's built-in scratch memory";
        default: return "BED_ERR_UNKNOWN";
    }
}

int bed_version(void) { return BED_VERSION; }

}  // extern "C"
