/*
 * bed -- batched symmetric eigendecomposition for AMD MI355X (gfx950).
 *
 * C ABI of libbed.so.  Every pointer marked "device" is GPU memory owned by
 * the caller; the library allocates nothing and keeps no state between calls
 * (one exception, stated there: bed_syevd_lockstep_static works in scratch
 * memory built into the library, which calls on the same GPU share).
 * All entry points are asynchronous: they enqueue their kernels (one, except
 * for the lock-step procedure) on `stream` (a hipStream_t passed as void*;
 * NULL = the default stream) and return.  Argument errors are detected on the
 * host, return a negative bed_status and enqueue nothing.  Entry points are
 * re-entrant and thread-safe (same exception).
 *
 * Method (arXiv 2207.04228, Sec. 3): Householder tridiagonalisation
 * A = P T P^T (Sec. 3.1), then QR iterations on T by Givens rotations with
 * the two Wilkinson shifts taken from the trailing 2x2 block (Sec. 3.2.1,
 * 3.2.2, App. A.1, A.3), per-matrix deflation of converged rows
 * (Sec. 3.2.3, generalised from the last row to any negligible off-diagonal),
 * and accumulation of all rotations into V = P Q_0 ... Q_k (closing equation
 * of Sec. 3.2.1, Sec. 3.2.5).
 */
#ifndef BED_H
#define BED_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BED_MAX_N 128
#define BED_VERSION 500 /* major*10000 + minor*100 + patch: 0.5.0 */

typedef enum {
    BED_OK = 0,
    BED_ERR_NULL = -1,   /* a required pointer is NULL                      */
    BED_ERR_BATCH = -2,  /* batch < 0                                       */
    BED_ERR_N = -3,      /* n < 1 or n > BED_MAX_N                          */
    BED_ERR_ALIGN = -4,  /* a pointer is not 4-byte aligned                 */
    BED_ERR_LAUNCH = -5, /* the HIP runtime refused the launch              */
    BED_ERR_ALIAS = -6,  /* an output buffer overlaps the input             */
    BED_ERR_ARG = -7,    /* an enumerated or scalar argument is out of range */
    BED_ERR_SCRATCH = -8 /* the problem does not fit the library's built-in scratch memory */
} bed_status;

/* Fields of the per-matrix `info` word of bed_syevd_info / bed_tridiag_qr / bed_spd_fn. */
#define BED_INFO_COUNT_MASK 0xFFFF
#define BED_INFO_RELAXED_SHIFT 16

typedef enum {
    BED_FN_SQRT = 0,     /* f(x) = x^(1/2)                                  */
    BED_FN_INV_SQRT = 1  /* f(x) = x^(-1/2)                                 */
} bed_fn;

/*
 * Eigendecomposition A_b = V_b diag(lambda_b) V_b^T of `batch` symmetric
 * n x n matrices (the problem stated in Sec. 3.1 Eq. (1) and the closing
 * equation of Sec. 3.2.1).
 *
 *   A      device, const, [batch][n][n] row-major fp32.  Only the LOWER
 *          triangle (i >= j) is read; it is mirrored.  Not modified.
 *   batch  >= 0; 0 is a no-op that returns BED_OK.
 *   n      1 .. BED_MAX_N.
 *   evals  device, [batch][n] fp32, ascending.
 *   evecs  device, [batch][n][n] row-major fp32; evecs[b][i][j] is component i
 *          of the eigenvector belonging to evals[b][j] (columns are
 *          eigenvectors, orthonormal).  May be NULL: eigenvalues only, the
 *          Householder accumulation and all rotations of V are skipped.
 *   stream hipStream_t or NULL.
 *
 * Numerical non-convergence never aborts: the QR loop is capped (30 sweeps
 * per row), a NaN/Inf input yields NaNs for that matrix only.  Use
 * bed_syevd_info to observe it.
 */
int bed_syevd(const float* A, int batch, int n, float* evals, float* evecs,
              void* stream);

/*
 * Same as bed_syevd, plus per-matrix diagnostics (either may be NULL):
 *   info       device, [batch] int32: 0 = converged to full accuracy.  Otherwise
 *              info = k + 65536 * w:
 *              k = info & BED_INFO_COUNT_MASK: k off-diagonal entries of T were
 *                  still not negligible when the sweep cap was reached, or k
 *                  eigenvalues came out non-finite (NaN/Inf input);
 *              w = info >> BED_INFO_RELAXED_SHIFT: w off-diagonal entries were
 *                  declared negligible only by the fallback test.  The deflation
 *                  test of Sec. 3.2.3 is relative here,
 *                  |e_k| <= 4 * 2^-23 (|d_k| + |d_k+1|); a window that has not
 *                  deflated anything for 12 (24) outer iterations (it sits at
 *                  the rounding noise of the rotations, which is relative to
 *                  ||A||, as happens for graded spectra) also accepts
 *                  |e_k| <= 2^-21 (2^-19) max|a_ij|.  Each such entry
 *                  perturbs the eigenvalues by at most 2e-6 ||A||_2 (a fifth of
 *                  the 1e-5 ||A||_2 accuracy bar), but eigenvalues far below
 *                  ||A||_2 lose their relative accuracy.
 *   rotations  device, [batch] uint32: number of Givens rotations applied to
 *              this matrix (the R of the flop model R*(6n+20); the paper
 *              reports the related "reduction times" in App. C.4).
 */
int bed_syevd_info(const float* A, int batch, int n, float* evals, float* evecs,
                   int* info, unsigned* rotations, void* stream);

/*
 * bed_syevd_info with the two run-time constants of the paper's procedure exposed (App. B
 * "Implementation Details": threshold 1e-5, a fixed number of iterations):
 *   epsilon_abs  > 0: the threshold of the paper, |e_k| <= epsilon_abs, ABSOLUTE in the units of A
 *                (Sec. 3.2.3; the paper uses 1e-5), applied to every off-diagonal of the active
 *                window after each outer iteration, per matrix.  It is used TOGETHER with the
 *                library's relative test (an entry is negligible if it passes either), because
 *                for ||A||_2 far above epsilon_abs / 1e-7 the rounding noise of float32 alone
 *                exceeds an absolute threshold and it could never be met.  Each entry deflated by
 *                it perturbs the eigenvalues by at most epsilon_abs, whatever ||A||: for ||A||_2
 *                near 1 that is at the edge of the 1e-5 ||A||_2 accuracy bar, for small ||A|| it
 *                is far outside.  0: the relative test alone (bed_syevd_info).  Finite and >= 0,
 *                else BED_ERR_ARG.
 *   sweep_cap    > 0: at most this many QR sweeps per matrix (two per outer iteration; App. B runs
 *                n outer iterations, i.e. 2 n sweeps); off-diagonals still live then are counted in
 *                info.  0: the default cap of 30 n.  < 0: BED_ERR_ARG.
 * Everything else as bed_syevd_info.
 */
int bed_syevd_tol(const float* A, int batch, int n, float* evals, float* evecs, int* info,
                  unsigned* rotations, float epsilon_abs, int sweep_cap, void* stream);

/*
 * bed_syevd_info through ONE kernel family, whatever the batch size (for parity tests of every
 * family at every batch size, and for measuring the batch sizes at which the automatic choice
 * should change).  Same method, arguments and outputs; the families differ in how matrices
 * map onto the machine:
 *   BED_FAMILY_AUTO    what bed_syevd does: chosen from n and batch (see bed_kernel_variant)
 *   BED_FAMILY_WAVE    one wavefront per matrix, n <= 64
 *   BED_FAMILY_PACKED  four matrices per wavefront (16 lanes each) for n <= 16, two (32 lanes each)
 *                      for 16 < n <= 32
 *   BED_FAMILY_LANE    one matrix per lane, n <= 8
 *   BED_FAMILY_BLOCK   four wavefronts per matrix, 64 < n <= 128
 *   BED_FAMILY_PAIR    two wavefronts per matrix, 32 < n <= 64, eigenvectors required
 *                      (BED_ERR_NULL without evecs)
 *   BED_FAMILY_PACKED_ROWS  four matrices per wavefront, 16 lanes each with two rows per lane,
 *                      n <= 32 (meant for 16 < n <= 32)
 * BED_ERR_N if the family does not serve this n, BED_ERR_ARG for an unknown family.
 */
typedef enum {
    BED_FAMILY_AUTO = 0,
    BED_FAMILY_WAVE = 1,
    BED_FAMILY_PACKED = 2,
    BED_FAMILY_LANE = 3,
    BED_FAMILY_BLOCK = 4,
    BED_FAMILY_PAIR = 5,
    BED_FAMILY_PACKED_ROWS = 6
} bed_family;
int bed_syevd_family(const float* A, int batch, int n, float* evals, float* evecs, int* info,
                     unsigned* rotations, int family, void* stream);

/*
 * Stage hook 1 -- Householder tridiagonalisation only (Sec. 3.1, Eqs. (2)-(7)):
 * A_b = P_b T_b P_b^T with T symmetric tridiagonal.
 *   d  device, [batch][n]   diagonal of T
 *   e  device, [batch][n]   e[b][k] = T[k+1][k] for k < n-1; e[b][n-1] = 0
 *   P  device, [batch][n][n] row-major, the product of the n-2 reflectors
 *      (first row and column are those of the identity).  May be NULL.
 */
int bed_tridiag(const float* A, int batch, int n, float* d, float* e, float* P,
                void* stream);

/*
 * Stage hook 2 -- shifted QR iterations on a given symmetric tridiagonal
 * matrix (Sec. 3.2): diag d, sub-diagonal e (same layout as bed_tridiag
 * writes; e[b][n-1] is ignored).  evals ascending; evecs (may be NULL) are
 * the eigenvectors of T as columns.
 */
int bed_tridiag_qr(const float* d, const float* e, int batch, int n,
                   float* evals, float* evecs, int* info, unsigned* rotations,
                   void* stream);

/*
 * Stage hook 3 -- a given number of shifted QR sweeps on a given symmetric tridiagonal
 * matrix, result left as it stands (Sec. 3.2.1, 3.2.2): one outer iteration is two sweeps
 * over the active window, the first with the eigenvalue of the trailing 2x2 block that is
 * closer to the last diagonal entry, the second with the other one, both taken from the
 * matrix as it was before the first sweep (Eq. (15), App. A.3).  Exists so that a test can
 * compare one iteration with T' = R Q + mu I of an explicit QR factorisation.
 *   d, e        as bed_tridiag_qr
 *   sweeps      >= 1: iterations run while fewer than this many sweeps have been done
 *               (2 = exactly one outer iteration on a matrix with no negligible entry)
 *   d_out,e_out device, [batch][n]: the tridiagonal after those sweeps (not sorted)
 *   Q           device, [batch][n][n] row-major: the product of the rotations, T_out = Q^T T Q
 *   rotations   device, [batch] or NULL
 *   n           1 .. 64 (BED_ERR_N beyond)
 */
int bed_tridiag_qr_sweeps(const float* d, const float* e, int batch, int n, int sweeps,
                          float* d_out, float* e_out, float* Q, unsigned* rotations,
                          void* stream);

/*
 * Fused spectral function of a batch of symmetric positive (semi-)definite
 * matrices: out_b = V_b f(max(Lambda_b, floor)) V_b^T, computed from the
 * eigendecomposition inside the same launch, without writing V.  This is what
 * the paper's applications do right after the decomposition: A^(-1/2) for ZCA
 * whitening / decorrelated batch normalisation and the whitening half of the
 * whitening-and-colouring transform, A^(1/2) for covariance pooling and the
 * colouring half (Sec. 4.2, 4.3, 4.4; App. B.1, B.2, B.3).
 *
 *   A      device, const, [batch][n][n] fp32, lower triangle read (as bed_syevd)
 *   fn     BED_FN_SQRT or BED_FN_INV_SQRT
 *   floor  eigenvalues below it are raised to it before f is applied; must be
 *          finite and >= 0, and > 0 for BED_FN_INV_SQRT (BED_ERR_ARG otherwise)
 *   out    device, [batch][n][n] row-major fp32, symmetric
 *   evals  device, [batch][n] ascending eigenvalues of A (not floored), or NULL
 *   info   device, [batch] as in bed_syevd_info, or NULL
 */
int bed_spd_fn(const float* A, int batch, int n, int fn, float floor, float* out,
               float* evals, int* info, void* stream);

typedef enum {
    BED_GRAD_EXACT = 0,  /* K_ij = 1/(lambda_j - lambda_i) where |lambda_j - lambda_i| >= gap_floor, else 0 */
    BED_GRAD_TAYLOR = 1  /* K_ij replaced by its truncated geometric series of the given degree          */
} bed_grad_mode;

/*
 * Gradient through the eigendecomposition A = V diag(lambda) V^T (Sec. 3.1 Eq. (1)): for a
 * loss with upstream gradients grad_evals (dL/dlambda) and grad_evecs (dL/dV),
 *
 *   grad_A = V ( diag(grad_evals) + sym( K o (V^T grad_evecs) ) ) V^T,   K_ii = 0,
 *
 * the symmetric gradient with respect to A (first-order perturbation theory).  The paper
 * does not derive a backward pass of its own; it uses a Taylor polynomial of degree 9 in
 * place of 1/(lambda_i - lambda_j), which stays finite for close and repeated eigenvalues
 * (Sec. 2; App. B "Implementation Details" and App. B.1).  BED_GRAD_TAYLOR is that choice:
 * for the pair (a, b) = (lambda_i, lambda_j) with b the larger in magnitude (for equal
 * magnitudes: the later index), K_ij = (1/b) sum_{k=0}^{degree} (a/b)^k, mirrored with the
 * opposite sign otherwise, so that K is antisymmetric and finite for repeated eigenvalues.  BED_GRAD_EXACT is the unmodified coupling
 * with pairs closer than gap_floor (absolute) dropped.
 *
 *   evals, evecs     device, const, [batch][n] and [batch][n][n] as written by bed_syevd
 *   grad_evals       device, const, [batch][n], or NULL (taken as zero)
 *   grad_evecs       device, const, [batch][n][n], or NULL (taken as zero); not both NULL
 *   mode, degree, gap_floor   see above; degree in 0..64 (BED_GRAD_TAYLOR), gap_floor finite
 *                    and >= 0 (BED_GRAD_EXACT); the unused one is ignored
 *   grad_A           device, [batch][n][n] row-major fp32; may alias none of the inputs
 */
int bed_syevd_backward(const float* evals, const float* evecs, const float* grad_evals,
                       const float* grad_evecs, int batch, int n, int mode, int degree,
                       float gap_floor, float* grad_A, void* stream);

/*
 * Gradient through bed_spd_fn: for F = V f(max(Lambda, floor)) V^T (Sec. 4.2-4.4, App.
 * B.1-B.3) and an upstream gradient grad_out = dL/dF,
 *
 *   grad_A = V ( Phi o (V^T sym(grad_out) V) ) V^T,
 *   Phi_ij = (f~(lambda_i) - f~(lambda_j)) / (lambda_i - lambda_j),  f~(x) = f(max(x, floor)),
 *
 * with the derivative of f~ where the two eigenvalues coincide.  For eigenvalues above the
 * floor the divided difference is evaluated without cancellation (1/(s_i + s_j) for the
 * square root, -1/(s_i s_j (s_i + s_j)) for the inverse square root, s = sqrt(lambda)), so
 * close and repeated eigenvalues need no special treatment.
 *
 *   evals, evecs   device, const, eigendecomposition of A as written by bed_syevd
 *   grad_out       device, const, [batch][n][n] (need not be symmetric)
 *   fn, floor      as in bed_spd_fn
 *   grad_A         device, [batch][n][n]; may alias none of the inputs
 */
int bed_spd_fn_backward(const float* evals, const float* evecs, const float* grad_out, int batch,
                        int n, int fn, float floor, float* grad_A, void* stream);

/*
 * The paper's fixed-budget procedure as written (Sec. 3.2.3, App. B), kept for comparison with
 * bed_syevd; it is NOT a solver to rely on (the budget can end far from convergence).  After the
 * tridiagonalisation of Sec. 3.1, `iterations` outer iterations (App. B: n), each two shifted QR
 * steps over the leading m x m window with the two eigenvalues of its trailing 2x2 block, both
 * taken from the matrix the iteration starts from (Sec. 3.2.2, App. A.3; the one closer to the
 * last diagonal entry first).  After an iteration the window shrinks by one row if the last
 * sub-diagonal entry of the window is at most `epsilon` in magnitude (App. B: 1e-5; absolute, that
 * entry only): with uniform = 1 for the whole batch at once, when every matrix passes, as a
 * batched tensor forces; with uniform = 0 for each matrix on its own.  No other deflation, no
 * convergence test, no pre-scaling of A (the test is absolute).  One launch per iteration.
 *
 *   A            device, const, [batch][n][n], lower triangle read, n in 1 .. 64 (BED_ERR_N beyond)
 *   epsilon      >= 0, finite;  iterations >= 0;  uniform 0 or 1   (else BED_ERR_ARG)
 *   evals        device, [batch][n]: diag(T) when the budget ends, ascending
 *   evecs        device, [batch][n][n] or NULL: P Q_1 Q_2 ..., columns in the order of evals
 *                (working storage between the launches)
 *   offdiag      device, [batch][n] or NULL: |sub-diagonal| of T when the budget ends, in the
 *                order of T before the sort (offdiag[b][k] couples rows k, k+1; last entry 0);
 *                ||A V - V diag(evals)||_F = sqrt(2 sum offdiag^2) up to rounding
 *   reductions   device, [batch] or NULL: rows dropped (equal for all matrices when uniform)
 *   workspace    device, at least bed_syevd_lockstep_workspace(batch, n, iterations) bytes, 4-byte
 *                aligned, owned by the caller, contents undefined afterwards; workspace_bytes is
 *                its size (BED_ERR_ARG if too small).  Calls that share a workspace must not overlap.
 * No buffer may alias another.  Asynchronous on `stream` like every other entry point.
 */
size_t bed_syevd_lockstep_workspace(int batch, int n, int iterations);
int bed_syevd_lockstep(const float* A, int batch, int n, float epsilon, int iterations, int uniform,
                       float* evals, float* evecs, float* offdiag, int* reductions,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * bed_syevd_lockstep for callers that can neither allocate nor bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and same results as bed_syevd_lockstep, but the per-iteration state lives in scratch
 * memory built into the library (a file-scope __device__ array, one copy per GPU, held until the
 * process ends) instead of a caller-owned workspace.  The call allocates nothing, on the host
 * side of the runtime or on the device.
 *
 *   capacity     bed_syevd_lockstep_static_capacity() bytes (1 MiB).  A problem fits when
 *                bed_syevd_lockstep_workspace(batch, n, iterations) <= capacity, i.e. roughly
 *                batch * n <= 130 000 (512 matrices of 32 x 32 use 133 KB); otherwise the call
 *                returns BED_ERR_SCRATCH and enqueues nothing.
 *   sharing      every call on a GPU uses that GPU's one scratch array: calls that may overlap
 *                in time on the same GPU (different streams, different host threads) race and
 *                must be serialised by the caller.  The array keeps the previous call's
 *                contents; everything a call reads from it is written by that call first
 *                (a fill kernel, no memset node, so the call may be captured into a graph).
 *   first call   the first call on each device looks up the array's device address
 *                (hipGetSymbolAddress); make that call outside graph capture.
 * All other arguments, layouts and error codes are those of bed_syevd_lockstep.
 */
size_t bed_syevd_lockstep_static_capacity(void);
int bed_syevd_lockstep_static(const float* A, int batch, int n, float epsilon, int iterations, int uniform,
                              float* evals, float* evecs, float* offdiag, int* reductions, void* stream);

/*
 * Measurement aids (not part of the method): the rates this build reaches on this machine, reported by
 * the benchmark beside the datasheet peaks.
 *
 * bed_ceiling_fma: every lane runs `chains` (1 or 16) independent chains of `iters` dependent
 *   v_fma_f32 (plain, not packed); 2 * blocks * threads * chains * iters flops in total.
 *   chains = 16 with several wavefronts per SIMD measures the vector ALU's plain-FMA throughput;
 *   chains = 1 with one 64-thread block per SIMD measures what one dependent instruction stream
 *   issues.  out: device, [blocks * threads] floats (written once at the end); threads a multiple
 *   of 64, <= 1024; iters a multiple of 64.
 * bed_ceiling_copy: plain device copy of `count` floats (count a multiple of 4, both pointers
 *   16-byte aligned, buffers must not overlap) by `blocks` blocks of 256 threads; 8 * count bytes
 *   of HBM traffic.
 */
int bed_ceiling_fma(float* out, int blocks, int threads, int chains, int iters, void* stream);
int bed_ceiling_copy(const float* src, float* dst, size_t count, int blocks, void* stream);

/*
 * Measurement aid: the duration of the library's own kernels, one figure per launch, taken from
 * the dispatch's begin and end timestamps (each timed kernel is launched with a start and a stop
 * event of its own; no marker is queued between the kernels of the stream, which a pair of
 * events recorded around a call would add, at 2-3 us per pair).  State is per host thread.
 * Not for launches into a stream that is being captured into a graph: disarm first.
 *   bed_timing_begin(capacity)  creates 2 * capacity events (host side; 1 <= capacity <= 2^20)
 *                               for the calling thread, not yet armed; BED_ERR_LAUNCH if the
 *                               runtime refuses, BED_ERR_ARG for a capacity out of range.
 *   bed_timing_arm(on)          on != 0: from now on every kernel that this thread launches
 *                               through the library is timed, until `capacity` launches have been
 *                               timed (later ones run untimed); 0: launches run untimed again.
 *                               BED_ERR_ARG without a bed_timing_begin.
 *   bed_timing_end(us, max_count, count)
 *                               waits for the timed kernels, writes their durations in
 *                               microseconds, in launch order, to us[0 .. min(*count, max_count))
 *                               (host memory), sets *count to the number of timed launches and
 *                               destroys the events.  BED_ERR_ARG without a bed_timing_begin or
 *                               for null pointers, BED_ERR_LAUNCH if an event could not be read.
 */
int bed_timing_begin(int capacity);
int bed_timing_arm(int on);
int bed_timing_end(float* microseconds, int max_count, int* count);

/*
 * Name of the kernel that bed_syevd (want_vectors = 1) or its eigenvalues-only form
 * (want_vectors = 0) launches for this batch and n, e.g. "wave_kernel<32>" (one wavefront per
 * matrix, register arrays of 32), "packed_kernel<16>" (several matrices per wavefront),
 * "lane_kernel<4>" (one matrix per lane), "pair_kernel<64>" (two wavefronts per matrix),
 * "block_kernel" (four wavefronts per matrix); static storage, NULL for arguments out of range.
 */
const char* bed_kernel_variant(int batch, int n, int want_vectors);

/* Human-readable name of a bed_status value (static storage). */
const char* bed_status_string(int status);

/* BED_VERSION the library was built with. */
int bed_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BED_H */
