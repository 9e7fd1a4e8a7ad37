#ifndef BED_WAVE_KERNEL_HPP
#define BED_WAVE_KERNEL_HPP
// Batched symmetric eigensolver kernels for gfx950 (MI355X), wave64.
//
// One wavefront owns one matrix from load to store; lane r holds row r of the
// working matrix and row r of the eigenvector accumulator in VGPRs.  The
// whole path of arXiv 2207.04228 Sec. 3 runs inside one launch:
//   Sec. 3.1   Householder tridiagonalisation (rank-2 update form, Eqs. (5)-(6)),
//              accumulation of P (Eq. (8)) as rank-1 updates of V
//   Sec. 3.2   QR iterations by Givens rotations (App. A.1) with the two
//              Wilkinson shifts of the trailing 2x2 block (Sec. 3.2.2, App. A.3),
//              per-matrix deflation (Sec. 3.2.3), O(1) update of the
//              tridiagonal per rotation (Sec. 3.2.4) and rotation of two
//              columns of V per rotation (Sec. 3.2.5)
// followed by an ascending sort and a coalesced store.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bed_kernel.h"

namespace bed {

namespace {

constexpr float kEps = 1.1920929e-7f;   // 2^-23: relative deflation tolerance
constexpr float kTinyE = 1.0e-18f;      // absolute floor for |e| (matrix is pre-scaled to max|a| in [0.5,1))
constexpr float kTinyH = 1.0e-37f;      // f^2+g^2 below this: rotation degenerates to the identity

// ---- cross-lane helpers ---------------------------------------------------

template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), CTRL, 0xF, 0xF, true));
}

constexpr int kQuadXor1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kQuadXor2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141;
constexpr int kRowMirror = 0x140;
constexpr int kWaveShl1 = 0x130;     // lane i reads lane i+1

// All-reduce (sum) over lanes [0, N) of the wave; every lane of that range
// ends with the total.  Butterfly: quad xor 1, xor 2, then mirrors act as
// xor 4 / xor 8 on quad-uniform values, then LDS-crossbar shuffles.
template <int N>
__device__ __forceinline__ float group_sum(float x) {
    x += dpp<kQuadXor1>(x);
    x += dpp<kQuadXor2>(x);
    if (N >= 8) x += dpp<kRowHalfMirror>(x);
    if (N >= 16) x += dpp<kRowMirror>(x);
    if (N >= 32) x += __shfl_xor(x, 16, 64);
    if (N >= 64) x += __shfl_xor(x, 32, 64);
    return x;
}

template <int N>
__device__ __forceinline__ float group_max(float x) {
    x = fmaxf(x, dpp<kQuadXor1>(x));
    x = fmaxf(x, dpp<kQuadXor2>(x));
    if (N >= 8) x = fmaxf(x, dpp<kRowHalfMirror>(x));
    if (N >= 16) x = fmaxf(x, dpp<kRowMirror>(x));
    if (N >= 32) x = fmaxf(x, __shfl_xor(x, 16, 64));
    if (N >= 64) x = fmaxf(x, __shfl_xor(x, 32, 64));
    return x;
}

__device__ __forceinline__ float uniform(float x) {
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x)));
}

__device__ __forceinline__ float read_lane(float x, int lane_uniform) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane_uniform));
}

// Monotone map float -> uint32 (total order; NaNs land at the ends).
__device__ __forceinline__ uint32_t sort_key(float x) {
    uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace

// ---------------------------------------------------------------------------
// N      padded dimension (8, 16, 32, 64); n <= N at run time
// WANT_V accumulate eigenvectors
// STAGE  kFull, kTridiagOnly (stage hook 1), kQrOnly (stage hook 2)
// SHIFT  kShiftDouble: both eigenvalues of the trailing 2x2 are taken once per
//        outer iteration (Sec. 3.2.2); the second sweep uses the second one
//        unless the first sweep already deflated the window.
//        kShiftSingle: the eigenvalue closer to the last diagonal entry is
//        recomputed before every sweep.
// ---------------------------------------------------------------------------
template <int N, bool WANT_V, int STAGE, int SHIFT>
__global__ __launch_bounds__(64) void wave_kernel(KernelArgs args) {
    constexpr int LD = N + 1;
    __shared__ float smat[N * LD];
    __shared__ float svec[64];

    const int lane = threadIdx.x;
    const int b = blockIdx.x;
    const int n = args.n;

    float a[N];
    float v[N];
    float d[N];
    float e[N];
    float dl = 0.f, el = 0.f;  // lane-distributed mirrors: lane k holds d[k], e[k]
    float inv_scale = 1.f;

#pragma unroll
    for (int c = 0; c < N; ++c) {
        v[c] = (c == lane) ? 1.f : 0.f;
        d[c] = 0.f;
        e[c] = 0.f;
    }

    if (STAGE != kQrOnly) {
        // ---- load: coalesced into LDS, then row `lane` (lower triangle mirrored)
        const float* __restrict__ Ab = args.A + (size_t)b * n * n;
        const float rcp_n = 1.0f / (float)n;
        for (int idx = lane; idx < n * n; idx += 64) {
            int i = (int)(((float)idx + 0.5f) * rcp_n);
            int j = idx - i * n;
            smat[i * LD + j] = Ab[idx];
        }
        __syncthreads();
        float amax = 0.f;
#pragma unroll
        for (int c = 0; c < N; ++c) {
            float x = 0.f;
            if (lane < n && c < n) x = (c <= lane) ? smat[lane * LD + c] : smat[c * LD + lane];
            a[c] = x;
            amax = fmaxf(amax, fabsf(x));   // fmaxf drops NaNs; they still reach the output through the arithmetic
        }
        __syncthreads();
        amax = uniform(group_max<N>(amax));
        // exact power-of-two pre-scaling: max|a| -> [0.5, 1)
        int ex = 0;
        if (amax > 0.f && amax < __builtin_inff()) ex = __builtin_amdgcn_frexp_expf(amax);
        ex = min(max(ex, -125), 126);
        const float scale = ldexpf(1.0f, -ex);
        inv_scale = ldexpf(1.0f, ex);
#pragma unroll
        for (int c = 0; c < N; ++c) a[c] *= scale;

        // ---- Householder tridiagonalisation, column J reduced at step J ----
#pragma unroll
        for (int J = 0; J < N; ++J) {
            // d[J] is final once columns 0..J-1 are reduced
            {
                float dj = read_lane(a[J], J);
                d[J] = dj;
                if (lane == J) dl = dj;
            }
            if (J < N - 2 && J < n - 2) {
                const float x = (lane > J) ? a[J] : 0.f;           // A[r][J], r > J
                const float alpha = uniform(group_sum<N>(x * x));    // |x|^2
                const float x0 = read_lane(a[J], J + 1);             // A[J+1][J]
                if (alpha > 0.f) {
                    const float nrm = sqrtf(alpha);
                    const float sigma = (x0 < 0.f) ? -nrm : nrm;     // sign chosen to avoid cancellation
                    const float ur = (lane == J + 1) ? (x0 + sigma) : ((lane > J + 1) ? x : 0.f);
                    const float beta = 1.0f / (alpha + fabsf(x0) * nrm);  // 2 / |u|^2
                    svec[lane] = ur;
                    __syncthreads();
                    float u[N];
#pragma unroll
                    for (int c = J + 1; c < N; ++c) u[c] = svec[c];
                    __syncthreads();
                    float p = 0.f, w = 0.f;
#pragma unroll
                    for (int c = J + 1; c < N; ++c) {
                        p = fmaf(a[c], u[c], p);
                        if (WANT_V) w = fmaf(v[c], u[c], w);
                    }
                    p *= beta;                                        // p = 2 A u / |u|^2
                    w *= beta;
                    const float K = 0.5f * beta * uniform(group_sum<N>(ur * p));
                    const float q = fmaf(-K, ur, p);                  // q = p - K u (symmetric rank-2 form)
                    svec[lane] = q;
                    __syncthreads();
#pragma unroll
                    for (int c = J + 1; c < N; ++c) {
                        const float qc = svec[c];
                        a[c] = fmaf(-q, u[c], a[c]);
                        a[c] = fmaf(-ur, qc, a[c]);
                        if (WANT_V) v[c] = fmaf(-w, u[c], v[c]);
                    }
                    __syncthreads();
                    e[J] = -sigma;
                } else {
                    e[J] = 0.f;
                }
                if (lane == J) el = e[J];
            } else if (J < N - 1 && J == n - 2) {
                const float ej = read_lane(a[J], J + 1);
                e[J] = ej;
                if (lane == J) el = ej;
            }
        }
    } else {
        // ---- stage hook 2: tridiagonal given ----
        float dv = 0.f, ev = 0.f;
        if (lane < n) dv = args.d_in[(size_t)b * n + lane];
        if (lane < n - 1) ev = args.e_in[(size_t)b * n + lane];
        float amax = uniform(group_max<N>(fmaxf(fabsf(dv), fabsf(ev))));
        int ex = 0;
        if (amax > 0.f && amax < __builtin_inff()) ex = __builtin_amdgcn_frexp_expf(amax);
        ex = min(max(ex, -125), 126);
        const float scale = ldexpf(1.0f, -ex);
        inv_scale = ldexpf(1.0f, ex);
        dl = dv * scale;
        el = ev * scale;
        svec[lane] = dl;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < N; ++c) d[c] = svec[c];
        __syncthreads();
        svec[lane] = el;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < N; ++c) e[c] = svec[c];
        __syncthreads();
    }

    uint32_t rotations = 0;
    int info = 0;

    if (STAGE == kTridiagOnly) {
        if (lane < n) {
            args.d_out[(size_t)b * n + lane] = dl * inv_scale;
            args.e_out[(size_t)b * n + lane] = (lane < n - 1) ? el * inv_scale : 0.f;
        }
    } else {
        // ---- shifted QR iterations on (d, e) ----
        const uint32_t cap = 30u * (uint32_t)n;
        uint32_t sweeps = 0;
        bool have_second = false;
        float mu_second = 0.f;
        int prev_lo = -1, prev_hi = -1;
        uint64_t nz = 0;
        while (true) {
            // deflation test, one off-diagonal per lane
            const float dnext = __shfl_down(dl, 1, 64);
            const bool live = (lane < n - 1) && (el != 0.f) &&
                              !(fabsf(el) <= fmaxf(kEps * (fabsf(dl) + fabsf(dnext)), kTinyE));
            if (!live) el = 0.f;
            nz = __ballot(live);
            if (nz == 0 || sweeps >= cap) break;
            const int hi = 64 - __builtin_clzll(nz);          // e[hi-1] is the last live entry
            const uint64_t below = ~nz & ((1ull << (hi - 1)) - 1ull);
            const int lo = below ? 64 - __builtin_clzll(below) : 0;

            float mu;
            if (SHIFT == kShiftDouble && have_second && lo == prev_lo && hi == prev_hi) {
                mu = mu_second;
                have_second = false;
            } else {
                // eigenvalues of [[ta, tb], [tb, td]] (App. A.3), smaller-angle root first
                const float ta = read_lane(dl, hi - 1);
                const float tb = read_lane(el, hi - 1);
                const float td = read_lane(dl, hi);
                const float delta = 0.5f * (ta - td);
                const float rt = sqrtf(fmaf(delta, delta, tb * tb));
                const float den = delta + ((delta >= 0.f) ? rt : -rt);
                const float t = (tb * tb) / den;
                mu = td - t;          // eigenvalue closer to the last diagonal entry
                mu_second = ta + t;   // the other eigenvalue of the block
                have_second = true;
                prev_lo = lo;
                prev_hi = hi;
            }

            // one implicit QR sweep over the window [lo, hi]
            float g = read_lane(dl, lo) - mu;
            float s = 1.f, c = 1.f, p = 0.f;
            const uint64_t act = ((1ull << hi) - 1ull) & ~((1ull << lo) - 1ull);  // bits lo..hi-1
#pragma unroll
            for (int k = 0; k < N; ++k) {
                if (k < N - 1 && ((act >> k) & 1ull)) {
                    const float ek = e[k];
                    const float f = s * ek;
                    const float bb = c * ek;
                    const float h = fmaf(f, f, g * g);
                    const bool ok = h > kTinyH;
                    float rinv = __builtin_amdgcn_rsqf(h);
                    rinv = ok ? rinv : 0.f;
                    const float r = h * rinv;
                    if (k > 0) {
                        e[k - 1] = r;
                        if (lane == k - 1) el = r;
                    }
                    s = f * rinv;
                    c = ok ? g * rinv : 1.f;
                    g = d[k] - p;
                    const float r2 = fmaf(d[k + 1] - g, s, 2.f * c * bb);
                    p = s * r2;
                    const float dk = g + p;
                    d[k] = dk;
                    if (lane == k) dl = dk;
                    g = fmaf(c, r2, -bb);
                    if (WANT_V) {
                        const float x = v[k], y = v[k + 1];
                        v[k] = fmaf(c, x, s * y);
                        v[k + 1] = fmaf(c, y, -s * x);
                    }
                } else if (k == hi) {
                    const float dk = d[k] - p;
                    d[k] = dk;
                    if (lane == k) dl = dk;
                    e[k - 1] = g;
                    if (lane == k - 1) el = g;
                }
            }
            // the first rotation wrote a value into the mirror of e[lo-1], which is outside the window
            if (lo > 0 && lane == lo - 1) el = 0.f;
            rotations += (uint32_t)(hi - lo);
            ++sweeps;
        }
        info = __builtin_popcountll(nz);
        {
            // a non-finite eigenvalue (NaN/Inf input) is reported even when every off-diagonal deflated
            const uint64_t bad = __ballot(lane < n && !(fabsf(dl) < __builtin_inff()));
            info = max(info, (int)__builtin_popcountll(bad));
        }

        // ---- ascending order ----
        const uint32_t mykey = sort_key(dl);
        int rank = 0;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            if (j < n) {
                const uint32_t kj = sort_key(d[j]);
                rank += (kj < mykey || (kj == mykey && j < lane)) ? 1 : 0;
            }
        }
        if (lane < n) args.evals[(size_t)b * n + rank] = dl * inv_scale;
        if (WANT_V) {
            int* srank = reinterpret_cast<int*>(svec);
            srank[lane] = rank;
            __syncthreads();
#pragma unroll
            for (int c = 0; c < N; ++c) {
                if (c < n && lane < n) smat[lane * LD + srank[c]] = v[c];
            }
            __syncthreads();
        }
    }

    if (STAGE == kTridiagOnly && WANT_V) {
        __syncthreads();
#pragma unroll
        for (int c = 0; c < N; ++c) {
            if (c < n && lane < n) smat[lane * LD + c] = v[c];
        }
        __syncthreads();
    }
    if (WANT_V) {
        float* __restrict__ Vb = args.evecs + (size_t)b * n * n;
        const float rcp_n = 1.0f / (float)n;
        for (int idx = lane; idx < n * n; idx += 64) {
            int i = (int)(((float)idx + 0.5f) * rcp_n);
            int j = idx - i * n;
            Vb[idx] = smat[i * LD + j];
        }
    }
    if (lane == 0) {
        if (args.info) args.info[b] = info;
        if (args.rotations) args.rotations[b] = rotations;
    }
}

// ---------------------------------------------------------------------------
// host-side dispatch for one padded size
// ---------------------------------------------------------------------------
template <int N, bool WANT_V, int STAGE, int SHIFT>
static hipError_t launch_one(const KernelArgs& args, hipStream_t stream) {
    hipLaunchKernelGGL((wave_kernel<N, WANT_V, STAGE, SHIFT>), dim3(args.batch), dim3(64), 0, stream, args);
    return hipGetLastError();
}

template <int N>
static hipError_t launch_n(const KernelArgs& args, int stage, int shift, bool want_v, hipStream_t stream) {
    if (stage == kTridiagOnly) {
        return want_v ? launch_one<N, true, kTridiagOnly, kShiftDouble>(args, stream)
                      : launch_one<N, false, kTridiagOnly, kShiftDouble>(args, stream);
    }
    if (stage == kQrOnly) {
        if (shift == kShiftSingle)
            return want_v ? launch_one<N, true, kQrOnly, kShiftSingle>(args, stream)
                          : launch_one<N, false, kQrOnly, kShiftSingle>(args, stream);
        return want_v ? launch_one<N, true, kQrOnly, kShiftDouble>(args, stream)
                      : launch_one<N, false, kQrOnly, kShiftDouble>(args, stream);
    }
    if (shift == kShiftSingle)
        return want_v ? launch_one<N, true, kFull, kShiftSingle>(args, stream)
                      : launch_one<N, false, kFull, kShiftSingle>(args, stream);
    return want_v ? launch_one<N, true, kFull, kShiftDouble>(args, stream)
                  : launch_one<N, false, kFull, kShiftDouble>(args, stream);
}

}  // namespace bed
#endif
