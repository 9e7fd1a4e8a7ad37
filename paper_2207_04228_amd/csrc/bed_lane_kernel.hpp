// One matrix per LANE, for tiny matrices (n <= 8): 64 matrices per wavefront.
//
// Same method as the one-wavefront-per-matrix kernel (arXiv 2207.04228 Sec. 3:
// Householder tridiagonalisation, then pairs of QR sweeps by Givens rotations
// with the two Wilkinson shifts of the trailing 2x2 block, per-matrix
// deflation, eigenvector accumulation), but every quantity is private to a
// lane, so there are no cross-lane reductions, broadcasts or barriers at all:
//   * the tridiagonalisation (Sec. 3.1) runs on register arrays with
//     compile-time indices (fully unrolled);
//   * the QR stage (Sec. 3.2) also stays in registers: a sweep is unrolled over
//     all N-1 rotation positions and a lane commits the results of position k
//     only if k lies inside its own window (selects, no branches), with an
//     identity rotation applied to V elsewhere.  Lanes whose matrix has
//     converged run with an empty window until the slowest lane is done.
// Global memory is read and written through an LDS staging buffer so that all
// accesses are coalesced.  This kernel is what makes large batches of 4x4 /
// 8x8 matrices (Fig. 1 left of the paper) run at a useful fraction of the
// memory roofline: no lane is idle.
#ifndef BED_LANE_KERNEL_HPP
#define BED_LANE_KERNEL_HPP
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bed_kernel.h"

namespace bed {

namespace lanek {

// 4 * 2^-23: relative deflation tolerance (well above the rounding level that the recurrence
// leaves on the off-diagonals inside a cluster of equal eigenvalues)
constexpr float kEps = 4.7683716e-7f;
constexpr float kTinyE = 1.0e-18f;      // absolute floor for |e| (matrix pre-scaled to max|a| in [0.5,1))
constexpr float kTinyG = 1.0e-18f;      // floor for the rotation pivot
constexpr float kTinyAlpha = 1.0e-35f;  // |x|^2 below this: column already reduced

__device__ __forceinline__ float guard_g(float g) {
    float mag;
    asm("v_max_f32 %0, |%1|, %2" : "=v"(mag) : "v"(g), "v"(kTinyG));
    return __uint_as_float((__float_as_uint(g) & 0x80000000u) | __float_as_uint(mag));
}

__device__ __forceinline__ uint32_t sort_key(float x) {
    uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace lanek

// STAGE: kFull, or kSpectral (the fused V f(max(Lambda, floor)) V^T of Sec. 4.2-4.4 / App.
// B.1-B.3: formed in registers from V and lambda, eigenvectors never written).
template <int N, bool WANT_V, int STAGE>
__global__ __launch_bounds__(64) void lane_kernel(KernelArgs args) {
    using namespace lanek;
    constexpr int NN = N * N;
    constexpr int MS = NN + 1;                 // staging stride per matrix (odd: conflict-free per-lane reads)
    __shared__ float stage[64 * MS];

    const int lane = threadIdx.x;
    const int n = args.n;
    const int nn = n * n;
    const long long b0 = (long long)blockIdx.x * 64;
    const int nb = (int)min((long long)64, (long long)args.batch - b0);   // matrices in this wavefront
    const bool mine = lane < nb;

    // ---- coalesced load into the staging buffer ----
    {
        const float* __restrict__ Ab = args.A + b0 * nn;
        const float rcp = 1.0f / (float)nn;
        chunked_copy<16>(
            nb * nn, lane, [&](int idx) { return Ab[idx]; },
            [&](int idx, float x) {
                const int m = (int)(((float)idx + 0.5f) * rcp);
                stage[m * MS + (idx - m * nn)] = x;
            });
    }
    __syncthreads();

    float a[N][N];
    float v[N][N];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) {
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            float x = 0.f;
            if (mine && i < n && j < n) x = stage[lane * MS + i * n + j];   // lower triangle, mirrored
            a[i][j] = x;
            a[j][i] = x;
            amax = fmaxf(amax, fabsf(x));
        }
    }
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int j = 0; j < N; ++j) v[i][j] = (i == j) ? 1.f : 0.f;
    __syncthreads();

    // exact power-of-two pre-scaling: max|a| -> [0.5, 1)
    int ex = 0;
    if (amax > 0.f && amax < __builtin_inff()) ex = __builtin_amdgcn_frexp_expf(amax);
    ex = min(max(ex, -125), 126);
    const float scale = ldexpf(1.0f, -ex);
    const float inv_scale = ldexpf(1.0f, ex);
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int j = 0; j < N; ++j) a[i][j] *= scale;

    // ---- Householder tridiagonalisation (Sec. 3.1), branch-free, fully unrolled ----
    float d[N], e[N];
#pragma unroll
    for (int k = 0; k < N; ++k) e[k] = 0.f;
#pragma unroll
    for (int J = 0; J < N - 2; ++J) {
        float alpha = 0.f;
#pragma unroll
        for (int r = J + 1; r < N; ++r) alpha = fmaf(a[r][J], a[r][J], alpha);
        const float x0 = a[J + 1][J];
        const bool active = (J < n - 2) && (alpha > kTinyAlpha);
        const float nrm = __builtin_amdgcn_sqrtf(alpha);
        const float sigma = (x0 < 0.f) ? -nrm : nrm;
        const float beta = active ? __builtin_amdgcn_rcpf(fmaf(fabsf(x0), nrm, alpha)) : 0.f;   // 2/|u|^2
        float u[N];
#pragma unroll
        for (int r = J + 1; r < N; ++r) u[r] = active ? ((r == J + 1) ? (x0 + sigma) : a[r][J]) : 0.f;
        // p = 2 A u / |u|^2 on the trailing block, K = u^T p / |u|^2, q = p - K u
        float q[N];
        float K = 0.f;
#pragma unroll
        for (int r = J + 1; r < N; ++r) {
            float p = 0.f;
#pragma unroll
            for (int c = J + 1; c < N; ++c) p = fmaf(a[r][c], u[c], p);
            p *= beta;
            q[r] = p;
            K = fmaf(u[r], p, K);
        }
        K *= 0.5f * beta;
#pragma unroll
        for (int r = J + 1; r < N; ++r) q[r] = fmaf(-K, u[r], q[r]);
        // A <- A - q u^T - u q^T on the trailing block (lower triangle, mirrored)
#pragma unroll
        for (int r = J + 1; r < N; ++r) {
#pragma unroll
            for (int c = J + 1; c <= r; ++c) {
                float x = a[r][c];
                x = fmaf(-q[r], u[c], x);
                x = fmaf(-u[r], q[c], x);
                a[r][c] = x;
                a[c][r] = x;
            }
        }
        if (WANT_V) {
            // V <- V (I - beta u u^T); row 0 of V stays e_0
#pragma unroll
            for (int r = 1; r < N; ++r) {
                float w = 0.f;
#pragma unroll
                for (int c = J + 1; c < N; ++c) w = fmaf(v[r][c], u[c], w);
                w *= beta;
#pragma unroll
                for (int c = J + 1; c < N; ++c) v[r][c] = fmaf(-w, u[c], v[r][c]);
            }
        }
        e[J] = active ? -sigma : x0;
    }
#pragma unroll
    for (int k = 0; k < N; ++k) d[k] = a[k][k];
    if (N >= 2) {
        // the last off-diagonal is never touched by a reflector
#pragma unroll
        for (int k = 0; k < N - 1; ++k)
            if (k == n - 2) e[k] = a[k + 1][k];
#pragma unroll
        for (int k = 0; k < N; ++k)
            if (k >= n - 1) e[k] = 0.f;
    }

    // ---- QR iterations (Sec. 3.2), everything in registers ----
    uint32_t live = 0;                     // bit k: e[k] not yet deflated
#pragma unroll
    for (int k = 0; k < N - 1; ++k)
        if (mine && k < n - 1) live |= (1u << k);
    uint32_t rotations = 0;
    uint32_t sweeps = 0;
    const uint32_t cap = args.sweep_cap ? args.sweep_cap : 30u * (uint32_t)n;

    // One sweep of the implicit shifted QR step over rows lo..hi (this lane's window; an
    // empty window, hi <= lo, leaves everything untouched).  Position k is committed only
    // when lo <= k < hi.
    auto sweep = [&](int lo, int hi, float mu) {
        float g = 0.f, s = 1.f, c = 1.f, p = 0.f;
#pragma unroll
        for (int k = 0; k < N - 1; ++k) {
            const bool act = (k >= lo) && (k < hi);
            // a position outside the window of every lane of the wavefront changes nothing
            if (__ballot(act) == 0) continue;
            const bool first = (k == lo);
            g = first ? (d[k] - mu) : g;
            const float ek = e[k];
            const float dk1 = d[k + 1];
            const float gg = guard_g(g);
            const float f = s * ek;
            const float bb = c * ek;
            const float h = fmaf(f, f, gg * gg);
            const float rinv = __builtin_amdgcn_rsqf(h);
            const float cn = gg * rinv;
            const float sn = f * rinv;
            const float gk = d[k] - p;
            const float r2 = fmaf(dk1 - gk, sn, 2.f * cn * bb);
            const float pn = sn * r2;
            if (k > 0) e[k - 1] = (act && !first) ? (h * rinv) : e[k - 1];
            d[k] = act ? (gk + pn) : d[k];
            g = act ? fmaf(cn, r2, -bb) : g;
            s = act ? sn : s;
            c = act ? cn : c;
            p = act ? pn : p;
            const bool last = act && (k + 1 == hi);
            d[k + 1] = last ? (dk1 - p) : d[k + 1];
            e[k] = last ? g : e[k];
            if (WANT_V) {
                const float ce = act ? cn : 1.f;
                const float se = act ? sn : 0.f;
#pragma unroll
                for (int r = 0; r < N; ++r) {
                    const float x = v[r][k], y = v[r][k + 1];
                    v[r][k] = fmaf(ce, x, se * y);
                    v[r][k + 1] = fmaf(ce, y, -se * x);
                }
            }
        }
        rotations += (hi > lo) ? (uint32_t)(hi - lo) : 0u;
        sweeps += (hi > lo) ? 1u : 0u;
    };

    // absolute part of the deflation test: the rounding-level floor, or the paper's threshold
    // epsilon (Sec. 3.2.3, App. B) in units of the pre-scaled matrix when the caller asked for it
    const float paper_eps = args.abs_eps * scale;
    const float tol0 = fmaxf(kTinyE, paper_eps), tol1 = fmaxf(2.3841858e-7f, paper_eps), tol2 = fmaxf(9.5367432e-7f, paper_eps);
    uint32_t live_prev = ~0u, stall = 0;      // iterations of this lane since its last deflation
    uint32_t relaxed = 0;                     // off-diagonals deflated only because the absolute fallback test accepted them
    while (true) {
        // deflation test over every live off-diagonal of this lane; a window that has not
        // deflated anything for 12 (24) iterations also accepts entries below an absolute
        // threshold of 2^-22 (2^-20) of the pre-scaled matrix (at most 2e-6 ||A||_2 per entry;
        // counted and reported through info)
        const float abs_tol = stall >= 24u ? tol2 : (stall >= 12u ? tol1 : tol0);
#pragma unroll
        for (int k = 0; k < N - 1; ++k) {
            const float dsum = fabsf(d[k]) + fabsf(d[k + 1]);
            const bool negl = fabsf(e[k]) <= fmaxf(kEps * dsum, abs_tol);
            const bool base = fabsf(e[k]) <= fmaxf(kEps * dsum, tol0);
            relaxed += ((live >> k) & 1u) && negl && !base ? 1u : 0u;
            live = negl ? (live & ~(1u << k)) : live;
        }
        stall = (live == live_prev) ? stall + 1u : 0u;
        live_prev = live;
        const bool active = (live != 0) && (sweeps < cap);
        if (__ballot(active) == 0) break;
        // this lane's window: the lowest run of live entries (empty for a finished lane)
        const uint32_t lv = active ? live : 0u;
        const int hi = lv ? (32 - __builtin_clz(lv)) : 0;          // e[hi-1] is the last live entry
        const uint32_t below = lv ? (~lv & ((1u << (hi - 1)) - 1u)) : 0u;
        const int lo = below ? 32 - __builtin_clz(below) : 0;
        // both eigenvalues of the trailing 2x2 block (App. A.3); the block is picked out of the
        // register arrays with selects
        float ta = 0.f, tb = 0.f, td = 1.f;
#pragma unroll
        for (int k = 0; k < N - 1; ++k) {
            const bool sel = (k + 1 == hi);
            ta = sel ? d[k] : ta;
            tb = sel ? e[k] : tb;
            td = sel ? d[k + 1] : td;
        }
        const float delta = 0.5f * (ta - td);
        const float rt = __builtin_amdgcn_sqrtf(fmaf(delta, delta, tb * tb));
        const float den = delta + ((delta >= 0.f) ? rt : -rt);
        const float tt = (tb * tb) * __builtin_amdgcn_rcpf(guard_g(den));
        const float mu1 = td - tt;
        // after 5 iterations without a deflation both sweeps use mu1: the pair (mu1, mu2) has
        // fixed points (diagonal 1, 0, 1 with off-diagonals 1 is one)
        const float mu2 = (stall >= 5u) ? mu1 : ta + tt;
        sweep(lo, hi, mu1);
        // a window that was the 2x2 block itself is diagonalised by the exact-shift step:
        // its off-diagonal is set to zero and the second sweep is skipped
        const bool single = (hi - lo == 1);
#pragma unroll
        for (int k = 0; k < N - 1; ++k) e[k] = (single && k == lo) ? 0.f : e[k];
        sweep(lo, single ? lo : hi, mu2);
    }
    int info = __builtin_popcount(live);

    // ---- ascending order, staging, coalesced store ----
    float lam[N];
#pragma unroll
    for (int k = 0; k < N; ++k) lam[k] = d[k];
    {
        int bad = 0;
#pragma unroll
        for (int k = 0; k < N; ++k) bad += (k < n && !(fabsf(lam[k]) < __builtin_inff())) ? 1 : 0;
        info = max(info, bad);
    }
    info |= (int)(relaxed << 16);
    int rank[N];
#pragma unroll
    for (int k = 0; k < N; ++k) {
        int rk = 0;
        const uint32_t key = sort_key(lam[k]);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const uint32_t kj = sort_key(lam[j]);
            rk += (j < n && (kj < key || (kj == key && j < k))) ? 1 : 0;
        }
        rank[k] = rk;
    }
    // eigenvalues through the staging buffer
    __syncthreads();
    if (mine) {
#pragma unroll
        for (int k = 0; k < N; ++k)
            if (k < n) stage[lane * MS + rank[k]] = lam[k] * inv_scale;
    }
    __syncthreads();
    if (args.evals) {
        float* __restrict__ Eb = args.evals + b0 * n;
        const float rcp = 1.0f / (float)n;
        for (int idx = lane; idx < nb * n; idx += 64) {
            const int m = (int)(((float)idx + 0.5f) * rcp);
            Eb[idx] = stage[m * MS + (idx - m * n)];
        }
    }
    if (STAGE == kSpectral) {
        // F = V f(Lambda) V^T in registers, row by row: t[k] = V[i][k] f(lambda_k), then
        // F[i][j] = sum_k t[k] V[j][k] for j <= i, mirrored into the staging buffer
        float fl[N];
#pragma unroll
        for (int k = 0; k < N; ++k) {
            const float x = fmaxf(lam[k] * inv_scale, args.fn_floor);
            fl[k] = (k < n) ? ((args.fn == kFnInvSqrt) ? __builtin_amdgcn_rsqf(x) : __builtin_amdgcn_sqrtf(x)) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < N; ++i) {
            float t[N];
#pragma unroll
            for (int k = 0; k < N; ++k) t[k] = v[i][k] * fl[k];
#pragma unroll
            for (int j = 0; j <= i; ++j) {
                float acc = 0.f;
#pragma unroll
                for (int k = 0; k < N; ++k) acc = fmaf(t[k], v[j][k], acc);
                if (mine && i < n && j < n) {
                    stage[lane * MS + i * n + j] = acc;
                    stage[lane * MS + j * n + i] = acc;
                }
            }
        }
        __syncthreads();
        float* __restrict__ Fb = args.fn_out + b0 * nn;
        const float rcp = 1.0f / (float)nn;
        chunked_copy<16>(
            nb * nn, lane,
            [&](int idx) {
                const int m = (int)(((float)idx + 0.5f) * rcp);
                return stage[m * MS + (idx - m * nn)];
            },
            [&](int idx, float x) { Fb[idx] = x; });
    }
    if (WANT_V && STAGE == kFull) {
        __syncthreads();
        if (mine) {
#pragma unroll
            for (int c = 0; c < N; ++c) {
#pragma unroll
                for (int r = 0; r < N; ++r)
                    if (c < n && r < n) stage[lane * MS + r * n + rank[c]] = v[r][c];
            }
        }
        __syncthreads();
        float* __restrict__ Vb = args.evecs + b0 * nn;
        const float rcp = 1.0f / (float)nn;
        chunked_copy<16>(
            nb * nn, lane,
            [&](int idx) {
                const int m = (int)(((float)idx + 0.5f) * rcp);
                return stage[m * MS + (idx - m * nn)];
            },
            [&](int idx, float x) { Vb[idx] = x; });
    }
    if (mine) {
        if (args.info) args.info[b0 + lane] = info;
        if (args.rotations) args.rotations[b0 + lane] = rotations;
    }
}

template <int N>
static hipError_t launch_lane_n(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    const unsigned blocks = (unsigned)((args.batch + 63) / 64);
    if (stage == kSpectral) return enqueue(lane_kernel<N, true, kSpectral>, dim3(blocks), dim3(64), stream, args);
    if (want_v) return enqueue(lane_kernel<N, true, kFull>, dim3(blocks), dim3(64), stream, args);
    return enqueue(lane_kernel<N, false, kFull>, dim3(blocks), dim3(64), stream, args);
}

}  // namespace bed
#endif
