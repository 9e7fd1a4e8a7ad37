// Two wavefronts per matrix, for 32 < n <= 64 in batches that leave most of the chip idle
// (config 5: 256 matrices of 48 x 48 / 64 x 64 on 1024 SIMDs).
//
// Same method and same arithmetic as the one-wavefront kernel (arXiv 2207.04228 Sec. 3), with
// the work of a matrix split so that neither wavefront repeats the other's instructions:
//   * Sec. 3.1: wavefront A holds the rows of the working matrix and runs the Householder
//     reduction (Eqs. (2)-(7)); it leaves u and 2/|u|^2 of every step in LDS.  Wavefront B holds
//     the rows of P (Eq. (8)) and applies the reflectors as they appear: P <- P - (2 P u/|u|^2) u^T.
//     A never waits for B; B waits (bounded spin on a step counter in LDS) for A.
//   * Sec. 3.2: each wavefront owns 32 rows of V and runs the role-lane QR loop of the
//     one-wavefront kernel (both sweeps in one instruction stream, 35.5 instructions per step
//     instead of 40 for 64 rows in one wavefront) on its OWN copy of the tridiagonal: the
//     arithmetic on the two copies is identical, so the wavefronts take the same shifts and
//     deflation decisions and never synchronise inside the phase.
// A workgroup is four wavefronts = two matrices (workgroups of four wavefronts always get one
// wavefront on each SIMD of their compute unit).
#ifndef BED_PAIR_KERNEL_HPP
#define BED_PAIR_KERNEL_HPP
#include "bed_wave_kernel.hpp"

namespace bed {

namespace pairk {

// Spin limit of wavefront B's wait for wavefront A (both belong to one workgroup, so A is
// resident and always progresses; the limit only makes sure that a mistake cannot hang the GPU).
constexpr int kSpinLimit = 1 << 22;

__device__ __forceinline__ bool wait_for_step(volatile int* step, int need) {
    for (int spin = 0; spin < kSpinLimit; ++spin) {
        if (*step >= need) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            return true;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    return false;
}

}  // namespace pairk

// N: register-array size (40, 48, 56, 64), 32 < n <= N at run time; eigenvectors always.
template <int N>
__global__ __launch_bounds__(256) void pair_kernel(KernelArgs args) {
    using namespace pairk;
    constexpr int LD = 65;                  // column stride of V (odd, >= 64)
    constexpr int VA = (N + 8) * LD;
    constexpr int PA = N + 10;
    __shared__ float sV_all[2 * VA];        // load staging, then P, then V (column-major)
    __shared__ float2 sP_all[4 * PA];       // one copy of T per wavefront: sP[k] = (e[k-1], d[k])
    __shared__ __align__(16) float sU_all[2 * (N - 2) * 64];   // u of every step
    __shared__ __align__(16) float sQ_all[2 * 64];             // p of the current step
    __shared__ float sBeta_all[2 * N];      // 2/|u|^2 of every step
    __shared__ int sStep_all[2];            // steps published by wavefront A
    __shared__ int sFail_all[2];
    __shared__ int sInv_all[2 * 64];
    __shared__ float sScale_all[2];         // 2^ex of the pre-scaling, for wavefront B

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;
    const int pr = wv >> 1;                 // which of the workgroup's two matrices
    const bool isB = (wv & 1) != 0;
    const int n = args.n;
    const long long m = 2ll * blockIdx.x + pr;
    const bool mine = m < args.batch;
    float* const sV = sV_all + pr * VA;
    float* const sU = sU_all + pr * (N - 2) * 64;
    float* const sQ = sQ_all + pr * 64;
    float* const sBeta = sBeta_all + pr * N;
    volatile int* const sStep = sStep_all + pr;

    if (tid < 2) {
        sStep_all[tid] = 0;
        sFail_all[tid] = 0;
    }
    __syncthreads();
    PhaseClock clk;
    clk.start();

    float inv_scale = 1.f;
    if (!isB) {
        // ---- wavefront A: load, pre-scale, Householder reduction of the working matrix ----
        float a[N];
        const float* __restrict__ Ab = args.A + (size_t)(mine ? m : 0) * n * n;
        const float rcp_n = 1.0f / (float)n;
        chunked_copy<16>(
            mine ? n * n : 0, lane, [&](int idx) { return Ab[idx]; },
            [&](int idx, float x) {
                const int i = (int)(((float)idx + 0.5f) * rcp_n);
                sV[i * LD + (idx - i * n)] = x;
            });
        wave_sync();
        float amax = 0.f;
#pragma unroll
        for (int c = 0; c < N; ++c) {
            float x = 0.f;
            if (mine && lane < n && c < n) x = (c <= lane) ? sV[lane * LD + c] : sV[c * LD + lane];
            a[c] = x;
            amax = fmaxf(amax, fabsf(x));
        }
        wave_sync();
        float scale;
        pow2_scale(wave_max_nonneg<64>(amax), scale, inv_scale);
#pragma unroll
        for (int c = 0; c < N; ++c) a[c] *= scale;
        clk.lap(kPhLoad);
        // publish the scale for wavefront B's later use (eigenvalues are un-scaled by A alone) and
        // tell B that the staging area has been read
        float2* const sPa = sP_all + (2 * pr) * PA;
        float2* const sPb = sPa + PA;
#pragma unroll
        for (int J = 0; J < N; ++J) {
            const float dJ = read_lane(a[J], J);
            float eJ = 0.f;
            if (J < N - 1) {
                const float x0 = read_lane(a[J], J + 1);
                eJ = x0;
                if (J < N - 2) {
                    const float x = (lane > J) ? a[J] : 0.f;
                    const float alpha = wave_sum<64>(x * x);
                    const bool active = (J < n - 2) && (alpha > kTinyAlpha);
                    const float nrm = __builtin_amdgcn_sqrtf(alpha);
                    const float sigma = (x0 < 0.f) ? -nrm : nrm;
                    float ur = (lane == J + 1) ? (x0 + sigma) : ((lane > J + 1) ? x : 0.f);
                    ur = active ? ur : 0.f;
                    const float beta = active ? __builtin_amdgcn_rcpf(fmaf(fabsf(x0), nrm, alpha)) : 0.f;
                    eJ = active ? -sigma : x0;
                    sU[J * 64 + lane] = ur;
                    if (lane == 0) sBeta[J] = beta;
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                    if (lane == 0) *sStep = J + 1;
                    float u[N];
#pragma unroll
                    for (int c = J + 1; c < N; ++c) u[c] = sU[J * 64 + c];
                    float pp[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int c = J + 1; c < N; ++c) pp[c & 3] = fmaf(a[c], u[c], pp[c & 3]);
                    const float p = beta * ((pp[0] + pp[1]) + (pp[2] + pp[3]));
                    sQ[lane] = p;
                    const float K2 = beta * wave_sum<64>(ur * p);
                    const float sr = fmaf(-K2, ur, p);
#pragma unroll
                    for (int c = J + 1; c < N; ++c) a[c] = fmaf(-sr, u[c], a[c]);
                    wave_sync();
#pragma unroll
                    for (int c = J + 1; c < N; ++c) a[c] = fmaf(-ur, sQ[c], a[c]);
                    wave_sync();
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (lane == 0) {
                const float ev = (J < n - 1) ? eJ : 0.f;
                sPa[J].y = dJ;
                sPa[J + 1].x = ev;
                sPb[J].y = dJ;
                sPb[J + 1].x = ev;
            }
        }
        if (lane == 0) {
            sPa[0].x = 0.f;
            sPb[0].x = 0.f;
            sScale_all[pr] = inv_scale;
        }
    } else {
        // ---- wavefront B: accumulation of P, one reflector behind A at most by what A has published ----
        float v[N];
#pragma unroll
        for (int c = 0; c < N; ++c) v[c] = (c == lane) ? 1.f : 0.f;
        bool ok = true;
#pragma unroll
        for (int J = 0; J < N - 2; ++J) {
            if (J < n - 2) {
                ok = wait_for_step(sStep, J + 1) && ok;
                const float beta = sBeta[J];
                float u[N];
#pragma unroll
                for (int c = J + 1; c < N; ++c) u[c] = sU[J * 64 + c];
                float ww[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = J + 1; c < N; ++c) ww[c & 3] = fmaf(v[c], u[c], ww[c & 3]);
                const float w = beta * ((ww[0] + ww[1]) + (ww[2] + ww[3]));
#pragma unroll
                for (int c = J + 1; c < N; ++c) v[c] = fmaf(-w, u[c], v[c]);
#pragma unroll
                for (int c = J + 1; c < N; ++c) asm volatile("" : "+v"(v[c]));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (!ok && lane == 0) sFail_all[pr] = 1;
        // A read the staging area before it published its first step (n > 32 here, so there is one)
#pragma unroll
        for (int c = 0; c < N; ++c) sV[c * LD + lane] = v[c];
    }
    __syncthreads();
    clk.lap(kPhTridiag);

    // ---- shifted QR iterations: 32 rows of V per wavefront, own copy of T ----
    uint32_t rotations = 0;
    int info = 0;
    float d_lane[1];
    qr_iterations<N, true, true, LD>(sP_all + wv * PA, sV, lane, 32 * (wv & 1) + (lane & 31), n, rotations, info, d_lane,
                                     args, sScale_all[pr], clk);
    __syncthreads();       // both wavefronts of a pair leave after the same iteration; V is complete

    // ---- ascending order (wavefront A), then both wavefronts of the pair store ----
    int* const sInv = sInv_all + pr * 64;
    if (!isB) {
        const float dl = d_lane[0];
        const uint32_t mykey = sort_key(dl);
        int rank = 0;
        const float2* const sPa = sP_all + wv * PA;
        for (int j = 0; j < n; ++j) {
            const uint32_t kj = sort_key(sPa[j].y);
            rank += (kj < mykey || (kj == mykey && j < lane)) ? 1 : 0;
        }
        if (mine && lane < n) {
            args.evals[(size_t)m * n + rank] = dl * inv_scale;
            sInv[rank] = lane;
        }
        if (mine && lane == 0) {
            if (sFail_all[pr]) info = n;        // wavefront B gave up waiting: nothing of this matrix is valid
            if (args.info) args.info[m] = info;
            if (args.rotations) args.rotations[m] = rotations;
        }
    }
    __syncthreads();
    if (mine) {
        float* __restrict__ Vb = args.evecs + (size_t)m * n * n;
        const float rcp_n = 1.0f / (float)n;
        const int t2 = (isB ? 64 : 0) + lane;      // 0 .. 127 within the pair
        for (int base = t2; base < n * n; base += 128 * 8) {
            float t[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int idx = base + 128 * k;
                const int i = (int)(((float)idx + 0.5f) * rcp_n);
                t[k] = idx < n * n ? sV[sInv[idx - i * n] * LD + i] : 0.f;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int idx = base + 128 * k;
                if (idx < n * n) Vb[idx] = t[k];
            }
        }
    }
    clk.lap(kPhStore);
    if (mine && !isB) clk.write(args.phases, (int)m, lane);
}

template <int N>
static hipError_t launch_pair_n(const KernelArgs& args, hipStream_t stream) {
    const unsigned blocks = (unsigned)((args.batch + 1) / 2);
    return enqueue(pair_kernel<N>, dim3(blocks), dim3(256), stream, args);
}

}  // namespace bed
#endif
