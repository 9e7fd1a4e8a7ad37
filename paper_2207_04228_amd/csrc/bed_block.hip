// 64 < n <= 128: one workgroup of four wavefronts per matrix.
//
// The matrix no longer fits one row per lane of a single wavefront, and its rows no longer
// fit in registers next to the rows of P, so the working matrix and P live in LDS (column
// major, odd stride; 136 KB of the 160 KB of a compute unit) and the loops run over the
// run-time n.
//   Sec. 3.1  tridiagonalisation: threads 0..127 own the rows of A, threads 128..255 the rows
//             of P; norms and u^T p are reduced per wavefront (DPP) and combined through LDS.
//   Sec. 3.2  QR iterations: every wavefront owns 32 rows of V and runs the same role-lane
//             loop as the single-wavefront kernel (qr_iterations, HALF) on its own copy of
//             the tridiagonal; the arithmetic on the copies is identical, so the four
//             wavefronts take the same shifts and deflation decisions without synchronising.
// followed by the ascending sort and a coalesced store by all 256 threads.
#include "bed_wave_kernel.hpp"

namespace bed {

namespace {

constexpr int BN = 128;              // rows covered
constexpr int BLD = 129;             // column stride in LDS (odd)
constexpr int BPA = BN + 10;         // float2 entries of one tridiagonal copy (with padding)
constexpr int BT = 256;              // threads per matrix

template <bool WANT_V, int STAGE>
__global__ __launch_bounds__(BT) void block_kernel(KernelArgs args) {
    __shared__ float sA[BN * BLD];               // A[r][c] at sA[c * BLD + r]; later V f(Lambda) (kSpectral)
    __shared__ float sV[(BN + 8) * BLD];         // P, then V: V[r][c] at sV[c * BLD + r]
    __shared__ float2 sP_all[4 * BPA];           // one copy of T per wavefront: sP[k] = (e[k-1], d[k])
    __shared__ float sd[BN], se[BN];             // T as produced by the tridiagonalisation
    __shared__ __align__(16) float svec[BN];     // u of the current step
    __shared__ __align__(16) float sq[BN];       // q of the current step
    __shared__ float sred[8];
    __shared__ int sinv[BN];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;
    const int b = blockIdx.x;
    const int n = args.n;
    float inv_scale = 1.f;

    if (STAGE != kQrOnly) {
        const float* __restrict__ Ab = args.A + (size_t)b * n * n;
        const float rcp_n = 1.0f / (float)n;
        // ---- power-of-two pre-scaling from max |a_ij| over the lower triangle ----
        float amax = 0.f;
        for (int idx = tid; idx < n * n; idx += BT) {
            const int i = (int)(((float)idx + 0.5f) * rcp_n);
            const int j = idx - i * n;
            if (j <= i) amax = fmaxf(amax, fabsf(Ab[idx]));
        }
        amax = wave_max_nonneg<64>(amax);
        if (lane == 0) sred[wv] = amax;
        __syncthreads();
        float scale;
        pow2_scale(fmaxf(fmaxf(sred[0], sred[1]), fmaxf(sred[2], sred[3])), scale, inv_scale);
        // ---- load: lower triangle mirrored, scaled; P = I.  Rows and columns n .. 127 are
        // zero, so the loops below can run over whole groups of eight columns. ----
        for (int idx = tid; idx < BN * BLD; idx += BT) {
            sA[idx] = 0.f;
            if (WANT_V) sV[idx] = 0.f;
        }
        __syncthreads();
        for (int idx = tid; idx < n * n; idx += BT) {
            const int i = (int)(((float)idx + 0.5f) * rcp_n);
            const int j = idx - i * n;
            if (j <= i) {
                const float a = Ab[idx] * scale;
                sA[j * BLD + i] = a;
                sA[i * BLD + j] = a;
            }
            if (WANT_V && i == j) sV[j * BLD + i] = 1.f;
        }
        __syncthreads();

        // ---- Householder tridiagonalisation, column J reduced at step J (Sec. 3.1) ----
        // The column loops run in groups of eight from the group that holds column J+1 to the
        // group that holds column n-1: eight independent LDS loads are in flight per group and
        // u, q come as 128-bit broadcast reads.  Columns <= J inside the first group are dead
        // for A (their entries of T are already recorded) and have u = 0, so P is untouched.
        // (Holding the rows in 128 VGPRs with unrolled column loops was measured too: the
        // step body then no longer fits the instruction cache and the phase gets slower.)
        const bool isA = tid < BN;
        const int row = tid & (BN - 1);
        float* const X = (isA ? sA : sV) + row;    // this thread's row: X[c * BLD]
        const bool works = isA || WANT_V;
        const int cend = (n + 7) & ~7;
        for (int J = 0; J < n - 2; ++J) {
            const int c0 = (J + 1) & ~7;
            float xc = 0.f;
            if (isA) {
                xc = (row > J) ? sA[J * BLD + row] : 0.f;
                const float part = wave_sum<64>(xc * xc);
                if (lane == 0) sred[wv] = part;
            }
            __syncthreads();
            const float alpha = sred[0] + sred[1];
            const float x0 = sA[J * BLD + J + 1];
            const bool active = alpha > kTinyAlpha;
            const float nrm = __builtin_amdgcn_sqrtf(alpha);
            const float sigma = (x0 < 0.f) ? -nrm : nrm;       // sign chosen to avoid cancellation
            const float beta = active ? __builtin_amdgcn_rcpf(fmaf(fabsf(x0), nrm, alpha)) : 0.f;   // 2/|u|^2
            float ur = 0.f;
            if (isA) {
                ur = (row == J + 1) ? (x0 + sigma) : ((row > J + 1) ? xc : 0.f);
                ur = active ? ur : 0.f;
                svec[row] = ur;
            }
            if (tid == 0) {
                sd[J] = sA[J * BLD + J];
                se[J] = active ? -sigma : x0;
            }
            __syncthreads();
            // p = 2 A u / |u|^2 (A rows), w = 2 P u / |u|^2 (P rows)
            float pw = 0.f;
            if (works) {
                float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
                for (int c = c0; c < cend; c += 8) {
                    float xv[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) xv[k] = X[(c + k) * BLD];
                    const float4 u0 = *reinterpret_cast<const float4*>(svec + c);
                    const float4 u1 = *reinterpret_cast<const float4*>(svec + c + 4);
                    acc[0] = fmaf(xv[0], u0.x, acc[0]);
                    acc[1] = fmaf(xv[1], u0.y, acc[1]);
                    acc[2] = fmaf(xv[2], u0.z, acc[2]);
                    acc[3] = fmaf(xv[3], u0.w, acc[3]);
                    acc[0] = fmaf(xv[4], u1.x, acc[0]);
                    acc[1] = fmaf(xv[5], u1.y, acc[1]);
                    acc[2] = fmaf(xv[6], u1.z, acc[2]);
                    acc[3] = fmaf(xv[7], u1.w, acc[3]);
                }
                pw = beta * ((acc[0] + acc[1]) + (acc[2] + acc[3]));
            }
            if (isA) {
                const float part = wave_sum<64>(ur * pw);
                if (lane == 0) sred[4 + wv] = part;
            } else if (WANT_V) {
                // P <- P - w u^T
#pragma unroll 2
                for (int c = c0; c < cend; c += 8) {
                    float xv[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) xv[k] = X[(c + k) * BLD];
                    const float4 u0 = *reinterpret_cast<const float4*>(svec + c);
                    const float4 u1 = *reinterpret_cast<const float4*>(svec + c + 4);
                    X[(c + 0) * BLD] = fmaf(-pw, u0.x, xv[0]);
                    X[(c + 1) * BLD] = fmaf(-pw, u0.y, xv[1]);
                    X[(c + 2) * BLD] = fmaf(-pw, u0.z, xv[2]);
                    X[(c + 3) * BLD] = fmaf(-pw, u0.w, xv[3]);
                    X[(c + 4) * BLD] = fmaf(-pw, u1.x, xv[4]);
                    X[(c + 5) * BLD] = fmaf(-pw, u1.y, xv[5]);
                    X[(c + 6) * BLD] = fmaf(-pw, u1.z, xv[6]);
                    X[(c + 7) * BLD] = fmaf(-pw, u1.w, xv[7]);
                }
            }
            __syncthreads();
            float q = 0.f;
            if (isA) {
                const float K = 0.5f * beta * (sred[4] + sred[5]);
                q = fmaf(-K, ur, pw);                          // q = p - K u (symmetric rank-2 form)
                sq[row] = q;
            }
            __syncthreads();
            if (isA) {
                // A <- A - q u^T - u q^T
#pragma unroll 2
                for (int c = c0; c < cend; c += 8) {
                    float xv[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) xv[k] = X[(c + k) * BLD];
                    const float4 u0 = *reinterpret_cast<const float4*>(svec + c);
                    const float4 u1 = *reinterpret_cast<const float4*>(svec + c + 4);
                    const float4 q0 = *reinterpret_cast<const float4*>(sq + c);
                    const float4 q1 = *reinterpret_cast<const float4*>(sq + c + 4);
                    X[(c + 0) * BLD] = fmaf(-ur, q0.x, fmaf(-q, u0.x, xv[0]));
                    X[(c + 1) * BLD] = fmaf(-ur, q0.y, fmaf(-q, u0.y, xv[1]));
                    X[(c + 2) * BLD] = fmaf(-ur, q0.z, fmaf(-q, u0.z, xv[2]));
                    X[(c + 3) * BLD] = fmaf(-ur, q0.w, fmaf(-q, u0.w, xv[3]));
                    X[(c + 4) * BLD] = fmaf(-ur, q1.x, fmaf(-q, u1.x, xv[4]));
                    X[(c + 5) * BLD] = fmaf(-ur, q1.y, fmaf(-q, u1.y, xv[5]));
                    X[(c + 6) * BLD] = fmaf(-ur, q1.z, fmaf(-q, u1.z, xv[6]));
                    X[(c + 7) * BLD] = fmaf(-ur, q1.w, fmaf(-q, u1.w, xv[7]));
                }
            }
            // the next step's first barrier orders these updates before other threads read them
        }
        __syncthreads();
        if (tid == 0) {
            if (n >= 2) {
                sd[n - 2] = sA[(n - 2) * BLD + n - 2];
                se[n - 2] = sA[(n - 2) * BLD + n - 1];
            }
            sd[n - 1] = sA[(n - 1) * BLD + n - 1];
            se[n - 1] = 0.f;
        }
        __syncthreads();
    } else {
        // ---- stage hook: tridiagonal given ----
        float dv = 0.f, ev = 0.f;
        if (tid < n) dv = args.d_in[(size_t)b * n + tid];
        if (tid < n - 1) ev = args.e_in[(size_t)b * n + tid];
        const float m = wave_max_nonneg<64>(fmaxf(fabsf(dv), fabsf(ev)));
        if (lane == 0) sred[wv] = m;
        __syncthreads();
        float scale;
        pow2_scale(fmaxf(fmaxf(sred[0], sred[1]), fmaxf(sred[2], sred[3])), scale, inv_scale);
        if (tid < BN) {
            sd[tid] = dv * scale;
            se[tid] = ev * scale;
        }
        if (WANT_V) {
            for (int idx = tid; idx < n * n; idx += BT) {
                const int i = idx / n, j = idx - i * n;
                sV[j * BLD + i] = (i == j) ? 1.f : 0.f;
            }
        }
        __syncthreads();
    }

    if (STAGE == kTridiagOnly) {
        if (tid < n) {
            args.d_out[(size_t)b * n + tid] = sd[tid] * inv_scale;
            args.e_out[(size_t)b * n + tid] = (tid < n - 1) ? se[tid] * inv_scale : 0.f;
        }
        if (WANT_V) {
            float* __restrict__ Vb = args.evecs + (size_t)b * n * n;
            const float rcp_n = 1.0f / (float)n;
            for (int idx = tid; idx < n * n; idx += BT) {
                const int i = (int)(((float)idx + 0.5f) * rcp_n);
                const int j = idx - i * n;
                Vb[idx] = sV[j * BLD + i];
            }
        }
        return;
    }

    // ---- one copy of T per wavefront ----
    for (int k = tid; k < BPA; k += BT) {
        const float2 v = make_float2((k >= 1 && k < n) ? se[k - 1] : 0.f, (k < n) ? sd[k] : 0.f);
#pragma unroll
        for (int w = 0; w < 4; ++w) sP_all[w * BPA + k] = v;
    }
    __syncthreads();

    // ---- shifted QR iterations: 32 rows of V per wavefront ----
    uint32_t rotations = 0;
    int info = 0;
    float d_lane[2];
    float2* const sP = sP_all + wv * BPA;
    PhaseClock clk;
    qr_iterations<BN, true, WANT_V, BLD>(sP, sV, lane, 32 * wv + (lane & 31), n, rotations, info, d_lane, args, inv_scale, clk);
    __syncthreads();       // all four wavefronts leave after the same iteration; V is complete

    if (STAGE == kSpectral) {
        // F = V f(max(Lambda, floor)) V^T: W = V diag(f) into the area of A, then F = W V^T
        if (tid < BN) {
            float lam = fmaxf(sP_all[tid].y * inv_scale, args.fn_floor);
            svec[tid] = (args.fn == kFnInvSqrt) ? __builtin_amdgcn_rsqf(lam) : __builtin_amdgcn_sqrtf(lam);
        }
        __syncthreads();
        const int row = tid & (BN - 1);
        for (int k = tid >> 7; k < n; k += 2) sA[k * BLD + row] = sV[k * BLD + row] * svec[k];
        __syncthreads();
        float* __restrict__ Fb = args.fn_out + (size_t)b * n * n;
        for (int c = tid >> 7; c < n; c += 2) {
            float acc0 = 0.f, acc1 = 0.f;
            int k = 0;
            for (; k + 1 < n; k += 2) {
                acc0 = fmaf(sA[k * BLD + row], sV[k * BLD + c], acc0);
                acc1 = fmaf(sA[(k + 1) * BLD + row], sV[(k + 1) * BLD + c], acc1);
            }
            if (k < n) acc0 = fmaf(sA[k * BLD + row], sV[k * BLD + c], acc0);
            if (row < n) Fb[c * n + row] = acc0 + acc1;     // F is symmetric: stored as F[c][row], coalesced
        }
    }

    // ---- ascending order: rank of d[k] among d[0..n) ----
    if (tid < n) {
        const float dk = sP_all[tid].y;
        const uint32_t key = sort_key(dk);
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const uint32_t kj = sort_key(sP_all[j].y);
            rank += (kj < key || (kj == key && j < tid)) ? 1 : 0;
        }
        if (args.evals) args.evals[(size_t)b * n + rank] = dk * inv_scale;
        sinv[rank] = tid;                                   // output column `rank` comes from column `tid`
    }
    if (STAGE != kSpectral && WANT_V) {
        __syncthreads();
        float* __restrict__ Vb = args.evecs + (size_t)b * n * n;
        const float rcp_n = 1.0f / (float)n;
        for (int idx = tid; idx < n * n; idx += BT) {
            const int i = (int)(((float)idx + 0.5f) * rcp_n);
            const int j = idx - i * n;
            Vb[idx] = sV[sinv[j] * BLD + i];
        }
    }
    if (tid == 0) {
        if (args.info) args.info[b] = info;
        if (args.rotations) args.rotations[b] = rotations;
    }
}

template <bool WANT_V, int STAGE>
hipError_t launch_block_one(const KernelArgs& args, hipStream_t stream) {
    return enqueue(block_kernel<WANT_V, STAGE>, dim3(args.batch), dim3(BT), stream, args);
}

}  // namespace

hipError_t launch_block(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (stage == kTridiagOnly)
        return want_v ? launch_block_one<true, kTridiagOnly>(args, stream) : launch_block_one<false, kTridiagOnly>(args, stream);
    if (stage == kQrOnly)
        return want_v ? launch_block_one<true, kQrOnly>(args, stream) : launch_block_one<false, kQrOnly>(args, stream);
    if (stage == kSpectral) return launch_block_one<true, kSpectral>(args, stream);
    return want_v ? launch_block_one<true, kFull>(args, stream) : launch_block_one<false, kFull>(args, stream);
}

}  // namespace bed
