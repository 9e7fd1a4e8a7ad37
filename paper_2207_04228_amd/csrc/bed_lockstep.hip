// The paper's fixed-budget procedure as written (Sec. 3.2.3, App. B), for an A/B against the
// per-matrix solver: after the tridiagonalisation (Sec. 3.1, the same kernel as everywhere
// else) a given number of outer iterations, each two shifted QR steps over the leading m x m
// window with the two eigenvalues of its trailing 2x2 block taken once per iteration
// (Sec. 3.2.2, App. A.3); after an iteration the window shrinks by one row when the last
// sub-diagonal entry is at most epsilon in magnitude (absolute test, that entry only): for the
// whole batch at once, when every matrix passes ("uniform", what a batched tensor forces), or
// per matrix.  No convergence test beyond that, no interior deflation, no pre-scaling.
//
// A batch-wide decision per iteration means one launch per iteration: the state (d, e in the
// workspace, V in the output buffer) lives in HBM between launches, and every matrix reports
// into one counter per iteration (flags[it] = matrices that did not pass), from which the next
// launches derive the window size.
//
// One wavefront per matrix, n <= 64.  A QR step T - mu I = QR, T' = RQ + mu I is computed with
// the O(1)-per-rotation recurrence of the explicit step (Sec. 3.2.4's constant cost per
// rotation): with a_k = d_k - mu, p_0 = a_0, q_0 = e_0,
//   r_k = hypot(p_k, e_k), c_k = p_k / r_k, s_k = e_k / r_k,
//   t_k = c_k q_k + s_k a_{k+1},   p_{k+1} = c_k a_{k+1} - s_k q_k,   q_{k+1} = c_k e_{k+1},
//   d'_k = c_k c_{k-1} r_k + s_k t_k + mu,   e'_{k-1} = s_{k-1} r_k,
//   d'_{m-1} = c_{m-2} p_{m-1} + mu,         e'_{m-2} = s_{m-2} p_{m-1},
// and columns k, k+1 of V become (c v_k + s v_{k+1}, -s v_k + c v_{k+1}).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "bed_kernel.h"

namespace bed {

namespace {

// Built-in scratch memory for callers that cannot bring a workspace of their own (code under
// HIP graph capture, serving loops and harnesses that must not allocate).  One copy per GPU,
// held until the process ends.  In host code the array's name is only a stand-in for the
// symbol: the device address is looked up once per device with hipGetSymbolAddress and every
// use goes through that pointer.
static __device__ __align__(256) unsigned char scratch[kLockstepScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

constexpr int LN = 64;               // largest n
constexpr int LLD = 65;              // column stride of V in LDS (odd)

__device__ __forceinline__ float lane_value(float x, int lane_uniform) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane_uniform));
}

// Window size at the start of iteration `it`: n minus the number of earlier iterations that
// every matrix passed, never below 1.
__device__ __forceinline__ int uniform_window(const int* flags, int it, int n, int lane) {
    int passed = 0;
    for (int base = 0; base < it; base += 64) {
        const int j = base + lane;
        passed += __builtin_popcountll(__ballot(j < it && flags[j] == 0));
    }
    return max(1, n - passed);
}

__global__ void lockstep_init(int* flags, int iterations, int* window, int batch, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < iterations) flags[i] = 0;
    if (i < batch) window[i] = n;
}

__global__ __launch_bounds__(64) void lockstep_iteration(LockstepArgs a, int it) {
    __shared__ float sV[LN * LLD];
    const int lane = threadIdx.x;
    const int b = blockIdx.x;
    const int n = a.n;
    const int m = a.uniform ? uniform_window(a.flags, it, n, lane) : a.window[b];
    if (m < 2) return;

    float d = (lane < n) ? a.d[(size_t)b * n + lane] : 0.f;     // lane k holds d[k], e[k]
    float e = (lane < n - 1) ? a.e[(size_t)b * n + lane] : 0.f;
    float* __restrict__ Vb = a.evecs ? a.evecs + (size_t)b * n * n : nullptr;
    const float rcp_n = 1.0f / (float)n;
    if (Vb) {
        for (int idx = lane; idx < n * n; idx += 64) {
            const int i = (int)(((float)idx + 0.5f) * rcp_n);
            const int j = idx - i * n;
            sV[j * LLD + i] = Vb[idx];                          // V[i][j] at sV[j * LLD + i]
        }
    }
    __builtin_amdgcn_wave_barrier();

    // both eigenvalues of the trailing block [[ta, tb], [tb, td]] (App. A.3); the first shift
    // is the one closer to td
    const float ta = lane_value(d, m - 2), tb = lane_value(e, m - 2), td = lane_value(d, m - 1);
    const float delta = 0.5f * (ta - td);
    const float rt = sqrtf(fmaf(delta, delta, tb * tb));
    const float den = delta + ((delta >= 0.f) ? rt : -rt);
    const float tt = (den != 0.f) ? (tb * tb) / den : 0.f;
    const float shifts[2] = {td - tt, ta + tt};

    for (int half = 0; half < 2; ++half) {
        const float mu = shifts[half];
        float p = lane_value(d, 0) - mu;
        float q = lane_value(e, 0);
        float c_prev = 1.f, s_prev = 0.f;
        float x = (Vb && lane < n) ? sV[lane] : 0.f;            // column k of this lane's row, carried
        for (int k = 0; k < m - 1; ++k) {
            const float ek = lane_value(e, k);
            // hypot with scaling: in a converged window both numbers can be at rounding level
            // (1e-20 and below), where p^2 + e^2 underflows and (c, s) would lose unit length
            const float mx = fmaxf(fabsf(p), fabsf(ek));
            float c = 1.f, s = 0.f, r = 0.f;
            if (mx > 0.f) {
                const float ps = p / mx, es = ek / mx;
                const float h = sqrtf(fmaf(ps, ps, es * es));
                c = ps / h;
                s = es / h;
                r = mx * h;
            }
            const float a1 = lane_value(d, k + 1) - mu;
            const float t = fmaf(c, q, s * a1);
            const float dk = fmaf(c * c_prev, r, s * t) + mu;
            const float ekm1 = s_prev * r;
            const float e_next = (k + 1 < m - 1) ? lane_value(e, k + 1) : 0.f;
            p = fmaf(c, a1, -s * q);
            q = c * e_next;
            d = (lane == k) ? dk : d;
            e = (lane == k - 1) ? ekm1 : e;
            if (Vb && lane < n) {
                const float y = sV[(k + 1) * LLD + lane];
                sV[k * LLD + lane] = fmaf(c, x, s * y);
                x = fmaf(c, y, -s * x);
            }
            c_prev = c;
            s_prev = s;
        }
        d = (lane == m - 1) ? fmaf(c_prev, p, mu) : d;
        e = (lane == m - 2) ? s_prev * p : e;
        if (Vb && lane < n) sV[(m - 1) * LLD + lane] = x;
        __builtin_amdgcn_wave_barrier();
    }

    const bool passes = fabsf(lane_value(e, m - 2)) <= a.epsilon;
    if (lane == 0) {
        if (a.uniform) {
            if (!passes) atomicAdd(&a.flags[it], 1);
        } else if (passes) {
            a.window[b] = m - 1;
        }
    }
    if (lane < n) a.d[(size_t)b * n + lane] = d;
    if (lane < n - 1) a.e[(size_t)b * n + lane] = e;
    if (Vb) {
        for (int idx = lane; idx < n * n; idx += 64) {
            const int i = (int)(((float)idx + 0.5f) * rcp_n);
            const int j = idx - i * n;
            Vb[idx] = sV[j * LLD + i];
        }
    }
}

__device__ __forceinline__ uint32_t order_key(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// diag(T) in ascending order, the columns of V permuted along, what is left of the
// sub-diagonal, and the number of rows dropped.
__global__ __launch_bounds__(64) void lockstep_finish(LockstepArgs a) {
    __shared__ float sV[LN * LLD];
    __shared__ float sd[LN];
    __shared__ int sinv[LN];
    const int lane = threadIdx.x;
    const int b = blockIdx.x;
    const int n = a.n;
    const int m = a.uniform ? uniform_window(a.flags, a.iterations, n, lane) : a.window[b];
    const float d = (lane < n) ? a.d[(size_t)b * n + lane] : 0.f;
    if (lane < n) sd[lane] = d;
    float* __restrict__ Vb = a.evecs ? a.evecs + (size_t)b * n * n : nullptr;
    const float rcp_n = 1.0f / (float)n;
    if (Vb) {
        for (int idx = lane; idx < n * n; idx += 64) {
            const int i = (int)(((float)idx + 0.5f) * rcp_n);
            const int j = idx - i * n;
            sV[j * LLD + i] = Vb[idx];
        }
    }
    __builtin_amdgcn_wave_barrier();
    const uint32_t key = order_key(d);
    int rank = 0;
    for (int j = 0; j < n; ++j) {
        const uint32_t kj = order_key(sd[j]);
        rank += (kj < key || (kj == key && j < lane)) ? 1 : 0;
    }
    if (lane < n) {
        a.evals[(size_t)b * n + rank] = d;
        sinv[rank] = lane;
        if (a.offdiag) a.offdiag[(size_t)b * n + lane] = (lane < n - 1) ? fabsf(a.e[(size_t)b * n + lane]) : 0.f;
    }
    if (lane == 0 && a.reductions) a.reductions[b] = n - m;
    __builtin_amdgcn_wave_barrier();
    if (Vb) {
        for (int idx = lane; idx < n * n; idx += 64) {
            const int i = (int)(((float)idx + 0.5f) * rcp_n);
            const int j = idx - i * n;
            Vb[idx] = sV[sinv[j] * LLD + i];
        }
    }
}

}  // namespace

hipError_t lockstep_scratch(void** ptr) {
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_lockstep(const LockstepArgs& a, hipStream_t stream) {
    // Sec. 3.1: d, e into the workspace, P into the eigenvector buffer
    KernelArgs t{};
    t.A = a.A;
    t.d_out = a.d;
    t.e_out = a.e;
    t.evecs = a.evecs;
    t.batch = a.batch;
    t.n = a.n;
    hipError_t err = launch(t, kTridiagOnly, a.evecs != nullptr, stream);
    if (err != hipSuccess) return err;
    const int items = a.batch > a.iterations ? a.batch : a.iterations;
    err = enqueue(lockstep_init, dim3((items + 255) / 256), dim3(256), stream, a.flags, a.iterations, a.window,
                  a.batch, a.n);
    for (int it = 0; it < a.iterations && err == hipSuccess; ++it)
        err = enqueue(lockstep_iteration, dim3(a.batch), dim3(64), stream, a, it);
    if (err != hipSuccess) return err;
    return enqueue(lockstep_finish, dim3(a.batch), dim3(64), stream, a);
}

}  // namespace bed
