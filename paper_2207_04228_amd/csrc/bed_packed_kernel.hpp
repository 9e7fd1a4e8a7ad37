// Several matrices per wavefront, for batches that fill the chip: four for n <= 16 (a matrix is
// owned by one DPP row of 16 lanes), two for 16 < n <= 32 (half a wavefront, two DPP rows).
//
// Same method as the one-wavefront-per-matrix kernel (arXiv 2207.04228 Sec. 3: Householder
// tridiagonalisation, Sec. 3.1; pairs of QR sweeps by Givens rotations with the two Wilkinson
// shifts of the trailing 2x2 block, Sec. 3.2.1, 3.2.2, App. A.1, A.3; per-matrix deflation,
// Sec. 3.2.3; O(1) update of T per rotation, Sec. 3.2.4; rotation of two columns of V per
// rotation, Sec. 3.2.5), but a matrix is owned by a GROUP of GW = 16 or 32 lanes instead of a
// whole wavefront:
//   * lane r of a group holds row r of the working matrix and of P in registers during the
//     tridiagonalisation; for GW = 16 broadcasts of u and p are DPP row broadcasts and reductions
//     DPP butterflies inside the row; for GW = 32 u and p go through LDS (128-bit reads of one
//     address per group) and reductions add a row exchange (v_permlane16_swap);
//   * in the QR phase the lower half of a group carries the scalar recurrence of the first sweep,
//     the upper half that of the second sweep two rotations behind, and every lane rotates its own
//     row of V for both sweeps with (c, s) broadcast inside the group;
//   * everything that is wave-uniform in the one-wavefront kernel (window, shifts, iteration
//     and sweep counts) is per-lane here and uniform only inside a group, and all control flow is
//     per group: the groups of a wavefront run different windows and stop at different times, the
//     wavefront runs until its slowest group is done.
// The instructions of the scalar recurrence, which every lane of the one-wavefront kernel
// repeats, are shared by four (two) matrices, which is what pays once every SIMD holds several
// wavefronts (config 4: 4096 matrices of 16 x 16; config 2 at batch 4096).
#ifndef BED_PACKED_KERNEL_HPP
#define BED_PACKED_KERNEL_HPP
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "bed_kernel.h"

namespace bed {

namespace packed {

// Same constants as the one-wavefront kernel (see there for the reasons).
constexpr float kEps = 4.7683716e-7f;       // 4 * 2^-23: relative deflation tolerance
constexpr uint32_t kExceptionalAfter = 5;   // iterations without deflation before both sweeps use mu1
constexpr uint32_t kStallIterations = 12;   // ... before the absolute threshold applies
constexpr float kAbsTol1 = 2.3841858e-7f;   // 2^-22 of the pre-scaled matrix
constexpr float kAbsTol2 = 9.5367432e-7f;   // 2^-20
constexpr float kTinyE = 1.0e-18f;
constexpr float kTinyG = 1.0e-18f;
constexpr float kTinyAlpha = 1.0e-35f;

// ---- data movement inside a group of GW lanes -----------------------------------

// Every lane of a DPP row receives the value of lane K of that row.  Every source lane exists, so
// the bound_ctrl form (which lets the compiler fold the move into the instruction that uses it)
// is the same operation.
template <int K>
__device__ __forceinline__ float row_bcast(float x) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x150 + K, 0xF, 0xF, true));
}

template <int CTRL>
__device__ __forceinline__ float row_perm(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kRowHalfMirror = 0x141, kRowMirror = 0x140;

// v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second:
// applied to two copies of x, the first result holds the even row's values in both rows of a pair
// of rows, the second result the odd row's.
__device__ __forceinline__ float even_row_to_pair(float x) {
    const unsigned u = __float_as_uint(x);
    return __uint_as_float(__builtin_amdgcn_permlane16_swap(u, u, false, false)[0]);
}
__device__ __forceinline__ float odd_row_to_pair(float x) {
    const unsigned u = __float_as_uint(x);
    return __uint_as_float(__builtin_amdgcn_permlane16_swap(u, u, false, false)[1]);
}

template <int GW>
struct Group;

// GW = 16: the group is one DPP row; lanes 0..7 are the first sweep's role lanes, 8..15 the second's.
template <>
struct Group<16> {
    // sum / max over the group, result in every lane of the group
    static __device__ __forceinline__ float sum(float x) {
        x += row_perm<kQuadXor1>(x);
        x += row_perm<kQuadXor2>(x);
        x += row_perm<kRowHalfMirror>(x);
        x += row_perm<kRowMirror>(x);
        return x;
    }
    static __device__ __forceinline__ float max_nonneg(float x) {
        x = fmaxf(x, row_perm<kQuadXor1>(x));
        x = fmaxf(x, row_perm<kQuadXor2>(x));
        x = fmaxf(x, row_perm<kRowHalfMirror>(x));
        x = fmaxf(x, row_perm<kRowMirror>(x));
        return x;
    }
    // value of lane K of the group, in every lane of the group
    template <int K>
    static __device__ __forceinline__ float bcast(float x) { return row_bcast<K>(x); }
    // lower half keeps `keep`; lane GW/2 + j receives the value lane j holds in `src`
    static __device__ __forceinline__ float upper_from_lower(float keep, float src) {
        return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(keep), __float_as_int(src),
                                                          0x118 /* row_shr:8 */, 0xF, 0xC, false));
    }
    // x is uniform over the lower half and over the upper half: both values to every lane
    static __device__ __forceinline__ void halves(float x, float& lower, float& upper) {
        lower = row_bcast<0>(x);
        upper = row_bcast<8>(x);
    }
};

// GW = 32: the group is a pair of DPP rows; the even row holds the first sweep's role lanes, the
// odd row the second's.
template <>
struct Group<32> {
    static __device__ __forceinline__ float sum(float x) {
        x = Group<16>::sum(x);
        return even_row_to_pair(x) + odd_row_to_pair(x);
    }
    static __device__ __forceinline__ float max_nonneg(float x) {
        x = Group<16>::max_nonneg(x);
        return fmaxf(even_row_to_pair(x), odd_row_to_pair(x));
    }
    template <int K>
    static __device__ __forceinline__ float bcast(float x) {
        const float y = row_bcast<(K & 15)>(x);       // lane K & 15 of each row, in that row
        return K < 16 ? even_row_to_pair(y) : odd_row_to_pair(y);
    }
    static __device__ __forceinline__ float upper_from_lower(float keep, float src) {
        return __uint_as_float(
            __builtin_amdgcn_permlane16_swap(__float_as_uint(keep), __float_as_uint(src), false, false)[0]);
    }
    static __device__ __forceinline__ void halves(float x, float& lower, float& upper) {
        const unsigned u = __float_as_uint(x);
        const auto both = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        lower = __uint_as_float(both[0]);
        upper = __uint_as_float(both[1]);
    }
};

__device__ __forceinline__ void wave_sync() { __builtin_amdgcn_wave_barrier(); }

// compile-time loop: f(integral_constant<int, B>), ..., f(integral_constant<int, E-1>)
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

__device__ __forceinline__ uint32_t sort_key(float x) {
    uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float guard_g(float g) {
    float mag;
    asm("v_max_f32 %0, |%1|, %2" : "=v"(mag) : "v"(g), "v"(kTinyG));
    return __uint_as_float((__float_as_uint(g) & 0x80000000u) | __float_as_uint(mag));
}

// Running state of one sweep (implicit shifted QR step as a chain of Givens rotations, App. A.1):
// rotation k consumes e[k], d[k+1] and emits the final e[k-1], d[k].
struct Chain {
    float g, s, c, p, dk;
};

__device__ __forceinline__ void chain_rotate(Chain& S, float ek, float dk1, float& e_out, float& d_out) {
    const float g = guard_g(S.g);
    const float f = S.s * ek;
    const float bb = S.c * ek;
    const float h = fmaf(f, f, g * g);
    const float rinv = __builtin_amdgcn_rsqf(h);
    const float gg = S.dk - S.p;
    S.c = g * rinv;
    S.s = f * rinv;
    e_out = h * rinv;
    const float r2 = fmaf(dk1 - gg, S.s, 2.f * S.c * bb);
    S.p = S.s * r2;
    S.g = fmaf(S.c, r2, -bb);
    d_out = gg + S.p;
    S.dk = dk1;
}

}  // namespace packed

// GW: lanes per matrix (16 or 32); N: register-array size (4, 8, 12, 16 for GW = 16; 20, 24, 28, 32
// for GW = 32), n <= N at run time.  One workgroup = one wavefront = up to 64 / GW consecutive
// matrices of the batch.  STAGE: kFull, or kSpectral (the fused V f(max(Lambda, floor)) V^T of
// Sec. 4.2-4.4 / App. B.1-B.3, eigenvectors never written).
template <int GW, int N, bool WANT_V, int STAGE>
__global__ __launch_bounds__(64) void packed_kernel(KernelArgs args) {
    using namespace packed;
    using G = Group<GW>;
    static_assert(N <= GW, "a matrix must fit its group of lanes");
    constexpr int PER_WAVE = 64 / GW;     // matrices per wavefront
    constexpr int HW = GW / 2;            // role lanes per sweep
    constexpr int LD = GW + 1;            // column stride of V in LDS (odd; every lane owns a row slot)
    constexpr int VA = (N + 8) * LD;      // V column-major, 8 padding columns (look-ahead reads, parked stores)
    constexpr int PA = N + 10;            // tridiagonal (e[k-1], d[k]) plus padding
    __shared__ float sV_all[PER_WAVE * VA];
    __shared__ float2 sP_all[PER_WAVE * PA];
    __shared__ float sE_all[PER_WAVE * GW];   // sorted eigenvalues, staged for the coalesced store
    __shared__ int sI_all[PER_WAVE * GW];     // output column -> column of V
    __shared__ __align__(16) float sU_all[PER_WAVE * GW];   // u of the current reflector (GW = 32)
    __shared__ __align__(16) float sQ_all[PER_WAVE * GW];   // p of the current reflector (GW = 32)

    const int lane = threadIdx.x;
    const int grp = lane / GW;            // which of the wavefront's matrices
    const int r = lane % GW;              // row of the matrix (and of V) this lane owns
    const int n = args.n;
    const int nn = n * n;
    const long long m0 = (long long)blockIdx.x * PER_WAVE;
    const int cnt = (int)min((long long)PER_WAVE, (long long)args.batch - m0);   // matrices in this wavefront
    const bool mine = grp < cnt;
    float* const sV = sV_all + grp * VA;
    float2* const sP = sP_all + grp * PA;

    // ---- load: the wavefront's matrices are one contiguous slab; coalesced into LDS (row-major) ----
    {
        const float* __restrict__ Ab = args.A + m0 * nn;
        const float rcp_nn = 1.0f / (float)nn, rcp_n = 1.0f / (float)n;
        chunked_copy<copy_chunk(PER_WAVE * N * N)>(
            cnt * nn, lane, [&](int idx) { return Ab[idx]; },
            [&](int idx, float x) {
                const int m = (int)(((float)idx + 0.5f) * rcp_nn);
                const int rem = idx - m * nn;
                const int i = (int)(((float)rem + 0.5f) * rcp_n);
                sV_all[m * VA + i * LD + (rem - i * n)] = x;
            });
    }
    wave_sync();
    float a[N], v[N];
    float amax = 0.f;
#pragma unroll
    for (int c = 0; c < N; ++c) {
        float x = 0.f;
        if (mine && r < n && c < n) x = (c <= r) ? sV[r * LD + c] : sV[c * LD + r];   // lower triangle, mirrored
        a[c] = x;
        v[c] = (c == r) ? 1.f : 0.f;
        amax = fmaxf(amax, fabsf(x));
    }
    wave_sync();
    amax = G::max_nonneg(amax);
    // exact power-of-two pre-scaling: max|a| -> [0.5, 1)
    int ex = 0;
    if (amax > 0.f && amax < __builtin_inff()) ex = __builtin_amdgcn_frexp_expf(amax);
    ex = min(max(ex, -125), 126);
    const float scale = ldexpf(1.0f, -ex);
    const float inv_scale = ldexpf(1.0f, ex);
#pragma unroll
    for (int c = 0; c < N; ++c) a[c] *= scale;

    // ---- Householder tridiagonalisation (Sec. 3.1), column J reduced at step J, branch-free ----
    // A step that has nothing to do (J >= n-2, or the column is already reduced) runs with u = 0
    // and beta = 0.  GW = 16: u[c] and p[c] are row broadcasts of lane c's value with a
    // compile-time c.  GW = 32: the group writes u and p to LDS and every lane reads them back
    // four at a time (one address per group).
    float* const sU = sU_all + grp * GW;
    float* const sQ = sQ_all + grp * GW;
    static_for<0, N>([&](auto j_) {
        constexpr int J = decltype(j_)::value;
        const float dJ = G::template bcast<J>(a[J]);         // A[J][J], final once columns 0..J-1 are reduced
        float eJ = 0.f;
        if constexpr (J < N - 1) {
            const float x0 = G::template bcast<J + 1>(a[J]); // A[J+1][J]
            eJ = x0;                                         // kept as is when no reflector is applied
            if constexpr (J < N - 2) {
                const float x = (r > J) ? a[J] : 0.f;        // A[r][J], r > J
                const float alpha = G::sum(x * x);           // |x|^2
                const bool active = (J < n - 2) && (alpha > kTinyAlpha);
                const float nrm = __builtin_amdgcn_sqrtf(alpha);
                const float sigma = (x0 < 0.f) ? -nrm : nrm;   // sign chosen to avoid cancellation
                float ur = (r == J + 1) ? (x0 + sigma) : ((r > J + 1) ? x : 0.f);
                ur = active ? ur : 0.f;
                const float beta = active ? __builtin_amdgcn_rcpf(fmaf(fabsf(x0), nrm, alpha)) : 0.f;   // 2/|u|^2
                eJ = active ? -sigma : x0;
                float u[N];
                if constexpr (GW == 32) {
                    sU[r] = ur;
                    wave_sync();
#pragma unroll
                    for (int c = J + 1; c < N; ++c) u[c] = sU[c];
                } else {
                    static_for<J + 1, N>([&](auto c_) { u[decltype(c_)::value] = row_bcast<decltype(c_)::value>(ur); });
                }
                // p = 2 A u / |u|^2 and w = 2 P u / |u|^2, four partial sums each
                float pp[4] = {0.f, 0.f, 0.f, 0.f}, ww[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = J + 1; c < N; ++c) {
                    pp[c & 3] = fmaf(a[c], u[c], pp[c & 3]);
                    if (WANT_V) ww[c & 3] = fmaf(v[c], u[c], ww[c & 3]);
                }
                const float p = beta * ((pp[0] + pp[1]) + (pp[2] + pp[3]));
                const float w = beta * ((ww[0] + ww[1]) + (ww[2] + ww[3]));
                if constexpr (GW == 32) sQ[r] = p;
                // A - q u^T - u q^T with q = p - K u, K = u^T p / |u|^2, regrouped as
                // A - (p - 2K u) u^T - u p^T; P <- P - w u^T
                const float K2 = beta * G::sum(ur * p);      // 2K
                const float sr = fmaf(-K2, ur, p);
#pragma unroll
                for (int c = J + 1; c < N; ++c) {
                    a[c] = fmaf(-sr, u[c], a[c]);
                    if (WANT_V) v[c] = fmaf(-w, u[c], v[c]);
                }
                if constexpr (GW == 32) {
                    wave_sync();
#pragma unroll
                    for (int c = J + 1; c < N; ++c) a[c] = fmaf(-ur, sQ[c], a[c]);
                    wave_sync();
                } else {
                    static_for<J + 1, N>([&](auto c_) {
                        constexpr int C = decltype(c_)::value;
                        a[C] = fmaf(-ur, row_bcast<C>(p), a[C]);
                    });
                }
                // Keep the steps apart.  The accumulation of P does not feed the reduction of A, and
                // the compiler would otherwise postpone all of it to the end of the reduction, with the
                // u of every step kept in registers until then: pin this step's P to this point.
                if (WANT_V) {
#pragma unroll
                    for (int c = J + 1; c < N; ++c) asm volatile("" : "+v"(v[c]));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (r == 0) {
            sP[J].y = dJ;                                    // sP[k] = (e[k-1], d[k])
            sP[J + 1].x = (J < n - 1) ? eJ : 0.f;
        }
    });
    if (r == 0) sP[0].x = 0.f;
    if (WANT_V) {
#pragma unroll
        for (int c = 0; c < N; ++c) sV[c * LD + r] = v[c];
    }
    wave_sync();

    // ---- shifted QR iterations (Sec. 3.2), control flow per group ----
    const bool roleB = r >= HW;
    const uint32_t cap = args.sweep_cap ? args.sweep_cap : 30u * (uint32_t)n;
    const int rshift = grp * GW;
    auto group_bits = [&](uint64_t ballot) -> uint32_t {
        return (uint32_t)(ballot >> rshift) & (GW == 32 ? 0xFFFFFFFFu : 0xFFFFu);
    };
    uint32_t sweeps = 0, rotations = 0, stall = 0, relaxed = 0;
    uint32_t nz = 0, nz_prev = 0xFFFFFFFFu;
    bool live = r < n - 1;                 // off-diagonal e[r] is watched by this lane
    float dl = 0.f;
    // absolute part of the deflation test: the rounding-level floor, or the paper's threshold
    // epsilon (Sec. 3.2.3, App. B) in units of the pre-scaled matrix when the caller asked for it
    const float paper_eps = args.abs_eps * scale;
    const float tol0 = fmaxf(kTinyE, paper_eps), tol1 = fmaxf(kAbsTol1, paper_eps), tol2 = fmaxf(kAbsTol2, paper_eps);
    while (true) {
        // deflation test (Sec. 3.2.3, per matrix, every off-diagonal): the lane looks at e[r], d[r], d[r+1]
        const bool widened = stall >= kStallIterations;
        const float abs_tol = stall >= 2 * kStallIterations ? tol2 : (widened ? tol1 : tol0);
        float el = 0.f, dnext = 0.f;
        if (r < N) {
            const float2 pk = sP[r];
            const float2 pk1 = sP[r + 1];
            dl = pk.y;
            el = pk1.x;
            dnext = pk1.y;
        }
        const float dsum = fabsf(dl) + fabsf(dnext);
        const bool negligible = fabsf(el) <= fmaxf(kEps * dsum, abs_tol);
        const bool by_fallback = widened && live && negligible && !(fabsf(el) <= fmaxf(kEps * dsum, tol0));
        relaxed += (uint32_t)__builtin_popcount(group_bits(__ballot(by_fallback)));
        live = live && !negligible;
        nz = group_bits(__ballot(live));
        stall = (nz == nz_prev) ? stall + 1 : 0;
        nz_prev = nz;
        if (nz == 0 || sweeps >= cap) break;
        // active window [lo, hi]: e[hi-1] is the last live entry, e[lo-1] the last dead one below it
        const int hi = 32 - __builtin_clz(nz);
        const uint32_t below = ~nz & ((1u << (hi - 1)) - 1u);
        const int lo = below ? 32 - __builtin_clz(below) : 0;

        // eigenvalues of the trailing block [[ta, tb], [tb, td]] (App. A.3), smaller-angle root first
        const float2 tA = sP[hi - 1];
        const float2 tB = sP[hi];
        const float ta = tA.y, tb = tB.x, td = tB.y;
        const float delta = 0.5f * (ta - td);
        const float rt = __builtin_amdgcn_sqrtf(fmaf(delta, delta, tb * tb));
        const float den = delta + ((delta >= 0.f) ? rt : -rt);
        const float tt = (tb * tb) * __builtin_amdgcn_rcpf(den);
        const float mu1 = td - tt;          // eigenvalue closer to the last diagonal entry
        const float mu2 = (stall >= kExceptionalAfter) ? mu1 : ta + tt;   // the other eigenvalue of the block

        // Inputs of rotation t: (e[t], d[t+1]) = sP[t+1] and column t+1 of V, fetched ahead into two
        // slots used in alternation.
        const float d_lo = sP[lo].y;
        float2 q0 = sP[lo + 1];
        float2 q1 = sP[lo + 2];
        float* xV = sV + lo * LD + r;       // this lane's row of V, at column lo
        float xA = WANT_V ? xV[0] : 0.f;    // sweep A's carried column
        float y0 = 0.f, y1 = 0.f;
        if (WANT_V) {
            y0 = xV[LD];
            y1 = xV[2 * LD];
        }
        Chain A;
        A.g = d_lo - mu1;
        A.s = 1.f;
        A.c = 1.f;
        A.p = 0.f;
        A.dk = d_lo;
        float pE, pD, pV = 0.f;             // A's outputs of the previous step
        // t = lo: A rotates row lo (computed by every lane)
        chain_rotate(A, q0.x, q0.y, pE, pD);
        if (WANT_V) {
            pV = fmaf(A.c, xA, A.s * y0);
            xA = fmaf(A.c, y0, -A.s * xA);
            y0 = xV[3 * LD];
        }
        q0 = sP[lo + 3];
        if (hi - lo == 1) {
            // The window is the 2x2 block the shifts were taken from: the step with its exact
            // eigenvalue mu1 diagonalises it (the rotation of App. A.3); the off-diagonal is set to
            // zero and no second sweep runs.
            if (r == 0) {
                sP[lo] = make_float2(pE, pD);
                sP[hi] = make_float2(0.f, A.dk - A.p);
            }
            if (WANT_V) {
                xV[0] = pV;
                xV[LD] = xA;
            }
            rotations += 1u;
            sweeps += 1;
        } else {
            // Two sweeps (shift mu1, then mu2) over the same window, software-pipelined: sweep B runs
            // two rotations behind sweep A and takes A's results from registers.  The recurrences run
            // in role lanes (lower half of the group: A, upper half: B); every lane owns a row of V and
            // applies both rotations to it with (c, s) broadcast inside the group.
            const float sD = pD;                       // d'[lo] as left by A
            float xB = pV;                             // column lo as left by A: B's carried column
            // t = lo + 1: A rotates row lo+1 (still computed by every lane)
            chain_rotate(A, q1.x, q1.y, pE, pD);
            if (WANT_V) {
                pV = fmaf(A.c, xA, A.s * y1);
                xA = fmaf(A.c, y1, -A.s * xA);
                y1 = xV[4 * LD];
            }
            q1 = sP[lo + 4];
            Chain S;                                   // this lane's recurrence: A or B
            S.g = roleB ? (sD - mu2) : A.g;
            S.s = roleB ? 1.f : A.s;
            S.c = roleB ? 1.f : A.c;
            S.p = roleB ? 0.f : A.p;
            S.dk = roleB ? sD : A.dk;
            float prevE = pE, prevD = pD;              // A's (e, d) of the previous step
            // T: one running pointer per lane; every lane stores at the pointer and loads three
            // positions above it.  A lanes: the pointer is at position t, the load fetches the inputs of
            // rotation t+2 and the store lands on a position A has consumed and B overwrites with the
            // final value two steps later.  B lanes: the pointer is at t-2, the store is the real one.
            float2* xP = sP + (roleB ? lo : (lo + 2));
            float oE, oD;
            auto step = [&](float2& q_, float& y_, const int k_) {
                const float e_in = G::upper_from_lower(q_.x, prevE);
                const float d_in = G::upper_from_lower(q_.y, prevD);
                chain_rotate(S, e_in, d_in, oE, oD);
                if (WANT_V) {
                    float cA, cB, sA, sB;
                    G::halves(S.c, cA, cB);
                    G::halves(S.s, sA, sB);
                    const float nV = fmaf(cA, xA, sA * y_);
                    xA = fmaf(cA, y_, -sA * xA);
                    const float vo = fmaf(cB, xB, sB * pV);
                    xB = fmaf(cB, pV, -sB * xB);
                    pV = nV;
                    xV[k_ * LD] = vo;
                    y_ = xV[(k_ + 5) * LD];
                }
                q_ = xP[k_ + 3];
                xP[k_] = make_float2(oE, oD);
                prevE = oE;
                prevD = oD;
            };
            int t = lo + 2;
            for (; t + 1 < hi; t += 2) {
                step(q0, y0, 0);
                step(q1, y1, 1);
                xV += 2 * LD;
                xP += 2;
            }
            if (t < hi) {
                step(q0, y0, 0);
                xV += LD;
                xP += 1;
            }
            // closing steps: B alone; the A lanes' T stores are parked in the padding
            xP = roleB ? xP : (sP + (N + 3));
            const float fE = S.g, fD = S.dk - S.p;       // A lanes: e[hi-1], d[hi] as left by A
            // t = hi: B rotates row hi-2 with A's outputs of row hi-1
            chain_rotate(S, G::upper_from_lower(prevE, prevE), G::upper_from_lower(prevD, prevD), oE, oD);
            xP[0] = make_float2(oE, oD);
            if (WANT_V) {
                float cA, cB, sA, sB;
                G::halves(S.c, cA, cB);
                G::halves(S.s, sA, sB);
                xV[0] = fmaf(cB, xB, sB * pV);
                xB = fmaf(cB, pV, -sB * xB);
            }
            // t = hi + 1: B rotates row hi-1 with A's closing values (column hi as left by A is xA)
            chain_rotate(S, G::upper_from_lower(fE, fE), G::upper_from_lower(fD, fD), oE, oD);
            xP[1] = make_float2(oE, oD);
            if (WANT_V) {
                float cA, cB, sA, sB;
                G::halves(S.c, cA, cB);
                G::halves(S.s, sA, sB);
                xV[LD] = fmaf(cB, xB, sB * xA);
                xB = fmaf(cB, xA, -sB * xB);
            }
            // t = hi + 2: B closes
            xP[2] = make_float2(S.g, S.dk - S.p);
            if (WANT_V) xV[2 * LD] = xB;
            rotations += 2u * (uint32_t)(hi - lo);
            sweeps += 2;
        }
        wave_sync();
    }

    // ---- info, (spectral function,) ascending order, coalesced store ----
    int info = (int)__builtin_popcount(nz);
    {
        const uint32_t bad = group_bits(__ballot(r < n && !(fabsf(dl) < __builtin_inff())));
        info = max(info, (int)__builtin_popcount(bad));
        info |= (int)(min(relaxed, 0x7FFFu) << 16);
    }
    if (STAGE == kSpectral) {
        // F = V f(Lambda) V^T straight from V and lambda in LDS: lane r forms w[k] = V[r][k] f(lambda_k)
        // once, then F[r][c] = sum_k w[k] V[c][k] for every c; F is symmetric, so the entry is stored
        // at F[c][r] and the lanes of a group write consecutive addresses.
        float w[N];
#pragma unroll
        for (int k = 0; k < N; ++k) {
            float lam = sP[k].y * inv_scale;
            lam = fmaxf(lam, args.fn_floor);
            const float fl = (args.fn == kFnInvSqrt) ? __builtin_amdgcn_rsqf(lam) : __builtin_amdgcn_sqrtf(lam);
            w[k] = (k < n) ? sV[k * LD + r] * fl : 0.f;
        }
        float* __restrict__ Fb = args.fn_out + (m0 + grp) * nn;
        for (int c = 0; c < n; ++c) {
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < N; ++k) acc[k & 3] = fmaf(w[k], sV[k * LD + c], acc[k & 3]);
            if (mine && r < n) Fb[c * n + r] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
        }
    }
    const uint32_t mykey = sort_key(dl);
    int rank = 0;
    for (int j = 0; j < n; ++j) {
        const uint32_t kj = sort_key(sP[j].y);
        rank += (kj < mykey || (kj == mykey && j < r)) ? 1 : 0;
    }
    float* const sE = sE_all + grp * GW;
    int* const sI = sI_all + grp * GW;
    if (r < n) {
        sE[rank] = dl * inv_scale;
        sI[rank] = r;                      // output column `rank` comes from column r of V
    }
    wave_sync();
    if (args.evals) {
        float* __restrict__ Eb = args.evals + m0 * n;
        const float rcp_n = 1.0f / (float)n;
        for (int idx = lane; idx < cnt * n; idx += 64) {
            const int m = (int)(((float)idx + 0.5f) * rcp_n);
            Eb[idx] = sE_all[m * GW + (idx - m * n)];
        }
    }
    if (WANT_V && STAGE == kFull) {
        float* __restrict__ Vb = args.evecs + m0 * nn;
        const float rcp_nn = 1.0f / (float)nn, rcp_n = 1.0f / (float)n;
        chunked_copy<copy_chunk(PER_WAVE * N * N)>(
            cnt * nn, lane,
            [&](int idx) {
                const int m = (int)(((float)idx + 0.5f) * rcp_nn);
                const int rem = idx - m * nn;
                const int i = (int)(((float)rem + 0.5f) * rcp_n);
                return sV_all[m * VA + sI_all[m * GW + (rem - i * n)] * LD + i];
            },
            [&](int idx, float x) { Vb[idx] = x; });
    }
    if (mine && r == 0) {
        if (args.info) args.info[m0 + grp] = info;
        if (args.rotations) args.rotations[m0 + grp] = rotations;
    }
}

template <int GW, int N>
static hipError_t launch_packed_n(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    constexpr int per_wave = 64 / GW;
    const unsigned blocks = (unsigned)((args.batch + per_wave - 1) / per_wave);
    if (stage == kSpectral)
        return enqueue(packed_kernel<GW, N, true, kSpectral>, dim3(blocks), dim3(64), stream, args);
    if (want_v) return enqueue(packed_kernel<GW, N, true, kFull>, dim3(blocks), dim3(64), stream, args);
    return enqueue(packed_kernel<GW, N, false, kFull>, dim3(blocks), dim3(64), stream, args);
}

}  // namespace bed
#endif
