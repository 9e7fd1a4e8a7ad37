// Four matrices per wavefront for 16 < n <= 32, for batches that fill the chip several times over.
//
// Same method as the other kernels (arXiv 2207.04228 Sec. 3) and the same organisation as
// packed_kernel<16, N>: a matrix is owned by one DPP row of 16 lanes, the scalar recurrences of the
// two sweeps run in the two halves of the row, control flow is per group.  The difference is
// that a lane owns TWO rows of the matrix, of P and of V (rows r and r + 16), so the instructions
// of the recurrence (19 of the 35 of a step in the one-wavefront kernel) are shared by four
// matrices of up to 32 rows instead of two, while the work on V per instruction stays what it
// is.  Broadcasts of u and p in the tridiagonalisation are DPP row broadcasts of one of the two
// values a lane holds; reductions add the lane's two contributions first.
#ifndef BED_PACKED_ROWS_KERNEL_HPP
#define BED_PACKED_ROWS_KERNEL_HPP
#include "bed_packed_kernel.hpp"

namespace bed {

// N: register-array size (20, 24, 28, 32), 16 < n <= N at run time (smaller n work, wastefully).
// STAGE: kFull (with or without eigenvectors), or kSpectral (the fused V f(max(Lambda, floor)) V^T of
// Sec. 4.2-4.4 / App. B.1-B.3, eigenvectors never written).
template <int N, bool WANT_V, int STAGE>
__global__ __launch_bounds__(64) void packed_rows_kernel(KernelArgs args) {
    static_assert(STAGE == kFull || (STAGE == kSpectral && WANT_V), "whole path or fused spectral function");
    using namespace packed;
    using G = Group<16>;
    static_assert(N > 16 && N <= 32, "two rows per lane of a group of 16");
    constexpr int GW = 16;                // lanes per matrix
    constexpr int R = 2;                  // rows per lane
    constexpr int PER_WAVE = 4;
    constexpr int HW = GW / 2;            // role lanes per sweep
    constexpr int LD = R * GW + 1;        // column stride of V in LDS (odd; every row has a slot)
    // V column-major.  The loop reads up to column N + 1 ahead of the window (lo <= N - 2: column
    // lo + 3; inside the loop: column hi + 2 with hi <= N - 1), so two padding columns are enough.
    // The LDS footprint also sets how many wavefronts share a compute unit: with two columns eight
    // wavefronts of N = 32 fit (two per SIMD, 1.35x faster than six at 16384 matrices); N = 24 with
    // two columns would fit ten, three on two of the four SIMDs, which measured 13 % slower than
    // eight, hence the wider padding there.
    constexpr int VA = (N + (N == 24 ? 8 : 2)) * LD;
    constexpr int PA = N + 10;
    constexpr int SW = R * GW;            // slots per matrix in the small staging arrays
    __shared__ float sV_all[PER_WAVE * VA];
    __shared__ float2 sP_all[PER_WAVE * PA];
    __shared__ float sE_all[PER_WAVE * SW];   // sorted eigenvalues, staged for the coalesced store
    __shared__ int sI_all[PER_WAVE * SW];     // output column -> column of V

    const int lane = threadIdx.x;
    const int grp = lane / GW;
    const int r = lane % GW;              // this lane owns rows r and r + GW
    const int n = args.n;
    const int nn = n * n;
    const long long m0 = (long long)blockIdx.x * PER_WAVE;
    const int cnt = (int)min((long long)PER_WAVE, (long long)args.batch - m0);
    const bool mine = grp < cnt;
    float* const sV = sV_all + grp * VA;
    float2* const sP = sP_all + grp * PA;
    int row[R];
#pragma unroll
    for (int h = 0; h < R; ++h) row[h] = r + h * GW;

    // ---- load: the wavefront's matrices are one contiguous slab; coalesced into LDS (row-major) ----
    {
        const float* __restrict__ Ab = args.A + m0 * nn;
        const float rcp_nn = 1.0f / (float)nn, rcp_n = 1.0f / (float)n;
        chunked_copy<16>(
            cnt * nn, lane, [&](int idx) { return Ab[idx]; },
            [&](int idx, float x) {
                const int m = (int)(((float)idx + 0.5f) * rcp_nn);
                const int rem = idx - m * nn;
                const int i = (int)(((float)rem + 0.5f) * rcp_n);
                sV_all[m * VA + i * LD + (rem - i * n)] = x;
            });
    }
    wave_sync();
    float a[R][N], v[R][N];
    float amax = 0.f;
    static_for<0, R>([&](auto h_) {
        constexpr int h = decltype(h_)::value;
        static_for<0, N>([&](auto c_) {
            constexpr int c = decltype(c_)::value;
            float x = 0.f;
            if (mine && row[h] < n && c < n) x = (c <= row[h]) ? sV[row[h] * LD + c] : sV[c * LD + row[h]];
            a[h][c] = x;
            v[h][c] = (c == row[h]) ? 1.f : 0.f;
            amax = fmaxf(amax, fabsf(x));
        });
    });
    wave_sync();
    amax = G::max_nonneg(amax);
    int ex = 0;
    if (amax > 0.f && amax < __builtin_inff()) ex = __builtin_amdgcn_frexp_expf(amax);
    ex = min(max(ex, -125), 126);
    const float scale = ldexpf(1.0f, -ex);
    const float inv_scale = ldexpf(1.0f, ex);
    static_for<0, R>([&](auto h_) {
        static_for<0, N>([&](auto c_) { a[decltype(h_)::value][decltype(c_)::value] *= scale; });
    });

    // ---- Householder tridiagonalisation (Sec. 3.1), column J reduced at step J, branch-free ----
    // Entry c of a vector that is distributed over the rows lives in lane c % 16 as that lane's
    // value number c / 16: its broadcast is a DPP row broadcast with both indices known at compile time.
    static_for<0, N>([&](auto j_) {
        constexpr int J = decltype(j_)::value;
        const float dJ = G::template bcast<J % GW>(a[J / GW][J]);
        float eJ = 0.f;
        if constexpr (J < N - 1) {
            const float x0 = G::template bcast<(J + 1) % GW>(a[(J + 1) / GW][J]);   // A[J+1][J]
            eJ = x0;
            if constexpr (J < N - 2) {
                float x[R], ur[R];
                float sq = 0.f;
                static_for<0, R>([&](auto h_) {
                    constexpr int h = decltype(h_)::value;
                    x[h] = (row[h] > J) ? a[h][J] : 0.f;
                    sq = fmaf(x[h], x[h], sq);
                });
                const float alpha = G::sum(sq);
                const bool active = (J < n - 2) && (alpha > kTinyAlpha);
                const float nrm = __builtin_amdgcn_sqrtf(alpha);
                const float sigma = (x0 < 0.f) ? -nrm : nrm;
                const float beta = active ? __builtin_amdgcn_rcpf(fmaf(fabsf(x0), nrm, alpha)) : 0.f;   // 2/|u|^2
                eJ = active ? -sigma : x0;
                static_for<0, R>([&](auto h_) {
                    constexpr int h = decltype(h_)::value;
                    const float t = (row[h] == J + 1) ? (x0 + sigma) : ((row[h] > J + 1) ? x[h] : 0.f);
                    ur[h] = active ? t : 0.f;
                });
                // p = 2 A u / |u|^2 and w = 2 P u / |u|^2 for both rows of the lane
                float pp[R][2] = {{0.f, 0.f}, {0.f, 0.f}}, ww[R][2] = {{0.f, 0.f}, {0.f, 0.f}};
                static_for<J + 1, N>([&](auto c_) {
                    constexpr int c = decltype(c_)::value;
                    const float uc = row_bcast<c % GW>(ur[c / GW]);
                    static_for<0, R>([&](auto h_) {
                        constexpr int h = decltype(h_)::value;
                        pp[h][c & 1] = fmaf(a[h][c], uc, pp[h][c & 1]);
                        if (WANT_V) ww[h][c & 1] = fmaf(v[h][c], uc, ww[h][c & 1]);
                    });
                });
                float p[R], w[R], sr[R];
                float up = 0.f;
                static_for<0, R>([&](auto h_) {
                    constexpr int h = decltype(h_)::value;
                    p[h] = beta * (pp[h][0] + pp[h][1]);
                    w[h] = beta * (ww[h][0] + ww[h][1]);
                    up = fmaf(ur[h], p[h], up);
                });
                // A - q u^T - u q^T with q = p - K u, K = u^T p / |u|^2, regrouped as
                // A - (p - 2K u) u^T - u p^T; P <- P - w u^T
                const float K2 = beta * G::sum(up);
                static_for<0, R>([&](auto h_) { sr[decltype(h_)::value] = fmaf(-K2, ur[decltype(h_)::value], p[decltype(h_)::value]); });
                static_for<J + 1, N>([&](auto c_) {
                    constexpr int c = decltype(c_)::value;
                    const float uc = row_bcast<c % GW>(ur[c / GW]);
                    const float pc = row_bcast<c % GW>(p[c / GW]);
                    static_for<0, R>([&](auto h_) {
                        constexpr int h = decltype(h_)::value;
                        a[h][c] = fmaf(-ur[h], pc, fmaf(-sr[h], uc, a[h][c]));
                        if (WANT_V) v[h][c] = fmaf(-w[h], uc, v[h][c]);
                    });
                });
                // keep the steps apart (the accumulation of P does not feed the reduction of A and
                // would otherwise be postponed as a whole, with every step's u kept alive)
                if (WANT_V) {
#pragma unroll
                    for (int c = J + 1; c < N; ++c) {
                        asm volatile("" : "+v"(v[0][c]));
                        asm volatile("" : "+v"(v[1][c]));
                    }
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
        static_for<0, R>([&](auto h_) {
            constexpr int h = decltype(h_)::value;
            static_for<0, N>([&](auto c_) { sV[decltype(c_)::value * LD + row[h]] = v[h][decltype(c_)::value]; });
        });
    }
    wave_sync();

    // ---- shifted QR iterations (Sec. 3.2), control flow per group ----
    const bool roleB = r >= HW;
    const uint32_t cap = args.sweep_cap ? args.sweep_cap : 30u * (uint32_t)n;
    const int rshift = grp * GW;
    auto group_bits = [&](uint64_t ballot) -> uint32_t { return (uint32_t)(ballot >> rshift) & 0xFFFFu; };
    uint32_t sweeps = 0, rotations = 0, stall = 0, relaxed = 0;
    uint32_t nz = 0, nz_prev = 0xFFFFFFFFu;
    bool live[R];
    float dl[R];
#pragma unroll
    for (int h = 0; h < R; ++h) {
        live[h] = row[h] < n - 1;          // off-diagonal e[row] is watched by this lane
        dl[h] = 0.f;
    }
    const float paper_eps = args.abs_eps * scale;
    const float tol0 = fmaxf(kTinyE, paper_eps), tol1 = fmaxf(kAbsTol1, paper_eps), tol2 = fmaxf(kAbsTol2, paper_eps);
    while (true) {
        // deflation test (Sec. 3.2.3, per matrix, every off-diagonal): the lane looks at e[k], d[k],
        // d[k+1] for its two indices k
        const bool widened = stall >= kStallIterations;
        const float abs_tol = stall >= 2 * kStallIterations ? tol2 : (widened ? tol1 : tol0);
        nz = 0;
#pragma unroll
        for (int h = 0; h < R; ++h) {
            float el = 0.f, dnext = 0.f;
            if (row[h] < N) {
                const float2 pk = sP[row[h]];
                const float2 pk1 = sP[row[h] + 1];
                dl[h] = pk.y;
                el = pk1.x;
                dnext = pk1.y;
            }
            const float dsum = fabsf(dl[h]) + fabsf(dnext);
            const bool negligible = fabsf(el) <= fmaxf(kEps * dsum, abs_tol);
            const bool by_fallback = widened && live[h] && negligible && !(fabsf(el) <= fmaxf(kEps * dsum, tol0));
            relaxed += (uint32_t)__builtin_popcount(group_bits(__ballot(by_fallback)));
            live[h] = live[h] && !negligible;
            nz |= group_bits(__ballot(live[h])) << (h * GW);
        }
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
        const float mu1 = td - tt;
        const float mu2 = (stall >= kExceptionalAfter) ? mu1 : ta + tt;

        // Inputs of rotation t: (e[t], d[t+1]) = sP[t+1] and column t+1 of V, fetched ahead into two
        // slots used in alternation.
        const float d_lo = sP[lo].y;
        float2 q0 = sP[lo + 1];
        float2 q1 = sP[lo + 2];
        float* xV = sV + lo * LD + r;       // this lane's first row of V, at column lo (second row: + GW)
        float xA[R], xB[R], pV[R], y0[R], y1[R];
#pragma unroll
        for (int h = 0; h < R; ++h) {
            xA[h] = WANT_V ? xV[h * GW] : 0.f;
            y0[h] = WANT_V ? xV[LD + h * GW] : 0.f;
            y1[h] = WANT_V ? xV[2 * LD + h * GW] : 0.f;
            pV[h] = 0.f;
            xB[h] = 0.f;
        }
        Chain A;
        A.g = d_lo - mu1;
        A.s = 1.f;
        A.c = 1.f;
        A.p = 0.f;
        A.dk = d_lo;
        float pE, pD;                       // A's outputs of the previous step
        // t = lo: A rotates row lo (computed by every lane)
        chain_rotate(A, q0.x, q0.y, pE, pD);
        if (WANT_V) {
#pragma unroll
            for (int h = 0; h < R; ++h) {
                pV[h] = fmaf(A.c, xA[h], A.s * y0[h]);
                xA[h] = fmaf(A.c, y0[h], -A.s * xA[h]);
                y0[h] = xV[3 * LD + h * GW];
            }
        }
        q0 = sP[lo + 3];
        if (hi - lo == 1) {
            // the window is the 2x2 block the shifts were taken from: the step with its exact
            // eigenvalue diagonalises it; the off-diagonal is set to zero, no second sweep
            if (r == 0) {
                sP[lo] = make_float2(pE, pD);
                sP[hi] = make_float2(0.f, A.dk - A.p);
            }
            if (WANT_V) {
#pragma unroll
                for (int h = 0; h < R; ++h) {
                    xV[h * GW] = pV[h];
                    xV[LD + h * GW] = xA[h];
                }
            }
            rotations += 1u;
            sweeps += 1;
        } else {
            const float sD = pD;                       // d'[lo] as left by A
#pragma unroll
            for (int h = 0; h < R; ++h) xB[h] = pV[h]; // column lo as left by A: B's carried column
            // t = lo + 1: A rotates row lo+1 (still computed by every lane)
            chain_rotate(A, q1.x, q1.y, pE, pD);
            if (WANT_V) {
#pragma unroll
                for (int h = 0; h < R; ++h) {
                    pV[h] = fmaf(A.c, xA[h], A.s * y1[h]);
                    xA[h] = fmaf(A.c, y1[h], -A.s * xA[h]);
                    y1[h] = xV[4 * LD + h * GW];
                }
            }
            q1 = sP[lo + 4];
            Chain S;                                   // this lane's recurrence: A or B
            S.g = roleB ? (sD - mu2) : A.g;
            S.s = roleB ? 1.f : A.s;
            S.c = roleB ? 1.f : A.c;
            S.p = roleB ? 0.f : A.p;
            S.dk = roleB ? sD : A.dk;
            float prevE = pE, prevD = pD;
            float2* xP = sP + (roleB ? lo : (lo + 2));
            float oE, oD;
            auto step = [&](float2& q_, float (&y_)[R], const int k_) {
                const float e_in = G::upper_from_lower(q_.x, prevE);
                const float d_in = G::upper_from_lower(q_.y, prevD);
                chain_rotate(S, e_in, d_in, oE, oD);
                if (WANT_V) {
                    float cA, cB, sA, sB;
                    G::halves(S.c, cA, cB);
                    G::halves(S.s, sA, sB);
#pragma unroll
                    for (int h = 0; h < R; ++h) {
                        const float nV = fmaf(cA, xA[h], sA * y_[h]);
                        xA[h] = fmaf(cA, y_[h], -sA * xA[h]);
                        const float vo = fmaf(cB, xB[h], sB * pV[h]);
                        xB[h] = fmaf(cB, pV[h], -sB * xB[h]);
                        pV[h] = nV;
                        xV[k_ * LD + h * GW] = vo;
                        y_[h] = xV[(k_ + 5) * LD + h * GW];
                    }
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
#pragma unroll
                for (int h = 0; h < R; ++h) {
                    xV[h * GW] = fmaf(cB, xB[h], sB * pV[h]);
                    xB[h] = fmaf(cB, pV[h], -sB * xB[h]);
                }
            }
            // t = hi + 1: B rotates row hi-1 with A's closing values (column hi as left by A is xA)
            chain_rotate(S, G::upper_from_lower(fE, fE), G::upper_from_lower(fD, fD), oE, oD);
            xP[1] = make_float2(oE, oD);
            if (WANT_V) {
                float cA, cB, sA, sB;
                G::halves(S.c, cA, cB);
                G::halves(S.s, sA, sB);
#pragma unroll
                for (int h = 0; h < R; ++h) {
                    xV[LD + h * GW] = fmaf(cB, xB[h], sB * xA[h]);
                    xB[h] = fmaf(cB, xA[h], -sB * xB[h]);
                }
            }
            // t = hi + 2: B closes
            xP[2] = make_float2(S.g, S.dk - S.p);
            if (WANT_V) {
#pragma unroll
                for (int h = 0; h < R; ++h) xV[2 * LD + h * GW] = xB[h];
            }
            rotations += 2u * (uint32_t)(hi - lo);
            sweeps += 2;
        }
        wave_sync();
    }

    // ---- info, ascending order, coalesced store ----
    int info = (int)__builtin_popcount(nz);
    {
        uint32_t bad = 0;
#pragma unroll
        for (int h = 0; h < R; ++h)
            bad |= group_bits(__ballot(row[h] < n && !(fabsf(dl[h]) < __builtin_inff()))) << (h * GW);
        info = max(info, (int)__builtin_popcount(bad));
        info |= (int)(min(relaxed, 0x7FFFu) << 16);
    }
    if (STAGE == kSpectral) {
        // F = V f(Lambda) V^T straight from V and lambda in LDS: the lane forms w[k] = V[row][k] f(lambda_k)
        // for its two rows once, then F[row][c] = sum_k w[k] V[c][k] for every c (V[c][k] is one address
        // per group); F is symmetric, so the entry is stored at F[c][row] and the lanes of a group write
        // consecutive addresses.
        float w[R][N];
        static_for<0, N>([&](auto k_) {
            constexpr int k = decltype(k_)::value;
            float lam = sP[k].y * inv_scale;
            lam = fmaxf(lam, args.fn_floor);
            const float fl = (args.fn == kFnInvSqrt) ? __builtin_amdgcn_rsqf(lam) : __builtin_amdgcn_sqrtf(lam);
            static_for<0, R>([&](auto h_) {
                constexpr int h = decltype(h_)::value;
                w[h][k] = (k < n) ? sV[k * LD + row[h]] * fl : 0.f;
            });
        });
        float* __restrict__ Fb = args.fn_out + (m0 + grp) * nn;
        for (int c = 0; c < n; ++c) {
            float acc[R][2] = {{0.f, 0.f}, {0.f, 0.f}};
            static_for<0, N>([&](auto k_) {
                constexpr int k = decltype(k_)::value;
                const float vc = sV[k * LD + c];
                static_for<0, R>([&](auto h_) {
                    constexpr int h = decltype(h_)::value;
                    acc[h][k & 1] = fmaf(w[h][k], vc, acc[h][k & 1]);
                });
            });
#pragma unroll
            for (int h = 0; h < R; ++h)
                if (mine && row[h] < n) Fb[c * n + row[h]] = acc[h][0] + acc[h][1];
        }
    }
    float* const sE = sE_all + grp * SW;
    int* const sI = sI_all + grp * SW;
#pragma unroll
    for (int h = 0; h < R; ++h) {
        const uint32_t mykey = sort_key(dl[h]);
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const uint32_t kj = sort_key(sP[j].y);
            rank += (kj < mykey || (kj == mykey && j < row[h])) ? 1 : 0;
        }
        if (row[h] < n) {
            sE[rank] = dl[h] * inv_scale;
            sI[rank] = row[h];             // output column `rank` comes from column row[h] of V
        }
    }
    wave_sync();
    if (args.evals) {
        float* __restrict__ Eb = args.evals + m0 * n;
        const float rcp_n = 1.0f / (float)n;
        for (int idx = lane; idx < cnt * n; idx += 64) {
            const int m = (int)(((float)idx + 0.5f) * rcp_n);
            Eb[idx] = sE_all[m * SW + (idx - m * n)];
        }
    }
    if (WANT_V && STAGE == kFull) {
        float* __restrict__ Vb = args.evecs + m0 * nn;
        const float rcp_nn = 1.0f / (float)nn, rcp_n = 1.0f / (float)n;
        chunked_copy<16>(
            cnt * nn, lane,
            [&](int idx) {
                const int m = (int)(((float)idx + 0.5f) * rcp_nn);
                const int rem = idx - m * nn;
                const int i = (int)(((float)rem + 0.5f) * rcp_n);
                return sV_all[m * VA + sI_all[m * SW + (rem - i * n)] * LD + i];
            },
            [&](int idx, float x) { Vb[idx] = x; });
    }
    if (mine && r == 0) {
        if (args.info) args.info[m0 + grp] = info;
        if (args.rotations) args.rotations[m0 + grp] = rotations;
    }
}

template <int N>
static hipError_t launch_packed_rows_n(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    const unsigned blocks = (unsigned)((args.batch + 3) / 4);
    if (stage == kSpectral) return enqueue(packed_rows_kernel<N, true, kSpectral>, dim3(blocks), dim3(64), stream, args);
    if (want_v) return enqueue(packed_rows_kernel<N, true, kFull>, dim3(blocks), dim3(64), stream, args);
    return enqueue(packed_rows_kernel<N, false, kFull>, dim3(blocks), dim3(64), stream, args);
}

}  // namespace bed
#endif
