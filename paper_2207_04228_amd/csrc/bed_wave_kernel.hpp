// Batched symmetric eigensolver kernels for gfx950 (MI355X), wave64.
//
// One wavefront owns one matrix from load to store.  The whole path of
// arXiv 2207.04228 Sec. 3 runs inside one launch:
//   Sec. 3.1   Householder tridiagonalisation (rank-2 update form, Eqs. (5)-(6));
//              the rows of the working matrix and of the accumulated reflector
//              product P (Eq. (8)) live in VGPRs, one row per lane (for n <= 32:
//              A in lanes 0..31, P in lanes 32..63)
//   Sec. 3.2   QR iterations by Givens rotations (App. A.1) with the two
//              Wilkinson shifts of the trailing 2x2 block (Sec. 3.2.2, App. A.3),
//              per-matrix deflation (Sec. 3.2.3), O(1) update of the
//              tridiagonal per rotation (Sec. 3.2.4) and rotation of two
//              columns of V per rotation (Sec. 3.2.5); the tridiagonal and V
//              (column-major) live in LDS, lane r owns row r of V
// followed by an ascending sort and a coalesced store.
#ifndef BED_WAVE_KERNEL_HPP
#define BED_WAVE_KERNEL_HPP
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bed_kernel.h"

namespace bed {

// Cycle counts per phase of one wavefront's work, for the phase-resolved profile
// (paper_2207_04228_amd/phase_profile.py builds a separate library with BED_PHASE_CLOCKS defined).
// In the product build every member is an empty inline function and the object holds nothing.
enum Phase { kPhLoad = 0, kPhTridiag, kPhBoundary, kPhFill, kPhSteady, kPhDrain, kPhStore, kPhIterations, kPhCount };
struct PhaseClock {
#ifdef BED_PHASE_CLOCKS
    unsigned long long last;
    unsigned long long acc[kPhCount];
    __device__ __forceinline__ void start() {
        for (int i = 0; i < kPhCount; ++i) acc[i] = 0;
        last = __builtin_readcyclecounter();
    }
    __device__ __forceinline__ void lap(int phase) {
        const unsigned long long t = __builtin_readcyclecounter();
        acc[phase] += t - last;
        last = t;
    }
    __device__ __forceinline__ void count(int phase) { acc[phase] += 1; }
    __device__ __forceinline__ void write(unsigned long long* out, int b, int lane) const {
        if (out && lane == 0)
            for (int i = 0; i < kPhCount; ++i) out[(size_t)b * kPhCount + i] = acc[i];
    }
#else
    __device__ __forceinline__ void start() {}
    __device__ __forceinline__ void lap(int) {}
    __device__ __forceinline__ void count(int) {}
    __device__ __forceinline__ void write(unsigned long long*, int, int) const {}
#endif
};

namespace {

// Relative deflation tolerance: |e_k| <= kEps (|d_k| + |d_k+1|), kEps = 4 * 2^-23.  Inside a
// cluster of (nearly) equal eigenvalues the recurrence leaves off-diagonals at the rounding
// level of the diagonal, one to two units in the last place of d; a tolerance of 2^-23 is only
// two such units when d is just above a power of two, and windows of repeated eigenvalues then
// hover around it without ever deflating.
constexpr float kEps = 4.7683716e-7f;
// The pair of sweeps with both eigenvalues of the trailing block has fixed points (the 3x3
// matrix with diagonal 1, 0, 1 and off-diagonals 1 is mapped onto itself up to signs), as the
// double-shift QR step has in general.  After this many iterations without any deflation both
// sweeps use the eigenvalue closer to the last diagonal entry, which leaves such a point.
constexpr uint32_t kExceptionalAfter = 5;
constexpr uint32_t kStallIterations = 12;   // iterations without any deflation before the absolute threshold applies
constexpr float kAbsTol1 = 2.3841858e-7f;   // 2^-22 of the pre-scaled matrix
constexpr float kAbsTol2 = 9.5367432e-7f;   // 2^-20
constexpr float kTinyE = 1.0e-18f;      // absolute floor for |e| (matrix is pre-scaled to max|a| in [0.5,1))
constexpr float kTinyG = 1.0e-18f;      // floor for |g| in a rotation (keeps f^2+g^2 a normal number)
constexpr float kTinyAlpha = 1.0e-35f;  // |x|^2 below this: column already reduced, reflector skipped

// ---- cross-lane helpers ---------------------------------------------------

template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp0(float x) {
    // lanes not selected by ROW_MASK (or reading out of range) receive 0
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xF, false));
}

constexpr int kQuadXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kQuadXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141;
constexpr int kRowMirror = 0x140;
constexpr int kRowBcast15 = 0x142;    // lane 15 of each row -> every lane of the next row
constexpr int kRowBcast31 = 0x143;    // lane 31 -> every lane of rows 2 and 3

// A workgroup is one wavefront, and a wavefront's LDS operations complete in
// program order, so data written to LDS by one lane is visible to a later read
// by another lane without a hardware barrier.  This only stops the compiler
// from moving memory operations across the point.
__device__ __forceinline__ void wave_sync() { __builtin_amdgcn_wave_barrier(); }

__device__ __forceinline__ float read_lane(float x, int lane_uniform) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane_uniform));
}

// Lanes 0..31 keep `keep`; lane 32 + i receives the value lane i holds in `src`
// (v_permlane32_swap exchanges the upper half of its first operand with the lower half of
// its second; the first result is the first operand after the exchange).
__device__ __forceinline__ float upper_from_lower(float keep, float src) {
    return __uint_as_float(
        __builtin_amdgcn_permlane32_swap(__float_as_uint(keep), __float_as_uint(src), false, false)[0]);
}

// Every lane receives the value lane 32 + (i & 31) holds: the second result of the same
// exchange applied to two copies of x is x with its upper half copied over its lower half.
__device__ __forceinline__ float from_upper_half(float x) {
    const unsigned u = __float_as_uint(x);
    return __uint_as_float(__builtin_amdgcn_permlane32_swap(u, u, false, false)[1]);
}

// Lanes 0..31 keep `keep`; lanes 32..63 receive the value lane 31 holds in `src`
// (DPP row_bcast31 restricted to rows 2 and 3): one instruction hands a value that is
// uniform over the lower half to the upper half.
__device__ __forceinline__ float upper_from_lane31(float keep, float src) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(__float_as_int(keep), __float_as_int(src), kRowBcast31, 0xC, 0xF, false));
}

// Sum over lanes [0, W) of the wave (W = 8, 16, 32 or 64, lanes outside must
// hold 0 or are ignored), returned as a wave-uniform value.  Quad butterflies,
// then mirrors (which act as xor 4 / xor 8 on quad-uniform values), then row
// broadcasts; no LDS traffic.
template <int W>
__device__ __forceinline__ float wave_sum(float x) {
    x += dpp0<kQuadXor1>(x);
    x += dpp0<kQuadXor2>(x);
    x += dpp0<kRowHalfMirror>(x);
    if (W >= 16) x += dpp0<kRowMirror>(x);
    if (W <= 16) return read_lane(x, 0);
    x += dpp0<kRowBcast15, 0xA>(x);
    if (W == 32) return read_lane(x, 31);
    x += dpp0<kRowBcast31, 0xC>(x);
    return read_lane(x, 63);
}

// Same for max of non-negative values.
template <int W>
__device__ __forceinline__ float wave_max_nonneg(float x) {
    x = fmaxf(x, dpp0<kQuadXor1>(x));
    x = fmaxf(x, dpp0<kQuadXor2>(x));
    x = fmaxf(x, dpp0<kRowHalfMirror>(x));
    if (W >= 16) x = fmaxf(x, dpp0<kRowMirror>(x));
    if (W <= 16) return read_lane(x, 0);
    x = fmaxf(x, dpp0<kRowBcast15, 0xA>(x));
    if (W == 32) return read_lane(x, 31);
    x = fmaxf(x, dpp0<kRowBcast31, 0xC>(x));
    return read_lane(x, 63);
}

constexpr int lanes_for(int n) { return n <= 8 ? 8 : (n <= 16 ? 16 : (n <= 32 ? 32 : 64)); }

// Monotone map float -> uint32 (total order; NaNs land at the ends).
__device__ __forceinline__ uint32_t sort_key(float x) {
    uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exact power-of-two scale bringing amax into [0.5, 1); 1 for 0 / non-finite
__device__ __forceinline__ void pow2_scale(float amax, float& scale, float& inv_scale) {
    int ex = 0;
    if (amax > 0.f && amax < __builtin_inff()) ex = __builtin_amdgcn_frexp_expf(amax);
    ex = min(max(ex, -125), 126);
    scale = ldexpf(1.0f, -ex);
    inv_scale = ldexpf(1.0f, ex);
}


// ---- one sweep's running state (all values are wave-uniform except x) ------
// Implicit shifted QR step written as a chain of Givens rotations (App. A.1):
// rotation k acts on rows/columns (k, k+1), consumes e[k], d[k+1] and column
// k+1 of V, and emits the final e[k-1], d[k] and column k of V.
struct Chain {
    float g, s, c, p;   // bulge-chase carries
    float dk;           // d[k] as left by the previous rotation
    float x;            // V[row][k], this lane's entry of the column being carried
};

template <bool WANT_V>
__device__ __forceinline__ void chain_start(Chain& S, float d_lo, float mu, float v_lo) {
    S.g = d_lo - mu;
    S.s = 1.f;
    S.c = 1.f;
    S.p = 0.f;
    S.dk = d_lo;
    S.x = v_lo;
}

// |g| is kept away from zero (by 1e-18 of the pre-scaled matrix, far below
// rounding) so that f^2 + g^2 is always a normal number: the rotation stays
// exactly normalised and no compare/select sits on the dependency chain.
__device__ __forceinline__ float guard_g(float g) {
    float mag;
    // max(|g|, floor) as one VALU instruction (the library fmaxf adds a NaN-quieting step)
    asm("v_max_f32 %0, |%1|, %2" : "=v"(mag) : "v"(g), "v"(kTinyG));
    return __uint_as_float((__float_as_uint(g) & 0x80000000u) | __float_as_uint(mag));
}

template <bool WANT_V>
__device__ __forceinline__ void chain_rotate(Chain& S, float ek, float dk1, float y,
                                             float& e_out, float& d_out, float& v_out) {
    const float g = guard_g(S.g);
    const float f = S.s * ek;
    const float bb = S.c * ek;
    const float h = fmaf(f, f, g * g);
    const float rinv = __builtin_amdgcn_rsqf(h);
    const float gg = S.dk - S.p;
    S.c = g * rinv;
    S.s = f * rinv;
    e_out = h * rinv;                        // e[k-1] = hypot(f, g)
    const float r2 = fmaf(dk1 - gg, S.s, 2.f * S.c * bb);
    S.p = S.s * r2;
    S.g = fmaf(S.c, r2, -bb);
    d_out = gg + S.p;                        // d[k] final
    if (WANT_V) {
        v_out = fmaf(S.c, S.x, S.s * y);     // column k final
        S.x = fmaf(S.c, y, -S.s * S.x);      // column k+1, carried
    }
    S.dk = dk1;
}

// end of a sweep at row hi: e[hi-1] = g, d[hi] -= p, column hi = carried column
__device__ __forceinline__ void chain_finish(const Chain& S, float& e_out, float& d_out, float& v_out) {
    e_out = S.g;
    d_out = S.dk - S.p;
    v_out = S.x;
}

}  // namespace

// ---------------------------------------------------------------------------
// Shifted QR iterations (Sec. 3.2) on the tridiagonal in sP, rotating the columns of V in
// sV, until every off-diagonal has deflated or the sweep cap is reached.  Runs in ONE
// wavefront; `vrow` is the row of V this lane owns.
//   HALF   the wavefront's rows of V fit in 32 lanes (lanes 32..63 shadow them): the two
//          sweeps of an iteration run in the two halves, each lane rotating its row for
//          its own sweep.  Otherwise every lane owns a row and rotates it for both sweeps.
// On return d_lane[bank] holds d[lane + 64 * bank].
// ---------------------------------------------------------------------------
template <int N, bool HALF, bool WANT_V, int LD, bool PAPER_EPS>
__device__ __forceinline__ void qr_iterations_impl(float2* const sP, float* const sV, const int lane, const int vrow,
                                              const int n, uint32_t& rotations, int& info,
                                              float (&d_lane)[(N + 63) / 64], const KernelArgs& args,
                                              const float paper_eps, PhaseClock& clk) {
    const bool roleB = lane >= 32;
    const uint32_t cap = args.sweep_cap ? args.sweep_cap : 30u * (uint32_t)n;
    uint32_t sweeps = 0;
    // Off-diagonal k = lane + 64 * bank is watched by this lane: e[k] not yet deflated.
    constexpr int NB = (N + 63) / 64;
    bool live[NB];
    float dl[NB];
#pragma unroll
    for (int bk = 0; bk < NB; ++bk) {
        live[bk] = lane + 64 * bk < n - 1;
        dl[bk] = 0.f;
    }
    uint64_t nz[NB], nz_prev[NB];
#pragma unroll
    for (int bk = 0; bk < NB; ++bk) nz_prev[bk] = ~0ull;
    uint32_t stall = 0;                 // iterations since the last deflation
    uint32_t relaxed = 0;               // off-diagonals deflated only because the absolute fallback test accepted them
    // Absolute part of the deflation test: the rounding-level floor, or the paper's threshold
    // epsilon (Sec. 3.2.3, App. B: 1e-5; here in units of the pre-scaled matrix) when the caller
    // asked for it; the fallback thresholds of a stalled window never fall below it.
    // Without a threshold from the caller (PAPER_EPS false) these are compile-time constants.
    const float tol0 = PAPER_EPS ? fmaxf(kTinyE, paper_eps) : kTinyE;
    const float tol1 = PAPER_EPS ? fmaxf(kAbsTol1, paper_eps) : kAbsTol1;
    const float tol2 = PAPER_EPS ? fmaxf(kAbsTol2, paper_eps) : kAbsTol2;
    while (true) {
        // A window that has not deflated anything for kStallIterations iterations is stuck at the
        // rounding noise of the rotations, which is relative to the norm of the matrix and not to
        // the neighbouring diagonal entries (windows with diagonal entries far below the norm:
        // graded spectra).  Such a window also accepts entries below an ABSOLUTE threshold
        // (2^-22, after twice as many iterations 2^-20, of the pre-scaled matrix, whose 2-norm is
        // at least 0.5): dropping one perturbs the eigenvalues by at most 2e-6 ||A||_2, so every
        // matrix finishes within the accuracy bar instead of using up the sweep cap.  Entries
        // accepted only by that threshold are counted and reported through info.
        const bool widened = stall >= kStallIterations;
        const float abs_tol = stall >= 2 * kStallIterations ? tol2 : (widened ? tol1 : tol0);
        // deflation test, lane-parallel: the lane looks at e[k], d[k], d[k+1]
        float el[NB], dnext[NB];
        uint64_t any = 0;
        bool same = true;
#pragma unroll
        for (int bk = 0; bk < NB; ++bk) {
            const int k = lane + 64 * bk;
            el[bk] = 0.f;
            dnext[bk] = 0.f;
            if (k < N) {
                const float2 pk = sP[k];
                const float2 pk1 = sP[k + 1];
                dl[bk] = pk.y;
                el[bk] = pk1.x;
                dnext[bk] = pk1.y;
            }
            const float dsum = fabsf(dl[bk]) + fabsf(dnext[bk]);
            const bool negligible = fabsf(el[bk]) <= fmaxf(kEps * dsum, abs_tol);
            if (widened)
                relaxed += (uint32_t)__builtin_popcountll(
                    __ballot(live[bk] && negligible && !(fabsf(el[bk]) <= fmaxf(kEps * dsum, tol0))));
            live[bk] = live[bk] && !negligible;
            nz[bk] = __ballot(live[bk]);
            any |= nz[bk];
            same = same && nz[bk] == nz_prev[bk];
            nz_prev[bk] = nz[bk];
        }
        stall = same ? stall + 1 : 0;
        if (any == 0 || sweeps >= cap) break;
        clk.count(kPhIterations);
        // active window [lo, hi]: e[hi-1] is the last live entry, e[lo-1] the last dead one below it
        int hi, lo;
        if (NB == 2 && nz[NB - 1] != 0) {
            hi = 128 - __builtin_clzll(nz[NB - 1]);
            const uint64_t below1 = ~nz[NB - 1] & ((1ull << (hi - 65)) - 1ull);
            const uint64_t below0 = ~nz[0];
            lo = below1 ? 128 - __builtin_clzll(below1) : (below0 ? 64 - __builtin_clzll(below0) : 0);
        } else {
            hi = 64 - __builtin_clzll(nz[0]);
            const uint64_t below = ~nz[0] & ((1ull << (hi - 1)) - 1ull);
            lo = below ? 64 - __builtin_clzll(below) : 0;
        }
        // value of a lane-distributed entry at a wave-uniform index
        auto at = [&](const float (&v)[NB], int idx) -> float {
            return (NB == 1 || idx < 64) ? read_lane(v[0], idx & 63) : read_lane(v[NB - 1], idx - 64);
        };

        // eigenvalues of the trailing block [[ta, tb], [tb, td]] (App. A.3), smaller-angle root first
        const float ta = at(dl, hi - 1);
        const float tb = at(el, hi - 1);
        const float td = at(dnext, hi - 1);
        const float delta = 0.5f * (ta - td);
        const float rt = __builtin_amdgcn_sqrtf(fmaf(delta, delta, tb * tb));
        const float den = delta + ((delta >= 0.f) ? rt : -rt);
        const float tt = (tb * tb) * __builtin_amdgcn_rcpf(den);
        const float mu1 = td - tt;          // eigenvalue closer to the last diagonal entry
        const float mu2 = (stall >= kExceptionalAfter) ? mu1 : ta + tt;   // the other eigenvalue of the block

        // Inputs of rotation t: (e[t], d[t+1]) = sP[t+1] and column t+1 of V.  They are
        // fetched two rotations ahead into two slots used in alternation (slot 0: rotations
        // lo, lo+2, ...; slot 1: rotations lo+1, lo+3, ...), so a slot is refilled right after
        // it has been consumed and no register shuffling is needed.
        const float d_lo = at(dl, lo);
        float2 q0 = make_float2(at(el, lo), at(dnext, lo));
        float2 q1 = sP[lo + 2];
        float y0 = 0.f, y1 = 0.f;
        Chain A;
        chain_start<WANT_V>(A, d_lo, mu1, WANT_V ? sV[lo * LD + vrow] : 0.f);
        if (WANT_V) {
            y0 = sV[(lo + 1) * LD + vrow];
            y1 = sV[(lo + 2) * LD + vrow];
        }
        // refill a slot with the inputs of rotation t_+2 (indices stay inside the padding)
#define BED_REFILL(q_, y_, t_)                                  \
        do {                                                \
            q_ = sP[(t_) + 3];                              \
            if (WANT_V) y_ = sV[((t_) + 3) * LD + vrow];    \
        } while (0)

        {
            // Two sweeps (shift mu1, then mu2) over the same window, software-pipelined:
            // sweep B runs two rotations behind sweep A and takes A's results straight
            // from registers.  At step t: B handles row t-2 with A's outputs of step t-1,
            // while A handles row t.
            float pE, pD, pV = 0.f;     // A's outputs of the previous step
            clk.lap(kPhBoundary);
            // t = lo: A rotates row lo
            chain_rotate<WANT_V>(A, q0.x, q0.y, y0, pE, pD, pV);
            BED_REFILL(q0, y0, lo);
            if (hi - lo == 1) {
                // The window is the 2x2 block the shifts were taken from: the step with
                // its exact eigenvalue mu1 diagonalises it (this is the rotation of
                // App. A.3), so the off-diagonal is set to zero and no second sweep runs.
                // (A second sweep here would start from (d'[lo] - mu2, e'[lo]) = rounding
                // noise and could rotate the converged block by an arbitrary angle.)
                sP[lo] = make_float2(pE, pD);
                if (WANT_V) sV[lo * LD + vrow] = pV;
                chain_finish(A, pE, pD, pV);
                sP[hi] = make_float2(0.f, pD);
                if (WANT_V) sV[hi * LD + vrow] = pV;
                rotations += 1u;
                sweeps += 1;
            } else if (HALF) {
                // Role lanes: lanes 0..31 carry sweep A, lanes 32..63 carry sweep B, so one
                // instruction stream advances both sweeps by one rotation per step.
                // B's inputs are A's outputs of the previous step, copied from the lower
                // half of the wavefront.
                const float sD = pD, sX = pV;              // d'[lo], column lo as left by A
                // t = lo + 1: A rotates row lo+1 (still computed by every lane)
                chain_rotate<WANT_V>(A, q1.x, q1.y, y1, pE, pD, pV);
                BED_REFILL(q1, y1, lo + 1);
                Chain S;                                   // this lane's chain: A or B
                S.g = roleB ? (sD - mu2) : A.g;
                S.s = roleB ? 1.f : A.s;
                S.c = roleB ? 1.f : A.c;
                S.p = roleB ? 0.f : A.p;
                S.dk = roleB ? sD : A.dk;
                S.x = roleB ? sX : A.x;
                // B's inputs are A's outputs of the previous step.  e and d are uniform over the
                // A lanes: one DPP broadcast of lane 31 into the upper half merges them with the A
                // lanes' own inputs.  The V entry is per row: a half swap does the same merge.
                float prevE = pE, prevD = pD, prevV = pV;
                // One running LDS pointer per lane and array; every lane stores at the pointer
                // and loads three positions above it.  A lanes: the pointer is at position t,
                // so the load fetches the inputs of rotation t+2 (position t+3) and the store
                // lands on a position A has already consumed and B overwrites with the final
                // value two steps later.  B lanes: the pointer is at position t-2, so the
                // store is the real one and the load is a valid address whose value is ignored.
                constexpr int AHEAD = 3;
                const float* xV = sV + (roleB ? lo : (lo + 2)) * LD + vrow;
                const float2* xP = sP + (roleB ? lo : (lo + 2));
                float oE, oD, oV = 0.f;
#define BED_STEPH(q_, y_, k_)                                                       \
                do {                                                            \
                    const float e_in = upper_from_lane31(q_.x, prevE);          \
                    const float d_in = upper_from_lane31(q_.y, prevD);          \
                    const float y_in = WANT_V ? upper_from_lower(y_, prevV) : 0.f; \
                    chain_rotate<WANT_V>(S, e_in, d_in, y_in, oE, oD, oV);      \
                    q_ = xP[(k_) + AHEAD];                                      \
                    if (WANT_V) y_ = xV[((k_) + AHEAD) * LD];                   \
                    const_cast<float2*>(xP)[(k_)] = make_float2(oE, oD);        \
                    if (WANT_V) const_cast<float*>(xV)[(k_) * LD] = oV;         \
                    prevE = oE;                                                 \
                    prevD = oD;                                                 \
                    prevV = oV;                                                 \
                } while (0)
                clk.lap(kPhFill);
                int t = lo + 2;
                for (; t + 1 < hi; t += 2) {
                    BED_STEPH(q0, y0, 0);
                    BED_STEPH(q1, y1, 1);
                    xV += 2 * LD;
                    xP += 2;
                }
                if (t < hi) {
                    BED_STEPH(q0, y0, 0);
                    xV += LD;
                    xP += 1;
                }
#undef BED_STEPH
                clk.lap(kPhSteady);
                // The three closing steps belong to B alone; the A lanes' stores would now land
                // beyond the window, so they are parked in the padding behind the arrays.
                xV = roleB ? xV : (sV + (N + 3) * LD + vrow);
                xP = roleB ? xP : (sP + (N + 3));
                // t = hi: A closes (values taken before its state is overwritten); B rotates row hi-2
                float fE, fD, fV;
                chain_finish(S, fE, fD, fV);
                chain_rotate<WANT_V>(S, upper_from_lane31(prevE, prevE), upper_from_lane31(prevD, prevD),
                                     WANT_V ? upper_from_lower(prevV, prevV) : 0.f, oE, oD, oV);
                const_cast<float2*>(xP)[0] = make_float2(oE, oD);
                if (WANT_V) const_cast<float*>(xV)[0] = oV;
                // t = hi + 1: B rotates row hi-1 with A's closing values
                chain_rotate<WANT_V>(S, upper_from_lane31(fE, fE), upper_from_lane31(fD, fD),
                                     WANT_V ? upper_from_lower(fV, fV) : 0.f, oE, oD, oV);
                const_cast<float2*>(xP)[1] = make_float2(oE, oD);
                if (WANT_V) const_cast<float*>(xV)[LD] = oV;
                // t = hi + 2: B closes
                chain_finish(S, fE, fD, fV);
                const_cast<float2*>(xP)[2] = make_float2(fE, fD);
                if (WANT_V) const_cast<float*>(xV)[2 * LD] = fV;
                rotations += 2u * (uint32_t)(hi - lo);
                sweeps += 2;
            } else {
                // Rows need the whole wavefront.  The scalar recurrences of the two sweeps
                // still run in the two halves (lanes 0..31 sweep A, lanes 32..63 sweep B, two
                // rotations behind), but every lane owns a row of V: the rotation coefficients
                // of both sweeps are broadcast with v_readlane and every lane applies both
                // rotations to its row.
                const float sD = pD;                       // d'[lo] as left by A
                float xB = pV;                             // column lo as left by A: B's carried column
                // t = lo + 1: A rotates row lo+1 (still computed by every lane)
                chain_rotate<WANT_V>(A, q1.x, q1.y, y1, pE, pD, pV);
                BED_REFILL(q1, y1, lo + 1);
                Chain S;                                   // this lane's recurrence: A or B (no V part)
                S.g = roleB ? (sD - mu2) : A.g;
                S.s = roleB ? 1.f : A.s;
                S.c = roleB ? 1.f : A.c;
                S.p = roleB ? 0.f : A.p;
                S.dk = roleB ? sD : A.dk;
                S.x = 0.f;
                float xA = A.x;                            // A's carried column
                float prevE = pE, prevD = pD;              // A's (e, d) of the previous step; pV is its column
                // T: one running pointer per lane as in the half-wavefront loop (store at the
                // pointer, load three positions above).  V: every lane stores column t-2 and
                // prefetches column t+3 of its own row.
                constexpr int AHEAD = 3;
                const float2* xP = sP + (roleB ? lo : (lo + 2));
                float* xVp = sV + lo * LD + vrow;
                float oE, oD, unused;
#define BED_STEPW(q_, y_, k_)                                                       \
                do {                                                            \
                    const float e_in = upper_from_lane31(q_.x, prevE);          \
                    const float d_in = upper_from_lane31(q_.y, prevD);          \
                    chain_rotate<false>(S, e_in, d_in, 0.f, oE, oD, unused);    \
                    if (WANT_V) {                                               \
                        const float cA = read_lane(S.c, 0), sA = read_lane(S.s, 0);   \
                        const float cB = read_lane(S.c, 32), sB = read_lane(S.s, 32); \
                        const float nV = fmaf(cA, xA, sA * y_);                 \
                        xA = fmaf(cA, y_, -sA * xA);                            \
                        const float vo = fmaf(cB, xB, sB * pV);                 \
                        xB = fmaf(cB, pV, -sB * xB);                            \
                        pV = nV;                                                \
                        xVp[(k_) * LD] = vo;                                    \
                        y_ = xVp[((k_) + 5) * LD];                              \
                    }                                                           \
                    q_ = xP[(k_) + AHEAD];                                      \
                    const_cast<float2*>(xP)[(k_)] = make_float2(oE, oD);        \
                    prevE = oE;                                                 \
                    prevD = oD;                                                 \
                } while (0)
                clk.lap(kPhFill);
                int t = lo + 2;
                for (; t + 1 < hi; t += 2) {
                    BED_STEPW(q0, y0, 0);
                    BED_STEPW(q1, y1, 1);
                    xVp += 2 * LD;
                    xP += 2;
                }
                if (t < hi) {
                    BED_STEPW(q0, y0, 0);
                    xVp += LD;
                    xP += 1;
                }
#undef BED_STEPW
                clk.lap(kPhSteady);
                // closing steps: B alone; the A lanes' T stores are parked in the padding
                xP = roleB ? xP : (sP + (N + 3));
                float fE, fD, fx;
                chain_finish(S, fE, fD, fx);               // A lanes: e[hi-1], d[hi] as left by A
                // t = hi: B rotates row hi-2 with A's outputs of row hi-1
                chain_rotate<false>(S, upper_from_lane31(prevE, prevE), upper_from_lane31(prevD, prevD), 0.f,
                                    oE, oD, unused);
                const_cast<float2*>(xP)[0] = make_float2(oE, oD);
                if (WANT_V) {
                    const float cB = read_lane(S.c, 32), sB = read_lane(S.s, 32);
                    xVp[0] = fmaf(cB, xB, sB * pV);
                    xB = fmaf(cB, pV, -sB * xB);
                }
                // t = hi + 1: B rotates row hi-1 with A's closing values (column hi as left by A is xA)
                chain_rotate<false>(S, upper_from_lane31(fE, fE), upper_from_lane31(fD, fD), 0.f, oE, oD, unused);
                const_cast<float2*>(xP)[1] = make_float2(oE, oD);
                if (WANT_V) {
                    const float cB = read_lane(S.c, 32), sB = read_lane(S.s, 32);
                    xVp[LD] = fmaf(cB, xB, sB * xA);
                    xB = fmaf(cB, xA, -sB * xB);
                }
                // t = hi + 2: B closes
                chain_finish(S, fE, fD, fx);
                const_cast<float2*>(xP)[2] = make_float2(fE, fD);
                if (WANT_V) xVp[2 * LD] = xB;
                rotations += 2u * (uint32_t)(hi - lo);
                sweeps += 2;
            }
        }
#undef BED_REFILL
        wave_sync();
        clk.lap(kPhDrain);
    }
    clk.lap(kPhBoundary);      // the last deflation test, which found nothing left
    info = 0;
#pragma unroll
    for (int bk = 0; bk < NB; ++bk) {
        // a non-finite eigenvalue (NaN/Inf input) is reported even when every off-diagonal deflated
        const uint64_t bad = __ballot(lane + 64 * bk < n && !(fabsf(dl[bk]) < __builtin_inff()));
        info += max((int)__builtin_popcountll(nz[bk]), (int)__builtin_popcountll(bad));
        d_lane[bk] = dl[bk];
    }
    info |= (int)(min(relaxed, 0x7FFFu) << 16);
}

// The two instantiations differ only in the thresholds above: the default path keeps them as
// literals, so a caller that passes no threshold runs the same loop as before the option existed.
template <int N, bool HALF, bool WANT_V, int LD>
__device__ __forceinline__ void qr_iterations(float2* const sP, float* const sV, const int lane, const int vrow,
                                              const int n, uint32_t& rotations, int& info,
                                              float (&d_lane)[(N + 63) / 64], const KernelArgs& args,
                                              const float inv_scale, PhaseClock& clk) {
    if (args.abs_eps > 0.f)   // uniform over the grid
        qr_iterations_impl<N, HALF, WANT_V, LD, true>(sP, sV, lane, vrow, n, rotations, info, d_lane, args,
                                                       args.abs_eps * pow2_reciprocal(inv_scale), clk);
    else
        qr_iterations_impl<N, HALF, WANT_V, LD, false>(sP, sV, lane, vrow, n, rotations, info, d_lane, args, 0.f, clk);
}

// ---------------------------------------------------------------------------
// N      register-array size (4, 8, 12, 16, 20, 24, 28, 32, 40, 48, 56, 64); n <= N at run time
// WANT_V accumulate eigenvectors
// STAGE  kFull, kTridiagOnly (stage hook 1), kQrOnly (stage hook 2), kQrPartial (stage hook 3:
//        a given number of sweeps on a given tridiagonal, result left unsorted)
// Shifts: both eigenvalues of the trailing 2x2 block of the active window are taken
// once per outer iteration and used by two sweeps over the same window (Sec. 3.2.2).
// ---------------------------------------------------------------------------
template <int N, bool WANT_V, int STAGE>
__global__ __launch_bounds__(64) void wave_kernel(KernelArgs args) {
    constexpr int W = lanes_for(N);
    // When the rows fit in half a wavefront (N <= 32), lane 32 + r works on the same row r as
    // lane r from load to store: in the tridiagonalisation the upper half holds the rows of P
    // (the lower half those of A), in the QR phase the halves carry the two sweeps of an
    // iteration.
    constexpr bool HALF = (N <= 32);
    // Column stride: odd (conflict-free rows and columns) and wide enough that every lane
    // owns a row slot, so no V access needs a lane predicate (rows >= n are idle lanes).
    constexpr int LD = HALF ? 33 : 65;
    // V, column-major: V[r][c] at sV[c * LD + r]; also the staging buffer for load and store.
    // Columns N .. N+7 and entries N .. N+9 of the tridiagonal are padding: the QR loop reads
    // up to three positions ahead of the window and parks idle stores there.
    constexpr int VA = (N + 8) * LD;
    constexpr int PA = N + 10;
    __shared__ float sV[VA];
    // tridiagonal: sP[k] = (e[k-1], d[k]); e[k] couples rows k and k+1
    __shared__ float2 sP[PA];
    __shared__ float svec[64];
    __shared__ float sq[64];

    const int lane = threadIdx.x;
    const int row = HALF ? (lane & 31) : lane;     // the row of the matrix and of V this lane owns
    const int b = blockIdx.x;
    const int n = args.n;

    float inv_scale = 1.f;
    PhaseClock clk;
    clk.start();

    constexpr bool GIVEN_T = (STAGE == kQrOnly || STAGE == kQrPartial);
    if (!GIVEN_T && HALF && WANT_V) {
        // ---- rows fit in half a wavefront and P is wanted: the lower half holds the rows of
        // the working matrix, the upper half the rows of the accumulated reflector product
        // P (Eq. (8)).  One instruction stream serves both: the dot product with u gives
        // p = 2Au/|u|^2 in the lower half and w = 2Pu/|u|^2 in the upper half, and the update
        // x <- x - q u^T is the first half of the rank-2 update of A (q = p - K u) and the whole
        // rank-1 update of P (q = w); the second half, x <- x - u q^T, runs with u = 0 in the
        // upper half.
        const bool roleP = lane >= 32;
        const int arow = roleP ? -1 : row;         // row index for the selections on A; none for the P lanes
        float x[N];
        const float* __restrict__ Ab = args.A + (size_t)b * n * n;
        const float rcp_n = 1.0f / (float)n;
        chunked_copy<copy_chunk(N * N)>(
            n * n, lane, [&](int idx) { return Ab[idx]; },
            [&](int idx, float x) {
                const int i = (int)(((float)idx + 0.5f) * rcp_n);
                sV[i * LD + (idx - i * n)] = x;
            });
        wave_sync();
        float amax = 0.f;
#pragma unroll
        for (int c = 0; c < N; ++c) {
            float aval = 0.f;
            if (row < n && c < n) aval = (c <= row) ? sV[row * LD + c] : sV[c * LD + row];
            amax = fmaxf(amax, fabsf(aval));   // fmaxf drops NaNs; they still reach the output through the arithmetic
            x[c] = roleP ? ((c == row) ? 1.f : 0.f) : aval;
        }
        wave_sync();
        float scale;
        pow2_scale(wave_max_nonneg<W>(amax), scale, inv_scale);
        const float myscale = roleP ? 1.f : scale;
#pragma unroll
        for (int c = 0; c < N; ++c) x[c] *= myscale;
        clk.lap(kPhLoad);
#pragma unroll
        for (int J = 0; J < N; ++J) {
            const float dJ = read_lane(x[J], J);      // final once columns 0..J-1 are reduced
            float eJ = 0.f;
            if (J < N - 1) {
                const float x0 = read_lane(x[J], J + 1);     // A[J+1][J]
                eJ = x0;                                      // kept as is when no reflector is applied
                if (J < N - 2) {
                    const float xc = (arow > J) ? x[J] : 0.f; // A[r][J], r > J
                    const float alpha = wave_sum<W>(xc * xc); // |x|^2 (the sum reads the lower half only)
                    const bool active = (J < n - 2) && (alpha > kTinyAlpha);
                    const float nrm = __builtin_amdgcn_sqrtf(alpha);
                    const float sigma = (x0 < 0.f) ? -nrm : nrm;   // sign chosen to avoid cancellation
                    float ur = (arow == J + 1) ? (x0 + sigma) : ((arow > J + 1) ? xc : 0.f);
                    ur = active ? ur : 0.f;
                    const float beta = active ? __builtin_amdgcn_rcpf(fmaf(fabsf(x0), nrm, alpha)) : 0.f;  // 2/|u|^2
                    eJ = active ? -sigma : x0;
                    // u and p are broadcast with v_readlane (the entries live in lanes 0..31; the
                    // results are scalars that the FMAs take as operands): no LDS round trip and no
                    // barrier in the whole reduction
                    float u[N];
#pragma unroll
                    for (int c = J + 1; c < N; ++c) u[c] = read_lane(ur, c);
                    float pp[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int c = J + 1; c < N; ++c) pp[c & 3] = fmaf(x[c], u[c], pp[c & 3]);
                    const float pw = beta * ((pp[0] + pp[1]) + (pp[2] + pp[3]));     // p (A lanes), w (P lanes)
                    // A - q u^T - u q^T with q = p - K u, K = u^T p / |u|^2, regrouped as
                    // A - (p - 2K u) u^T - u p^T: the broadcast of p does not wait for K.
                    const float K2 = beta * wave_sum<W>(ur * pw);                    // 2K
                    const float sr = fmaf(-K2, ur, pw);       // p - 2K u; stays w in the P lanes (u = 0 there)
#pragma unroll
                    for (int c = J + 1; c < N; ++c) x[c] = fmaf(-ur, read_lane(pw, c), fmaf(-sr, u[c], x[c]));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (lane == 0) {
                sP[J].y = dJ;
                sP[J + 1].x = (J < n - 1) ? eJ : 0.f;
            }
        }
        if (lane == 0) sP[0].x = 0.f;
        // every lane stores the P lanes' row (the upper half's value copied over the lower half)
#pragma unroll
        for (int c = 0; c < N; ++c) sV[c * LD + row] = from_upper_half(x[c]);
        wave_sync();
    } else if (!GIVEN_T) {
        float a[N];
        float v[N];
#pragma unroll
        for (int c = 0; c < N; ++c) v[c] = (c == row) ? 1.f : 0.f;

        // ---- load: coalesced into LDS, then row `row` (lower triangle mirrored)
        const float* __restrict__ Ab = args.A + (size_t)b * n * n;
        const float rcp_n = 1.0f / (float)n;
        chunked_copy<copy_chunk(N * N)>(
            n * n, lane, [&](int idx) { return Ab[idx]; },
            [&](int idx, float x) {
                const int i = (int)(((float)idx + 0.5f) * rcp_n);
                sV[i * LD + (idx - i * n)] = x;
            });
        wave_sync();
        float amax = 0.f;
#pragma unroll
        for (int c = 0; c < N; ++c) {
            float x = 0.f;
            if (row < n && c < n) x = (c <= row) ? sV[row * LD + c] : sV[c * LD + row];
            a[c] = x;
            amax = fmaxf(amax, fabsf(x));   // fmaxf drops NaNs; they still reach the output through the arithmetic
        }
        wave_sync();
        float scale;
        pow2_scale(wave_max_nonneg<W>(amax), scale, inv_scale);
#pragma unroll
        for (int c = 0; c < N; ++c) a[c] *= scale;
        clk.lap(kPhLoad);

        // ---- Householder tridiagonalisation, column J reduced at step J ----
        // Branch-free: a step that has nothing to do (J >= n-2, or the column is
        // already reduced) runs with u = 0 and beta = 0.
        // u and q are broadcast through LDS (one write, then 128-bit reads that every lane
        // issues for the same address); the latency of each round trip is covered by
        // independent work: the rank-1 update of V is deferred by one step and runs while
        // the next u is in flight, and the part of the rank-2 update of A that needs only
        // this lane's q runs while q is in flight.
        float ud[N];          // u of the previous step (for the deferred update of V)
        float wd = 0.f;       // its 2 V u / |u|^2
#pragma unroll
        for (int c = 0; c < N; ++c) ud[c] = 0.f;
#pragma unroll
        for (int J = 0; J < N; ++J) {
            const float dJ = read_lane(a[J], J);      // final once columns 0..J-1 are reduced
            float eJ = 0.f;
            if (J < N - 1) {
                const float x0 = read_lane(a[J], J + 1);     // A[J+1][J]
                eJ = x0;                                      // kept as is when no reflector is applied
                if (J < N - 2) {
                    const float x = (row > J) ? a[J] : 0.f;   // A[r][J], r > J
                    const float alpha = wave_sum<W>(x * x);   // |x|^2
                    const bool active = (J < n - 2) && (alpha > kTinyAlpha);
                    const float nrm = __builtin_amdgcn_sqrtf(alpha);
                    const float sigma = (x0 < 0.f) ? -nrm : nrm;   // sign chosen to avoid cancellation
                    float ur = (row == J + 1) ? (x0 + sigma) : ((row > J + 1) ? x : 0.f);
                    ur = active ? ur : 0.f;
                    const float beta = active ? __builtin_amdgcn_rcpf(fmaf(fabsf(x0), nrm, alpha)) : 0.f;  // 2/|u|^2
                    eJ = active ? -sigma : x0;
                    // Up to 32 rows, u and p are broadcast with v_readlane (scalar operands of the
                    // FMAs); beyond, through LDS (one write, then 128-bit reads of one address).
                    constexpr bool RL = (N <= 32);
                    if (!RL) svec[lane] = ur;
                    if (WANT_V && J > 0) {
                        // deferred: V <- V - w u^T of step J-1 (columns J .. N-1)
#pragma unroll
                        for (int c = J; c < N; ++c) v[c] = fmaf(-wd, ud[c], v[c]);
                    }
                    if (!RL) __syncthreads();
                    float u[N];
#pragma unroll
                    for (int c = J + 1; c < N; ++c) u[c] = RL ? read_lane(ur, c) : svec[c];
                    // p = 2 A u / |u|^2, w = 2 V u / |u|^2; four partial sums each
                    float pp[4] = {0.f, 0.f, 0.f, 0.f}, ww[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int c = J + 1; c < N; ++c) {
                        pp[c & 3] = fmaf(a[c], u[c], pp[c & 3]);
                        if (WANT_V) ww[c & 3] = fmaf(v[c], u[c], ww[c & 3]);
                    }
                    const float p = beta * ((pp[0] + pp[1]) + (pp[2] + pp[3]));
                    wd = beta * ((ww[0] + ww[1]) + (ww[2] + ww[3]));
                    // A - q u^T - u q^T with q = p - K u, regrouped as A - (p - 2K u) u^T - u p^T
                    // (p is broadcast before K is known; same arithmetic as the role-lane variant)
                    if (!RL) sq[lane] = p;
                    const float K2 = beta * wave_sum<W>(ur * p);  // 2K
                    const float sr = fmaf(-K2, ur, p);
#pragma unroll
                    for (int c = J + 1; c < N; ++c) a[c] = fmaf(-sr, u[c], a[c]);
                    if (!RL) __syncthreads();
#pragma unroll
                    for (int c = J + 1; c < N; ++c) {
                        a[c] = fmaf(-ur, RL ? read_lane(p, c) : sq[c], a[c]);
                        ud[c] = u[c];
                    }
                    // keep the steps apart: interleaving them makes the compiler hoist the next
                    // steps' loads and run out of registers
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // sP[J+1].x = e[J], sP[J].y = d[J]
            if (lane == 0) {
                sP[J].y = dJ;
                sP[J + 1].x = (J < n - 1) ? eJ : 0.f;
            }
        }
        if (WANT_V && N > 2) {
            // the last reflector's deferred update of V
#pragma unroll
            for (int c = N - 2; c < N; ++c) v[c] = fmaf(-wd, ud[c], v[c]);
        }
        if (lane == 0) sP[0].x = 0.f;
        if (WANT_V) {
#pragma unroll
            for (int c = 0; c < N; ++c) sV[c * LD + row] = v[c];
        }
        wave_sync();
    } else {
        // ---- stage hook 2: tridiagonal given ----
        float dv = 0.f, ev = 0.f;
        if (lane < n) dv = args.d_in[(size_t)b * n + lane];
        if (lane < n - 1) ev = args.e_in[(size_t)b * n + lane];
        float scale;
        pow2_scale(wave_max_nonneg<64>(fmaxf(fabsf(dv), fabsf(ev))), scale, inv_scale);
        if (lane < N) {
            sP[lane].y = dv * scale;
            sP[lane + 1].x = ev * scale;
        }
        if (lane == 0) sP[0].x = 0.f;
        if (WANT_V) {
            for (int c = 0; c < N; ++c) sV[c * LD + row] = (c == row) ? 1.f : 0.f;
        }
        wave_sync();
    }

    uint32_t rotations = 0;
    int info = 0;
    clk.lap(kPhTridiag);

    if (STAGE == kTridiagOnly) {
        if (lane < n) {
            args.d_out[(size_t)b * n + lane] = sP[lane].y * inv_scale;
            args.e_out[(size_t)b * n + lane] = (lane < n - 1) ? sP[lane + 1].x * inv_scale : 0.f;
        }
        if (WANT_V) {
            float* __restrict__ Vb = args.evecs + (size_t)b * n * n;
            const float rcp_n = 1.0f / (float)n;
            chunked_copy<copy_chunk(N * N)>(
                n * n, lane,
                [&](int idx) {
                    const int i = (int)(((float)idx + 0.5f) * rcp_n);
                    return sV[(idx - i * n) * LD + i];
                },
                [&](int idx, float x) { Vb[idx] = x; });
        }
    } else {
        // ---- shifted QR iterations on the tridiagonal in sP ----
        float d_lane[1];
        qr_iterations<N, HALF, WANT_V, LD>(sP, sV, lane, row, n, rotations, info, d_lane, args, inv_scale, clk);
        const float dl = d_lane[0];
        const int vrow = row;
        if (STAGE == kQrPartial) {
            // stage hook 3: the tridiagonal and the accumulated rotations as they stand
            if (lane < n) {
                args.d_out[(size_t)b * n + lane] = sP[lane].y * inv_scale;
                args.e_out[(size_t)b * n + lane] = (lane < n - 1) ? sP[lane + 1].x * inv_scale : 0.f;
            }
            if (WANT_V) {
                float* __restrict__ Vb = args.evecs + (size_t)b * n * n;
                const float rcp_n = 1.0f / (float)n;
                chunked_copy<copy_chunk(N * N)>(
                    n * n, lane,
                    [&](int idx) {
                        const int i = (int)(((float)idx + 0.5f) * rcp_n);
                        return sV[(idx - i * n) * LD + i];
                    },
                    [&](int idx, float x) { Vb[idx] = x; });
            }
            if (lane == 0 && args.rotations) args.rotations[b] = rotations;
            return;
        }

        if (STAGE == kSpectral) {
            // ---- F = V f(Lambda) V^T (Sec. 4.2-4.4, App. B: A^{-1/2} for whitening, A^{1/2} for
            // covariance pooling / colouring), straight from V and lambda in LDS; no sort needed.
            // Lane r forms w[k] = V[r][k] f(lambda_k) once, then F[r][c] = sum_k w[k] V[c][k] for
            // every c; F is symmetric, so the entry is stored at F[c][r] and consecutive lanes
            // write consecutive addresses.  With rows shadowed in both halves of the wavefront
            // (n <= 32) the halves split the columns.
            float w[N];
#pragma unroll
            for (int k = 0; k < N; ++k) {
                float lam = sP[k].y * inv_scale;
                lam = fmaxf(lam, args.fn_floor);
                const float fl = (args.fn == kFnInvSqrt) ? __builtin_amdgcn_rsqf(lam) : __builtin_amdgcn_sqrtf(lam);
                w[k] = (k < n) ? sV[k * LD + row] * fl : 0.f;
            }
            float* __restrict__ Fb = args.fn_out + (size_t)b * n * n;
            const int c0 = HALF ? (lane >> 5) : 0;
            const int cstep = HALF ? 2 : 1;
            for (int c = c0; c < n; c += cstep) {
                float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k = 0; k < N; ++k) acc[k & 3] = fmaf(w[k], sV[k * LD + c], acc[k & 3]);
                if (row < n) Fb[c * n + row] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
            }
            if (args.evals) {
                // eigenvalues as a by-product (ascending)
                const uint32_t key = sort_key(dl);
                int rk = 0;
                for (int j = 0; j < n; ++j) {
                    const uint32_t kj = sort_key(sP[j].y);
                    rk += (kj < key || (kj == key && j < lane)) ? 1 : 0;
                }
                if (lane < n) args.evals[(size_t)b * n + rk] = dl * inv_scale;
            }
            if (lane == 0 && args.info) args.info[b] = info;
            return;
        }

        // ---- ascending order: rank of d[lane] among d[0..n) ----
        // (keys from LDS: taking them from the lanes with v_readlane was measured 2 % slower at n = 32)
        const uint32_t mykey = sort_key(dl);
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const uint32_t kj = sort_key(sP[j].y);
            rank += (kj < mykey || (kj == mykey && j < lane)) ? 1 : 0;
        }
        if (lane < n) args.evals[(size_t)b * n + rank] = dl * inv_scale;
        if (WANT_V) {
            int* sinv = reinterpret_cast<int*>(svec);
            if (lane < n) sinv[rank] = lane;       // output column `rank` comes from column `lane`
            wave_sync();
            float* __restrict__ Vb = args.evecs + (size_t)b * n * n;
            const float rcp_n = 1.0f / (float)n;
            chunked_copy<copy_chunk(N * N)>(
                n * n, lane,
                [&](int idx) {
                    const int i = (int)(((float)idx + 0.5f) * rcp_n);
                    return sV[sinv[idx - i * n] * LD + i];
                },
                [&](int idx, float x) { Vb[idx] = x; });
        }
    }

    if (lane == 0) {
        if (args.info) args.info[b] = info;
        if (args.rotations) args.rotations[b] = rotations;
    }
    clk.lap(kPhStore);
    clk.write(args.phases, b, lane);
}

// ---------------------------------------------------------------------------
// host-side dispatch for one register-array size
// ---------------------------------------------------------------------------
template <int N, bool WANT_V, int STAGE>
static hipError_t launch_one(const KernelArgs& args, hipStream_t stream) {
    return enqueue(wave_kernel<N, WANT_V, STAGE>, dim3(args.batch), dim3(64), stream, args);
}

template <int N>
static hipError_t launch_n(const KernelArgs& args, int stage, bool want_v, hipStream_t stream) {
    if (stage == kTridiagOnly) {
        return want_v ? launch_one<N, true, kTridiagOnly>(args, stream)
                      : launch_one<N, false, kTridiagOnly>(args, stream);
    }
    if (stage == kQrOnly) {
        return want_v ? launch_one<N, true, kQrOnly>(args, stream)
                      : launch_one<N, false, kQrOnly>(args, stream);
    }
    if (stage == kSpectral) return launch_one<N, true, kSpectral>(args, stream);
    if (stage == kQrPartial) return launch_one<N, true, kQrPartial>(args, stream);
    return want_v ? launch_one<N, true, kFull>(args, stream)
                  : launch_one<N, false, kFull>(args, stream);
}

}  // namespace bed
#endif
