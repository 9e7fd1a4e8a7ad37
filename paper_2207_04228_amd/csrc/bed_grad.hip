// Gradients through the eigendecomposition on the matrix cores (gfx950, wave64).
//
// For A = V diag(lambda) V^T (Sec. 3.1 Eq. (1)) and a loss with upstream
// gradients g_lambda, g_V, first-order perturbation theory gives
//   g_A = V ( diag(g_lambda) + sym(K o (V^T g_V)) ) V^T,  K_ij = 1/(lambda_j - lambda_i),
// where the coupling K is either exact with a gap floor or replaced by its
// truncated geometric series (the Taylor polynomial the paper uses for the
// backward pass, App. B / App. B.1: degree 9).  For F = V f(max(Lambda, floor)) V^T
// (Sec. 4.2-4.4, App. B.1-B.3) the same structure holds with divided
// differences of f in place of K:
//   g_A = V ( Phi o (V^T sym(G) V) ) V^T.
//
// One wavefront owns one matrix (four wavefronts, one row block of 32 each, for n > 64).
// The three (four) n x n x n products are dense
// contractions and run on v_mfma_f32_32x32x2_f32 (full fp32 operands and
// accumulation); operands are staged in LDS with an odd row stride so that row
// and column (transposed) operand reads are both conflict-free, and every
// product's result is written back to LDS in row-major order to become an
// operand of the next one.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bed_kernel.h"

namespace bed {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void wave_sync() { __builtin_amdgcn_wave_barrier(); }

// Operand and result layout of v_mfma_f32_32x32x2_f32 (A is 32x2, B is 2x32, D is 32x32):
//   A: lane l holds A[l % 32][l / 32]
//   B: lane l holds B[l / 32][l % 32]
//   D: register v (0..15) of lane l holds D[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32]
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// acc[tr][tj] = sum_k X[i][k] * Y[k][j] over k < kdim (kdim even), tiles of 32x32; the
// wavefront computes the TR row tiles that start at tile row0.
// XT / YT: the operand is stored transposed in its LDS buffer.
template <int NT, int TR, bool XT, bool YT>
__device__ __forceinline__ void product(floatx16 (&acc)[TR][NT], const float* X, const float* Y, int kdim, int lane,
                                        int row0) {
    constexpr int LD = 32 * NT + 1;
    const int lo = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int ti = 0; ti < TR; ++ti)
#pragma unroll
        for (int tj = 0; tj < NT; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ti][tj][v] = 0.f;
    for (int k0 = 0; k0 < kdim; k0 += 2) {
        const int k = k0 + hi;
        float a[TR], b[NT];
#pragma unroll
        for (int t = 0; t < TR; ++t) {
            const int r = 32 * (row0 + t) + lo;
            a[t] = XT ? X[k * LD + r] : X[r * LD + k];
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int r = 32 * t + lo;
            b[t] = YT ? Y[r * LD + k] : Y[k * LD + r];
        }
#pragma unroll
        for (int ti = 0; ti < TR; ++ti)
#pragma unroll
            for (int tj = 0; tj < NT; ++tj)
                acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
    }
}

template <int NT, int TR>
__device__ __forceinline__ void spill_to_lds(const floatx16 (&acc)[TR][NT], float* dst, int lane, int row0) {
    constexpr int LD = 32 * NT + 1;
#pragma unroll
    for (int ti = 0; ti < TR; ++ti)
#pragma unroll
        for (int tj = 0; tj < NT; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                dst[(32 * (row0 + ti) + acc_row(v, lane)) * LD + 32 * tj + (lane & 31)] = acc[ti][tj][v];
}

// Coupling of the pair (a, b) = (lambda_i, lambda_j), i != j.
__device__ __forceinline__ float coupling(float a, float b, bool j_later, int mode, int degree, float gap_floor) {
    if (mode == kGradExact) {
        const float d = b - a;
        return (fabsf(d) >= gap_floor && d != 0.f) ? 1.0f / d : 0.f;
    }
    // truncated series: with b the larger in magnitude, 1/(b - a) ~ (1/b) sum_{k<=degree} (a/b)^k;
    // mirrored otherwise.  Equal magnitudes: the later index counts as the larger, which keeps
    // K antisymmetric.
    const bool big_b = fabsf(b) > fabsf(a) || (fabsf(b) == fabsf(a) && j_later);
    const float num = big_b ? a : b, den = big_b ? b : a;
    if (den == 0.f) return 0.f;
    const float rden = 1.0f / den;
    const float rho = num * rden;
    float s = 1.f;
    for (int k = 0; k < degree; ++k) s = fmaf(s, rho, 1.f);
    const float kk = s * rden;
    return big_b ? kk : -kk;
}

// Divided difference of f~(x) = f(max(x, floor)) at (lambda_i, lambda_j); the derivative when they coincide.
__device__ __forceinline__ float divided_difference(float li, float lj, int mode, float floor) {
    const float ai = fmaxf(li, floor), aj = fmaxf(lj, floor);
    const float si = sqrtf(ai), sj = sqrtf(aj);
    // for unclamped arguments: (f(ai) - f(aj)) / (ai - aj) in a form without cancellation
    float phi = (mode == kGradSqrt) ? 1.0f / (si + sj) : -1.0f / (si * sj * (si + sj));
    if (li < floor || lj < floor) {
        // f~(li) - f~(lj) = (f(ai) - f(aj)); the denominator is the distance of the true eigenvalues
        phi = (ai == aj) ? 0.f : phi * ((ai - aj) / (li - lj));
    }
    return phi;
}

// NT tiles of 32 per side (1: n <= 32, 2: n <= 64, 4: n <= 128); NWV wavefronts per matrix,
// each owning NT / NWV row tiles of every product.
// PB > 0 (n <= PB <= 16, NT = NWV = 1): 32 / PB matrices share the wavefront as the diagonal
// blocks of one 32 x 32 operand; products of block-diagonal matrices are block diagonal, so
// the same instruction stream serves all of them.
template <int NT, int NWV, int PB>
__global__ __launch_bounds__(64 * NWV) void grad_kernel(GradArgs args) {
    static_assert(PB == 0 || (NT == 1 && NWV == 1 && 32 % PB == 0), "packing needs one 32 x 32 tile");
    constexpr int NMAT = PB ? 32 / PB : 1;       // matrices per workgroup
    constexpr int NP = 32 * NT;
    constexpr int LD = NP + 1;
    constexpr int TR = NT / NWV;
    constexpr int NTH = 64 * NWV;
    __shared__ float sV[NP * LD];      // V, row-major, zero padded
    __shared__ float sW[NP * LD];      // G, then the intermediate products
    __shared__ float sL[NP];           // eigenvalues
    __shared__ float sGl[NP];          // upstream gradient of the eigenvalues

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int row0 = (NWV == 1) ? 0 : (tid >> 6) * TR;     // first row tile of this wavefront
    const int b = blockIdx.x * NMAT;           // first matrix of this workgroup
    const int count = min(NMAT, args.batch - b);
    const int n = args.n;
    const int kdim = PB ? 32 : ((n + 1) & ~1);
    const bool ed = (args.mode == kGradExact || args.mode == kGradTaylor);
    // position p of the (padded) operand -> matrix p / PB, local index p % PB
    auto blk = [](int p) { return PB ? p / (PB ? PB : 1) : 0; };
    auto loc = [](int p) { return PB ? p % (PB ? PB : 1) : p; };
    // LDS written by one wavefront and read by another needs a workgroup barrier
    auto sync = [&]() {
        if (NWV == 1) wave_sync();
        else __syncthreads();
    };

    for (int idx = tid; idx < NP * LD; idx += NTH) {
        sV[idx] = 0.f;
        sW[idx] = 0.f;
    }
    if (tid < NP) {
        const bool ok = blk(tid) < count && loc(tid) < n;
        const size_t at = (size_t)(b + blk(tid)) * n + loc(tid);
        sL[tid] = ok ? args.evals[at] : 0.f;
        sGl[tid] = (ok && args.g_evals) ? args.g_evals[at] : 0.f;
    }
    sync();
    {
        // the workgroup's matrices are contiguous in memory: one coalesced pass over all of them
        const float* __restrict__ Vb = args.evecs + (size_t)b * n * n;
        const float* __restrict__ Gb = args.g_mat ? args.g_mat + (size_t)b * n * n : nullptr;
        const float rcp_n = 1.0f / (float)n;
        const float rcp_nn = rcp_n * rcp_n;
        for (int idx = tid; idx < count * n * n; idx += NTH) {
            const int m = PB ? (int)(((float)idx + 0.5f) * rcp_nn) : 0;
            const int r = idx - m * n * n;
            const int i = (int)(((float)r + 0.5f) * rcp_n);
            const int j = r - i * n;
            const int at = (m * PB + i) * LD + m * PB + j;
            sV[at] = Vb[idx];
            if (Gb) sW[at] = Gb[idx];
        }
    }
    sync();

    floatx16 acc[TR][NT];
    if (!ed) {
        // spectral function: T = G V first, so that C = V^T G V
        product<NT, TR, false, false>(acc, sW, sV, kdim, lane, row0);
        sync();
        spill_to_lds<NT, TR>(acc, sW, lane, row0);
        sync();
    }
    // C = V^T T  (T = g_V for the eigendecomposition itself)
    product<NT, TR, true, false>(acc, sV, sW, kdim, lane, row0);
    sync();
    spill_to_lds<NT, TR>(acc, sW, lane, row0);
    sync();
    // M: element (i, j) needs C_ij (own register), C_ji, lambda_i, lambda_j
#pragma unroll
    for (int ti = 0; ti < TR; ++ti)
#pragma unroll
        for (int tj = 0; tj < NT; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 32 * (row0 + ti) + acc_row(v, lane);
                const int j = 32 * tj + (lane & 31);
                const float cij = acc[ti][tj][v];
                const float cji = sW[j * LD + i];
                const float li = sL[i], lj = sL[j];
                float m;
                if (ed) {
                    m = (i == j) ? sGl[i]
                                 : 0.5f * coupling(li, lj, j > i, args.mode, args.degree, args.param) * (cij - cji);
                } else {
                    m = 0.5f * divided_difference(li, lj, args.mode, args.param) * (cij + cji);
                }
                const bool inside = blk(i) == blk(j) && blk(i) < count && loc(i) < n && loc(j) < n;
                acc[ti][tj][v] = inside ? m : 0.f;
            }
    sync();
    spill_to_lds<NT, TR>(acc, sW, lane, row0);
    sync();
    // U = V M
    product<NT, TR, false, false>(acc, sV, sW, kdim, lane, row0);
    sync();
    spill_to_lds<NT, TR>(acc, sW, lane, row0);
    sync();
    // g_A = U V^T
    product<NT, TR, false, true>(acc, sW, sV, kdim, lane, row0);
    float* __restrict__ Ob = args.g_A + (size_t)b * n * n;
#pragma unroll
    for (int ti = 0; ti < TR; ++ti)
#pragma unroll
        for (int tj = 0; tj < NT; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 32 * (row0 + ti) + acc_row(v, lane);
                const int j = 32 * tj + (lane & 31);
                const bool inside = blk(i) == blk(j) && blk(i) < count && loc(i) < n && loc(j) < n;
                if (inside) Ob[(size_t)blk(i) * n * n + loc(i) * n + loc(j)] = acc[ti][tj][v];
            }
}

}  // namespace

hipError_t launch_grad(const GradArgs& args, hipStream_t stream) {
    if (args.batch == 0) return hipSuccess;
    const int n = args.n, B = args.batch;
    if (n <= 4)
        return enqueue(grad_kernel<1, 1, 4>, dim3((B + 7) / 8), dim3(64), stream, args);
    else if (n <= 8)
        return enqueue(grad_kernel<1, 1, 8>, dim3((B + 3) / 4), dim3(64), stream, args);
    else if (n <= 16)
        return enqueue(grad_kernel<1, 1, 16>, dim3((B + 1) / 2), dim3(64), stream, args);
    else if (n <= 32)
        return enqueue(grad_kernel<1, 1, 0>, dim3(B), dim3(64), stream, args);
    else if (n <= 64)
        return enqueue(grad_kernel<2, 1, 0>, dim3(B), dim3(64), stream, args);
    else
        return enqueue(grad_kernel<4, 4, 0>, dim3(B), dim3(256), stream, args);
}

}  // namespace bed
