// Generic fp64 GEMM on the CDNA matrix cores (v_mfma_f64_16x16x4_f64), used for
// the rank-B (deferred) updates of the path that are not fused into a
// factorization kernel: the triangular inverse, L^-T L^-1, the general-block
// form of the shared-Hinv elimination (Eq. 12 applied B columns at a time) and
// the deferred weight compensation (Eq. 9 / 11 applied B columns at a time).
//
// One workgroup = 512 threads = 8 wavefronts computes a 64 x 64 tile of C; each wavefront owns a
// 16 x 32 part = 1 x 2 MFMA tiles (two wavefronts per SIMD: one alone issues an fp64 MFMA only every
// ~140 cycles, two interleave to the pipe's rate of one per ~64).  K is walked in chunks of
// 64: a chunk of both operand tiles is fetched with one round of loads (lane index
// along the contiguous dimension), held in registers while the previous chunk is
// multiplied out of LDS (32 MFMAs per wavefront, about one memory round trip), and
// then stored to LDS.  The C tile is prefetched with the first chunk.  The rank-64
// updates (K = 64) are latency bound -- a few tiles per launch -- so a single
// exposed memory round trip is what matters there.
#include <hip/hip_ext.h>

#include "fobq_internal.h"

namespace fobq {

typedef double d4 __attribute__((ext_vector_type(4)));

constexpr int GT = 512;   // threads per workgroup
constexpr int TM = 64, TN = 64, K1 = 64, K1_LD = K1 + 2;   // +2 doubles: conflict-free 8-byte fragment reads

template <bool TA, bool TB>
__global__ __launch_bounds__(GT) void gemm64_kernel(GemmP p)
{
    const int b = blockIdx.z;
    int M = p.M, K = p.K;
    const int N = p.N;
    if (p.Mtot >= 0) M = min(M, p.Mtot - b * p.mstep);
    if (p.Ktot >= 0) K = min(K, p.Ktot - b * p.kstep);
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    if (M <= 0 || N <= 0 || m0 >= M || n0 >= N) return;
    if (p.cmode == CMODE_LOWER && n0 > m0 + TM - 1) return;
    if (p.cmode == CMODE_UPPER && n0 + TN - 1 < m0) return;
    int k_lo = 0, k_hi = K;
    if (p.kmode == KMODE_GE_MAX_MN) k_lo = max(m0, n0);      // multiples of 64
    else if (p.kmode == KMODE_GE_N) k_lo = n0;
    else if (p.kmode == KMODE_LT_M) k_hi = min(K, m0 + TM);
    k_lo = max(k_lo, p.kmin);

    const double* __restrict__ A = p.A + (int64_t)b * p.sA;
    const double* __restrict__ B = p.B + (int64_t)b * p.sB;
    double* C = p.C + (int64_t)b * p.sC;
    double* C2 = p.C2 ? p.C2 + (int64_t)b * p.sC : nullptr;

    __shared__ double As[TM][K1_LD];
    __shared__ double Bs[TN][K1_LD];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wn = wave & 1;     // 16-row slice, 32-column half of the tile

    double ra[8], rb[8];
    auto gload = [&](int kk) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int x = lane, y = wave + 8 * u;    // x: contiguous index, y: strided index (0..63)
            if (!TA) { const int gm = m0 + y, gk = kk + x; ra[u] = (gm < M && gk < k_hi) ? A[(int64_t)gm * p.lda + gk] : 0.0; }
            else     { const int gm = m0 + x, gk = kk + y; ra[u] = (gm < M && gk < k_hi) ? A[(int64_t)gk * p.lda + gm] : 0.0; }
            if (!TB) { const int gn = n0 + x, gk = kk + y; rb[u] = (gn < N && gk < k_hi) ? B[(int64_t)gk * p.ldb + gn] : 0.0; }
            else     { const int gn = n0 + y, gk = kk + x; rb[u] = (gn < N && gk < k_hi) ? B[(int64_t)gn * p.ldb + gk] : 0.0; }
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int x = lane, y = wave + 8 * u;
            if (!TA) As[y][x] = ra[u]; else As[x][y] = ra[u];
            if (!TB) Bs[x][y] = rb[u]; else Bs[y][x] = rb[u];
        }
    };

    if (k_lo < k_hi) gload(k_lo);
    d4 cin[2];
    const bool use_c = p.beta != 0.0 && (p.beta_ncols < 0 || n0 < p.beta_ncols);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gm = m0 + wr * 16 + 4 * v + (lane >> 4);
            const int gn = n0 + wn * 32 + j * 16 + (lane & 15);
            cin[j][v] = (use_c && gm < M && gn < N) ? C[(int64_t)gm * p.ldc + gn] : 0.0;
        }

    d4 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[j] = d4{0.0, 0.0, 0.0, 0.0};

    for (int kk = k_lo; kk < k_hi; kk += K1) {
        __syncthreads();                      // previous chunk fully consumed
        sstore();
        __syncthreads();
        if (kk + K1 < k_hi) gload(kk + K1);   // in flight while this chunk is multiplied
        const int ksteps = (min(K1, k_hi - kk) + 3) / 4;
        for (int ks = 0; ks < ksteps; ++ks) {
            const double a = As[wr * 16 + (lane & 15)][ks * 4 + (lane >> 4)];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, Bs[wn * 32 + j * 16 + (lane & 15)][ks * 4 + (lane >> 4)],
                                                              acc[j], 0, 0, 0);
        }
    }

    // accumulator layout of v_mfma_f64_16x16x4_f64: lane l, element v holds D[4 * v + l / 16][l % 16]
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gm = m0 + wr * 16 + 4 * v + (lane >> 4);
            const int gn = n0 + wn * 32 + j * 16 + (lane & 15);
            if (gm < M && gn < N) {
                const int64_t off = (int64_t)gm * p.ldc + gn;
                double r = p.alpha * acc[j][v];
                if (use_c) r += p.beta * cin[j][v];
                C[off] = r;
                if (C2) C2[off] = p.rowscale[gm] * r;
            }
        }
}

hipError_t gemm64(hipStream_t s, const GemmP& p, bool TA, bool TB, hipEvent_t done)
{
    if (p.M <= 0 || p.N <= 0 || p.batches <= 0) {
        if (done) return hipEventRecord(done, s);
        return hipSuccess;
    }
    dim3 grid((p.N + TN - 1) / TN, (p.M + TM - 1) / TM, p.batches), block(GT);
    // `done` rides on the launch as its stop event (see fobq_internal.h)
    if (!TA && !TB) hipExtLaunchKernelGGL((gemm64_kernel<false, false>), grid, block, 0, s, nullptr, done, 0, p);
    else if (!TA && TB) hipExtLaunchKernelGGL((gemm64_kernel<false, true>), grid, block, 0, s, nullptr, done, 0, p);
    else if (TA && !TB) hipExtLaunchKernelGGL((gemm64_kernel<true, false>), grid, block, 0, s, nullptr, done, 0, p);
    else hipExtLaunchKernelGGL((gemm64_kernel<true, true>), grid, block, 0, s, nullptr, done, 0, p);
    return hipGetLastError();
}

}  // namespace fobq
