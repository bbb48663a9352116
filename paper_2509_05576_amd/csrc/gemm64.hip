// Generic fp64 GEMM on the CDNA matrix cores (v_mfma_f64_16x16x4_f64), used for
// every rank-B (deferred) update of the path: Cholesky panel/trailing updates,
// the triangular inverse, L^-T L^-1, the blocked form of the shared-Hinv
// elimination (Eq. 12 applied B columns at a time) and of the weight
// compensation (Eq. 9 / 11 applied B columns at a time).
//
// One workgroup = 256 threads = 4 wavefronts computes a 64 x 64 tile of C; each
// wavefront owns a 32 x 32 sub-tile = 2 x 2 MFMA tiles.  K is walked in chunks
// of 16 staged through LDS (double-buffered, one barrier per chunk).
#include "fobq_internal.h"

namespace fobq {

typedef double d4 __attribute__((ext_vector_type(4)));

constexpr int TM = 64, TN = 64, KC = 16, LDS_LD = KC + 2;  // +2 doubles: conflict-free b64 fragment reads

template <bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm64_kernel(GemmP p)
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
    if (p.kmode == KMODE_GE_MAX_MN) k_lo = max(m0, n0);
    else if (p.kmode == KMODE_GE_N) k_lo = n0;
    else if (p.kmode == KMODE_LT_M) k_hi = min(K, m0 + TM);
    k_lo &= ~(KC - 1);

    const double* __restrict__ A = p.A + (int64_t)b * p.sA;
    const double* __restrict__ B = p.B + (int64_t)b * p.sB;
    double* C = p.C + (int64_t)b * p.sC;
    double* C2 = p.C2 ? p.C2 + (int64_t)b * p.sC : nullptr;

    __shared__ double As[2][TM][LDS_LD];
    __shared__ double Bs[2][TN][LDS_LD];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // per-thread staging slots: 4 elements of the A tile and 4 of the B tile
    double ra[4], rb[4];
    auto gload = [&](int kk) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (!TA) {   // A[m][k], k contiguous
                const int r = (tid >> 4) + 16 * u, k = tid & 15;
                const int gm = m0 + r, gk = kk + k;
                ra[u] = (gm < M && gk < k_hi) ? A[(int64_t)gm * p.lda + gk] : 0.0;
            } else {     // A[k][m], m contiguous
                const int k = (tid >> 6) + 4 * u, r = tid & 63;
                const int gm = m0 + r, gk = kk + k;
                ra[u] = (gm < M && gk < k_hi) ? A[(int64_t)gk * p.lda + gm] : 0.0;
            }
            if (!TB) {   // B[k][n], n contiguous
                const int k = (tid >> 6) + 4 * u, c = tid & 63;
                const int gn = n0 + c, gk = kk + k;
                rb[u] = (gn < N && gk < k_hi) ? B[(int64_t)gk * p.ldb + gn] : 0.0;
            } else {     // B[n][k], k contiguous
                const int c = (tid >> 4) + 16 * u, k = tid & 15;
                const int gn = n0 + c, gk = kk + k;
                rb[u] = (gn < N && gk < k_hi) ? B[(int64_t)gn * p.ldb + gk] : 0.0;
            }
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (!TA) As[buf][(tid >> 4) + 16 * u][tid & 15] = ra[u];
            else     As[buf][tid & 63][(tid >> 6) + 4 * u] = ra[u];
            if (!TB) Bs[buf][tid & 63][(tid >> 6) + 4 * u] = rb[u];
            else     Bs[buf][(tid >> 4) + 16 * u][tid & 15] = rb[u];
        }
    };

    d4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = d4{0.0, 0.0, 0.0, 0.0};

    if (k_lo < k_hi) {
        gload(k_lo);
        sstore(0);
        __syncthreads();
        int cur = 0;
        for (int kk = k_lo; kk < k_hi; kk += KC) {
            const bool more = kk + KC < k_hi;
            if (more) gload(kk + KC);
#pragma unroll
            for (int ks = 0; ks < KC / 4; ++ks) {
                double a[2], bb[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) a[i] = As[cur][wm * 32 + i * 16 + (lane & 15)][ks * 4 + (lane >> 4)];
#pragma unroll
                for (int j = 0; j < 2; ++j) bb[j] = Bs[cur][wn * 32 + j * 16 + (lane & 15)][ks * 4 + (lane >> 4)];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], bb[j], acc[i][j], 0, 0, 0);
            }
            if (more) sstore(cur ^ 1);
            __syncthreads();
            cur ^= 1;
        }
    }

    // accumulator layout of v_mfma_f64_16x16x4_f64: lane l, element v holds
    // D[4 * v + l / 16][l % 16]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = m0 + wm * 32 + i * 16 + 4 * v + (lane >> 4);
                const int gn = n0 + wn * 32 + j * 16 + (lane & 15);
                if (gm < M && gn < N) {
                    const int64_t off = (int64_t)gm * p.ldc + gn;
                    double r = p.alpha * acc[i][j][v];
                    if (p.beta != 0.0) r += p.beta * C[off];
                    C[off] = r;
                    if (C2) C2[off] = p.rowscale[gm] * r;
                }
            }
}

// Single-stage variant for K <= 64 (the rank-64 panel and trailing updates): the whole
// K extent of both operand tiles is fetched with one round of loads, C is prefetched at
// the same time, and the 16 k-steps run out of LDS with a single barrier.  These launches
// are latency bound (a few tiles each), so one exposed memory round trip instead of four
// is what matters.  K-range restrictions (kmode) are ignored: the operands hold explicit
// zeros where a restriction would skip.
constexpr int K1 = 64, K1_LD = K1 + 2;

template <bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm64_k64_kernel(GemmP p)
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

    const double* __restrict__ A = p.A + (int64_t)b * p.sA;
    const double* __restrict__ B = p.B + (int64_t)b * p.sB;
    double* C = p.C + (int64_t)b * p.sC;
    double* C2 = p.C2 ? p.C2 + (int64_t)b * p.sC : nullptr;

    __shared__ double As[TM][K1_LD];
    __shared__ double Bs[TN][K1_LD];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // one round of loads: lane index runs along the contiguous dimension of each operand
    double ra[16], rb[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int x = lane, y = wave + 4 * u;        // x: contiguous index, y: strided index (0..63)
        if (!TA) { const int gm = m0 + y, gk = x; ra[u] = (gm < M && gk < K) ? A[(int64_t)gm * p.lda + gk] : 0.0; }
        else     { const int gm = m0 + x, gk = y; ra[u] = (gm < M && gk < K) ? A[(int64_t)gk * p.lda + gm] : 0.0; }
        if (!TB) { const int gn = n0 + x, gk = y; rb[u] = (gn < N && gk < K) ? B[(int64_t)gk * p.ldb + gn] : 0.0; }
        else     { const int gn = n0 + y, gk = x; rb[u] = (gn < N && gk < K) ? B[(int64_t)gn * p.ldb + gk] : 0.0; }
    }
    d4 cin[2][2];
    const bool use_c = p.beta != 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = m0 + wm * 32 + i * 16 + 4 * v + (lane >> 4);
                const int gn = n0 + wn * 32 + j * 16 + (lane & 15);
                cin[i][j][v] = (use_c && gm < M && gn < N) ? C[(int64_t)gm * p.ldc + gn] : 0.0;
            }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int x = lane, y = wave + 4 * u;
        if (!TA) As[y][x] = ra[u]; else As[x][y] = ra[u];
        if (!TB) Bs[x][y] = rb[u]; else Bs[y][x] = rb[u];
    }
    __syncthreads();

    d4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = d4{0.0, 0.0, 0.0, 0.0};
    const int ksteps = (K + 3) / 4;
    for (int ks = 0; ks < ksteps; ++ks) {
        double a[2], bb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = As[wm * 32 + i * 16 + (lane & 15)][ks * 4 + (lane >> 4)];
#pragma unroll
        for (int j = 0; j < 2; ++j) bb[j] = Bs[wn * 32 + j * 16 + (lane & 15)][ks * 4 + (lane >> 4)];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], bb[j], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = m0 + wm * 32 + i * 16 + 4 * v + (lane >> 4);
                const int gn = n0 + wn * 32 + j * 16 + (lane & 15);
                if (gm < M && gn < N) {
                    const int64_t off = (int64_t)gm * p.ldc + gn;
                    double r = p.alpha * acc[i][j][v];
                    if (use_c) r += p.beta * cin[i][j][v];
                    C[off] = r;
                    if (C2) C2[off] = p.rowscale[gm] * r;
                }
            }
}

hipError_t gemm64(hipStream_t s, const GemmP& p, bool TA, bool TB)
{
    if (p.M <= 0 || p.N <= 0 || p.batches <= 0) return hipSuccess;
    dim3 grid((p.N + TN - 1) / TN, (p.M + TM - 1) / TM, p.batches), block(256);
    if (p.K <= K1) {
        if (!TA && !TB) hipLaunchKernelGGL((gemm64_k64_kernel<false, false>), grid, block, 0, s, p);
        else if (!TA && TB) hipLaunchKernelGGL((gemm64_k64_kernel<false, true>), grid, block, 0, s, p);
        else if (TA && !TB) hipLaunchKernelGGL((gemm64_k64_kernel<true, false>), grid, block, 0, s, p);
        else hipLaunchKernelGGL((gemm64_k64_kernel<true, true>), grid, block, 0, s, p);
        return hipGetLastError();
    }
    if (!TA && !TB) hipLaunchKernelGGL((gemm64_kernel<false, false>), grid, block, 0, s, p);
    else if (!TA && TB) hipLaunchKernelGGL((gemm64_kernel<false, true>), grid, block, 0, s, p);
    else if (TA && !TB) hipLaunchKernelGGL((gemm64_kernel<true, false>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((gemm64_kernel<true, true>), grid, block, 0, s, p);
    return hipGetLastError();
}

}  // namespace fobq
