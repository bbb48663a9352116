// Hessian of the layer objective (Section 3, Eq. 2): H = (2/N) X X^T.
//
// xxt_kernel: fp32 X is read from HBM, staged through LDS as fp32, widened to
// fp64 when the MFMA fragments are formed (products of two fp32 values are
// exact in fp64), and accumulated with v_mfma_f64_16x16x4_f64.  Only tiles on
// or below the diagonal are computed.  The calibration dimension is split over
// blockIdx.y; each split owns its own d x d slab of partial sums, so the
// result does not depend on the order in which workgroups finish.
#include "fobq_internal.h"

namespace fobq {

typedef double d4 __attribute__((ext_vector_type(4)));

constexpr int XT = 128;          // tile edge
constexpr int XK = 32;           // calibration columns per LDS stage
constexpr int XLD = XK + 4;      // fp32 row stride in LDS: 16B-aligned rows, conflict-free fragment reads

__device__ __forceinline__ void tile_decode(int t, int& I, int& J)
{
    // t = I (I + 1) / 2 + J, 0 <= J <= I
    int i = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while ((i + 1) * (i + 2) / 2 <= t) ++i;
    while (i * (i + 1) / 2 > t) --i;
    I = i;
    J = t - i * (i + 1) / 2;
}

template <bool VEC>
__global__ __launch_bounds__(256) void xxt_kernel(const float* __restrict__ X, int64_t ld, int d, int64_t n,
                                                  double* __restrict__ Hpart, int64_t kper)
{
    int I, J;
    tile_decode(blockIdx.x, I, J);
    const int split = blockIdx.y;
    const int64_t k_begin = (int64_t)split * kper;
    const int64_t k_end = min(n, k_begin + kper);
    if (k_begin >= k_end) return;
    const int i0 = I * XT, j0 = J * XT;

    __shared__ float As[XT][XLD];
    __shared__ float Bs[XT][XLD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = tid >> 3;          // 0..31: row within a group of 32 rows
    const int lk = (tid & 7) * 4;     // 0..28: first of 4 consecutive calibration columns

    float4 pa[4], pb[4];
    auto gload = [&](int64_t kk) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ra = i0 + lr + 32 * u, rb = j0 + lr + 32 * u;
            const int64_t k = kk + lk;
            float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va;
            if (VEC && k + 3 < k_end) {
                if (ra < d) va = *reinterpret_cast<const float4*>(X + (int64_t)ra * ld + k);
                if (rb < d) vb = *reinterpret_cast<const float4*>(X + (int64_t)rb * ld + k);
            } else {
                if (ra < d) {
                    const float* src = X + (int64_t)ra * ld;
                    if (k + 0 < k_end) va.x = src[k + 0];
                    if (k + 1 < k_end) va.y = src[k + 1];
                    if (k + 2 < k_end) va.z = src[k + 2];
                    if (k + 3 < k_end) va.w = src[k + 3];
                }
                if (rb < d) {
                    const float* src = X + (int64_t)rb * ld;
                    if (k + 0 < k_end) vb.x = src[k + 0];
                    if (k + 1 < k_end) vb.y = src[k + 1];
                    if (k + 2 < k_end) vb.z = src[k + 2];
                    if (k + 3 < k_end) vb.w = src[k + 3];
                }
            }
            pa[u] = va;
            pb[u] = vb;
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *reinterpret_cast<float4*>(&As[lr + 32 * u][lk]) = pa[u];
            *reinterpret_cast<float4*>(&Bs[lr + 32 * u][lk]) = pb[u];
        }
    };

    d4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = d4{0.0, 0.0, 0.0, 0.0};

    gload(k_begin);
    for (int64_t kk = k_begin; kk < k_end; kk += XK) {
        __syncthreads();          // previous stage fully consumed
        sstore();
        __syncthreads();
        if (kk + XK < k_end) gload(kk + XK);
#pragma unroll
        for (int ks = 0; ks < XK / 4; ++ks) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = (double)As[wm * 64 + i * 16 + (lane & 15)][ks * 4 + (lane >> 4)];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = (double)Bs[wn * 64 + j * 16 + (lane & 15)][ks * 4 + (lane >> 4)];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }

    double* __restrict__ out = Hpart + (int64_t)split * d * d;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gr = i0 + wm * 64 + i * 16 + 4 * v + (lane >> 4);
                const int gc = j0 + wn * 64 + j * 16 + (lane & 15);
                if (gr < d && gc < d) out[(int64_t)gr * d + gc] += acc[i][j][v];
            }
}

int xxt_pick_splits(int d)
{
    const int nt = (d + XT - 1) / XT;
    const int tiles = nt * (nt + 1) / 2;
    int s = (1024 + tiles - 1) / tiles;   // aim at ~4 workgroups per compute unit
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return s;
}

hipError_t launch_xxt(hipStream_t s, const float* X, int64_t ld, int d, int64_t n, double* Hpart, int splits)
{
    const int nt = (d + XT - 1) / XT;
    const int tiles = nt * (nt + 1) / 2;
    int64_t kper = (n + splits - 1) / splits;
    kper = (kper + XK - 1) / XK * XK;
    dim3 grid(tiles, splits), block(256);
    const bool vec = (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    if (vec) hipLaunchKernelGGL((xxt_kernel<true>), grid, block, 0, s, X, ld, d, n, Hpart, kper);
    else     hipLaunchKernelGGL((xxt_kernel<false>), grid, block, 0, s, X, ld, d, n, Hpart, kper);
    return hipGetLastError();
}

// H[a][b] = H[b][a] = factor * sum_s Hpart[s][a][b]   for b <= a (lower slabs hold the sums)
__global__ __launch_bounds__(256) void hessian_finalize_kernel(const double* __restrict__ Hpart, int splits, int d,
                                                               double factor, double* __restrict__ H)
{
    const int b = blockIdx.x * 16 + (threadIdx.x & 15);
    const int a = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (a >= d || b >= d || b > a) return;
    double s = 0.0;
    for (int k = 0; k < splits; ++k) s += Hpart[(int64_t)k * d * d + (int64_t)a * d + b];
    s *= factor;
    H[(int64_t)a * d + b] = s;
    H[(int64_t)b * d + a] = s;
}

hipError_t launch_hessian_finalize(hipStream_t s, const double* Hpart, int splits, int d, double factor, double* H)
{
    dim3 grid((d + 15) / 16, (d + 15) / 16), block(256);
    hipLaunchKernelGGL(hessian_finalize_kernel, grid, block, 0, s, Hpart, splits, d, factor, H);
    return hipGetLastError();
}

// lambda = damp * mean(diag H) + damp_abs   (Section 6.1: damping added to the diagonal)
__global__ __launch_bounds__(256) void damp_lambda_kernel(const double* __restrict__ H, int d, double damp,
                                                          double damp_abs, double* __restrict__ lam)
{
    __shared__ double part[256];
    double s = 0.0;
    for (int a = threadIdx.x; a < d; a += 256) s += H[(int64_t)a * d + a];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *lam = damp * (part[0] / (double)d) + damp_abs;
}

__global__ __launch_bounds__(256) void damp_copy_kernel(const double* __restrict__ H, int d,
                                                        const double* __restrict__ lam, double* __restrict__ Hd)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)d * d;
    if (idx >= total) return;
    const int a = (int)(idx / d), b = (int)(idx % d);
    double v = H[idx];
    if (a == b) v += *lam;
    Hd[idx] = v;
}

hipError_t launch_damp(hipStream_t s, const double* H, int d, double damp, double damp_abs, double* Hd, double* lam_out)
{
    hipLaunchKernelGGL(damp_lambda_kernel, dim3(1), dim3(256), 0, s, H, d, damp, damp_abs, lam_out);
    const int64_t total = (int64_t)d * d;
    hipLaunchKernelGGL(damp_copy_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, H, d, lam_out, Hd);
    return hipGetLastError();
}

}  // namespace fobq
