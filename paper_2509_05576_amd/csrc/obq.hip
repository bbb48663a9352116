// The baseline the method replaces (Section 4.2, first paragraphs): OBQ, every row on its own -- its own
// running inverse Hessian and its own greedy order (the not-yet-quantized weight with the smallest loss
// term of Eq. 10 first).  A measurement baseline for small layers: one workgroup per row walks the d
// steps of its row; the row's d x d inverse sits in LDS up to d = 128 and in device scratch beyond.
#include <hip/hip_ext.h>

#include "fobq_internal.h"

namespace fobq {

constexpr int OBQ_THREADS = 256;
constexpr int OBQ_LDS_D = 128;        // largest d whose running inverse fits LDS (128 KiB)

// One step's choice: the smallest loss term, the first index among equal ones.
struct ObqPick { double s; int k; };
__device__ __forceinline__ ObqPick obq_better(ObqPick a, ObqPick b)
{
    return (b.s < a.s || (b.s == a.s && b.k < a.k)) ? b : a;
}

// LDSM: the running inverse in LDS (d <= OBQ_LDS_D), else in Hscratch (d x d per workgroup); MAXD: capacity
// of the per-row arrays.  Arithmetic in the order of the definition, no contraction into fused multiply-adds:
// the greedy choice compares loss terms that can be equal to the last bit.
template <bool LDSM, int MAXD>
__global__ __launch_bounds__(OBQ_THREADS) void obq_rows_kernel(const float* __restrict__ W, int d, int gs, int G,
                                                               const double* __restrict__ Hinv0,
                                                               const double* __restrict__ scale,
                                                               const double* __restrict__ zero, double maxq, int row_begin,
                                                               double* __restrict__ Hscratch, uint8_t* __restrict__ codes,
                                                               float* __restrict__ Q, int* __restrict__ order,
                                                               double* __restrict__ lossrow, int* __restrict__ flag)
{
#pragma clang fp contract(off)
    __shared__ double Hl[LDSM ? OBQ_LDS_D * OBQ_LDS_D : 1];
    __shared__ double w[MAXD], rowj[MAXD];
    __shared__ unsigned char done[MAXD];
    __shared__ ObqPick wave_pick[OBQ_THREADS / 64];
    __shared__ double bcast[2];        // hjj, e
    __shared__ int stop;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = row_begin + (int)blockIdx.x;
    double* Hc = LDSM ? Hl : Hscratch + (int64_t)blockIdx.x * d * d;
    for (int64_t e = tid; e < (int64_t)d * d; e += OBQ_THREADS) Hc[e] = Hinv0[e];
    for (int k = tid; k < d; k += OBQ_THREADS) {
        w[k] = (double)W[(int64_t)row * d + k];
        done[k] = 0;
    }
    if (tid == 0) stop = 0;
    __syncthreads();
    const double* __restrict__ sc = scale + (int64_t)row * G;
    const double* __restrict__ ze = zero + (int64_t)row * G;
    double loss = 0.0;                 // thread 0's
    for (int t = 0; t < d; ++t) {
        // the remaining weight with the smallest (quant(w) - w)^2 / (2 [Hinv]_kk), first index among equal ones
        ObqPick best{0.0, 0x7fffffff};
        for (int k = tid; k < d; k += OBQ_THREADS) {
            if (done[k]) continue;
            const double s = sc[k / gs], z = ze[k / gs];
            const double diff = s * (grid_code(w[k], s, z, maxq) - z) - w[k];
            const ObqPick c{diff * diff / (2.0 * Hc[(int64_t)k * d + k]), k};
            best = best.k == 0x7fffffff ? c : obq_better(best, c);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            ObqPick o;
            o.s = __shfl_xor(best.s, off);
            o.k = __shfl_xor(best.k, off);
            if (o.k != 0x7fffffff) best = best.k == 0x7fffffff ? o : obq_better(best, o);
        }
        if (lane == 0) wave_pick[wave] = best;
        __syncthreads();
        ObqPick pick = wave_pick[0];
#pragma unroll
        for (int v = 1; v < OBQ_THREADS / 64; ++v) {
            const ObqPick o = wave_pick[v];
            if (o.k != 0x7fffffff) pick = pick.k == 0x7fffffff ? o : obq_better(pick, o);
        }
        const int j = pick.k;          // a remaining index exists at every step
        const double hjj = Hc[(int64_t)j * d + j];
        for (int k = tid; k < d; k += OBQ_THREADS) rowj[k] = Hc[(int64_t)j * d + k];
        if (tid == 0) {
            if (!(hjj > 0.0)) { stop = 1; atomicExch(flag, 1); }
            done[j] = 1;
            if (order) order[(int64_t)row * d + t] = j;
            const double s = sc[j / gs], z = ze[j / gs];
            const double c = grid_code(w[j], s, z, maxq);
            const double q = s * (c - z);
            codes[(int64_t)row * d + j] = (uint8_t)c;
            Q[(int64_t)row * d + j] = (float)q;
            const double diff = w[j] - q;
            loss += diff * diff / (2.0 * hjj);
            bcast[0] = hjj;
            bcast[1] = diff / hjj;
        }
        __syncthreads();
        if (stop) break;               // the same for every thread: a pivot that is not positive
        const double e = bcast[1];
        // Eq. 9 / 11 on the rest of the row, Eq. 12 on the row's own inverse
        for (int k = tid; k < d; k += OBQ_THREADS)
            if (!done[k]) w[k] -= e * rowj[k];
        for (int a = wave; a < d; a += OBQ_THREADS / 64) {
            if (done[a]) continue;
            const double f = rowj[a] / hjj;
            double* __restrict__ ra = Hc + (int64_t)a * d;
            for (int b = lane; b < d; b += 64)
                if (!done[b]) ra[b] -= f * rowj[b];
        }
        __syncthreads();
    }
    if (tid == 0) lossrow[row] = loss;
}

hipError_t launch_obq_rows(hipStream_t s, const float* W, int d, int bits, int group, const double* Hinv0, const double* scale,
                           const double* zero, int row_begin, int rows, double* Hscratch, uint8_t* codes, float* Q, int* order,
                           double* lossrow, int* flag)
{
    const int gs = group > 0 ? group : d;
    const int G = group > 0 ? d / group : 1;
    const double maxq = (double)((1 << bits) - 1);
    if (d <= OBQ_LDS_D)
        hipLaunchKernelGGL((obq_rows_kernel<true, OBQ_LDS_D>), dim3(rows), dim3(OBQ_THREADS), 0, s, W, d, gs, G, Hinv0, scale, zero,
                           maxq, row_begin, Hscratch, codes, Q, order, lossrow, flag);
    else
        hipLaunchKernelGGL((obq_rows_kernel<false, OBQ_MAX_D>), dim3(rows), dim3(OBQ_THREADS), 0, s, W, d, gs, G, Hinv0, scale, zero,
                           maxq, row_begin, Hscratch, codes, Q, order, lossrow, flag);
    return hipGetLastError();
}

// bytes of device scratch per row of a launch (0: the inverse lives in LDS)
size_t obq_scratch_per_row(int d) { return d <= OBQ_LDS_D ? 0 : (size_t)d * d * sizeof(double); }

}  // namespace fobq
