// Grid, sensitivity, ordering, permutation and the column loop (Section 4.2).
#include <hip/hip_ext.h>

#include "fobq_internal.h"

namespace fobq {

// ---------------------------------------------------------------------------
// Min-max grid per (row, group) from the original W (Section 3, "fixed grid of
// width Delta"): lo = min(min w, 0), hi = max(max w, 0), scale = (hi - lo) / maxq,
// zero = rint(-lo / scale); an all-zero group gets scale 1, zero 0.
// One wavefront per (row, group); min / max by wavefront shuffles.
__global__ __launch_bounds__(256) void grid_kernel(const float* __restrict__ W, int R, int d, int gs, int G,
                                                   double maxq, double* __restrict__ scale, double* __restrict__ zero,
                                                   float* __restrict__ scales_out, float* __restrict__ zeros_out)
{
    const int lane = threadIdx.x & 63;
    const int64_t pair = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= (int64_t)R * G) return;
    const int i = (int)(pair / G), g = (int)(pair % G);
    const float* __restrict__ src = W + (int64_t)i * d + (int64_t)g * gs;
    float lo = 0.f, hi = 0.f;
    for (int j = lane; j < gs; j += 64) {
        const float w = src[j];
        lo = fminf(lo, w);
        hi = fmaxf(hi, w);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
    }
    if (lane == 0) {
        double s = 1.0, z = 0.0;
        if (hi != lo) {
            s = ((double)hi - (double)lo) / maxq;
            z = rint(-(double)lo / s);
        }
        scale[pair] = s;
        zero[pair] = z;
        if (scales_out) scales_out[pair] = (float)s;
        if (zeros_out) zeros_out[pair] = (float)z;
    }
}

hipError_t launch_grid(hipStream_t s, const float* W, int R, int d, int bits, int group,
                       double* scale, double* zero, float* scales_out, float* zeros_out)
{
    const int gs = group > 0 ? group : d;
    const int G = group > 0 ? d / group : 1;
    const int64_t pairs = (int64_t)R * G;
    const double maxq = (double)((1 << bits) - 1);
    hipLaunchKernelGGL(grid_kernel, dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, s, W, R, d, gs, G, maxq,
                       scale, zero, scales_out, zeros_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Column scores (Eq. 10 summed over rows, Section 4.2 steps 1-2):
//   S_j = sum_i (quant(w_ij) - w_ij)^2 / (2 [Hinv]_jj)
// Pass 1: thread = column, block row-chunk c sums rows [c*RC, (c+1)*RC).
// Pass 2: chunks are added in index order, then divided by 2 [Hinv]_jj.
constexpr int SENS_RC = 64;

// kind 0 / 1: sum of squared quantization errors ("sensi" divides by 2 [Hinv]_jj in pass 2, "err" does
// not); kind 2: sum of squared weights ("w").  Section 4.1, Table 3.
__global__ __launch_bounds__(256) void sens_partial_kernel(const float* __restrict__ W, int R, int d, int gs, int G,
                                                           double maxq, const double* __restrict__ scale,
                                                           const double* __restrict__ zero, double* __restrict__ Spart,
                                                           int kind)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= d) return;
    const int g = j / gs;
    const int r0 = blockIdx.y * SENS_RC, r1 = min(R, r0 + SENS_RC);
    double acc = 0.0;
    for (int i = r0; i < r1; ++i) {
        const double w = (double)W[(int64_t)i * d + j];
        const double s = scale[(int64_t)i * G + g], z = zero[(int64_t)i * G + g];
        const double q = s * (grid_code(w, s, z, maxq) - z);
        acc += (kind == 2) ? w * w : (q - w) * (q - w);
    }
    Spart[(int64_t)blockIdx.y * d + j] = acc;
}

__global__ __launch_bounds__(256) void sens_reduce_kernel(const double* __restrict__ Spart, int chunks, int d,
                                                          const double* __restrict__ Hinv, double* __restrict__ S,
                                                          int kind)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= d) return;
    double acc = 0.0;
    for (int c = 0; c < chunks; ++c) acc += Spart[(int64_t)c * d + j];
    S[j] = (kind == 0) ? acc / (2.0 * Hinv[(int64_t)j * d + j]) : acc;
}

int sens_chunks(int R) { return (R + SENS_RC - 1) / SENS_RC; }

// pass 1: per-chunk sums over the rows (needs W and the grid only)
hipError_t launch_sens_partial(hipStream_t s, const float* W, int R, int d, int bits, int group,
                               const double* scale, const double* zero, double* Spart, int chunks, int kind,
                               hipEvent_t done)
{
    const int gs = group > 0 ? group : d;
    const int G = group > 0 ? d / group : 1;
    const double maxq = (double)((1 << bits) - 1);
    hipExtLaunchKernelGGL(sens_partial_kernel, dim3((d + 255) / 256, chunks), dim3(256), 0, s, nullptr, done, 0, W, R, d,
                          gs, G, maxq, scale, zero, Spart, kind);
    return hipGetLastError();
}

// pass 2: sum of the chunks, and for "sensi" the division by 2 [Hinv]_jj (Hinv: d x d, its diagonal is read)
hipError_t launch_sens_reduce(hipStream_t s, const double* Spart, int chunks, int d, const double* Hinv, double* S,
                              int kind)
{
    hipLaunchKernelGGL(sens_reduce_kernel, dim3((d + 255) / 256), dim3(256), 0, s, Spart, chunks, d, Hinv, S, kind);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Order (Section 4.2 step 3): descending S (or ascending), equal scores keep index order.
// rank_j = #{k : S_k before S_j or (S_k == S_j and k < j)}; perm[rank_j] = j.  Ascending order
// is the descending order of the negated keys.
// A score that is not finite compares as -infinity so that perm stays a permutation.
__device__ __forceinline__ double sort_key(double v)
{
    return (!(v == v) || v > 1.0e300 || v < -1.0e300) ? -1.0e308 : v;
}

// One workgroup ranks 32 columns j against all d columns k (staged through LDS 256 at a time), eight
// threads per column each taking every eighth k, and writes both directions of the order: no zero-filled
// counters, no atomics, no second pass.
__global__ __launch_bounds__(256) void rank_sort_kernel(const double* __restrict__ S, int d, int* __restrict__ perm,
                                                        int* __restrict__ invperm, double sign)
{
    __shared__ double tile[256];
    __shared__ int part_cnt[8][32];
    const int jl = threadIdx.x & 31, part = threadIdx.x >> 5;
    const int j = blockIdx.x * 32 + jl;
    const double sj = (j < d) ? sort_key(sign * S[j]) : 0.0;
    int cnt = 0;
    for (int base = 0; base < d; base += 256) {
        const int k = base + threadIdx.x;
        __syncthreads();
        tile[threadIdx.x] = (k < d) ? sort_key(sign * S[k]) : 0.0;
        __syncthreads();
        const int lim = min(256, d - base);
        // columns before j win ties: up to j - base of the tile's entries count when equal
        const int before = min(max(j - base, 0), lim);
#pragma unroll 4
        for (int u = part; u < lim; u += 8) {
            const double v = tile[u];
            cnt += (v > sj || (v == sj && u < before)) ? 1 : 0;
        }
    }
    part_cnt[part][jl] = cnt;
    __syncthreads();
    if (part == 0 && j < d) {
        int r = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) r += part_cnt[q][jl];
        r = min(max(r, 0), d - 1);
        perm[r] = j;
        invperm[j] = r;
    }
}

hipError_t launch_rank_sort(hipStream_t s, const double* S, int d, int* perm, int* invperm, int ascending)
{
    hipLaunchKernelGGL(rank_sort_kernel, dim3((d + 31) / 32), dim3(256), 0, s, S, d, perm, invperm,
                       ascending ? -1.0 : 1.0);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void iota_kernel(int d, int* __restrict__ perm, int* __restrict__ invperm)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j < d) { perm[j] = j; invperm[j] = j; }
}

hipError_t launch_iota(hipStream_t s, int d, int* perm, int* invperm)
{
    hipLaunchKernelGGL(iota_kernel, dim3((d + 255) / 256), dim3(256), 0, s, d, perm, invperm);
    return hipGetLastError();
}

// Custom order: copy, and verify that it is a permutation of 0..d-1.  Entries out
// of range are replaced by a valid index so that later gathers stay in bounds;
// the flag makes the call fail.
__global__ __launch_bounds__(256) void perm_copy_kernel(const int* __restrict__ perm_in, int d, int* __restrict__ perm,
                                                        int* __restrict__ invperm, int* __restrict__ flag)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= d) return;
    int j = perm_in[t];
    if (j < 0 || j >= d) { *flag = 1; j = t; }
    perm[t] = j;
    invperm[j] = t;     // duplicates: last writer wins, detected by the check pass
}

__global__ __launch_bounds__(256) void perm_check_kernel(const int* __restrict__ perm, const int* __restrict__ invperm,
                                                         int d, int* __restrict__ flag)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= d) return;
    const int j = perm[t];
    if (j < 0 || j >= d || invperm[j] != t) *flag = 1;
}

hipError_t launch_check_perm(hipStream_t s, const int* perm_in, int d, int* perm, int* invperm, int* flag)
{
    // invperm starts at -1 so that an index that never appears is detected
    (void)launch_fill_i32(s, invperm, d, -1);
    hipLaunchKernelGGL(perm_copy_kernel, dim3((d + 255) / 256), dim3(256), 0, s, perm_in, d, perm, invperm, flag);
    hipLaunchKernelGGL(perm_check_kernel, dim3((d + 255) / 256), dim3(256), 0, s, perm, invperm, d, flag);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Put W and Hinv into processing order (Section 4.2 step 3):
//   Wp[i][t] = W[i][perm[t]] (widened),  A[a][b] = Hinv[perm[a]][perm[b]]
// Hinv is read from its upper triangle.  Both gathers in one launch: blockIdx.x < R walks the
// rows of W, the rest the rows of Hinv (blockIdx.y: 256 columns).
__global__ __launch_bounds__(256) void gather_kernel(const float* __restrict__ W, int R, int d,
                                                     const int* __restrict__ perm, const double* __restrict__ Hu,
                                                     double* __restrict__ Wp, double* __restrict__ A)
{
    const int t = blockIdx.y * 256 + threadIdx.x;
    if (t >= d) return;
    int pt = perm[t];
    pt = min(max(pt, 0), d - 1);
    if ((int)blockIdx.x < R) {
        const int i = blockIdx.x;
        Wp[(int64_t)i * d + t] = (double)W[(int64_t)i * d + pt];
        return;
    }
    // the elimination maintains (and reads) the upper triangle only, plus the whole 64 x 64 tiles on the
    // diagonal that its tile updates load and store
    const int a = (int)blockIdx.x - R;
    if (t < (a & ~63)) return;
    int pa = perm[a];
    pa = min(max(pa, 0), d - 1);
    const int lo = min(pa, pt), hi = max(pa, pt);
    A[(int64_t)a * d + t] = Hu[(int64_t)lo * d + hi];
}

hipError_t launch_gather(hipStream_t s, const float* W, int R, int d, const int* perm,
                         const double* Hinv_upper, double* Wp, double* A, hipEvent_t done)
{
    hipExtLaunchKernelGGL(gather_kernel, dim3(R + d, (d + 255) / 256), dim3(256), 0, s, nullptr, done, 0, W, R, d, perm,
                          Hinv_upper, Wp, A);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Blocked column loop, the sequential part (Section 4.2 steps 4-5 inside one
// block of nb <= 64 columns o .. o+nb-1).  One wavefront owns one row of W; lane k
// holds the row's entry in block column k, its grid (scale, zero), and the block's
// pivot-row entries Un[o+j][o+k] for every j.  Rows never interact.  For each
// column j of the block, in order:
//   q    = quant(w_j)                                   (every row at once: one row per wavefront)
//   diff = w_j - q ;  loss += diff^2 / (2 U[t,t])       (Eq. 10)
//   w_k -= diff * Un[t, k]  for the later columns k     (Eq. 9 / 11;
//          e * Hinv[t,k] = (diff / U[t,t]) * U[t,k] = diff * Un[t,k])
// Every lane evaluates the quantizer on its own entry each step; lane j's result is
// the one that counts and is broadcast with v_readlane.  The loop is fully
// unrolled, so there is no memory access on the sequential chain.  diff is stored
// (DT) for the deferred rank-nb update of the columns right of the block.
constexpr int CB = 64;
constexpr int CHAIN_WAVES = 8;

__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// The 64 sequential steps of one row.  EXACT = false forms the quotient w / s as w * (1 / s)
// (the product is within 2 ulp of the true quotient, so rint of it can differ from
// rint(w / s) only when it lies within 2 ulp of a half-integer) and reports through `suspect`
// whether any lane came that close; EXACT = true uses the true division.  The dependent chain
// per step is: multiply, rint, max, min, fma, readlane, fma.
template <bool EXACT>
__device__ __forceinline__ void chain_steps(double& w, const double (*Us)[CB + 1], double s, double z, double maxq,
                                            int nb, int lane, double& mycode, double& mydiff, bool& suspect)
{
    const double rcp_s = 1.0 / s;
    const double lo = -z, hi = maxq - z;          // clamp(c + z, 0, maxq) - z = clamp(c, -z, maxq - z)
    // This lane's pivot-row entries u_j = Us[j][lane] (0 for lanes <= j: they keep the value they were
    // quantized at) come from LDS 16 steps ahead of their use, so that no memory access sits on the
    // sequential chain and only 32 of the 64 are in registers at a time.
    double ub[2][16];
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) ub[0][jj] = Us[jj][lane];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        if (g < 3) {
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) ub[(g + 1) & 1][jj] = Us[16 * (g + 1) + jj][lane];
        }
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int j = 16 * g + jj;
            if (j < nb) {                             // uniform
                const double tq = EXACT ? w / s : w * rcp_s;
                const double c0 = rint(tq);
                if (!EXACT) suspect = suspect || (fabs(fabs(tq - c0) - 0.5) < 1.0e-9 * fmax(1.0, fabs(tq)));
                const double cz = fmin(fmax(c0, lo), hi);        // code - zero
                const double df = w - s * cz;
                const double dj = readlane_f64(df, j);
                if (lane == j) { mycode = cz + z; mydiff = df; }
                w -= dj * ub[g & 1][jj];
            }
        }
        __builtin_amdgcn_sched_barrier(0);            // keeps the loads of the group after the next from moving up here
    }
}

// One launch per column block k does two things that do not depend on each other:
//   (chain role, workgroups 0 .. n_chain-1)   the 64 sequential steps of block k, one row of W per wavefront;
//   (update role, the remaining workgroups)   the deferred compensation of block k-1 for the columns from
//                                             block k+1 on:  W[:, c0:] -= D_{k-1} Un[block k-1, c0:]
// Block k's own columns get block k-1's compensation without waiting for that product: a row's share of it,
// sum_j diff_j Un[o'+j][o+c], is row-local, so the wavefront that has produced the diff_j of its row in launch
// k-1 computes it there (64 fmas per lane, `corr_out`) and this launch subtracts it when it loads its
// columns (`corr_in`).  The sequential loop is therefore one launch per block instead of chain, product,
// chain, ... with the product on the critical path.
struct ColChainP {
    double* Wp; int R, d, o, nb;
    const double* Un; const double* U; const double* scale; const double* zero; int G, gs;
    const int* perm; double maxq; uint8_t* codesT; double* DT; int Rp; double* lossrow;
    const double* corr_in; double* corr_out; int nb_next;
};
struct ColUpdateP {
    int tiles_n;                 // column tiles of the update (0: no update in this launch)
    int o, nb, c0;               // block whose compensation is applied, first column it is applied to
};

__device__ __forceinline__ void col_chain_role(const ColChainP& c, double* lds, int wg)
{
    // the block's pivot rows, fetched once per workgroup (every row of W needs all of them): the part
    // inside the block, and (corr_out != null) the part above the next block's columns
    double (*Us)[CB + 1] = reinterpret_cast<double (*)[CB + 1]>(lds);
    double (*Vs)[CB + 1] = reinterpret_cast<double (*)[CB + 1]>(lds + CB * (CB + 1));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int o = c.o, nb = c.nb, d = c.d;
    const bool col_ok = lane < nb;
    const int cl = col_ok ? lane : 0;        // safe column for address arithmetic
    {
        double t[CB / CHAIN_WAVES], v[CB / CHAIN_WAVES];
        const int cn = min(lane, max(c.nb_next, 1) - 1);
#pragma unroll
        for (int i = 0; i < CB / CHAIN_WAVES; ++i) {
            const int j = wave + CHAIN_WAVES * i;
            t[i] = c.Un[(int64_t)(o + min(j, nb - 1)) * d + o + cl];
            v[i] = c.corr_out ? c.Un[(int64_t)(o + min(j, nb - 1)) * d + o + nb + cn] : 0.0;
        }
#pragma unroll
        for (int i = 0; i < CB / CHAIN_WAVES; ++i) {
            const int j = wave + CHAIN_WAVES * i;
            Us[j][lane] = (j < nb && lane > j && col_ok) ? t[i] : 0.0;    // as the chain uses it: see chain_steps
            Vs[j][lane] = v[i];
        }
    }
    const int row = wg * CHAIN_WAVES + wave;
    const int rw = min(row, c.R - 1);
    double* __restrict__ wptr = c.Wp + (int64_t)rw * d + o + cl;
    double w0 = *wptr;
    if (c.corr_in) w0 -= c.corr_in[(int64_t)rw * CB + cl];
    int pj = c.perm[o + cl];
    pj = min(max(pj, 0), d - 1);
    const int64_t gi = (int64_t)rw * c.G + pj / c.gs;
    const double s = c.scale[gi], z = c.zero[gi];
    const double hp = 0.5 / c.U[(int64_t)(o + cl) * d + o + cl];
    __syncthreads();
    if (row >= c.R) return;                  // whole wavefront leaves; no barrier after this point
    double w = w0, mycode = 0.0, mydiff = 0.0;
    bool suspect = false;
    chain_steps<false>(w, Us, s, z, c.maxq, nb, lane, mycode, mydiff, suspect);
    if (__any(suspect)) {                    // wavefront-uniform; practically never taken
        w = w0;
        chain_steps<true>(w, Us, s, z, c.maxq, nb, lane, mycode, mydiff, suspect);
    }
    if (col_ok) {
        c.codesT[(int64_t)(o + lane) * c.Rp + row] = (uint8_t)mycode;
        c.DT[(int64_t)(o + lane) * c.Rp + row] = mydiff;
        *wptr = w;
    }
    if (c.corr_out) {
        // lane n: sum over the block's columns j of diff_j Un[o+j][o+nb+n]   (lanes >= nb hold diff 0)
        const double dk = col_ok ? mydiff : 0.0;
        double acc = 0.0;
#pragma unroll
        for (int k = 0; k < CB; ++k) acc = fma(readlane_f64(dk, k), Vs[k][lane], acc);
        if (lane < c.nb_next) c.corr_out[(int64_t)row * CB + lane] = acc;
    }
    double loss = col_ok ? mydiff * mydiff * hp : 0.0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) loss += __shfl_xor(loss, off);
    if (lane == 0) c.lossrow[row] += loss;
}

// 64 x 64 tile (ty, tx) of W[:, c0:] -= D^T Un[o : o+nb, c0:], D = DT[o : o+nb, :] (nb x Rp): one chunk of K.
__device__ __forceinline__ void col_update_role(const ColChainP& c, const ColUpdateP& u, double* lds, int t)
{
    typedef double d4 __attribute__((ext_vector_type(4)));
    constexpr int LD = CB + 2;
    double (*As)[LD] = reinterpret_cast<double (*)[LD]>(lds);            // As[m][k] = D[k][m0 + m]
    double (*Bs)[LD] = reinterpret_cast<double (*)[LD]>(lds + CB * LD);   // Bs[n][k] = Un[o + k][n0 + n]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ty = t / u.tiles_n, tx = t - ty * u.tiles_n;
    const int m0 = ty * 64, n0 = u.c0 + tx * 64;
    const int d = c.d;
    double ra[8], rb[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int k = wave + 8 * i;
        const bool kv = k < u.nb;
        const int kk = u.o + min(k, u.nb - 1);
        ra[i] = (kv && m0 + lane < c.R) ? c.DT[(int64_t)kk * c.Rp + m0 + lane] : 0.0;
        rb[i] = (kv && n0 + lane < d) ? c.Un[(int64_t)kk * d + min(n0 + lane, d - 1)] : 0.0;
    }
    const int wr = wave >> 1, wn = wave & 1, fr = lane & 15, fq = lane >> 4;
    d4 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gm = m0 + wr * 16 + 4 * v + fq, gn = n0 + wn * 32 + j * 16 + fr;
            acc[j][v] = (gm < c.R && gn < d) ? c.Wp[(int64_t)gm * d + gn] : 0.0;
        }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        As[lane][wave + 8 * i] = -ra[i];
        Bs[lane][wave + 8 * i] = rb[i];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const double a = As[wr * 16 + fr][4 * ks + fq];
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, Bs[wn * 32 + j * 16 + fr][4 * ks + fq], acc[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gm = m0 + wr * 16 + 4 * v + fq, gn = n0 + wn * 32 + j * 16 + fr;
            if (gm < c.R && gn < d) c.Wp[(int64_t)gm * d + gn] = acc[j][v];
        }
}

__global__ __launch_bounds__(64 * CHAIN_WAVES, 4) void col_block_kernel(ColChainP c, ColUpdateP u, int n_chain)
{
    __shared__ double lds[2 * CB * (CB + 2)];
    if ((int)blockIdx.x < n_chain) col_chain_role(c, lds, (int)blockIdx.x);
    else col_update_role(c, u, lds, (int)blockIdx.x - n_chain);
}

// chain: block [o, o+nb) (nb = 0: no chain in this launch); update: the compensation of block [uo, uo+unb) for
// the columns from c0 on (unb = 0 or c0 >= d: no update in this launch)
hipError_t launch_col_block(hipStream_t s, double* Wp, int R, int d, int o, int nb,
                            const double* Un, const double* U, const double* scale, const double* zero,
                            int G, int group, const int* perm, int bits,
                            uint8_t* codesT, double* DT, int Rp, double* lossrow,
                            const double* corr_in, double* corr_out, int nb_next,
                            int uo, int unb, int c0, hipEvent_t done)
{
    ColChainP c;
    c.Wp = Wp; c.R = R; c.d = d; c.o = o; c.nb = nb; c.Un = Un; c.U = U; c.scale = scale; c.zero = zero;
    c.G = G; c.gs = group > 0 ? group : d; c.perm = perm; c.maxq = (double)((1 << bits) - 1);
    c.codesT = codesT; c.DT = DT; c.Rp = Rp; c.lossrow = lossrow;
    c.corr_in = corr_in; c.corr_out = corr_out; c.nb_next = nb_next;
    ColUpdateP u;
    u.o = uo; u.nb = unb; u.c0 = c0;
    u.tiles_n = (unb > 0 && c0 < d) ? (d - c0 + 63) / 64 : 0;
    const int n_chain = nb > 0 ? (R + CHAIN_WAVES - 1) / CHAIN_WAVES : 0;
    const int n_upd = u.tiles_n * ((R + 63) / 64);
    if (n_chain + n_upd == 0) return done ? hipEventRecord(done, s) : hipSuccess;
    hipExtLaunchKernelGGL(col_block_kernel, dim3(n_chain + n_upd), dim3(64 * CHAIN_WAVES), 0, s, nullptr, done, 0, c, u,
                          n_chain);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Unblocked column step t (Section 4.2 steps 4-5 with Eq. 9 / 11 and Eq. 12
// literally, one launch per column): with p = A[t][t] (A = running shared Hinv in
// processing order, upper triangle maintained),
//   rows of W :  q = quant(W[i][t]); e = (W[i][t] - q) / p;  W[i][k] -= e * A[t][k]     k > t
//   rows of A :  A[a][b] -= (A[t][a] / p) * A[t][b]                                    t < a <= b
// blockIdx.y walks groups of 4 rows, first the R rows of W then the d-t-1 rows of
// A; each wavefront takes one row; blockIdx.x walks strips of 1024 columns whose
// boundaries are fixed multiples of 1024, so that with an even d every lane can move
// 16 bytes at a time.  Row t of A and column t of W are read-only during the step.
// This is the streaming, HBM-bound form: every step reads and writes the whole
// remaining part of W and of the upper triangle of A.
constexpr int STEP_SW = 1024;                  // columns per strip
constexpr int STEP_U = STEP_SW / 128;          // 16-byte pairs per lane

template <bool VEC2>
__global__ __launch_bounds__(256) void step_kernel(double* __restrict__ Wp, int R, int d, int t, double* __restrict__ A,
                                                   const double* __restrict__ scale, const double* __restrict__ zero,
                                                   int G, int gs, const int* __restrict__ perm, double maxq,
                                                   uint8_t* __restrict__ codesT, int Rp, double* __restrict__ lossrow,
                                                   int* __restrict__ flag)
{
    const int lane = threadIdx.x & 63;
    const int rid = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int strip0 = (t + 1) / STEP_SW;
    const int c_base = (strip0 + blockIdx.x) * STEP_SW;
    const double* __restrict__ rowt = A + (int64_t)t * d;
    const double p = rowt[t];
    // the pivot of Eq. 12 must be positive and finite (the call then fails; the arithmetic below goes on
    // with whatever the division gives, every access stays in bounds)
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0 && !(p > 0.0 && p < 1.0e300)) *flag = 1;
    double* __restrict__ row;      // the row this wavefront updates
    double f;                      // row[k] -= f * rowt[k]
    int first;                     // first column to update
    if (rid < R) {
        const int i = rid;
        row = Wp + (int64_t)i * d;
        int pj = perm[t];
        pj = min(max(pj, 0), d - 1);
        const int g = pj / gs;
        const double s = scale[(int64_t)i * G + g], z = zero[(int64_t)i * G + g];
        const double wt = row[t];
        const double c = grid_code(wt, s, z, maxq);
        const double q = s * (c - z);
        const double diff = wt - q;
        if (blockIdx.x == 0 && lane == 0) {
            codesT[(int64_t)t * Rp + i] = (uint8_t)c;
            lossrow[i] += diff * diff / (2.0 * p);
        }
        f = diff / p;
        first = t + 1;
    } else {
        const int a = t + 1 + (rid - R);
        if (a >= d) return;
        if (c_base + STEP_SW <= a) return;          // strip entirely left of the diagonal
        row = A + (int64_t)a * d;
        f = rowt[a] / p;
        first = a;
    }
    if (VEC2) {
        // all loads first (16 in flight per lane), then the updates
        double2 v[STEP_U], r[STEP_U];
#pragma unroll
        for (int u = 0; u < STEP_U; ++u) {
            const int k = c_base + u * 128 + 2 * lane;
            v[u] = make_double2(0.0, 0.0);
            r[u] = make_double2(0.0, 0.0);
            if (k + 1 >= first && k < d) {           // d is even: k + 1 < d as well
                v[u] = *reinterpret_cast<const double2*>(row + k);
                r[u] = *reinterpret_cast<const double2*>(rowt + k);
            }
        }
#pragma unroll
        for (int u = 0; u < STEP_U; ++u) {
            const int k = c_base + u * 128 + 2 * lane;
            if (k + 1 >= first && k < d) {
                if (k >= first) {
                    v[u].x -= f * r[u].x;
                    v[u].y -= f * r[u].y;
                    *reinterpret_cast<double2*>(row + k) = v[u];
                } else {
                    row[k + 1] = v[u].y - f * r[u].y;   // pair straddles the first column
                }
            }
        }
    } else {
        double v[2 * STEP_U], r[2 * STEP_U];
#pragma unroll
        for (int u = 0; u < 2 * STEP_U; ++u) {
            const int k = c_base + u * 64 + lane;
            const bool ok = k >= first && k < d;
            v[u] = ok ? row[k] : 0.0;
            r[u] = ok ? rowt[k] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < 2 * STEP_U; ++u) {
            const int k = c_base + u * 64 + lane;
            if (k >= first && k < d) row[k] = v[u] - f * r[u];
        }
    }
}

// ---------------------------------------------------------------------------
// Dynamic order (the reading of Section 5 in which the sorting is repeated for every
// column): before step t the scores of Eq. 10 are recomputed for the columns at
// positions t .. d-1 from the current weights and the diagonal of the current shared
// inverse, and the column with the largest score is swapped into position t.
//
// Pass 1 (dyn_score_kernel): thread = position, block row-chunk c sums the squared
// quantization errors of rows [c*SENS_RC, (c+1)*SENS_RC).
// Pass 2 (dyn_select_kernel, one workgroup): chunks are added in index order and divided
// by 2 [Hinv]_kk; the largest score wins, the smaller original column index among equal
// scores; then positions t and the winner's are exchanged in W (columns), in the upper
// triangle of the running inverse (rows and columns) and in perm.
__global__ __launch_bounds__(256) void dyn_score_kernel(const double* __restrict__ Wp, int R, int d, int t, int gs,
                                                        int G, double maxq, const double* __restrict__ scale,
                                                        const double* __restrict__ zero,
                                                        const int* __restrict__ perm, double* __restrict__ Spart)
{
    const int k = t + blockIdx.x * 256 + threadIdx.x;
    if (k >= d) return;
    const int g = min(max(perm[k], 0), d - 1) / gs;
    const int r0 = blockIdx.y * SENS_RC, r1 = min(R, r0 + SENS_RC);
    double acc = 0.0;
    for (int i = r0; i < r1; ++i) {
        const double w = Wp[(int64_t)i * d + k];
        const double s = scale[(int64_t)i * G + g], z = zero[(int64_t)i * G + g];
        const double q = s * (grid_code(w, s, z, maxq) - z);
        acc += (q - w) * (q - w);
    }
    Spart[(int64_t)blockIdx.y * d + k] = acc;
}

__global__ __launch_bounds__(1024) void dyn_select_kernel(double* __restrict__ Wp, int R, int d, int t,
                                                          double* __restrict__ A, const double* __restrict__ Spart,
                                                          int chunks, int* __restrict__ perm)
{
    __shared__ double bs[1024];
    __shared__ int bo[1024], bp[1024];
    const int tid = threadIdx.x;
    // a score that is not a number is never taken; position t stands in when none qualifies
    double best = -1.0;
    int borig = 0x7fffffff, bpos = -1;
    for (int k = t + tid; k < d; k += 1024) {
        double acc = 0.0;
        for (int c = 0; c < chunks; ++c) acc += Spart[(int64_t)c * d + k];
        const double sc = acc / (2.0 * A[(int64_t)k * d + k]);
        const int orig = perm[k];
        if (sc > best || (sc == best && orig < borig)) { best = sc; borig = orig; bpos = k; }
    }
    bs[tid] = best; bo[tid] = borig; bp[tid] = bpos;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (tid < w) {
            const double s2 = bs[tid + w];
            const int o2 = bo[tid + w];
            if (bp[tid + w] >= 0 && (bp[tid] < 0 || s2 > bs[tid] || (s2 == bs[tid] && o2 < bo[tid]))) {
                bs[tid] = s2; bo[tid] = o2; bp[tid] = bp[tid + w];
            }
        }
        __syncthreads();
    }
    const int c = bp[0] < 0 ? t : bp[0];
    if (c == t) return;
    // exchange positions t < c
    if (tid == 0) { const int a = perm[t]; perm[t] = perm[c]; perm[c] = a; }
    for (int i = tid; i < R; i += 1024) {
        const double a = Wp[(int64_t)i * d + t];
        Wp[(int64_t)i * d + t] = Wp[(int64_t)i * d + c];
        Wp[(int64_t)i * d + c] = a;
    }
    // symmetric exchange in the upper triangle; rows and columns left of t are no longer read
    for (int m = t + tid; m < d; m += 1024) {
        if (m == c) continue;
        double *x, *y;
        if (m == t) { x = A + (int64_t)t * d + t; y = A + (int64_t)c * d + c; }           // diagonal entries
        else if (m < c) { x = A + (int64_t)t * d + m; y = A + (int64_t)m * d + c; }       // [t][m] <-> [m][c]
        else { x = A + (int64_t)t * d + m; y = A + (int64_t)c * d + m; }                  // [t][m] <-> [c][m]
        const double a = *x;
        *x = *y;
        *y = a;
    }
}

__global__ __launch_bounds__(256) void invert_perm_kernel(const int* __restrict__ perm, int d, int* __restrict__ invperm)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < d) invperm[min(max(perm[t], 0), d - 1)] = t;
}

hipError_t launch_invert_perm(hipStream_t s, const int* perm, int d, int* invperm)
{
    hipLaunchKernelGGL(invert_perm_kernel, dim3((d + 255) / 256), dim3(256), 0, s, perm, d, invperm);
    return hipGetLastError();
}

hipError_t launch_dyn_select(hipStream_t s, double* Wp, int R, int d, int t, double* A, const double* scale,
                             const double* zero, int G, int group, int* perm, int bits, double* Spart, int chunks)
{
    const int gs = group > 0 ? group : d;
    const double maxq = (double)((1 << bits) - 1);
    hipLaunchKernelGGL(dyn_score_kernel, dim3((d - t + 255) / 256, chunks), dim3(256), 0, s, Wp, R, d, t, gs, G, maxq,
                       scale, zero, perm, Spart);
    hipLaunchKernelGGL(dyn_select_kernel, dim3(1), dim3(1024), 0, s, Wp, R, d, t, A, Spart, chunks, perm);
    return hipGetLastError();
}

hipError_t launch_step(hipStream_t s, double* Wp, int R, int d, int t, double* A,
                       const double* scale, const double* zero, int G, int group, const int* perm, int bits,
                       uint8_t* codesT, int Rp, double* lossrow, int* flag)
{
    const int gs = group > 0 ? group : d;
    const double maxq = (double)((1 << bits) - 1);
    const int r = d - t - 1;
    const int strip0 = (t + 1) / STEP_SW;
    const int strips = r > 0 ? (d - 1) / STEP_SW - strip0 + 1 : 1;
    const int rows = R + (r > 0 ? r : 0);
    dim3 grid(strips, (rows + 3) / 4), block(256);
    if (d % 2 == 0)
        hipLaunchKernelGGL((step_kernel<true>), grid, block, 0, s, Wp, R, d, t, A, scale, zero, G, gs, perm, maxq,
                           codesT, Rp, lossrow, flag);
    else
        hipLaunchKernelGGL((step_kernel<false>), grid, block, 0, s, Wp, R, d, t, A, scale, zero, G, gs, perm, maxq,
                           codesT, Rp, lossrow, flag);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Outputs in original column order: codes[i][c] and Q[i][c] = scale * (code - zero)
// for the column c processed at step invperm[c] < steps; others get code 0, Q 0.
// Workgroup (0, 0) also adds up the per-row loss terms (loss != null).
__global__ __launch_bounds__(256) void emit_kernel(const uint8_t* __restrict__ codesT, int Rp, int R, int d, int steps,
                                                   const int* __restrict__ invperm, const double* __restrict__ scale,
                                                   const double* __restrict__ zero, int G, int gs,
                                                   uint8_t* __restrict__ codes, float* __restrict__ Q,
                                                   const double* __restrict__ lossrow, double* __restrict__ loss)
{
    if (loss && blockIdx.x == 0 && blockIdx.y == 0) {       // uniform over the workgroup
        __shared__ double part[256];
        double s = 0.0;
        for (int i = threadIdx.x; i < R; i += 256) s += lossrow[i];
        part[threadIdx.x] = s;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) *loss = part[0];
    }
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int i = blockIdx.y;
    if (c >= d) return;
    int t = invperm[c];
    uint8_t code = 0;
    double q = 0.0;
    if (t >= 0 && t < steps) {
        code = codesT[(int64_t)t * Rp + i];
        const int g = c / gs;
        q = scale[(int64_t)i * G + g] * ((double)code - zero[(int64_t)i * G + g]);
    }
    if (codes) codes[(int64_t)i * d + c] = code;
    if (Q) Q[(int64_t)i * d + c] = (float)q;
}

hipError_t launch_emit(hipStream_t s, const uint8_t* codesT, int Rp, int R, int d, int steps,
                       const int* invperm, const double* scale, const double* zero, int G, int group,
                       uint8_t* codes, float* Q, const double* lossrow, double* loss)
{
    const int gs = group > 0 ? group : d;
    hipLaunchKernelGGL(emit_kernel, dim3((d + 255) / 256, R), dim3(256), 0, s, codesT, Rp, R, d, steps, invperm,
                       scale, zero, G, gs, codes, Q, lossrow, loss);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void loss_kernel(const double* __restrict__ lossrow, int R, double* __restrict__ loss)
{
    __shared__ double part[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < R; i += 256) s += lossrow[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = part[0];
}

hipError_t launch_loss(hipStream_t s, const double* lossrow, int R, double* loss)
{
    hipLaunchKernelGGL(loss_kernel, dim3(1), dim3(256), 0, s, lossrow, R, loss);
    return hipGetLastError();
}

// Running shared inverse after `steps` columns, processing order, full symmetric;
// rows and columns of processed steps are 0.  A holds valid data on and above the
// diagonal of the trailing square.
__global__ __launch_bounds__(256) void hinv_work_kernel(const double* __restrict__ A, int d, int steps,
                                                        double* __restrict__ out)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    const int a = blockIdx.y;
    if (b >= d) return;
    double v = 0.0;
    if (a >= steps && b >= steps) v = A[(int64_t)min(a, b) * d + max(a, b)];
    out[(int64_t)a * d + b] = v;
}

hipError_t launch_hinv_work(hipStream_t s, const double* A, int d, int steps, double* out)
{
    hipLaunchKernelGGL(hinv_work_kernel, dim3((d + 255) / 256, d), dim3(256), 0, s, A, d, steps, out);
    return hipGetLastError();
}

// Zero two buffers of 4-byte words in one launch (n2 may be 0).  A kernel rather than hipMemsetAsync: one
// launch for both, and safe inside a stream capture.
__global__ __launch_bounds__(256) void clear_words_kernel(uint32_t* __restrict__ p1, int64_t n1,
                                                          uint32_t* __restrict__ p2, int64_t n2)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n1 + n2; i += stride) {
        if (i < n1) p1[i] = 0u; else p2[i - n1] = 0u;
    }
}
hipError_t launch_clear_words(hipStream_t s, void* p1, int64_t n1, void* p2, int64_t n2, hipEvent_t done)
{
    const int64_t n = n1 + n2;
    if (n <= 0) return done ? hipEventRecord(done, s) : hipSuccess;
    const int64_t blocks = (n + 255) / 256;
    hipExtLaunchKernelGGL(clear_words_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, nullptr,
                          done, 0, (uint32_t*)p1, n1, (uint32_t*)p2, n2);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int* __restrict__ p, int64_t n, int v)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}
hipError_t launch_fill_i32(hipStream_t s, int* p, int64_t n, int v)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Batched small layers (see batch_inverse_kernel): the same stages with one grid dimension over the layers
// of the batch, each layer's shapes and pointers in its BatchLayer; workgroups past a layer's own extent leave.

// Grid per (row, group) as grid_kernel; the first workgroup of a layer also clears its status words and
// per-row loss terms.
__global__ __launch_bounds__(256) void batch_grid_kernel(const BatchLayer* __restrict__ layers)
{
    const BatchLayer L = layers[blockIdx.y];
    if (blockIdx.x == 0) {
        if (threadIdx.x < 4) L.flags[threadIdx.x] = 0;
        for (int i = threadIdx.x; i < L.R; i += 256) L.lossrow[i] = 0.0;
    }
    const int lane = threadIdx.x & 63;
    const int64_t pair = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= (int64_t)L.R * L.G) return;
    const int i = (int)(pair / L.G), g = (int)(pair % L.G);
    const float* __restrict__ src = L.W + (int64_t)i * L.d + (int64_t)g * L.gs;
    float lo = 0.f, hi = 0.f;
    for (int j = lane; j < L.gs; j += 64) {
        const float w = src[j];
        lo = fminf(lo, w);
        hi = fmaxf(hi, w);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
    }
    if (lane == 0) {
        double s = 1.0, z = 0.0;
        if (hi != lo) {
            s = ((double)hi - (double)lo) / L.maxq;
            z = rint(-(double)lo / s);
        }
        L.scale[pair] = s;
        L.zero[pair] = z;
        if (L.scales) L.scales[pair] = (float)s;
        if (L.zeros) L.zeros[pair] = (float)z;
    }
}

// Per-chunk column sums as sens_partial_kernel; blockIdx.x = chunk of 64 rows, thread = column (d <= 256).
__global__ __launch_bounds__(256) void batch_sens_partial_kernel(const BatchLayer* __restrict__ layers)
{
    const BatchLayer L = layers[blockIdx.y];
    const int j = threadIdx.x;
    if ((int)blockIdx.x >= L.chunks || j >= L.d) return;
    const int g = j / L.gs;
    const int r0 = blockIdx.x * SENS_RC, r1 = min(L.R, r0 + SENS_RC);
    double acc = 0.0;
    for (int i = r0; i < r1; ++i) {
        const double w = (double)L.W[(int64_t)i * L.d + j];
        const double s = L.scale[(int64_t)i * L.G + g], z = L.zero[(int64_t)i * L.G + g];
        const double q = s * (grid_code(w, s, z, L.maxq) - z);
        acc += (L.kind == 2) ? w * w : (q - w) * (q - w);
    }
    L.Spart[(int64_t)blockIdx.x * L.d + j] = acc;
}

// Scores and order of one layer by one workgroup (d <= 256: thread = column): the chunks are added in index
// order, "sensi" divides by 2 [Hinv]_jj; rank by counting, equal keys keep index order.
__global__ __launch_bounds__(256) void batch_order_kernel(const BatchLayer* __restrict__ layers)
{
    __shared__ double key[BATCH_MAX_D];
    const BatchLayer L = layers[blockIdx.x];
    const int j = threadIdx.x, d = L.d;
    if (j < d) {
        double acc = 0.0;
        for (int c = 0; c < L.chunks; ++c) acc += L.Spart[(int64_t)c * d + j];
        const double sj = (L.kind == 0) ? acc / (2.0 * L.Hinv[(int64_t)j * d + j]) : acc;
        L.S[j] = sj;
        key[j] = sort_key((L.ascending ? -1.0 : 1.0) * sj);
    }
    __syncthreads();
    if (L.order == FOBQ_ORDER_NATURAL) {
        if (j < d) { L.perm[j] = j; L.invperm[j] = j; }
    } else if (j < d) {
        const double sj = key[j];
        int r = 0;
        for (int k = 0; k < d; ++k) {
            const double v = key[k];
            r += (v > sj || (v == sj && k < j)) ? 1 : 0;
        }
        L.perm[r] = j;
        L.invperm[j] = r;
    }
    __syncthreads();
    if (L.perm_out && j < d) L.perm_out[j] = L.perm[j];
}

// The whole column loop of a small layer in one launch.  Rows never interact (Section 4.2 step 4: all rows
// at once), and with the pivot rows complete a workgroup of 8 wavefronts owns 8 rows from the first column to
// the last: it gathers them into processing order, then block by block runs the 64 sequential steps
// (col_chain_role) and applies the block's deferred compensation (Eq. 9 / 11) to its own rows' later columns;
// at the end it writes its rows' codes and dequantized weights in the original column order.
__global__ __launch_bounds__(64 * CHAIN_WAVES) void batch_columns_kernel(const BatchLayer* __restrict__ layers)
{
    __shared__ double lds[2 * CB * (CB + 2)];
    const BatchLayer L = layers[blockIdx.y];
    const int wg = blockIdx.x;
    if (wg * CHAIN_WAVES >= L.R) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = wg * CHAIN_WAVES + wave, d = L.d;
    const bool row_ok = row < L.R;
    if (row_ok) {
        for (int t = lane; t < d; t += 64) {
            const int pt = min(max(L.perm[t], 0), d - 1);
            L.Wp[(int64_t)row * d + t] = (double)L.W[(int64_t)row * d + pt];
        }
    }
    __syncthreads();
    ColChainP c;
    c.Wp = L.Wp; c.R = L.R; c.d = d; c.Un = L.Un; c.U = L.U; c.scale = L.scale; c.zero = L.zero;
    c.G = L.G; c.gs = L.gs; c.perm = L.perm; c.maxq = L.maxq; c.codesT = L.codesT; c.DT = L.DT; c.Rp = L.Rp;
    c.lossrow = L.lossrow; c.corr_in = nullptr; c.corr_out = nullptr; c.nb_next = 0;
    for (int o = 0; o < d; o += CB) {
        const int nb = min(CB, d - o);
        c.o = o; c.nb = nb;
        col_chain_role(c, lds, wg);
        __syncthreads();               // the chain's stores of this workgroup's rows are visible to it
        // W[row][k] -= sum_j diff_j Un[o + j][k] for the columns k right of the block, 64 columns at a time: the
        // block's pivot rows above those columns go through LDS once for the workgroup's 8 rows; lane j holds diff_j
        const double dj = (row_ok && lane < nb) ? L.DT[(int64_t)(o + lane) * L.Rp + row] : 0.0;
        double (*Us)[CB + 1] = reinterpret_cast<double (*)[CB + 1]>(lds);
        for (int k0 = o + nb; k0 < d; k0 += CB) {
            const int nk = min(CB, d - k0);
#pragma unroll
            for (int i = 0; i < CB / CHAIN_WAVES; ++i) {
                const int j = wave + CHAIN_WAVES * i;
                Us[j][lane] = (j < nb && lane < nk) ? L.Un[(int64_t)(o + j) * d + k0 + lane] : 0.0;
            }
            __syncthreads();
            double acc = 0.0;
#pragma unroll
            for (int j = 0; j < CB; ++j) acc = fma(readlane_f64(dj, j), Us[j][lane], acc);
            if (row_ok && lane < nk) L.Wp[(int64_t)row * d + k0 + lane] -= acc;
            __syncthreads();
        }
    }
    if (!row_ok) return;
    for (int cidx = lane; cidx < d; cidx += 64) {
        const int t = min(max(L.invperm[cidx], 0), d - 1);
        const uint8_t code = L.codesT[(int64_t)t * L.Rp + row];
        const int g = cidx / L.gs;
        const double q = L.scale[(int64_t)row * L.G + g] * ((double)code - L.zero[(int64_t)row * L.G + g]);
        if (L.codes) L.codes[(int64_t)row * d + cidx] = code;
        if (L.Q) L.Q[(int64_t)row * d + cidx] = (float)q;
    }
}

__global__ __launch_bounds__(256) void batch_loss_kernel(const BatchLayer* __restrict__ layers)
{
    __shared__ double part[256];
    const BatchLayer L = layers[blockIdx.x];
    if (!L.loss) return;
    double s = 0.0;
    for (int i = threadIdx.x; i < L.R; i += 256) s += L.lossrow[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *L.loss = part[0];
}

hipError_t launch_batch_grid(hipStream_t s, const BatchLayer* layers, int n, int max_pairs)
{
    hipLaunchKernelGGL(batch_grid_kernel, dim3((max_pairs + 3) / 4, n), dim3(256), 0, s, layers);
    return hipGetLastError();
}

hipError_t launch_batch_sens_partial(hipStream_t s, const BatchLayer* layers, int n, int max_chunks)
{
    hipLaunchKernelGGL(batch_sens_partial_kernel, dim3(max_chunks, n), dim3(256), 0, s, layers);
    return hipGetLastError();
}

hipError_t launch_batch_order(hipStream_t s, const BatchLayer* layers, int n)
{
    hipLaunchKernelGGL(batch_order_kernel, dim3(n), dim3(256), 0, s, layers);
    return hipGetLastError();
}

hipError_t launch_batch_columns(hipStream_t s, const BatchLayer* layers, int n, int max_rows)
{
    hipLaunchKernelGGL(batch_columns_kernel, dim3((max_rows + CHAIN_WAVES - 1) / CHAIN_WAVES, n), dim3(64 * CHAIN_WAVES), 0, s,
                       layers);
    return hipGetLastError();
}

hipError_t launch_batch_loss(hipStream_t s, const BatchLayer* layers, int n)
{
    hipLaunchKernelGGL(batch_loss_kernel, dim3(n), dim3(256), 0, s, layers);
    return hipGetLastError();
}

}  // namespace fobq
