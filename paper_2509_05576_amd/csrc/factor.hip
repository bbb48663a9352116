// Dense factorizations of the path, all fp64, all blocked with 64-wide panels:
//   cholesky_lower   H_d = L L^T                       (Section 5, item 1)
//   trtri_lower      L^-1 by recursive doubling of the block size
//   lauum_upper      Hinv = L^-T L^-1
//   eliminate_blocked the shared-Hinv elimination of Eq. 12, B columns at a time:
//                    after column t is processed, Hinv -= Hinv[:,t] Hinv[t,:] / Hinv[t,t].
//                    The pivot rows are kept:  U[t, t:]  = Hinv^(t)[t, t:]  and
//                    Un[t, :] = U[t, :] / U[t, t]; the weight compensation of Eq. 9 / 11
//                    for step t is  W[:, k] -= (w_t - q_t) * Un[t, k].
// The 64 x 64 diagonal blocks are handled by one workgroup in LDS; everything
// else is a rank-64 update on the matrix cores (gemm64).
#include "fobq_internal.h"

namespace fobq {

constexpr int NB = 64;
constexpr int DLD = NB + 1;

// ---------------------------------------------------------------------------
// Diagonal block of the Cholesky factorization.
//   in : A[o:o+nb, o:o+nb] (lower triangle read)
//   out: L[o:o+nb, o:o+nb] = L11 (lower, upper part zeroed)
//        Linv[o:o+nb, o:o+nb] = L11^-1 (lower, upper part zeroed)
//        Dinv (64 x 64, ld 64) = L11^-1 zero padded
//   flag: set to 1 when a pivot is <= 0 or not finite (the pivot is replaced by 1
//         so that the arithmetic stays finite; the caller reports ENOTPD).
__global__ __launch_bounds__(256) void chol_diag_kernel(const double* __restrict__ A, int64_t ld, int o, int nb,
                                                        double* __restrict__ L, double* __restrict__ Linv,
                                                        double* __restrict__ Dinv, int* __restrict__ flag)
{
    __shared__ double a[NB][DLD];
    __shared__ double x[NB][DLD];
    const int tid = threadIdx.x;
    for (int idx = tid; idx < NB * NB; idx += 256) {
        const int i = idx / NB, j = idx % NB;
        a[i][j] = (i < nb && j <= i) ? A[(int64_t)(o + i) * ld + o + j] : 0.0;
        x[i][j] = 0.0;
    }
    __syncthreads();
    for (int j = 0; j < nb; ++j) {
        if (tid == 0) {
            double piv = a[j][j];
            if (!(piv > 0.0) || !(piv < 1.0e300)) { *flag = 1; piv = 1.0; }
            a[j][j] = sqrt(piv);
        }
        __syncthreads();
        const double ljj = a[j][j];
        if (tid > j && tid < nb) a[tid][j] /= ljj;
        __syncthreads();
        const int rem = nb - j - 1;
        for (int idx = tid; idx < rem * rem; idx += 256) {
            const int i = j + 1 + idx / rem, k = j + 1 + idx % rem;
            if (k <= i) a[i][k] -= a[i][j] * a[k][j];
        }
        __syncthreads();
    }
    // column c of L11^-1 by forward substitution (one thread per column)
    if (tid < nb) {
        const int c = tid;
        x[c][c] = 1.0 / a[c][c];
        for (int i = c + 1; i < nb; ++i) {
            double s = 0.0;
            for (int k = c; k < i; ++k) s += a[i][k] * x[k][c];
            x[i][c] = -s / a[i][i];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < NB * NB; idx += 256) {
        const int i = idx / NB, j = idx % NB;
        Dinv[idx] = x[i][j];
        if (i < nb && j < nb) {
            L[(int64_t)(o + i) * ld + o + j] = (j <= i) ? a[i][j] : 0.0;
            Linv[(int64_t)(o + i) * ld + o + j] = x[i][j];
        }
    }
}

hipError_t cholesky_lower(fobq_ctx* c, double* Hd, double* L, int d, double* Linv, int* flag)
{
    hipStream_t s = c->stream;
    double* Dinv = c->Dblk.as<double>();
    for (int o = 0; o < d; o += NB) {
        const int nb = min(NB, d - o);
        hipLaunchKernelGGL(chol_diag_kernel, dim3(1), dim3(256), 0, s, Hd, (int64_t)d, o, nb, L, Linv, Dinv, flag);
        const int r = d - o - nb;
        if (r <= 0) break;
        // L21 = A21 * L11^-T
        GemmP p;
        p.M = r; p.N = nb; p.K = nb;
        p.A = Hd + (int64_t)(o + nb) * d + o; p.lda = d;
        p.B = Dinv; p.ldb = NB;
        p.C = L + (int64_t)(o + nb) * d + o; p.ldc = d;
        hipError_t e = gemm64(s, p, false, true);
        if (e != hipSuccess) return e;
        // A22 -= L21 L21^T  (lower tiles)
        GemmP q;
        q.M = r; q.N = r; q.K = nb;
        q.A = L + (int64_t)(o + nb) * d + o; q.lda = d;
        q.B = q.A; q.ldb = d;
        q.C = Hd + (int64_t)(o + nb) * d + (o + nb); q.ldc = d;
        q.alpha = -1.0; q.beta = 1.0; q.cmode = CMODE_LOWER;
        e = gemm64(s, q, false, true);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

// Linv holds the inverses of the 64 x 64 diagonal blocks of L and zeros elsewhere.
// Level s: for every pair of adjacent s-blocks [[A, 0], [C, B]] with A^-1, B^-1 known,
// the missing block of the inverse is -B^-1 C A^-1.
hipError_t trtri_lower(fobq_ctx* c, const double* L, int d, double* Linv, double* T)
{
    hipStream_t st = c->stream;
    for (int64_t s = NB; s < d; s *= 2) {
        const int batches = (int)((d - s + 2 * s - 1) / (2 * s));
        const int64_t stride = 2 * s * (int64_t)d + 2 * s;
        GemmP p;   // T_blk = C * A^-1
        p.M = (int)s; p.N = (int)s; p.K = (int)s;
        p.A = L + s * d; p.lda = d;
        p.B = Linv; p.ldb = d;
        p.C = T + s * d; p.ldc = d;
        p.kmode = KMODE_GE_N;
        p.batches = batches; p.sA = stride; p.sB = stride; p.sC = stride;
        p.Mtot = (int)(d - s); p.mstep = (int)(2 * s);
        hipError_t e = gemm64(st, p, false, false);
        if (e != hipSuccess) return e;
        GemmP q;   // Linv_blk = -B^-1 * T_blk
        q.M = (int)s; q.N = (int)s; q.K = (int)s;
        q.A = Linv + s * d + s; q.lda = d;
        q.B = T + s * d; q.ldb = d;
        q.C = Linv + s * d; q.ldc = d;
        q.alpha = -1.0; q.kmode = KMODE_LT_M;
        q.batches = batches; q.sA = stride; q.sB = stride; q.sC = stride;
        q.Mtot = (int)(d - s); q.mstep = (int)(2 * s);
        q.Ktot = (int)(d - s); q.kstep = (int)(2 * s);
        e = gemm64(st, q, false, false);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

// Hinv = Linv^T Linv, tiles on or above the diagonal.
hipError_t lauum_upper(fobq_ctx* c, const double* Linv, int d, double* Hinv)
{
    GemmP p;
    p.M = d; p.N = d; p.K = d;
    p.A = Linv; p.lda = d;
    p.B = Linv; p.ldb = d;
    p.C = Hinv; p.ldc = d;
    p.cmode = CMODE_UPPER; p.kmode = KMODE_GE_MAX_MN;
    return gemm64(c->stream, p, true, false);
}

// ---------------------------------------------------------------------------
// Diagonal block of the shared-Hinv elimination (Eq. 12 for nb consecutive steps
// restricted to the block).  With A11 the current block and U11 its pivot rows,
// A11 = U11^T D^-1 U11, D = diag(U11).
//   out: U[o+j, o+j : o+nb]  = pivot row j inside the block
//        Un = U / pivot
//        G (64 x 64, ld 64)  = D U11^-T  (unit lower): pivot rows right of the
//                              block are G * A[o:o+nb, o+nb:]
//        rinv[j] = 1 / pivot_j
__global__ __launch_bounds__(256) void elim_diag_kernel(const double* __restrict__ A, int64_t ld, int o, int nb,
                                                        double* __restrict__ U, double* __restrict__ Un,
                                                        double* __restrict__ G, double* __restrict__ rinv,
                                                        int* __restrict__ flag)
{
    __shared__ double a[NB][DLD];
    __shared__ double x[NB][DLD];
    const int tid = threadIdx.x;
    for (int idx = tid; idx < NB * NB; idx += 256) {
        const int i = idx / NB, j = idx % NB;
        a[i][j] = (j < nb && i <= j) ? A[(int64_t)(o + i) * ld + o + j] : 0.0;
        x[i][j] = 0.0;
    }
    __syncthreads();
    for (int j = 0; j < nb; ++j) {
        if (tid == 0) {
            const double piv = a[j][j];
            if (!(piv > 0.0) || !(piv < 1.0e300)) { *flag = 1; a[j][j] = 1.0; }
        }
        __syncthreads();
        const double pinv = 1.0 / a[j][j];
        const int rem = nb - j - 1;
        for (int idx = tid; idx < rem * rem; idx += 256) {
            const int r = j + 1 + idx / rem, k = j + 1 + idx % rem;
            if (k >= r) a[r][k] -= a[j][r] * pinv * a[j][k];
        }
        __syncthreads();
    }
    // G = D * (U11^T)^-1: column c by forward substitution with Lh[i][k] = a[k][i]
    if (tid < nb) {
        const int c = tid;
        x[c][c] = 1.0 / a[c][c];
        for (int i = c + 1; i < nb; ++i) {
            double s = 0.0;
            for (int k = c; k < i; ++k) s += a[k][i] * x[k][c];
            x[i][c] = -s / a[i][i];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < NB * NB; idx += 256) {
        const int i = idx / NB, j = idx % NB;
        G[idx] = (i < nb && j < nb) ? a[i][i] * x[i][j] : 0.0;
        if (i < nb && j < nb && j >= i) {
            U[(int64_t)(o + i) * ld + o + j] = a[i][j];
            Un[(int64_t)(o + i) * ld + o + j] = a[i][j] / a[i][i];
        }
    }
    if (tid < NB) rinv[tid] = (tid < nb) ? 1.0 / a[tid][tid] : 0.0;
}

hipError_t eliminate_blocked(fobq_ctx* c, double* A, int d, int steps, int block, double* U, double* Un, int* flag)
{
    hipStream_t s = c->stream;
    double* G = c->Dblk.as<double>() + NB * NB;
    double* rinv = c->Dblk.as<double>() + 2 * NB * NB;
    for (int o = 0; o < steps; o += block) {
        const int nb = min(block, steps - o);
        hipLaunchKernelGGL(elim_diag_kernel, dim3(1), dim3(256), 0, s, A, (int64_t)d, o, nb, U, Un, G, rinv, flag);
        const int r = d - o - nb;
        if (r <= 0) break;
        // pivot rows right of the block: U12 = G * A12, Un12 = D^-1 U12
        GemmP p;
        p.M = nb; p.N = r; p.K = nb;
        p.A = G; p.lda = NB;
        p.B = A + (int64_t)o * d + (o + nb); p.ldb = d;
        p.C = U + (int64_t)o * d + (o + nb); p.ldc = d;
        p.C2 = Un + (int64_t)o * d + (o + nb); p.rowscale = rinv;
        hipError_t e = gemm64(s, p, false, false);
        if (e != hipSuccess) return e;
        // trailing update  A22 -= Un12^T U12  (tiles on or above the diagonal)
        GemmP q;
        q.M = r; q.N = r; q.K = nb;
        q.A = Un + (int64_t)o * d + (o + nb); q.lda = d;
        q.B = U + (int64_t)o * d + (o + nb); q.ldb = d;
        q.C = A + (int64_t)(o + nb) * d + (o + nb); q.ldc = d;
        q.alpha = -1.0; q.beta = 1.0; q.cmode = CMODE_UPPER;
        e = gemm64(s, q, true, false);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

}  // namespace fobq
