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
// 64 x 64 diagonal blocks.  Both diagonal-block kernels use the same scheme: the
// block lives in registers, thread (ti, tj) of a 16 x 16 grid owning the 4 x 4
// micro-tile rows 4 ti.., columns 4 tj.. of the (full symmetric) block and of a
// second 64 x 64 matrix X that starts as the identity.  Step k of the
// factorization is a rank-1 update of both; the only data exchanged per step are
// column k of the block and row k of X, through LDS, behind one barrier (the LDS
// slots alternate with the parity of k so that one barrier per step is enough).
// Applying the elementary eliminations to the identity yields the inverse of the
// triangular factor in the same sweep.

// Diagonal block of the Cholesky factorization.
//   in : A[o:o+nb, o:o+nb] (symmetric; only the lower triangle is read)
//   out: L[o:o+nb, o:o+nb] = L11 (lower, upper part zeroed)
//        Linv[o:o+nb, o:o+nb] = L11^-1 (lower, upper part zeroed)
//        Dinv (64 x 64, ld 64) = L11^-1 zero padded
//   flag: set to 1 when a pivot is <= 0 or not finite (the pivot is replaced by 1
//         so that the arithmetic stays finite; the caller reports ENOTPD).
// Column k of L and row k of L^-1 are final at step k and are stored right then by
// the threads that hold them.
__global__ __launch_bounds__(256) void chol_diag_kernel(const double* __restrict__ A, int64_t ld, int o, int nb,
                                                        double* __restrict__ L, double* __restrict__ Linv,
                                                        double* __restrict__ Dinv, int* __restrict__ flag)
{
    __shared__ double col[2][NB];
    __shared__ double xrow[2][NB];
    const int tid = threadIdx.x;
    const int ti = tid >> 4, tj = tid & 15;
    const int i0 = ti * 4, j0 = tj * 4;
    double a[4][4], x[4][4];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int i = i0 + ii, j = j0 + jj;
            double v = (i == j) ? 1.0 : 0.0;           // identity padding past nb
            if (i < nb && j < nb) {
                const int lo = min(i, j), hi = max(i, j);
                v = A[(int64_t)(o + hi) * ld + o + lo];
                if (j > i) {                            // strictly upper part of the outputs is zero
                    L[(int64_t)(o + i) * ld + o + j] = 0.0;
                    Linv[(int64_t)(o + i) * ld + o + j] = 0.0;
                }
            }
            a[ii][jj] = v;
            x[ii][jj] = (i == j) ? 1.0 : 0.0;
            if (j > i || i >= nb || j >= nb) Dinv[i * NB + j] = 0.0;
        }
    // k = 4 kb + kk with kk unrolled, so that the micro-tile column / row handed to LDS
    // has a compile-time register index (the tiles must stay in registers)
    for (int kb = 0; kb < (nb + 3) / 4; ++kb) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int k = kb * 4 + kk, slot = kk & 1;
        if (k >= nb) break;
        if (tj == kb) {
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) col[slot][i0 + ii] = a[ii][kk];
        }
        if (ti == kb) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) xrow[slot][j0 + jj] = x[kk][jj];
        }
        __syncthreads();
        double piv = col[slot][k];
        if (!(piv > 0.0) || !(piv < 1.0e300)) { if (tid == 0) *flag = 1; piv = 1.0; }
        const double rs = rsqrt(piv);
        double li[4], lj[4], xs[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const double ci = col[slot][i0 + u] * rs;
            li[u] = (i0 + u > k) ? ci : 0.0;           // rows <= k are finished: zero multiplier
            lj[u] = (j0 + u > k) ? col[slot][j0 + u] * rs : 0.0;
            xs[u] = xrow[slot][j0 + u] * rs;
            if (tj == kb) {                             // this thread holds column k: store L[:, k]
                const int i = i0 + u;
                if (i >= k && i < nb) L[(int64_t)(o + i) * ld + o + k] = (i == k) ? piv * rs : ci;
            }
            if (ti == kb) {                             // this thread holds row k of X: store L^-1[k, :]
                const int j = j0 + u;
                if (j <= k) {
                    Linv[(int64_t)(o + k) * ld + o + j] = xs[u];
                    Dinv[k * NB + j] = xs[u];
                }
            }
        }
#pragma unroll
        for (int ii = 0; ii < 4; ++ii)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                a[ii][jj] -= li[ii] * lj[jj];
                x[ii][jj] -= li[ii] * xs[jj];
            }
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
// Same register scheme as chol_diag_kernel; X accumulates (U11^T)^-1, whose row k
// before its division by the pivot is row k of G.  Pivot row k and row k of G are
// final at step k and are stored right then.
__global__ __launch_bounds__(256) void elim_diag_kernel(const double* __restrict__ A, int64_t ld, int o, int nb,
                                                        double* __restrict__ U, double* __restrict__ Un,
                                                        double* __restrict__ G, double* __restrict__ rinv,
                                                        int* __restrict__ flag)
{
    __shared__ double col[2][NB];
    __shared__ double xrow[2][NB];
    const int tid = threadIdx.x;
    const int ti = tid >> 4, tj = tid & 15;
    const int i0 = ti * 4, j0 = tj * 4;
    double a[4][4], x[4][4];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int i = i0 + ii, j = j0 + jj;
            double v = (i == j) ? 1.0 : 0.0;
            if (i < nb && j < nb) {
                const int lo = min(i, j), hi = max(i, j);
                v = A[(int64_t)(o + lo) * ld + o + hi];      // upper triangle is the maintained one
            }
            a[ii][jj] = v;
            x[ii][jj] = (i == j) ? 1.0 : 0.0;
            if (j > i || i >= nb || j >= nb) G[i * NB + j] = 0.0;
        }
    if (tid < NB && tid >= nb) rinv[tid] = 0.0;
    for (int kb = 0; kb < (nb + 3) / 4; ++kb) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int k = kb * 4 + kk, slot = kk & 1;
        if (k >= nb) break;
        if (tj == kb) {
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) col[slot][i0 + ii] = a[ii][kk];
        }
        if (ti == kb) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) xrow[slot][j0 + jj] = x[kk][jj];
        }
        __syncthreads();
        double piv = col[slot][k];
        if (!(piv > 0.0) || !(piv < 1.0e300)) { if (tid == 0) *flag = 1; piv = 1.0; }
        const double pinv = 1.0 / piv;
        if (tid == 0) rinv[k] = pinv;
        double fi[4], cj[4], xr[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            fi[u] = (i0 + u > k) ? col[slot][i0 + u] * pinv : 0.0;   // rows <= k are finished
            const double c = col[slot][j0 + u];                       // = A[k][j] by symmetry
            cj[u] = (j0 + u > k) ? c : 0.0;
            xr[u] = xrow[slot][j0 + u];
            const int j = j0 + u;
            if (ti == kb) {                              // one thread row stores pivot row k and row k of G
                if (j >= k && j < nb) {
                    const double uv = (j == k) ? piv : c;
                    U[(int64_t)(o + k) * ld + o + j] = uv;
                    Un[(int64_t)(o + k) * ld + o + j] = (j == k) ? 1.0 : c * pinv;
                }
                if (j <= k) G[k * NB + j] = xr[u];
            }
        }
#pragma unroll
        for (int ii = 0; ii < 4; ++ii)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                a[ii][jj] -= fi[ii] * cj[jj];
                x[ii][jj] -= fi[ii] * xr[jj];
            }
      }
    }
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
