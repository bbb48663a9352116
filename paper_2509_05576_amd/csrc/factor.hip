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

// ---------------------------------------------------------------------------
// 64 x 64 diagonal blocks.  Both diagonal-block kernels keep the block in LDS and
// work on it as a 4 x 4 grid of 16 x 16 tiles: the only sequential arithmetic is
// the unblocked factorization of a 16 x 16 diagonal tile (one wavefront, one tile
// row per lane, pivot rows broadcast with v_readlane, the tile's triangular
// inverse obtained in the same sweep by applying the eliminations to the
// identity); everything else -- panel, trailing update, assembly of the 64 x 64
// triangular inverse from the tile inverses -- is 16 x 16 x 16 products on the
// matrix cores (4 MFMAs each), one tile per wavefront.
typedef double d4 __attribute__((ext_vector_type(4)));
constexpr int DL = 66;    // LDS row stride (doubles): conflict-free 8-byte MFMA fragment reads per half-wave

__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ d4 mfma4(double a, double b, d4 c)
{
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// Assembly of the inverse X of a 64 x 64 lower triangular matrix T from the inverses of
// its four 16 x 16 diagonal tiles (already in Xm):  X_ij = -X_ii sum_{m=j}^{i-1} T_im X_mj,
// by distance from the diagonal.  tfetch(i, m, ks) returns this lane's A-operand element
// of tile T_im for k-step ks, i.e. T_im[fr][4 ks + fq].
template <class TF>
__device__ __forceinline__ void assemble_inverse(double* Xm, TF tfetch, int wave, int fr, int fq)
{
    for (int dist = 1; dist < 4; ++dist) {
        const int i = dist + wave, j = i - dist;
        if (i < 4) {
            d4 t = {0.0, 0.0, 0.0, 0.0};
            for (int m = j; m < i; ++m)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    t = mfma4(tfetch(i, m, ks), Xm[(16 * m + 4 * ks + fq) * DL + 16 * j + fr], t);
            // the accumulator layout (row 4 v + fq, column fr) is the B-operand layout of k-step v
            d4 r = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) r = mfma4(Xm[(16 * i + fr) * DL + 16 * i + 4 * ks + fq], t[ks], r);
#pragma unroll
            for (int v = 0; v < 4; ++v) Xm[(16 * i + 4 * v + fq) * DL + 16 * j + fr] = -r[v];
        }
        __syncthreads();
    }
}

// Diagonal block of the Cholesky factorization.
//   in : A[o:o+nb, o:o+nb] (symmetric; only the lower triangle is read)
//   out: L[o:o+nb, o:o+nb] = L11 (lower, upper part zeroed)
//        Linv[o:o+nb, o:o+nb] = L11^-1 (lower, upper part zeroed)
//        Dinv (64 x 64, ld 64) = L11^-1 zero padded
//   flag: set to 1 when a pivot is <= 0 or not finite (the pivot is replaced by 1
//         so that the arithmetic stays finite; the caller reports ENOTPD).
__global__ __launch_bounds__(256) void chol_diag_kernel(const double* __restrict__ A, int64_t ld, int o, int nb,
                                                        double* __restrict__ L, double* __restrict__ Linv,
                                                        double* __restrict__ Dinv, int* __restrict__ flag)
{
    __shared__ double Am[NB * DL];
    __shared__ double Xm[NB * DL];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, fq = lane >> 4;
    for (int idx = tid; idx < NB * NB; idx += 256) {
        const int i = idx >> 6, j = idx & 63;
        double v = (i == j) ? 1.0 : 0.0;                    // identity padding past nb
        if (i < nb && j < nb) v = (j <= i) ? A[(int64_t)(o + i) * ld + o + j] : 0.0;
        Am[i * DL + j] = v;
        Xm[i * DL + j] = 0.0;
    }
    __syncthreads();
    for (int b = 0; b < 4; ++b) {
        const int base = 16 * b;
        if (wave == 0) {
            // unblocked Cholesky of the 16 x 16 diagonal tile; lane r (mod 16) holds row r of the
            // symmetric tile
            const int r = fr;
            double a[16], rsv[16];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                a[j] = (j <= r) ? Am[(base + r) * DL + base + j] : Am[(base + j) * DL + base + r];
            // the pivot of step k+1 is final as soon as column k+1 has been updated in step k, so
            // that update is done first and the next reciprocal square root is started before the
            // remaining updates of step k (they fill its latency)
            bool bad = false;
            double piv = readlane_f64(a[0], 0);
            bad = bad || !(piv > 0.0) || !(piv < 1.0e300);
            piv = bad ? 1.0 : piv;
            double rs = rsqrt(piv);
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                rsv[k] = rs;                                           // 1 / L[k][k]
                const double t = (r == k) ? piv * rs : a[k] * rs;      // l_rk for r >= k
                const double lm = (r > k) ? t : 0.0;
                a[k] = t;
                if (k + 1 < 16) {
                    a[k + 1] -= lm * readlane_f64(t, k + 1);
                    piv = readlane_f64(a[k + 1], k + 1);
                    const bool b2 = !(piv > 0.0) || !(piv < 1.0e300);
                    bad = bad || b2;
                    piv = b2 ? 1.0 : piv;
                    rs = rsqrt(piv);
                }
#pragma unroll
                for (int j = k + 2; j < 16; ++j) a[j] -= lm * readlane_f64(t, j);
            }
            if (bad && lane == 0) *flag = 1;
            if (lane < 16) {
#pragma unroll
                for (int j = 0; j < 16; ++j) Am[(base + r) * DL + base + j] = (j <= r) ? a[j] : 0.0;
            }
            __builtin_amdgcn_wave_barrier();
            // the tile's inverse by forward substitution: lane c (mod 16) solves L x = e_c; the
            // entries of L are wavefront-uniform LDS reads
            double sv[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) sv[i] = (i == r) ? 1.0 : 0.0;
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                const double xm = sv[m] * rsv[m];
                sv[m] = xm;
#pragma unroll
                for (int i = m + 1; i < 16; ++i) sv[i] -= Am[(base + i) * DL + base + m] * xm;
            }
            if (lane < 16) {
#pragma unroll
                for (int i = 0; i < 16; ++i) Xm[(base + i) * DL + base + r] = sv[i];
            }
        }
        __syncthreads();
        // panel: L_ib = A_ib * Linv_bb^T for the tiles below the diagonal tile
        {
            const int i = b + 1 + wave;
            if (i < 4) {
                d4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    acc = mfma4(Am[(16 * i + fr) * DL + base + 4 * ks + fq], Xm[(base + fr) * DL + base + 4 * ks + fq], acc);
#pragma unroll
                for (int v = 0; v < 4; ++v) Am[(16 * i + 4 * v + fq) * DL + base + fr] = acc[v];
            }
        }
        __syncthreads();
        // trailing tiles: A_ij -= L_ib L_jb^T for b < j <= i
        {
            int t = 0;
            for (int i = b + 1; i < 4; ++i)
                for (int j = b + 1; j <= i; ++j, ++t) {
                    if ((t & 3) != wave) continue;
                    d4 acc;
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[v] = Am[(16 * i + 4 * v + fq) * DL + 16 * j + fr];
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        acc = mfma4(-Am[(16 * i + fr) * DL + base + 4 * ks + fq], Am[(16 * j + fr) * DL + base + 4 * ks + fq], acc);
#pragma unroll
                    for (int v = 0; v < 4; ++v) Am[(16 * i + 4 * v + fq) * DL + 16 * j + fr] = acc[v];
                }
        }
        __syncthreads();
    }
    assemble_inverse(Xm, [&](int i, int m, int ks) { return Am[(16 * i + fr) * DL + 16 * m + 4 * ks + fq]; }, wave, fr, fq);
    for (int idx = tid; idx < NB * NB; idx += 256) {
        const int i = idx >> 6, j = idx & 63;
        const bool in = i < nb && j < nb;
        const double xv = (in && j <= i) ? Xm[i * DL + j] : 0.0;
        Dinv[idx] = xv;
        if (in) {
            L[(int64_t)(o + i) * ld + o + j] = (j <= i) ? Am[i * DL + j] : 0.0;
            Linv[(int64_t)(o + i) * ld + o + j] = xv;
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
// restricted to the block).  With A11 the current block, U11 its pivot rows,
// D = diag(U11) and Un11 = D^-1 U11 (unit upper):  A11 = Un11^T D Un11.
//   out: U[o+j, o+j : o+nb]  = pivot row j inside the block
//        Un = U / pivot
//        G (64 x 64, ld 64)  = (Un11^T)^-1 (unit lower): pivot rows right of the
//                              block are G * A[o:o+nb, o+nb:]
//        rinv[j] = 1 / pivot_j
// Same tile scheme as chol_diag_kernel, without square roots.
__global__ __launch_bounds__(256) void elim_diag_kernel(const double* __restrict__ A, int64_t ld, int o, int nb,
                                                        double* __restrict__ U, double* __restrict__ Un,
                                                        double* __restrict__ G, double* __restrict__ rinv,
                                                        int* __restrict__ flag)
{
    __shared__ double Am[NB * DL];     // current block (full symmetric); rows become pivot rows U
    __shared__ double Um[NB * DL];     // Un
    __shared__ double Xm[NB * DL];     // G
    __shared__ double rv[NB];          // 1 / pivot
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, fq = lane >> 4;
    for (int idx = tid; idx < NB * NB; idx += 256) {
        const int i = idx >> 6, j = idx & 63;
        double v = (i == j) ? 1.0 : 0.0;
        if (i < nb && j < nb) v = A[(int64_t)(o + min(i, j)) * ld + o + max(i, j)];   // upper triangle is the maintained one
        Am[i * DL + j] = v;
        Um[i * DL + j] = 0.0;
        Xm[i * DL + j] = 0.0;
    }
    __syncthreads();
    for (int b = 0; b < 4; ++b) {
        const int base = 16 * b;
        if (wave == 0) {
            // unblocked elimination of the 16 x 16 diagonal tile; lane r (mod 16) holds row r of
            // the symmetric tile
            const int r = fr;
            double a[16], pinv[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) a[j] = Am[(base + min(r, j)) * DL + base + max(r, j)];
            // as in chol_diag_kernel: update column k+1 first, start the next reciprocal, then the rest
            bool bad = false;
            double piv = readlane_f64(a[0], 0);
            bad = bad || !(piv > 0.0) || !(piv < 1.0e300);
            piv = bad ? 1.0 : piv;
            double pi = 1.0 / piv;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                pinv[k] = pi;
                const double cr = (r == k) ? piv : a[k];          // A[k][r] = U[k][r] for r >= k
                const double fm = (r > k) ? cr * pi : 0.0;        // Un[k][r]
                a[k] = cr;
                if (k + 1 < 16) {
                    a[k + 1] -= fm * readlane_f64(cr, k + 1);
                    piv = readlane_f64(a[k + 1], k + 1);
                    const bool b2 = !(piv > 0.0) || !(piv < 1.0e300);
                    bad = bad || b2;
                    piv = b2 ? 1.0 : piv;
                    pi = 1.0 / piv;
                }
#pragma unroll
                for (int j = k + 2; j < 16; ++j) a[j] -= fm * readlane_f64(cr, j);
            }
            if (bad && lane == 0) *flag = 1;
            if (lane < 16) {
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    // lane r holds column r of the pivot rows: U[k][r] for k <= r
                    if (k <= r) {
                        Am[(base + k) * DL + base + r] = a[k];
                        Um[(base + k) * DL + base + r] = (k == r) ? 1.0 : a[k] * pinv[k];
                    }
                    if (k == r) rv[base + k] = pinv[k];
                }
            }
            __builtin_amdgcn_wave_barrier();
            // G_bb = (Un_bb^T)^-1 (unit lower) by forward substitution: lane c (mod 16) solves
            // Un_bb^T x = e_c; entry [i][m] of Un_bb^T is Un[m][i], a wavefront-uniform LDS read
            double sv[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) sv[i] = (i == r) ? 1.0 : 0.0;
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                const double xm = sv[m];
#pragma unroll
                for (int i = m + 1; i < 16; ++i) sv[i] -= Um[(base + m) * DL + base + i] * xm;
            }
            if (lane < 16) {
#pragma unroll
                for (int i = 0; i < 16; ++i) Xm[(base + i) * DL + base + r] = sv[i];
            }
        }
        __syncthreads();
        // pivot rows right of the diagonal tile: U_bj = G_bb * A_bj, Un_bj = D^-1 U_bj
        {
            const int j = b + 1 + wave;
            if (j < 4) {
                d4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    acc = mfma4(Xm[(base + fr) * DL + base + 4 * ks + fq], Am[(base + 4 * ks + fq) * DL + 16 * j + fr], acc);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    Am[(base + 4 * v + fq) * DL + 16 * j + fr] = acc[v];
                    Um[(base + 4 * v + fq) * DL + 16 * j + fr] = acc[v] * rv[base + 4 * v + fq];
                }
            }
        }
        __syncthreads();
        // trailing tiles: A_ij -= Un_bi^T U_bj for b < i <= j
        {
            int t = 0;
            for (int i = b + 1; i < 4; ++i)
                for (int j = i; j < 4; ++j, ++t) {
                    if ((t & 3) != wave) continue;
                    d4 acc;
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[v] = Am[(16 * i + 4 * v + fq) * DL + 16 * j + fr];
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        acc = mfma4(-Um[(base + 4 * ks + fq) * DL + 16 * i + fr], Am[(base + 4 * ks + fq) * DL + 16 * j + fr], acc);
#pragma unroll
                    for (int v = 0; v < 4; ++v) Am[(16 * i + 4 * v + fq) * DL + 16 * j + fr] = acc[v];
                }
        }
        __syncthreads();
    }
    // G = (Un11^T)^-1: tile T_im of Un11^T is Un_mi transposed
    assemble_inverse(Xm, [&](int i, int m, int ks) { return Um[(16 * m + 4 * ks + fq) * DL + 16 * i + fr]; }, wave, fr, fq);
    for (int idx = tid; idx < NB * NB; idx += 256) {
        const int i = idx >> 6, j = idx & 63;
        const bool in = i < nb && j < nb;
        G[idx] = (in && j <= i) ? Xm[i * DL + j] : 0.0;
        if (in && j >= i) {
            U[(int64_t)(o + i) * ld + o + j] = Am[i * DL + j];
            Un[(int64_t)(o + i) * ld + o + j] = Um[i * DL + j];
        }
    }
    if (tid < NB) rinv[tid] = (tid < nb) ? rv[tid] : 0.0;
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
