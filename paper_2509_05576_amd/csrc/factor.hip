// Dense factorizations of the path, all fp64, all blocked with 64-wide panels:
//   cholesky_lower   H_d = L L^T                       (Section 5, item 1); for d up to a limit its panel
//                    launches also carry L^-1 and Hinv = L^-T L^-1 (tiles in the shadow of the
//                    critical path), otherwise:
//   trtri_lower      L^-1 by recursive doubling of the block size
//   lauum_upper      Hinv = L^-T L^-1
//   eliminate_blocked the shared-Hinv elimination of Eq. 12, B columns at a time:
//                    after column t is processed, Hinv -= Hinv[:,t] Hinv[t,:] / Hinv[t,t].
//                    The pivot rows are kept:  U[t, t:]  = Hinv^(t)[t, t:]  and
//                    Un[t, :] = U[t, :] / U[t, t]; the weight compensation of Eq. 9 / 11
//                    for step t is  W[:, k] -= (w_t - q_t) * Un[t, k].
// The 64 x 64 diagonal blocks are handled by one workgroup in LDS; everything
// else is a rank-64 update on the matrix cores, fused into the panel launches
// (chol_iter_kernel, elim_iter_kernel) or through gemm64.
#include <hip/hip_ext.h>

#include "fobq_internal.h"

namespace fobq {

constexpr int NB = 64;

// ---------------------------------------------------------------------------
// 64 x 64 diagonal blocks.  Both diagonal-block kernels keep the block in LDS and
// work on it as a 4 x 4 grid of 16 x 16 tiles.  The only sequential arithmetic is
// the unblocked sweep over the 16 pivots of a diagonal tile: one wavefront, one
// row (Cholesky) or column (elimination) of the whole block per lane, so the same
// sweep also produces the tiles below (right of) the diagonal tile; pivot rows are
// broadcast with v_readlane (next column) and LDS reads (the columns after it).  A
// wavefront on its own issues one instruction of any kind per 5 to 8 cycles, so the
// sweep costs its instruction count.  The triangular inverse of a diagonal tile comes out
// of the same sweep, in lanes it would leave idle (the first tile's: a forward
// substitution on a second wavefront during the next sweep).  Everything else --
// trailing update, assembly of the 64 x 64 triangular inverse from the tile
// inverses -- is 16 x 16 x 16 products on the matrix cores (4 MFMAs each), one tile
// per wavefront, one interval behind the sweeps.
typedef double d4 __attribute__((ext_vector_type(4)));
constexpr int NT = 512;   // threads per workgroup of every kernel in this file (8 wavefronts)
// launches with more tiles than this use the two-workgroups-per-compute-unit variant of the panel kernels
constexpr int DENSE_LAUNCH_TILES = 300;
// launches with at least this many trailing tiles are bound by tile throughput: the panel is stored by a launch of
// its own and every tile does one product instead of three (see chol_iter_kernel)
constexpr int STORED_PANEL_TILES = 800;
// The workgroup that holds the place beside workgroup 0 (see chol_iter_kernel) has the index `mate_slot` = the number
// of compute units of the device (the first that many workgroups of a launch go to distinct compute units).
constexpr int MATE_MAX_NAPS = 64;
constexpr int DL = 66;    // LDS row stride (doubles): conflict-free 8-byte MFMA fragment reads per half-wave
constexpr int CB0 = 48, CB_LEN = CB0 + 16 * 16 + 48;   // sweep column buffer: see chol_block
constexpr int SWEEP_LDS = NB + CB_LEN + 16 * DL;   // doubles of LDS that chol_block / elim_block need besides the two tiles

__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// Reciprocal and reciprocal square root of a pivot (a normal, positive number): the hardware
// approximation r0 (good to about 2^-24) with one third-order correction,
//   1/x       = r0 (1 + e + e^2 + ...),            e = 1 - x r0
//   1/sqrt(x) = y0 (1 + e/2 + 3 e^2 / 8 + ...),    e = 1 - x y0^2
// accurate to about one ulp (measured 1.00 / 1.24 ulp, the same as two Newton steps).  Four / five
// dependent operations: these sit on the sequential path of the tile sweeps.
__device__ __forceinline__ double pivot_rcp(double x)
{
    const double r0 = __builtin_amdgcn_rcp(x);
    const double e = fma(-x, r0, 1.0);
    return fma(r0 * e, 1.0 + e, r0);
}

__device__ __forceinline__ double pivot_rsqrt(double x)
{
    const double y0 = __builtin_amdgcn_rsq(x);
    const double e = fma(-(x * y0), y0, 1.0);
    return fma(y0 * e, fma(0.375, e, 0.5), y0);
}

__device__ __forceinline__ d4 mfma4(double a, double b, d4 c)
{
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// One off-diagonal 16 x 16 tile of the inverse X of a 64 x 64 lower triangular matrix T:
//   X_ij = -X_ii sum_{m=j}^{i-1} T_im X_mj        (X_ii and the X_mj already in Xm).
// tfetch(i, m, ks) returns this lane's A-operand element of tile T_im for k-step ks, i.e.
// T_im[fr][4 ks + fq].  One wavefront.  inv_tile_sum adds the terms m0 <= m < m1 to t,
// inv_tile_finish multiplies by -X_ii and stores the tile.
template <class TF>
__device__ __forceinline__ d4 inv_tile_sum(const double* Xm, TF tfetch, int i, int j, int m0, int m1, d4 t, int fr,
                                           int fq)
{
    for (int m = m0; m < m1; ++m)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            t = mfma4(tfetch(i, m, ks), Xm[(16 * m + 4 * ks + fq) * DL + 16 * j + fr], t);
    return t;
}

__device__ __forceinline__ void inv_tile_finish(double* Xm, int i, int j, d4 t, int fr, int fq)
{
    // the accumulator layout (row 4 v + fq, column fr) is the B-operand layout of k-step v
    d4 r = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) r = mfma4(Xm[(16 * i + fr) * DL + 16 * i + 4 * ks + fq], t[ks], r);
#pragma unroll
    for (int v = 0; v < 4; ++v) Xm[(16 * i + 4 * v + fq) * DL + 16 * j + fr] = -r[v];
    __builtin_amdgcn_wave_barrier();
}

template <class TF>
__device__ __forceinline__ void inv_tile(double* Xm, TF tfetch, int i, int j, int fr, int fq)
{
    inv_tile_finish(Xm, i, j, inv_tile_sum(Xm, tfetch, i, j, j, i, d4{0.0, 0.0, 0.0, 0.0}, fr, fq), fr, fq);
}

// Schedule shared by chol_block and elim_block.  sweep(b): pivots of diagonal tile b and the
// tiles below / right of it -- and, for b >= 1, the inverse X_bb of the diagonal tile, carried along in
// 16 lanes that the sweep leaves idle; tinv(0): triangular inverse of diagonal tile 0 into Xm;
// trail(b): update of the tiles behind tile row/column b; tf: tile fetch for inv_tile.
//   interval   wavefront 0        wavefront 1   wavefront 2   wavefronts 3, 4, 5
//   b = 0      sweep(0)
//   b = 1      sweep(1) + X_11    tinv(0)
//   b = 2      sweep(2) + X_22                  X_10
//   b = 3      sweep(3) + X_33    X_21          X_20          the sums of X_30, X_31, X_32 as far as they
//                                                             do not need this interval's tiles
//   then                                                      rest of the sums, times -X_33
//   (after each of b = 0..2: trail(b) on all wavefronts)
// Called by all NT threads of the workgroup (at least 6 wavefronts); ends with a barrier.
template <class SW, class TI, class TR, class TF>
__device__ __forceinline__ void block_schedule(double* Xm, SW sweep, TI tinv, TR trail, TF tf)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fr = lane & 15, fq = lane >> 4;
    d4 t = {0.0, 0.0, 0.0, 0.0};
    const int j3 = wave - 3;                       // wavefronts 3, 4, 5: column tile of X_3j
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (wave == 0) sweep(b);
        else if (wave == 1 && b == 1) tinv(0);
        else if (wave == 2 && b == 2) inv_tile(Xm, tf, 1, 0, fr, fq);
        else if (wave == 1 && b == 3) inv_tile(Xm, tf, 2, 1, fr, fq);
        else if (wave == 2 && b == 3) inv_tile(Xm, tf, 2, 0, fr, fq);
        else if (wave >= 3 && wave <= 5 && b == 3)
            t = inv_tile_sum(Xm, tf, 3, j3, j3, j3 == 2 ? 3 : 2, t, fr, fq);   // X_2j is not there yet
        __syncthreads();
        if (b < 3) {
            trail(b);
            __syncthreads();
        }
    }
    if (wave >= 3 && wave <= 5) {
        if (j3 < 2) t = inv_tile_sum(Xm, tf, 3, j3, 2, 3, t, fr, fq);
        inv_tile_finish(Xm, 3, j3, t, fr, fq);
    }
    __syncthreads();
}

// Cholesky of the 64 x 64 block held in LDS.
//   in : Am lower triangle = the block (identity padding past its size); Xm need not be initialised (every
//        entry of its lower triangle, whole diagonal 16 x 16 tiles included, is written before it is read)
//   out: Am = L (lower; what is above the diagonal is not defined),
//        Xm = L^-1 (lower);  rq (SWEEP_LDS doubles of LDS) is scratch: 1 / L[k][k], then the sweep columns
//   flag: set to 1 when a pivot is <= 0 or not finite (the pivot is replaced by 1 so that
//         the arithmetic stays finite; the caller reports ENOTPD).
// Called by all NT threads of the workgroup; ends with a barrier.
__device__ __forceinline__ void chol_block(double* Am, double* Xm, double* rq, int* __restrict__ flag)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, fq = lane >> 4;
    // The columns of the running sweep: column k at cb[CB0 + 16 k + r], r = row - tile base.  Only the
    // 16 tile rows are read; what the other lanes write falls into the slots of neighbouring columns,
    // which is harmless: a column is read right after it is written, before the next one is written.
    double* cb = rq + NB;
    double* idt = cb + CB_LEN; // 16 rows of the identity, row stride DL (read from the second sweep on)
    if (tid < 256) idt[(tid >> 4) * DL + (tid & 15)] = (tid >> 4) == (tid & 15) ? 1.0 : 0.0;

    // Right-looking Cholesky of the 16 columns base .. base+15 of the block over all rows
    // >= base: lane rho holds row rho.  Rows inside the diagonal tile (0 <= r < 16) hold the
    // tile row (what lies right of its diagonal is carried along and never used); rows below it
    // (r >= 16) get their part of L in the same sweep (l_rho,k = (a_rho,k - sum l l) / l_kk);
    // rows above (r < 0) idle on harmless values.
    auto sweep = [&](int b) {
        const int base = 16 * b, rho = lane, r = rho - base;
        // For b >= 1 the lanes 0..15 (rows above the tile, otherwise idle) carry the rows of the identity
        // as if they were rows below the tile: those become I L_bb^-T, i.e. lane c ends with column c of
        // X_bb = L_bb^-1, for the price of no extra instruction.
        const bool idl = b > 0 && lane < 16;
        // one row of 16 per lane: its own (columns j > r of a tile row are never used), or a row of the identity
        const double* src = idl ? idt + lane * DL : Am + rho * DL + base;
        double a[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) a[j] = src[j];
        // Each lane of the tile also keeps its own diagonal entry in `dg` and updates it locally
        // (dg -= l_rk^2), so the pivot of step k+1 is available one fma after l_rk: the
        // sequential chain per step is readlane, reciprocal square root, multiply, fma.  A wavefront on
        // its own issues an instruction of any kind every 5 to 8 cycles, so the sweep costs its
        // instruction count: nothing sits in the loop that can be done once after it.
        double dg = Am[rho * DL + rho];
        double tp = 0.0, lb[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const double rs = pivot_rsqrt(readlane_f64(dg, base + k));     // 1 / L[k][k]
            // l_rk for r >= k (lane k's a[k] has had the same updates as its dg: it is the pivot).  Lanes
            // of rows above the pivot go through the same arithmetic on entries that are never stored.
            const double t = a[k] * rs;
            dg -= t * t;
            a[k] = t;
            // Rank-1 update of the columns behind: the next column takes l_jk by readlane (it is on the
            // sequential path), the others take it one step late as a broadcast read of the column that
            // every lane leaves in LDS: half an instruction per column instead of two readlanes.
            cb[CB0 + 16 * k + r] = t;
            if (k > 0) {
#pragma unroll
                for (int j = k + 1; j < 16; ++j) a[j] -= tp * lb[j];
            }
            if (k < 15) a[k + 1] -= t * readlane_f64(t, base + k + 1);
#pragma unroll
            for (int j = k + 2; j < 16; ++j) lb[j] = cb[CB0 + 16 * k + j];   // in flight during the next pivot
            tp = t;
        }
        if (r >= 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) Am[rho * DL + base + j] = a[j];
            if (r < 16) {
                // A pivot that is not a positive normal number (nor anything after it) leaves no positive
                // finite L[r][r] behind: one test per tile row after the sweep instead of one per pivot.
                const double lrr = Am[rho * DL + rho];
                if (!(lrr > 0.0) || !(lrr < 1.0e300)) *flag = 1;
                rq[rho] = pivot_rcp(lrr);
            }
        }
        if (idl) {
#pragma unroll
            for (int k = 0; k < 16; ++k) Xm[(base + k) * DL + base + lane] = a[k];
        }
    };
    // the diagonal tile's inverse by forward substitution: lane c (mod 16) solves L x = e_c;
    // the entries of L and the pivot reciprocals are wavefront-uniform LDS reads
    auto tinv = [&](int b) {
        const int base = 16 * b, c = fr;
        double sv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) sv[i] = (i == c) ? 1.0 : 0.0;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const double xm = sv[m] * rq[base + m];
            sv[m] = xm;
#pragma unroll
            for (int i = m + 1; i < 16; ++i) sv[i] -= Am[(base + i) * DL + base + m] * xm;
        }
        if (lane < 16) {
#pragma unroll
            for (int i = 0; i < 16; ++i) Xm[(base + i) * DL + base + c] = sv[i];
        }
        __builtin_amdgcn_wave_barrier();
    };
    // trailing tiles: A_ij -= L_ib L_jb^T for b < j <= i
    auto trail = [&](int b) {
        const int base = 16 * b;
        int t = 0;
        for (int i = b + 1; i < 4; ++i)
            for (int j = b + 1; j <= i; ++j, ++t) {
                if ((t & (NT / 64 - 1)) != wave) continue;
                d4 acc;
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[v] = Am[(16 * i + 4 * v + fq) * DL + 16 * j + fr];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    acc = mfma4(-Am[(16 * i + fr) * DL + base + 4 * ks + fq], Am[(16 * j + fr) * DL + base + 4 * ks + fq], acc);
#pragma unroll
                for (int v = 0; v < 4; ++v) Am[(16 * i + 4 * v + fq) * DL + 16 * j + fr] = acc[v];
            }
    };
    block_schedule(Xm, sweep, tinv, trail,
                   [&](int i, int m, int ks) { return Am[(16 * i + fr) * DL + 16 * m + 4 * ks + fq]; });
}

// Fragment layout of a 64 x 64 block inverse M that the next launch uses as an MFMA operand:
//   F[((w * 16 + ks) * 2 + h) * 64 + lane] = M[w * 32 + h * 16 + (lane & 15)][4 * ks + (lane >> 4)]
// so that the 64 lanes of a wavefront read 512 contiguous bytes per operand element instead of
// 16 scattered 32-byte pieces.  frag_source returns the (row, column) of M stored at F[idx].
__device__ __forceinline__ void frag_source(int idx, int& row, int& col)
{
    const int lane = idx & 63, h = (idx >> 6) & 1, ks = (idx >> 7) & 15, w = idx >> 11;
    row = w * 32 + h * 16 + (lane & 15);
    col = 4 * ks + (lane >> 4);
}

__device__ __forceinline__ void chol_block_store(const double* Am, const double* Xm, int64_t ld, int o, int nb,
                                                 double* __restrict__ L, double* __restrict__ Linv,
                                                 double* __restrict__ Dinv)
{
    for (int idx = threadIdx.x; idx < NB * NB; idx += NT) {
        const int i = idx >> 6, j = idx & 63;
        const bool in = i < nb && j < nb;
        const double xv = (in && j <= i) ? Xm[i * DL + j] : 0.0;
        int fi, fj;
        frag_source(idx, fi, fj);
        Dinv[idx] = (fi < nb && fj <= fi) ? Xm[fi * DL + fj] : 0.0;     // fj <= fi < nb
        if (in) {
            if (L) L[(int64_t)(o + i) * ld + o + j] = (j <= i) ? Am[i * DL + j] : 0.0;
            Linv[(int64_t)(o + i) * ld + o + j] = xv;
        }
    }
}

// Diagonal block of the Cholesky factorization (stand-alone launch: first block, and every
// block of the unfused path).
//   in : A[o:o+nb, o:o+nb] (symmetric; only the lower triangle is read)
//   out: L[o:o+nb, o:o+nb] = L11 (lower, upper part zeroed)
//        Linv[o:o+nb, o:o+nb] = L11^-1 (lower, upper part zeroed)
//        Dinv (4096 doubles) = L11^-1 zero padded, in the fragment layout
__global__ __launch_bounds__(NT) void chol_diag_kernel(const double* __restrict__ A, int64_t ld, int o, int nb,
                                                        double* __restrict__ L, double* __restrict__ Linv,
                                                        double* __restrict__ Dinv, int* __restrict__ flag)
{
    __shared__ double Am[NB * DL];
    __shared__ double Xm[NB * DL];
    __shared__ double rq[SWEEP_LDS];
    for (int idx = threadIdx.x; idx < NB * NB; idx += NT) {
        const int i = idx >> 6, j = idx & 63;
        double v = (i == j) ? 1.0 : 0.0;                    // identity padding past nb
        if (i < nb && j < nb) v = (j <= i) ? A[(int64_t)(o + i) * ld + o + j] : 0.0;
        Am[i * DL + j] = v;
    }
    __syncthreads();
    chol_block(Am, Xm, rq, flag);
    chol_block_store(Am, Xm, ld, o, nb, L, Linv, Dinv);
}

// t = big (big + 1) / 2 + small, 0 <= small <= big
__device__ __forceinline__ void tri_decode(int t, int& big, int& small)
{
    int i = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while ((i + 1) * (i + 2) / 2 <= t) ++i;
    while (i * (i + 1) / 2 > t) --i;
    big = i;
    small = t - i * (i + 1) / 2;
}

// A 64 x 64 lower-triangular block T in the fragment layout (frag_source) as an MFMA operand: operand tile
// t (of 4; 16 rows of T as A-operand, or 16 columns of T^T as B-operand) only needs the k-steps 0 .. 4 t + 3.
// A wavefront takes the two operand tiles {W, 3 - W}, W = 0 or 1: 20 of 32 (k-step, tile) pairs either way.
// W is a template parameter so that the k-loops below are straight-line code: with a run-time W
// every skipped pair is a branch, and the branches keep the LDS reads of one k-step from being
// issued under the MFMAs of the one before.
template <int W>
__device__ __forceinline__ void tri_frag_load(const double* __restrict__ F, int lane, double (&g)[16][2])
{
    constexpr int t[2] = {W, 3 - W};
#pragma unroll
    for (int ks = 0; ks < 16; ++ks)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            g[ks][j] = (ks <= 4 * t[j] + 3) ? F[(((t[j] >> 1) * 16 + ks) * 2 + (t[j] & 1)) * 64 + lane] : 0.0;
}

// li (+ lj if TWO) += P T^T for the wavefront's 16 rows (from row0) and its two column tiles {W, 3 - W}:
// A-operand rows out of LDS (Pi / Pj, row-major [row][k]), B-operand = g.
template <int W, bool TWO>
__device__ __forceinline__ void tri_right_product(const double* Pi, const double* Pj, const double (&g)[16][2],
                                                  int row0, int fr, int fq, d4 (&li)[2], d4 (&lj)[2])
{
    constexpr int t[2] = {W, 3 - W};
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const double ai = Pi[(row0 + fr) * DL + 4 * ks + fq];
        double aj = 0.0;
        if (TWO) aj = Pj[(row0 + fr) * DL + 4 * ks + fq];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if (ks > 4 * t[j] + 3) continue;
            li[j] = mfma4(ai, g[ks][j], li[j]);
            if (TWO) lj[j] = mfma4(aj, g[ks][j], lj[j]);
        }
    }
}

// ui (+ uj if TWO) += T P for the wavefront's two row tiles {W, 3 - W} and its 16 columns (from col0):
// A-operand = g, B-operand columns out of LDS (Pi / Pj, row-major [k][column]).
template <int W, bool TWO>
__device__ __forceinline__ void tri_left_product(const double* Pi, const double* Pj, const double (&g)[16][2],
                                                 int col0, int fr, int fq, d4 (&ui)[2], d4 (&uj)[2])
{
    constexpr int t[2] = {W, 3 - W};
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const double bi = Pi[(4 * ks + fq) * DL + col0 + fr];
        double bj = 0.0;
        if (TWO) bj = Pj[(4 * ks + fq) * DL + col0 + fr];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (ks > 4 * t[i] + 3) continue;
            ui[i] = mfma4(g[ks][i], bi, ui[i]);
            if (TWO) uj[i] = mfma4(g[ks][i], bj, uj[i]);
        }
    }
}

// Work split of the fused panel kernels below: NT = 512 threads = 8 wavefronts per 64 x 64 tile, two per
// SIMD.  One wavefront alone issues a v_mfma_f64_16x16x4_f64 only every ~140 cycles (measured: 59 ns per
// instruction per wavefront whatever the number of independent accumulators); two wavefronts on a SIMD
// interleave to the pipe's own rate of one per ~64 cycles.  The products of workgroup 0 are on the critical
// path of the whole factorization, so they are spread over twice the wavefronts a 64 x 64 tile needs.
// Wavefront w: wr = w / 2 is its 16-row slice of the tile, w2 = w % 2 its 32-column half (and the parity
// W of its operand tiles in the triangular products).

// Triangular inverse alongside the factorization (right-looking): with S_ij = sum_{m=j}^{i-1} L_im Linv_mj
// the blocks of L^-1 below the diagonal are Linv_ij = -Linv_ii S_ij.  In the launch of panel p, once
// per tile (i, j), i > p >= j:
//     L_ip    = A_ip Linv_pp^T                      (the same panel product as the trailing tiles)
//     Linv_pj = -Linv_pp S_pj  (j < p),  Linv_pp    (j = p)     -- S_pj is complete after launch p - 1
//     S_ij   += L_ip Linv_pj                        (first touched, from zero, when j = p)
// and the tiles of row i = p + 1 store Linv_pj.  S lives in Sacc (d x d, lower blocks); the last block
// row of L^-1 is finished by the caller.  These tiles run in the shadow of workgroup 0, like the
// trailing tiles, so the inverse costs no launches of its own.
__device__ __forceinline__ void chol_inverse_tile(double* lds, const double* __restrict__ Hd, int d, int o, int it,
                                                  int jt, const double* __restrict__ Dinv,
                                                  double* __restrict__ Linv, double* __restrict__ Sacc)
{
    double* Pi = lds;
    double* Pj = lds + NB * DL;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, w2 = wave & 1, fr = lane & 15, fq = lane >> 4;
    const int mi0 = NB * it, n0 = NB * jt;
    const bool at_panel = n0 == o;                     // j = p
    // Linv_pp is the B-operand (transposed) of the first product and the A-operand of the second: the
    // same fragment elements serve both
    const int t2[2] = {w2, 3 - w2};
    double g[16][2];
    if (w2 == 0) tri_frag_load<0>(Dinv, lane, g); else tri_frag_load<1>(Dinv, lane, g);
    double pa[8], pb[8];
    const double* __restrict__ src = at_panel ? Linv + (int64_t)o * d + o : Sacc + (int64_t)o * d + n0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        pa[u] = Hd[(int64_t)min(mi0 + y, d - 1) * d + o + x];          // A_ip (rows past d: see chol_iter_kernel)
        pb[u] = src[(int64_t)y * d + x];                               // S_pj, or Linv_pp itself
    }
    d4 c[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gm = mi0 + wr * 16 + 4 * v + fq, gn = n0 + w2 * 32 + j * 16 + fr;
            c[j][v] = at_panel ? 0.0 : Sacc[(int64_t)min(gm, d - 1) * d + gn];
        }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        Pi[y * DL + x] = pa[u];
        Pj[y * DL + x] = pb[u];
    }
    __syncthreads();
    d4 li[2], xp[2], none[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) { li[j] = d4{0.0, 0.0, 0.0, 0.0}; xp[j] = d4{0.0, 0.0, 0.0, 0.0}; }
    if (w2 == 0) {
        tri_right_product<0, false>(Pi, Pi, g, wr * 16, fr, fq, li, none);
        if (!at_panel) tri_left_product<0, false>(Pj, Pj, g, wr * 16, fr, fq, xp, none);
    } else {
        tri_right_product<1, false>(Pi, Pi, g, wr * 16, fr, fq, li, none);
        if (!at_panel) tri_left_product<1, false>(Pj, Pj, g, wr * 16, fr, fq, xp, none);
    }
    __syncthreads();
    // Pi := L_ip (row m, panel column k), Pj := Linv_pj (panel row k, column n)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            Pi[(wr * 16 + 4 * v + fq) * DL + t2[j] * 16 + fr] = li[j][v];
            if (!at_panel) {
                const int m = t2[j] * 16 + 4 * v + fq, n = wr * 16 + fr;
                Pj[m * DL + n] = -xp[j][v];
                if (mi0 == o + NB) Linv[(int64_t)(o + m) * d + n0 + n] = -xp[j][v];
            }
        }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const double a = Pi[(wr * 16 + fr) * DL + 4 * ks + fq];
#pragma unroll
        for (int j = 0; j < 2; ++j) c[j] = mfma4(a, Pj[(4 * ks + fq) * DL + w2 * 32 + j * 16 + fr], c[j]);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gm = mi0 + wr * 16 + 4 * v + fq, gn = n0 + w2 * 32 + j * 16 + fr;
            if (gm < d) Sacc[(int64_t)gm * d + gn] = c[j][v];
        }
}

// Hinv = Linv^T Linv alongside the factorization: block row k of L^-1 is complete one launch after its
// panel, and adds Linv_km^T Linv_kn to every tile (m, n), m <= n <= k, of the upper triangle of Hinv
// (first touched, from zero, when n = k).  One tile per workgroup, again in the shadow of workgroup 0.
__device__ __forceinline__ void chol_lauum_tile(double* lds, int d, int kt, int mt, int nt,
                                                const double* __restrict__ Linv, double* __restrict__ Hinv)
{
    double* Pi = lds;
    double* Pj = lds + NB * DL;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, w2 = wave & 1, fr = lane & 15, fq = lane >> 4;
    const bool first = nt == kt;
    const double* __restrict__ rowk = Linv + (int64_t)NB * kt * d;
    double pa[8], pb[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        pa[u] = rowk[(int64_t)y * d + NB * mt + x];
        pb[u] = rowk[(int64_t)y * d + NB * nt + x];
    }
    d4 c[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gm = NB * mt + wr * 16 + 4 * v + fq, gn = NB * nt + w2 * 32 + j * 16 + fr;
            c[j][v] = first ? 0.0 : Hinv[(int64_t)gm * d + gn];
        }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        Pi[y * DL + x] = pa[u];
        Pj[y * DL + x] = pb[u];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const double a = Pi[(4 * ks + fq) * DL + wr * 16 + fr];
#pragma unroll
        for (int j = 0; j < 2; ++j) c[j] = mfma4(a, Pj[(4 * ks + fq) * DL + w2 * 32 + j * 16 + fr], c[j]);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gm = NB * mt + wr * 16 + 4 * v + fq, gn = NB * nt + w2 * 32 + j * 16 + fr;
            Hinv[(int64_t)gm * d + gn] = c[j][v];
        }
}

// One whole iteration of the blocked Cholesky factorization in a single launch.  The panel is
// the 64 columns o .. o+63, whose diagonal block has already been factored (Dinv = L11^-1).
// Workgroup (ti, tj), ti >= tj, owns the 64 x 64 tile (ti, tj) of the trailing matrix:
//   1. it recomputes the two panel blocks it needs, L21_i = A21_i L11^-T and L21_j (three
//      rank-64 MFMA products per tile instead of one, in exchange for not waiting on a
//      separate panel launch); the tiles of the first tile column also store L21_i into L;
//   2. A22(ti, tj) -= L21_i L21_j^T;
//   3. workgroup 0 owns tile (0, 0), the next diagonal block: it does not write it back but
//      factors it right away (chol_block) and stores L11, L11^-1 and Dinv_next for the next
//      launch, overlapped with the other tiles of this launch.
// Workgroups past the ntrail trailing tiles (when Sacc != null) are first the ninv tiles of the triangular
// inverse (chol_inverse_tile): (row block, column block) = (o / 64 + 1 + e / (o / 64 + 1), e % (o / 64 + 1)),
// then the tiles of Hinv that block row o / 64 - 1 of L^-1 contributes to (chol_lauum_tile).
// WPS = wavefronts per SIMD the register budget allows: 2 (one workgroup per compute unit, workgroup 0 has
// its matrix pipes to itself: faster while the launch's tiles fit in workgroup 0's shadow anyway) or 4
// (two workgroups per compute unit: more tile throughput for the large launches).
// MODE: PANEL_FUSED as described; for launches so large that tile throughput, not workgroup 0, bounds them, the
// panel is stored once instead of being recomputed by every tile (one product per tile instead of three):
// PANEL_ONLY = workgroup i computes and stores L21_i (nothing else), PANEL_STORED = the trailing launch that
// follows it and takes L21_i, L21_j from L (L must not be null; no inverse tiles ride along).
// Two such panels can share one pass over the trailing matrix, which is what bounds those launches: after the
// first panel of a pair only the next panel's tiles are updated (PANEL_NEAR: one launch, workgroup i owns tile (i, 0),
// recomputes L21_i and L21_0 like PANEL_FUSED and stores L21_i), after the second every trailing tile takes both
// panels, the older one first (PANEL_STORED2: the 128 columns o - 64 .. o + 63 of L) -- the same operations on every
// element in the same order as two single-panel launches.
enum { PANEL_FUSED = 0, PANEL_ONLY = 1, PANEL_STORED = 2, PANEL_NEAR = 3, PANEL_STORED2 = 4 };
template <int WPS, int MODE>
__global__ __launch_bounds__(NT, WPS) void chol_iter_kernel(double* __restrict__ Hd, int d, int o,
                                                       const double* __restrict__ Dinv, double* __restrict__ L,
                                                       double* __restrict__ Linv, double* __restrict__ Dinv_next,
                                                       int* __restrict__ flag, int ntrail, int ninv,
                                                       double* __restrict__ Sacc, double* __restrict__ Hinv,
                                                       int* __restrict__ mate_flag, int epoch, int mate_slot)
{
    // sweep scratch first (its broadcast reads then have constant addresses below 64 KB, i.e. no address
    // register), then two tiles: 2 workgroups per compute unit
    __shared__ double lds[SWEEP_LDS + 2 * NB * DL];
    double* tiles = lds + SWEEP_LDS;
    // Two workgroups fit a compute unit in this variant, and the one that lands beside workgroup 0 takes
    // matrix-pipe and LDS time from the launch's critical path.  The first 256 workgroups go to distinct
    // compute units, so that neighbour is workgroup `mate_slot` (measured: leaving that index idle is the only
    // one that shortens the launch).  It is not a tile: one of its wavefronts sleeps, holding the place,
    // until workgroup 0 says that it is done (mate_flag reaches this launch's epoch) or MATE_MAX_NAPS naps of
    // about 0.4 us have passed -- a bounded wait, it ends whatever workgroup 0 does.
    if (WPS == 4 && (int)blockIdx.x == mate_slot) {
        if (threadIdx.x >= 64) return;
        for (int i = 0; i < MATE_MAX_NAPS; ++i) {
            if (__hip_atomic_load(mate_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch >= 0) break;
            __builtin_amdgcn_s_sleep(16);
        }
        return;
    }
    const int bid = (int)blockIdx.x - ((WPS == 4 && (int)blockIdx.x > mate_slot) ? 1 : 0);
    if (MODE == PANEL_FUSED && bid >= ntrail + ninv) {
        // tiles of the Hinv role in this launch; a workgroup past them has nothing to do
        const int nlau = Sacc ? (o / NB) * (o / NB + 1) / 2 : 0;
        if (bid - ntrail - ninv >= nlau) return;
        int nt, mt;
        tri_decode(bid - ntrail - ninv, nt, mt);          // mt <= nt <= o / 64 - 1
        chol_lauum_tile(tiles, d, o / NB - 1, mt, nt, Linv, Hinv);
        return;
    }
    if (MODE == PANEL_FUSED && bid >= ntrail) {
        const int pcols = o / NB + 1, e = bid - ntrail;
        chol_inverse_tile(tiles, Hd, d, o, o / NB + 1 + e / pcols, e % pcols, Dinv, Linv, Sacc);
        return;
    }
    if (MODE != PANEL_FUSED && bid >= ntrail) return;
    double* Pi = tiles;
    double* Pj = tiles + NB * DL;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wn = wave & 1, fr = lane & 15, fq = lane >> 4;
    const int r0 = o + NB;
    int ti, tj;
    if (MODE == PANEL_ONLY) { ti = bid; tj = bid; }      // workgroup i: row tile i of the panel (ntrail = row tiles)
    else if (MODE == PANEL_NEAR) { ti = bid; tj = 0; }   // workgroup i: tile (i, 0), the next panel (ntrail = row tiles)
    else tri_decode(bid, ti, tj);
    const bool diag_tile = ti == tj;
    const int mi0 = r0 + NB * ti, mj0 = r0 + NB * tj;
    constexpr bool STORED = MODE == PANEL_STORED || MODE == PANEL_STORED2;

    d4 c[2];
    if (STORED) {
        // the panel blocks L21_i, L21_j as the panel launch(es) stored them; the tile itself in flight meanwhile
        const int o1 = MODE == PANEL_STORED2 ? o - NB : o;      // the panel that is applied first
        double pa[8], pb[8], qa[8], qb[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int y = wave + 8 * u, x = lane;
            pa[u] = L[(int64_t)min(mi0 + y, d - 1) * d + o1 + x];
            pb[u] = L[(int64_t)min(mj0 + y, d - 1) * d + o1 + x];
        }
        if (MODE == PANEL_STORED2) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int y = wave + 8 * u, x = lane;
                qa[u] = L[(int64_t)min(mi0 + y, d - 1) * d + o + x];
                qb[u] = L[(int64_t)min(mj0 + y, d - 1) * d + o + x];
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = mi0 + wr * 16 + 4 * v + fq, gn = mj0 + wn * 32 + j * 16 + fr;
                c[j][v] = Hd[(int64_t)min(gm, d - 1) * d + min(gn, d - 1)];
            }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int y = wave + 8 * u, x = lane;
            Pi[y * DL + x] = pa[u];
            if (!diag_tile) Pj[y * DL + x] = pb[u];
        }
        __syncthreads();
        if (MODE == PANEL_STORED2) {
            // the older panel's product here, then the newer panel takes its place in LDS for the product below
            const double* Q1 = diag_tile ? Pi : Pj;
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) {
                const double a = -Pi[(wr * 16 + fr) * DL + 4 * ks + fq];
#pragma unroll
                for (int j = 0; j < 2; ++j) c[j] = mfma4(a, Q1[(wn * 32 + j * 16 + fr) * DL + 4 * ks + fq], c[j]);
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int y = wave + 8 * u, x = lane;
                Pi[y * DL + x] = qa[u];
                if (!diag_tile) Pj[y * DL + x] = qb[u];
            }
            __syncthreads();
        }
    } else {
    // Panel product L21 = A21 L11^-T: L11^-1 is lower triangular, so the 16 columns of column tile ct
    // (of 4) only need the k-steps 0 .. 4 ct + 3.  The wavefronts with wn = 0 take the column tiles
    // 0 and 3, those with wn = 1 the tiles 1 and 2: 20 of 32 (k-step, tile) pairs each.
    const int ct[2] = {wn, 3 - wn};
    // this lane's B-operand elements of L11^-T for those k-steps, straight from global memory
    // (32 KB shared by every workgroup of the launch: cache hits)
    double gb[16][2];
    if (wn == 0) tri_frag_load<0>(Dinv, lane, gb); else tri_frag_load<1>(Dinv, lane, gb);
    // one round of loads (all in flight together), then the stores to LDS
    double pa[8], pb[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        // Rows past d are read from row d - 1 (clamped address, no branch per load): they only
        // reach outputs past d, which are never stored or are replaced by the identity padding.
        pa[u] = Hd[(int64_t)min(mi0 + y, d - 1) * d + o + x];
    }
    if (!diag_tile) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int y = wave + 8 * u, x = lane;
            pb[u] = Hd[(int64_t)min(mj0 + y, d - 1) * d + o + x];
        }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        Pi[y * DL + x] = pa[u];
        if (!diag_tile) Pj[y * DL + x] = pb[u];
    }
    __syncthreads();
    // the tile itself: in flight during the panel product
    if (MODE == PANEL_FUSED || MODE == PANEL_NEAR) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = mi0 + wr * 16 + 4 * v + fq, gn = mj0 + wn * 32 + j * 16 + fr;
                c[j][v] = Hd[(int64_t)min(gm, d - 1) * d + min(gn, d - 1)];
            }
    }

    d4 li[2], lj[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) { li[j] = d4{0.0, 0.0, 0.0, 0.0}; lj[j] = d4{0.0, 0.0, 0.0, 0.0}; }
    if (wn == 0) {
        if (diag_tile) tri_right_product<0, false>(Pi, Pj, gb, wr * 16, fr, fq, li, lj);
        else tri_right_product<0, true>(Pi, Pj, gb, wr * 16, fr, fq, li, lj);
    } else {
        if (diag_tile) tri_right_product<1, false>(Pi, Pj, gb, wr * 16, fr, fq, li, lj);
        else tri_right_product<1, true>(Pi, Pj, gb, wr * 16, fr, fq, li, lj);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int m = wr * 16 + 4 * v + fq, n = ct[j] * 16 + fr;
            Pi[m * DL + n] = li[j][v];
            if (!diag_tile) Pj[m * DL + n] = lj[j][v];
            if (L && (tj == 0 || MODE == PANEL_ONLY) && mi0 + m < d) L[(int64_t)(mi0 + m) * d + o + n] = li[j][v];
        }
    if (MODE == PANEL_ONLY) return;
    __syncthreads();
    }
    const double* Qj = diag_tile ? Pi : Pj;
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const double a = -Pi[(wr * 16 + fr) * DL + 4 * ks + fq];
#pragma unroll
        for (int j = 0; j < 2; ++j) c[j] = mfma4(a, Qj[(wn * 32 + j * 16 + fr) * DL + 4 * ks + fq], c[j]);
    }
    if (bid != 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = mi0 + wr * 16 + 4 * v + fq, gn = mj0 + wn * 32 + j * 16 + fr;
                if (gm < d && gn < d) Hd[(int64_t)gm * d + gn] = c[j][v];
            }
        return;
    }
    // tile (0, 0): the next diagonal block, of size nbn
    const int nbn = min(NB, d - r0);
    __syncthreads();
    double* Am = Pi;
    double* Xm = Pj;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int m = wr * 16 + 4 * v + fq, n = wn * 32 + j * 16 + fr;
            Am[m * DL + n] = (m < nbn && n < nbn) ? c[j][v] : (m == n ? 1.0 : 0.0);
        }
    __syncthreads();
    chol_block(Am, Xm, lds, flag);
    chol_block_store(Am, Xm, d, r0, nbn, L, Linv, Dinv_next);
    if (WPS == 4 && threadIdx.x == 0) __hip_atomic_store(mate_flag, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// H_d = L L^T.  One stand-alone launch for the first diagonal block, then one fused launch
// per 64-column panel.  L may be null when only the inverse is wanted (Sacc != null): it is not stored then.
hipError_t cholesky_lower(fobq_ctx* c, double* Hd, double* L, int d, double* Linv, int* flag, double* Sacc,
                          double* Hinv)
{
    hipStream_t s = c->stream;
    double* Dinv[2] = {c->Dblk.as<double>(), c->Dblk.as<double>() + NB * NB};
    int* mate_flag = c->flags.as<int>() + FLAG_WORD_MATE;
    hipLaunchKernelGGL(chol_diag_kernel, dim3(1), dim3(NT), 0, s, Hd, (int64_t)d, 0, min(NB, d), L, Linv, Dinv[0],
                       flag);
    int it = 0;
    for (int o = 0; o + NB < d; o += NB, ++it) {
        const int T = (d - o - NB + NB - 1) / NB;
        const int ntrail = T * (T + 1) / 2;
        const int ninv = Sacc ? T * (it + 1) : 0;      // tiles of the triangular inverse (row below, column up to the panel)
        const int nlau = Sacc ? it * (it + 1) / 2 : 0;  // tiles of Hinv that block row it - 1 of L^-1 adds to
        const int tiles = ntrail + ninv + nlau;
        if (!Sacc && L && ntrail >= STORED_PANEL_TILES) {
            const int T2 = T - 1, ntrail2 = T2 * (T2 + 1) / 2;
            if (ntrail2 >= STORED_PANEL_TILES) {
                // two panels, one pass over the trailing matrix: after this panel only the next panel's tiles (and its
                // diagonal block, workgroup 0) are updated; the launch after the next panel applies both to the rest
                hipLaunchKernelGGL((chol_iter_kernel<2, PANEL_NEAR>), dim3(T), dim3(NT), 0, s, Hd, d, o, Dinv[it & 1], L, Linv,
                                   Dinv[(it + 1) & 1], flag, T, 0, Sacc, Hinv, mate_flag, 0, c->cus);
                o += NB;
                ++it;
                hipLaunchKernelGGL((chol_iter_kernel<2, PANEL_ONLY>), dim3(T2), dim3(NT), 0, s, Hd, d, o, Dinv[it & 1], L, Linv,
                                   Dinv[(it + 1) & 1], flag, T2, 0, Sacc, Hinv, mate_flag, 0, c->cus);
                hipLaunchKernelGGL((chol_iter_kernel<4, PANEL_STORED2>), dim3(ntrail2 + 1), dim3(NT), 0, s, Hd, d, o, Dinv[it & 1],
                                   L, Linv, Dinv[(it + 1) & 1], flag, ntrail2, 0, Sacc, Hinv, mate_flag, ++c->mate_epoch, c->cus);
            } else {
                // throughput-bound launch: the panel once (T workgroups), then one product per trailing tile
                hipLaunchKernelGGL((chol_iter_kernel<2, PANEL_ONLY>), dim3(T), dim3(NT), 0, s, Hd, d, o, Dinv[it & 1], L, Linv,
                                   Dinv[(it + 1) & 1], flag, T, 0, Sacc, Hinv, mate_flag, 0, c->cus);
                hipLaunchKernelGGL((chol_iter_kernel<4, PANEL_STORED>), dim3(ntrail + 1), dim3(NT), 0, s, Hd, d, o, Dinv[it & 1],
                                   L, Linv, Dinv[(it + 1) & 1], flag, ntrail, 0, Sacc, Hinv, mate_flag, ++c->mate_epoch, c->cus);
            }
        } else if (tiles <= DENSE_LAUNCH_TILES)
            hipLaunchKernelGGL((chol_iter_kernel<2, PANEL_FUSED>), dim3(tiles), dim3(NT), 0, s, Hd, d, o, Dinv[it & 1], L, Linv,
                               Dinv[(it + 1) & 1], flag, ntrail, ninv, Sacc, Hinv, mate_flag, 0, c->cus);
        else
            // one workgroup more than tiles: the place holder (when the device has more compute units than the launch has
            // tiles, the extra workgroup has no tile and returns)
            hipLaunchKernelGGL((chol_iter_kernel<4, PANEL_FUSED>), dim3(tiles + 1), dim3(NT), 0, s, Hd, d, o, Dinv[it & 1], L, Linv,
                               Dinv[(it + 1) & 1], flag, ntrail, ninv, Sacc, Hinv, mate_flag, ++c->mate_epoch, c->cus);
    }
    if (Sacc && it > 0) {
        // last block row of L^-1: Linv[last][0 : last] = -Linv[last][last] S[last][0 : last]
        const int o = it * NB;                          // first row of the last block
        GemmP q;
        q.M = d - o; q.N = o; q.K = d - o;
        q.A = Linv + (int64_t)o * d + o; q.lda = d;
        q.B = Sacc + (int64_t)o * d; q.ldb = d;
        q.C = Linv + (int64_t)o * d; q.ldc = d;
        q.alpha = -1.0;
        hipError_t e = gemm64(s, q, false, false);
        if (e != hipSuccess) return e;
    }
    if (Sacc) {
        // what the launches above have not added to Hinv: the last two block rows of L^-1 (all of it if
        // there are at most two); the tiles right of those rows' first column are touched for the first time
        const int k0 = max(0, it - 1) * NB;
        GemmP q;
        q.M = d; q.N = d; q.K = d;
        q.A = Linv; q.lda = d;
        q.B = Linv; q.ldb = d;
        q.C = Hinv; q.ldc = d;
        q.cmode = CMODE_UPPER; q.kmode = KMODE_GE_MAX_MN; q.kmin = k0;
        q.beta = 1.0; q.beta_ncols = k0;
        hipError_t e = gemm64(s, q, true, false);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

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
// Shared-Hinv elimination (Eq. 12) of the 64 x 64 block held in LDS.  With A11 the block,
// U11 its pivot rows, D = diag(U11) and Un11 = D^-1 U11 (unit upper):  A11 = Un11^T D Un11.
//   in : Am upper triangle = the block (identity padding past its size; what is below the diagonal is
//        not used); Xm need not be initialised
//   out: Am upper triangle = U11 (pivot row j = row j; below the diagonal: not defined), rv[j] = 1 / pivot_j
//        (so Un11[i][j] = Am[i][j] * rv[i]),  Xm = G = (Un11^T)^-1 (unit lower)
// Called by all NT threads of the workgroup; ends with a barrier.
__device__ __forceinline__ void elim_block(double* Am, double* Xm, double* rv, int* __restrict__ flag)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, fq = lane >> 4;
    double* cb = rv + NB;      // the pivot rows of the running sweep, laid out as in chol_block
    double* idt = cb + CB_LEN; // 16 rows of the identity, row stride DL (read from the second sweep on)
    if (tid < 256) idt[(tid >> 4) * DL + (tid & 15)] = (tid >> 4) == (tid & 15) ? 1.0 : 0.0;

    // Elimination of the 16 pivots base .. base+15 over all columns >= base: lane c holds
    // column c of the 16 pivot rows.  Columns inside the diagonal tile (0 <= r < 16) hold the
    // tile column (what lies below its diagonal is carried along and never used); columns right
    // of it (r >= 16) get their part of the pivot rows
    // in the same sweep; columns left of it (r < 0) idle on harmless values.
    auto sweep = [&](int b) {
        const int base = 16 * b, c = lane, r = c - base;
        // For b >= 1 the lanes 0..15 (columns left of the tile, otherwise idle) carry the columns of the
        // identity as if they were columns right of the tile: those become G_bb I, i.e. lane c ends with
        // column c of G_bb = (Un_bb^T)^-1.
        const bool idl = b > 0 && lane < 16;
        // one column of 16 per lane: its own (rows j > r of a tile column are never used), or one of the identity
        const double* src = idl ? idt + lane : Am + base * DL + c;
        double a[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) a[j] = src[j * DL];
        // as in chol_block: every lane of the tile keeps its own diagonal entry in `dg`
        double dg = Am[c * DL + c];
        double fp = 0.0, lb[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const double pi = pivot_rcp(readlane_f64(dg, base + k));
            // A[k][c] = U[k][c] for c >= k (lane k's a[k] has had the same updates as its dg: it is the
            // pivot).  Lanes of columns left of the pivot go through the same arithmetic on entries that
            // are never stored.
            const double cr = a[k];
            const double fm = cr * pi;                        // Un[k][c]
            dg -= fm * cr;
            // as in chol_block: the next row by readlane, the others one step late from LDS
            cb[CB0 + 16 * k + r] = cr;
            if (k > 0) {
#pragma unroll
                for (int j = k + 1; j < 16; ++j) a[j] -= fp * lb[j];
            }
            if (k < 15) a[k + 1] -= fm * readlane_f64(cr, base + k + 1);
#pragma unroll
            for (int j = k + 2; j < 16; ++j) lb[j] = cb[CB0 + 16 * k + j];   // in flight during the next pivot
            fp = fm;
        }
        if (r >= 0) {
#pragma unroll
            for (int k = 0; k < 16; ++k) Am[(base + k) * DL + c] = a[k];   // U[k][c] for k <= c
            if (r < 16) {
                // a pivot that is not a positive normal number leaves such a value, or a NaN, on the diagonal
                const double piv = Am[c * DL + c];
                if (!(piv > 0.0) || !(piv < 1.0e300)) *flag = 1;
                rv[c] = pivot_rcp(piv);
            }
        }
        if (idl) {
#pragma unroll
            for (int k = 0; k < 16; ++k) Xm[(base + k) * DL + base + lane] = a[k];
        }
    };
    // G_bb = (Un_bb^T)^-1 (unit lower) by forward substitution: lane c (mod 16) solves
    // Un_bb^T x = e_c; entry [i][m] of Un_bb^T is Un[m][i], a wavefront-uniform LDS read
    auto tinv = [&](int b) {
        const int base = 16 * b, c = fr;
        double sv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) sv[i] = (i == c) ? 1.0 : 0.0;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const double xm = sv[m] * rv[base + m];
#pragma unroll
            for (int i = m + 1; i < 16; ++i) sv[i] -= Am[(base + m) * DL + base + i] * xm;
        }
        if (lane < 16) {
#pragma unroll
            for (int i = 0; i < 16; ++i) Xm[(base + i) * DL + base + c] = sv[i];
        }
        __builtin_amdgcn_wave_barrier();
    };
    // trailing tiles: A_ij -= Un_bi^T U_bj for b < i <= j
    auto trail = [&](int b) {
        const int base = 16 * b;
        int t = 0;
        for (int i = b + 1; i < 4; ++i)
            for (int j = i; j < 4; ++j, ++t) {
                if ((t & (NT / 64 - 1)) != wave) continue;
                d4 acc;
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[v] = Am[(16 * i + 4 * v + fq) * DL + 16 * j + fr];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    acc = mfma4(-Am[(base + 4 * ks + fq) * DL + 16 * i + fr] * rv[base + 4 * ks + fq],
                                Am[(base + 4 * ks + fq) * DL + 16 * j + fr], acc);
#pragma unroll
                for (int v = 0; v < 4; ++v) Am[(16 * i + 4 * v + fq) * DL + 16 * j + fr] = acc[v];
            }
    };
    // G = (Un11^T)^-1: tile T_im of Un11^T is Un_mi transposed
    block_schedule(Xm, sweep, tinv, trail, [&](int i, int m, int ks) {
        return Am[(16 * m + 4 * ks + fq) * DL + 16 * i + fr] * rv[16 * m + 4 * ks + fq]; });
}

__device__ __forceinline__ void elim_block_store(const double* Am, const double* Xm, const double* rv,
                                                 int64_t ld, int o, int nb, double* __restrict__ U,
                                                 double* __restrict__ Un, double* __restrict__ G,
                                                 double* __restrict__ Gf, double* __restrict__ rinv)
{
    for (int idx = threadIdx.x; idx < NB * NB; idx += NT) {
        const int i = idx >> 6, j = idx & 63;
        const bool in = i < nb && j < nb;
        if (G) G[idx] = (in && j <= i) ? Xm[i * DL + j] : 0.0;
        if (Gf) {
            int fi, fj;
            frag_source(idx, fi, fj);
            Gf[idx] = (fi < nb && fj <= fi) ? Xm[fi * DL + fj] : 0.0;
        }
        if (in && j >= i) {
            U[(int64_t)(o + i) * ld + o + j] = Am[i * DL + j];
            Un[(int64_t)(o + i) * ld + o + j] = (i == j) ? 1.0 : Am[i * DL + j] * rv[i];
        }
    }
    if (threadIdx.x < NB) rinv[threadIdx.x] = (threadIdx.x < nb) ? rv[threadIdx.x] : 0.0;
}

// Diagonal block of the elimination (stand-alone launch).
//   out: U[o+j, o+j : o+nb]  = pivot row j inside the block
//        Un = U / pivot
//        G (64 x 64, ld 64)  = (Un11^T)^-1: pivot rows right of the block are G * A[o:o+nb, o+nb:];
//        Gf = the same in the fragment layout (either may be null)
//        rinv[j] = 1 / pivot_j
__global__ __launch_bounds__(NT) void elim_diag_kernel(const double* __restrict__ A, int64_t ld, int o, int nb,
                                                        double* __restrict__ U, double* __restrict__ Un,
                                                        double* __restrict__ G, double* __restrict__ Gf,
                                                        double* __restrict__ rinv, int* __restrict__ flag)
{
    __shared__ double Am[NB * DL];
    __shared__ double Xm[NB * DL];
    __shared__ double rv[SWEEP_LDS];
    for (int idx = threadIdx.x; idx < NB * NB; idx += NT) {
        const int i = idx >> 6, j = idx & 63;
        double v = (i == j) ? 1.0 : 0.0;
        if (i < nb && j < nb) v = A[(int64_t)(o + min(i, j)) * ld + o + max(i, j)];   // upper triangle is the maintained one
        Am[i * DL + j] = v;
    }
    __syncthreads();
    elim_block(Am, Xm, rv, flag);
    elim_block_store(Am, Xm, rv, ld, o, nb, U, Un, G, Gf, rinv);
}

// One whole iteration of the blocked shared-Hinv elimination in a single launch (same scheme
// as chol_iter_kernel).  The panel is the 64 rows/columns o .. o+63 whose diagonal block has
// been eliminated (G in the fragment layout, rinv).  Workgroup (ti, tj), ti <= tj, owns tile (ti, tj) of the trailing
// matrix (upper triangle):
//   1. pivot rows right of the block for its two tile columns: U12_i = G A12_i, U12_j, and
//      Un12 = D^-1 U12; the tiles of the first tile row also store them into U and Un;
//   2. A22(ti, tj) -= Un12_i^T U12_j        (Eq. 12 for the 64 columns of the panel at once);
//   3. workgroup 0 eliminates tile (0, 0), the next diagonal block, right away.
// MODE as for chol_iter_kernel: PANEL_ONLY = workgroup j computes and stores the pivot rows U12_j, Un12_j right of the
// block for its tile column; PANEL_STORED = the trailing launch that follows and takes them from U and Un;
// PANEL_NEAR = only the tiles (0, j) of the next panel's rows, each recomputing and storing its pivot rows;
// PANEL_STORED2 = the 128 pivot rows o - 64 .. o + 63 at once.
template <int WPS, int MODE>
__global__ __launch_bounds__(NT, WPS) void elim_iter_kernel(double* __restrict__ A, int d, int o,
                                                       const double* __restrict__ G, const double* __restrict__ rinv,
                                                       double* __restrict__ U, double* __restrict__ Un,
                                                       double* __restrict__ G_next, double* __restrict__ rinv_next,
                                                       int* __restrict__ flag, int* __restrict__ mate_flag, int epoch, int mate_slot)
{
    __shared__ double lds[SWEEP_LDS + 2 * NB * DL];   // sweep scratch, two tiles: 2 workgroups per compute unit
    // epoch != 0: the launch has one workgroup more than tiles, and workgroup `mate_slot` only holds the place
    // beside workgroup 0 (see chol_iter_kernel; both variants of this kernel fit two workgroups per compute unit)
    if (epoch != 0 && (int)blockIdx.x == mate_slot) {
        if (threadIdx.x >= 64) return;
        for (int i = 0; i < MATE_MAX_NAPS; ++i) {
            if (__hip_atomic_load(mate_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch >= 0) break;
            __builtin_amdgcn_s_sleep(16);
        }
        return;
    }
    const int bid = (int)blockIdx.x - ((epoch != 0 && (int)blockIdx.x > mate_slot) ? 1 : 0);
    double* Pi = lds + SWEEP_LDS;
    double* Pj = Pi + NB * DL;
    double* rs = lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, w2 = wave & 1, fr = lane & 15, fq = lane >> 4;
    const int r0 = o + NB;
    int ti, tj;
    if (MODE == PANEL_ONLY) { ti = bid; tj = bid; }      // workgroup j: tile column j of the pivot rows
    else if (MODE == PANEL_NEAR) { ti = 0; tj = bid; }   // workgroup j: tile (0, j), the rows of the next panel
    else tri_decode(bid, tj, ti);     // ti <= tj
    const bool diag_tile = ti == tj;
    const int ci0 = r0 + NB * ti, cj0 = r0 + NB * tj;
    constexpr bool STORED = MODE == PANEL_STORED || MODE == PANEL_STORED2;

    d4 c[2];
    if (STORED) {
        // Un12_i and U12_j as the panel launch(es) stored them; the trailing tile itself in flight meanwhile
        const int o1 = MODE == PANEL_STORED2 ? o - NB : o;      // the panel that is applied first
        double pa[8], pb[8], qa[8], qb[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int y = wave + 8 * u, x = lane;
            pa[u] = Un[(int64_t)(o1 + y) * d + min(ci0 + x, d - 1)];
            pb[u] = U[(int64_t)(o1 + y) * d + min(cj0 + x, d - 1)];
        }
        if (MODE == PANEL_STORED2) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int y = wave + 8 * u, x = lane;
                qa[u] = Un[(int64_t)(o + y) * d + min(ci0 + x, d - 1)];
                qb[u] = U[(int64_t)(o + y) * d + min(cj0 + x, d - 1)];
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = ci0 + wr * 16 + 4 * v + fq, gn = cj0 + w2 * 32 + j * 16 + fr;
                c[j][v] = A[(int64_t)min(gm, d - 1) * d + min(gn, d - 1)];
            }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int y = wave + 8 * u, x = lane;
            Pi[y * DL + x] = pa[u];
            Pj[y * DL + x] = pb[u];
        }
        __syncthreads();
        if (MODE == PANEL_STORED2) {
            // the older panel's product here, then the newer panel takes its place in LDS for the product below
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) {
                const double a = -Pi[(4 * ks + fq) * DL + wr * 16 + fr];
#pragma unroll
                for (int j = 0; j < 2; ++j) c[j] = mfma4(a, Pj[(4 * ks + fq) * DL + w2 * 32 + j * 16 + fr], c[j]);
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int y = wave + 8 * u, x = lane;
                Pi[y * DL + x] = qa[u];
                Pj[y * DL + x] = qb[u];
            }
            __syncthreads();
        }
    } else {
    // Pivot rows U12 = G A12: G is lower triangular, so the 16 rows of row tile rt (of 4) only need
    // the k-steps 0 .. 4 rt + 3.  The wavefronts with w2 = 0 take the row tiles 0 and 3, those with
    // w2 = 1 the tiles 1 and 2 (20 of 32 (k-step, tile) pairs each), for the 16 columns of slice wr.
    const int rt[2] = {w2, 3 - w2};
    // this lane's A-operand elements of G for those k-steps, straight from global memory
    double ga[16][2];
    if (w2 == 0) tri_frag_load<0>(G, lane, ga); else tri_frag_load<1>(G, lane, ga);
    // one round of loads (all in flight together), then the stores to LDS
    double pa[8], pb[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        // Columns past d are read from column d - 1 (clamped address, no branch per load): they
        // only reach outputs past d, which are never stored or are replaced by the identity padding.
        pa[u] = A[(int64_t)(o + y) * d + min(ci0 + x, d - 1)];
    }
    if (!diag_tile) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int y = wave + 8 * u, x = lane;
            pb[u] = A[(int64_t)(o + y) * d + min(cj0 + x, d - 1)];
        }
    }
    const double rsv = (tid < NB) ? rinv[tid] : 0.0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        Pi[y * DL + x] = pa[u];
        if (!diag_tile) Pj[y * DL + x] = pb[u];
    }
    if (tid < NB) rs[tid] = rsv;
    __syncthreads();
    // the trailing tile itself (rows of slice wr, the 32 columns of half w2): in flight during the product
    if (MODE == PANEL_FUSED || MODE == PANEL_NEAR) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = ci0 + wr * 16 + 4 * v + fq, gn = cj0 + w2 * 32 + j * 16 + fr;
                c[j][v] = A[(int64_t)min(gm, d - 1) * d + min(gn, d - 1)];
            }
    }

    d4 ui[2], uj[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) { ui[i] = d4{0.0, 0.0, 0.0, 0.0}; uj[i] = d4{0.0, 0.0, 0.0, 0.0}; }
    if (w2 == 0) {
        if (diag_tile) tri_left_product<0, false>(Pi, Pj, ga, wr * 16, fr, fq, ui, uj);
        else tri_left_product<0, true>(Pi, Pj, ga, wr * 16, fr, fq, ui, uj);
    } else {
        if (diag_tile) tri_left_product<1, false>(Pi, Pj, ga, wr * 16, fr, fq, ui, uj);
        else tri_left_product<1, true>(Pi, Pj, ga, wr * 16, fr, fq, ui, uj);
    }
    __syncthreads();
    // Pi := Un12_i (rows scaled by 1 / pivot), Pj := U12_j
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int m = rt[i] * 16 + 4 * v + fq, n = wr * 16 + fr;
            const double uiv = ui[i][v];
            const double ujv = diag_tile ? uiv : uj[i][v];
            Pi[m * DL + n] = uiv * rs[m];
            Pj[m * DL + n] = ujv;
            if ((ti == 0 || MODE == PANEL_ONLY) && cj0 + n < d) {
                U[(int64_t)(o + m) * d + cj0 + n] = ujv;
                Un[(int64_t)(o + m) * d + cj0 + n] = ujv * rs[m];
            }
        }
    if (MODE == PANEL_ONLY) return;
    __syncthreads();
    }
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const double a = -Pi[(4 * ks + fq) * DL + wr * 16 + fr];
#pragma unroll
        for (int j = 0; j < 2; ++j) c[j] = mfma4(a, Pj[(4 * ks + fq) * DL + w2 * 32 + j * 16 + fr], c[j]);
    }
    if (bid != 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gm = ci0 + wr * 16 + 4 * v + fq, gn = cj0 + w2 * 32 + j * 16 + fr;
                if (gm < d && gn < d) A[(int64_t)gm * d + gn] = c[j][v];
            }
        return;
    }
    // tile (0, 0): the next diagonal block, of size nbn
    const int nbn = min(NB, d - r0);
    __syncthreads();
    double* Am = Pi;
    double* Xm = Pj;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int m = wr * 16 + 4 * v + fq, n = w2 * 32 + j * 16 + fr;
            Am[m * DL + n] = (m < nbn && n < nbn) ? c[j][v] : (m == n ? 1.0 : 0.0);
        }
    __syncthreads();
    elim_block(Am, Xm, rs, flag);
    elim_block_store(Am, Xm, rs, d, r0, nbn, U, Un, nullptr, G_next, rinv_next);
    if (epoch != 0 && threadIdx.x == 0) __hip_atomic_store(mate_flag, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Shared-Hinv elimination of the first `steps` columns, `block` columns at a time.
hipError_t eliminate_blocked(fobq_ctx* c, double* A, int d, int steps, int block, double* U, double* Un, int* flag,
                             const std::vector<hipEvent_t>* rows_ready)
{
    hipStream_t s = c->stream;
    auto ready = [&](int k) {
        if (rows_ready && k < (int)rows_ready->size())
            (void)hipEventRecord((*rows_ready)[k], s);
    };
    double* Gb[2] = {c->Dblk.as<double>() + 2 * NB * NB, c->Dblk.as<double>() + 3 * NB * NB};
    double* rb[2] = {c->Dblk.as<double>() + 4 * NB * NB, c->Dblk.as<double>() + 4 * NB * NB + NB};
    if (block == NB && steps == d) {
        // one stand-alone launch for the first diagonal block, then one fused launch per panel
        hipLaunchKernelGGL(elim_diag_kernel, dim3(1), dim3(NT), 0, s, A, (int64_t)d, 0, min(NB, d), U, Un,
                           (double*)nullptr, Gb[0], rb[0], flag);
        int it = 0;
        for (int o = 0; o + NB < d; o += NB, ++it) {
            const int T = (d - o - NB + NB - 1) / NB;
            // rows of block `it` are complete when this launch is (its diagonal part came from the previous
            // one): the block's event rides on the launch itself as its stop event -- a separate
            // hipEventRecord between two dependent launches costs about 4 us of bubble
            hipEvent_t done = (rows_ready && it < (int)rows_ready->size()) ? (*rows_ready)[it] : nullptr;
            const int tiles = T * (T + 1) / 2;
            // a launch with a workgroup of index `cus` gets one more, which holds the place beside workgroup 0
            const bool mate = tiles > c->cus;
            const int epoch = mate ? ++c->mate_epoch : 0;
            int* mate_flag = c->flags.as<int>() + FLAG_WORD_MATE;
            if (tiles >= STORED_PANEL_TILES) {
                const int T2 = T - 1, tiles2 = T2 * (T2 + 1) / 2;
                if (tiles2 >= STORED_PANEL_TILES) {
                    // two panels, one pass over the trailing matrix (see chol_iter_kernel): the next panel's rows now,
                    // both panels' update of everything else after the next panel
                    hipExtLaunchKernelGGL((elim_iter_kernel<2, PANEL_NEAR>), dim3(T), dim3(NT), 0, s, nullptr, done, 0, A, d, o,
                                          (const double*)Gb[it & 1], (const double*)rb[it & 1], U, Un, Gb[(it + 1) & 1],
                                          rb[(it + 1) & 1], flag, mate_flag, 0, c->cus);
                    o += NB;
                    ++it;
                    hipEvent_t done2 = (rows_ready && it < (int)rows_ready->size()) ? (*rows_ready)[it] : nullptr;
                    hipLaunchKernelGGL((elim_iter_kernel<2, PANEL_ONLY>), dim3(T2), dim3(NT), 0, s, A, d, o,
                                       (const double*)Gb[it & 1], (const double*)rb[it & 1], U, Un, Gb[(it + 1) & 1],
                                       rb[(it + 1) & 1], flag, mate_flag, 0, c->cus);
                    hipExtLaunchKernelGGL((elim_iter_kernel<4, PANEL_STORED2>), dim3(tiles2 + 1), dim3(NT), 0, s, nullptr, done2, 0,
                                          A, d, o, (const double*)Gb[it & 1], (const double*)rb[it & 1], U, Un, Gb[(it + 1) & 1],
                                          rb[(it + 1) & 1], flag, mate_flag, ++c->mate_epoch, c->cus);
                } else {
                    // throughput-bound launch: the pivot rows once (T workgroups), then one product per trailing tile
                    hipLaunchKernelGGL((elim_iter_kernel<2, PANEL_ONLY>), dim3(T), dim3(NT), 0, s, A, d, o,
                                       (const double*)Gb[it & 1], (const double*)rb[it & 1], U, Un, Gb[(it + 1) & 1],
                                       rb[(it + 1) & 1], flag, mate_flag, 0, c->cus);
                    hipExtLaunchKernelGGL((elim_iter_kernel<4, PANEL_STORED>), dim3(tiles + 1), dim3(NT), 0, s, nullptr, done, 0, A,
                                          d, o, (const double*)Gb[it & 1], (const double*)rb[it & 1], U, Un, Gb[(it + 1) & 1],
                                          rb[(it + 1) & 1], flag, mate_flag, epoch, c->cus);
                }
            } else if (tiles <= DENSE_LAUNCH_TILES)
                hipExtLaunchKernelGGL((elim_iter_kernel<2, PANEL_FUSED>), dim3(tiles + (mate ? 1 : 0)), dim3(NT), 0, s, nullptr, done, 0, A,
                                      d, o, (const double*)Gb[it & 1], (const double*)rb[it & 1], U, Un, Gb[(it + 1) & 1],
                                      rb[(it + 1) & 1], flag, mate_flag, epoch, c->cus);
            else
                hipExtLaunchKernelGGL((elim_iter_kernel<4, PANEL_FUSED>), dim3(tiles + (mate ? 1 : 0)), dim3(NT), 0, s, nullptr, done, 0, A,
                                      d, o, (const double*)Gb[it & 1], (const double*)rb[it & 1], U, Un, Gb[(it + 1) & 1],
                                      rb[(it + 1) & 1], flag, mate_flag, epoch, c->cus);
        }
        ready(it);              // last block: only a diagonal part
        return hipGetLastError();
    }
    // general form (any block width, partial elimination): diagonal block, pivot rows, trailing update
    double* G = Gb[0];
    double* rinv = rb[0];
    int it = 0;
    for (int o = 0; o < steps; o += block, ++it) {
        const int nb = min(block, steps - o);
        hipLaunchKernelGGL(elim_diag_kernel, dim3(1), dim3(NT), 0, s, A, (int64_t)d, o, nb, U, Un, G,
                           (double*)nullptr, rinv, flag);
        const int r = d - o - nb;
        if (r <= 0) { ready(it); break; }
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
        ready(it);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Batched small layers (d <= 256, at most 4 panels).  A layer this small never fills the GPU: its whole
// factor path is a chain of dependent steps on one workgroup's worth of work.  Here ONE workgroup per layer
// walks that chain by itself -- blocked with the same 64 x 64 diagonal-block routines, the tile products on
// the matrix cores with operands straight from global memory (everything sits in L2) -- so that a single
// launch factors every layer of a batch, and the launch count no longer grows with the number of layers.
//
// tile_mm: C (m x n) = beta C + alpha op(A) op(B), op(A) m x k, op(B) k x n, all <= 64, row-major in global memory.
//   TA: op(A)[r][q] = A[q * lda + r] (else A[r * lda + q]);  TB: op(B)[q][c] = B[c * ldb + q] (else B[q * ldb + c]).
//   C2 / rowscale (may be null): C2[r][c] = rowscale[r] * result.
// The two operand tiles are staged in LDS as they lie in memory (coalesced rows; Pa, Pb: NB * DL doubles each)
// and the MFMA fragments are read in the orientation the product needs.  Called by all NT threads; every
// operand is in LDS before anything is stored (C may alias A or B); ends with a barrier.
template <bool TA, bool TB>
__device__ __forceinline__ void tile_mm(double* Pa, double* Pb, double* C, int64_t ldc, const double* A, int64_t lda,
                                        const double* B, int64_t ldb, int m, int n, int k, double alpha, double beta,
                                        double* C2 = nullptr, const double* rowscale = nullptr)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wr = wave >> 1, w2 = wave & 1, fr = lane & 15, fq = lane >> 4;
    const int arows = TA ? k : m, acols = TA ? m : k, brows = TB ? n : k, bcols = TB ? k : n;
    double pa[8], pb[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int y = wave + 8 * u, x = lane;
        pa[u] = (y < arows && x < acols) ? A[(int64_t)y * lda + x] : 0.0;
        pb[u] = (y < brows && x < bcols) ? B[(int64_t)y * ldb + x] : 0.0;
    }
    d4 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = wr * 16 + 4 * v + fq, c = w2 * 32 + 16 * j + fr;
            acc[j][v] = (beta != 0.0 && r < m && c < n) ? beta * C[(int64_t)r * ldc + c] : 0.0;
        }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        Pa[(wave + 8 * u) * DL + lane] = alpha * pa[u];
        Pb[(wave + 8 * u) * DL + lane] = pb[u];
    }
    __syncthreads();
    const int ar = wr * 16 + fr;
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const int q = 4 * ks + fq;
        const double av = TA ? Pa[q * DL + ar] : Pa[ar * DL + q];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int bc = w2 * 32 + 16 * j + fr;
            acc[j] = mfma4(av, TB ? Pb[bc * DL + q] : Pb[q * DL + bc], acc[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = wr * 16 + 4 * v + fq, c = w2 * 32 + 16 * j + fr;
            if (r < m && c < n) {
                C[(int64_t)r * ldc + c] = acc[j][v];
                if (C2) C2[(int64_t)r * ldc + c] = acc[j][v] * rowscale[r];
            }
        }
    __syncthreads();
}

// Damped Hessian -> Hinv = L^-T L^-1 (upper tiles; Section 5 item 1, Section 6.1), one workgroup per layer.
__global__ __launch_bounds__(NT) void batch_inverse_kernel(const BatchLayer* __restrict__ layers)
{
    __shared__ double Am[NB * DL];
    __shared__ double Xm[NB * DL];
    __shared__ double rq[SWEEP_LDS];
    const BatchLayer L = layers[blockIdx.x];
    const int d = L.d, T = (d + NB - 1) / NB, tid = threadIdx.x;
    // lambda = damp * mean(diag H) + damp_abs; the diagonal is summed in index order by one wavefront-sized tree
    {
        double s = 0.0;
        for (int a = tid; a < d; a += NT) s += L.H[(int64_t)a * d + a];
        Xm[tid] = s;
        __syncthreads();
        for (int w = NT / 2; w > 0; w >>= 1) {
            if (tid < w) Xm[tid] += Xm[tid + w];
            __syncthreads();
        }
    }
    const double lam = L.damp * (Xm[0] / (double)d) + L.damp_abs;
    __syncthreads();
    for (int idx = tid; idx < d * d; idx += NT) {
        const int a = idx / d, b = idx - a * d;
        L.Hd[idx] = L.H[idx] + (a == b ? lam : 0.0);
    }
    __syncthreads();
    // H_d = L L^T, right-looking over the panels; L overwrites the lower tiles of Hd
    for (int p = 0; p < T; ++p) {
        const int o = NB * p, nb = min(NB, d - o);
        for (int idx = tid; idx < NB * NB; idx += NT) {
            const int i = idx >> 6, j = idx & 63;
            double v = (i == j) ? 1.0 : 0.0;                    // identity padding past nb
            if (i < nb && j < nb) v = (j <= i) ? L.Hd[(int64_t)(o + i) * d + o + j] : 0.0;
            Am[i * DL + j] = v;
        }
        __syncthreads();
        chol_block(Am, Xm, rq, L.flags + 0);
        for (int idx = tid; idx < NB * NB; idx += NT) {
            const int i = idx >> 6, j = idx & 63;
            if (i < nb && j < nb) {
                L.Hd[(int64_t)(o + i) * d + o + j] = (j <= i) ? Am[i * DL + j] : 0.0;
                L.Linv[(int64_t)(o + i) * d + o + j] = (j <= i) ? Xm[i * DL + j] : 0.0;
            }
        }
        __syncthreads();
        for (int i = p + 1; i < T; ++i) {        // L_ip = A_ip L_pp^-T
            double* t = L.Hd + (int64_t)(NB * i) * d + o;
            tile_mm<false, true>(Am, Xm, t, d, t, d, L.Linv + (int64_t)o * d + o, d, min(NB, d - NB * i), nb, nb, 1.0, 0.0);
        }
        for (int i = p + 1; i < T; ++i)          // A_ij -= L_ip L_jp^T
            for (int j = p + 1; j <= i; ++j)
                tile_mm<false, true>(Am, Xm, L.Hd + (int64_t)(NB * i) * d + NB * j, d, L.Hd + (int64_t)(NB * i) * d + o, d,
                                     L.Hd + (int64_t)(NB * j) * d + o, d, min(NB, d - NB * i), min(NB, d - NB * j), nb, -1.0, 1.0);
    }
    // L^-1 below the diagonal blocks: X_ij = -X_ii sum_{m=j}^{i-1} L_im X_mj
    for (int j = 0; j < T; ++j)
        for (int i = j + 1; i < T; ++i) {
            const int mi = min(NB, d - NB * i), nj = min(NB, d - NB * j);
            double* t = L.T + (int64_t)(NB * i) * d + NB * j;
            for (int m = j; m < i; ++m)
                tile_mm<false, false>(Am, Xm, t, d, L.Hd + (int64_t)(NB * i) * d + NB * m, d, L.Linv + (int64_t)(NB * m) * d + NB * j, d,
                                      mi, nj, min(NB, d - NB * m), 1.0, m > j ? 1.0 : 0.0);
            tile_mm<false, false>(Am, Xm, L.Linv + (int64_t)(NB * i) * d + NB * j, d, L.Linv + (int64_t)(NB * i) * d + NB * i, d, t, d,
                                  mi, nj, mi, -1.0, 0.0);
        }
    // Hinv = L^-T L^-1, tiles on and above the diagonal: Hinv_ij = sum_{m >= j} X_mi^T X_mj
    for (int i = 0; i < T; ++i)
        for (int j = i; j < T; ++j)
            for (int m = j; m < T; ++m)
                tile_mm<true, false>(Am, Xm, L.Hinv + (int64_t)(NB * i) * d + NB * j, d, L.Linv + (int64_t)(NB * m) * d + NB * i, d,
                                     L.Linv + (int64_t)(NB * m) * d + NB * j, d, min(NB, d - NB * i), min(NB, d - NB * j),
                                     min(NB, d - NB * m), 1.0, m > j ? 1.0 : 0.0);
}

// The shared-Hinv elimination (Eq. 12) of a whole small layer: A = Hinv in processing order (gathered here
// through perm), then panel by panel the diagonal block, the pivot rows right of it, the trailing update.
// Leaves U (pivot rows) and Un = U / pivot, both on and above the diagonal.  One workgroup per layer.
__global__ __launch_bounds__(NT) void batch_eliminate_kernel(const BatchLayer* __restrict__ layers)
{
    __shared__ double Am[NB * DL];
    __shared__ double Xm[NB * DL];
    __shared__ double rv[SWEEP_LDS];
    const BatchLayer L = layers[blockIdx.x];
    const int d = L.d, T = (d + NB - 1) / NB, tid = threadIdx.x;
    for (int idx = tid; idx < d * d; idx += NT) {
        const int a = idx / d, b = idx - a * d;
        const int pa = min(max(L.perm[a], 0), d - 1), pb = min(max(L.perm[b], 0), d - 1);
        L.A[idx] = L.Hinv[(int64_t)min(pa, pb) * d + max(pa, pb)];
    }
    __syncthreads();
    for (int p = 0; p < T; ++p) {
        const int o = NB * p, nb = min(NB, d - o);
        for (int idx = tid; idx < NB * NB; idx += NT) {
            const int i = idx >> 6, j = idx & 63;
            double v = (i == j) ? 1.0 : 0.0;
            if (i < nb && j < nb) v = L.A[(int64_t)(o + min(i, j)) * d + o + max(i, j)];
            Am[i * DL + j] = v;
        }
        __syncthreads();
        elim_block(Am, Xm, rv, L.flags + 1);
        for (int idx = tid; idx < NB * NB; idx += NT) {
            const int i = idx >> 6, j = idx & 63;
            const bool in = i < nb && j < nb;
            L.Gs[idx] = (in && j <= i) ? Xm[i * DL + j] : 0.0;
            if (in && j >= i) {
                L.U[(int64_t)(o + i) * d + o + j] = Am[i * DL + j];
                L.Un[(int64_t)(o + i) * d + o + j] = (i == j) ? 1.0 : Am[i * DL + j] * rv[i];
            }
        }
        if (tid < NB) L.rinv[tid] = (tid < nb) ? rv[tid] : 0.0;
        __syncthreads();
        for (int j = p + 1; j < T; ++j)          // pivot rows right of the block: U_pj = G A_pj, Un_pj = D^-1 U_pj
            tile_mm<false, false>(Am, Xm, L.U + (int64_t)o * d + NB * j, d, L.Gs, NB, L.A + (int64_t)o * d + NB * j, d, nb,
                                  min(NB, d - NB * j), nb, 1.0, 0.0, L.Un + (int64_t)o * d + NB * j, L.rinv);
        for (int i = p + 1; i < T; ++i)          // A_ij -= Un_pi^T U_pj
            for (int j = i; j < T; ++j)
                tile_mm<true, false>(Am, Xm, L.A + (int64_t)(NB * i) * d + NB * j, d, L.Un + (int64_t)o * d + NB * i, d,
                                     L.U + (int64_t)o * d + NB * j, d, min(NB, d - NB * i), min(NB, d - NB * j), nb, -1.0, 1.0);
    }
}

hipError_t launch_batch_inverse(hipStream_t s, const BatchLayer* layers, int n)
{
    hipLaunchKernelGGL(batch_inverse_kernel, dim3(n), dim3(NT), 0, s, layers);
    return hipGetLastError();
}

hipError_t launch_batch_eliminate(hipStream_t s, const BatchLayer* layers, int n)
{
    hipLaunchKernelGGL(batch_eliminate_kernel, dim3(n), dim3(NT), 0, s, layers);
    return hipGetLastError();
}

}  // namespace fobq
