// X X^T of the layer Hessian (Section 3, Eq. 2) on the int8 matrix cores, by exact integer slices.
//
// Every row i of the fp32 X handed to one accumulate call is written as a fixed-point integer under a
// per-row power of two, Y = rint(x * 2^sh_i), |Y| <= 2^38, and Y is cut into NS = 5 balanced base-256
// digits D_0 (most significant) .. D_4, each in [-128, 127]:  Y = sum_s D_s 256^(4 - s).  Then
//     x_i . x_j  =  2^-(sh_i + sh_j)  sum_{s,t} 256^(8 - s - t)  (D_s[i] . D_t[j])
// and every slice product D_s[i] . D_t[j] is an int8 dot product that the matrix cores accumulate
// exactly in int32 (v_mfma_i32_32x32x32_i8).  Products with the same s + t = m share a scale and an
// accumulator; the antidiagonals m = 0 .. 5 are kept (19 slice products), m >= 6 dropped.  (Splitting a
// floating-point product into exact integer slice products is the published "Ozaki scheme" for matrix
// units; the choice of 5 digits and 6 antidiagonals is this library's.)  What that costs in accuracy,
// measured against the fp64 sum on the benchmark layers: H differs by 3e-13 relative, the column scores
// by 2e-11 relative at most; with one antidiagonal less (15 products) the scores move by 1e-9, which is
// the size of the smallest gap between two column scores of those layers -- the processing order must
// not change, so the sixth antidiagonal stays.
//
// int32 accumulators are folded into the fp64 slabs of partial sums after at most I8_FOLD_STEPS k-steps:
// at most 5 products per accumulator, |D D'| <= 2^14, 2^14 columns  ->  |sum| <= 5 * 2^28 < 2^31.
//
// Three kernels: row_shift_kernel (per-row exponent of a call), slice_kernel (digits, in the order the
// matrix kernel wants them), xxt_i8_kernel (persistent workgroups, 128 x 128 tiles on and below the diagonal,
// operands copied global -> LDS without passing through registers; a workgroup takes one contiguous range of
// (tile, k-step) items, or, for wide layers whose digits no cache holds, whole tiles in step with the others).
#include <hip/hip_ext.h>

#include <type_traits>

#include "fobq_internal.h"

namespace fobq {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

constexpr int NS = 5;               // digits per value
constexpr int NM = 6;               // antidiagonals s + t = 0 .. NM - 1 kept
constexpr int YBITS = 8 * NS - 2;   // |Y| <= 2^YBITS
constexpr int IK = 32;              // calibration columns per k-step (one MFMA)
constexpr int IT = 128;             // tile edge
constexpr int I8_FOLD_STEPS = 512;  // k-steps between folds (16384 columns)
constexpr int I8_WGS = 256;         // persistent workgroups: one per compute unit (8 wavefronts, two per SIMD)

// Digit storage.  For k-step q (32 columns), block of 32 rows b, digit s: one 1 KiB block of 64 slots of
// 16 bytes; slot l holds row 32 b + (l % 32), columns 32 q + 16 (l / 32) .. + 15.  That is the order in which
// the 64 lanes of a wavefront hold one MFMA operand (lane l: row l % 32, k = 16 (l / 32) ..), so a block
// goes global -> LDS -> registers as 64 consecutive 16-byte pieces at every stage.
// Block index = (q * (dpad / 32) + b) * NS + s;  dpad = d rounded up to 128 (rows past d hold zeros).
int i8_dpad(int d) { return (d + IT - 1) / IT * IT; }
int64_t i8_ksteps(int64_t n) { return (n + IK - 1) / IK; }
// most columns per launch: 2 GiB of digits
int64_t i8_block_columns(int d) { return ((int64_t)2 << 30) / ((int64_t)i8_dpad(d) * NS) / 256 * 256; }
size_t i8_planes_bytes(int d, int64_t n) { return (size_t)i8_ksteps(n) * (size_t)(i8_dpad(d) / 32) * NS * 1024; }

// ---------------------------------------------------------------------------
// sh[row] = YBITS - e, 2^e > max_j |x_row,j| (e from the exponent field of the largest magnitude).
// A row with an Inf or NaN raises *nonfinite (the Hessian is then poisoned by the finalize kernel).
// One workgroup per row; VEC: rows are 16-byte aligned (ld % 4 == 0, base aligned).
template <bool VEC>
__global__ __launch_bounds__(256) void row_shift_kernel(const float* __restrict__ X, int64_t ld, int d, int64_t n,
                                                        int* __restrict__ sh, int* __restrict__ nonfinite)
{
    __shared__ unsigned part[256];
    const int row = blockIdx.x;
    const float* __restrict__ x = X + (int64_t)row * ld;
    unsigned m = 0;
    if (VEC) {
        const int64_t n4 = n >> 2;
        const uint4* __restrict__ x4 = reinterpret_cast<const uint4*>(x);
        int64_t j = threadIdx.x;
        auto mag4 = [](const uint4& a) {
            return max(max(a.x & 0x7fffffffu, a.y & 0x7fffffffu), max(a.z & 0x7fffffffu, a.w & 0x7fffffffu));
        };
        for (; j + 768 < n4; j += 1024) {
            const uint4 a = x4[j], b = x4[j + 256], c = x4[j + 512], e = x4[j + 768];
            m = max(max(m, mag4(a)), max(mag4(b), max(mag4(c), mag4(e))));
        }
        for (; j < n4; j += 256) m = max(m, mag4(x4[j]));
        for (int64_t k = (n4 << 2) + threadIdx.x; k < n; k += 256) m = max(m, __float_as_uint(x[k]) & 0x7fffffffu);
    } else {
        for (int64_t j = threadIdx.x; j < n; j += 256) m = max(m, __float_as_uint(x[j]) & 0x7fffffffu);
    }
    part[threadIdx.x] = m;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] = max(part[threadIdx.x], part[threadIdx.x + w]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        int E = (int)(part[0] >> 23);
        if (E == 255) { *nonfinite = 1; E = 254; }
        E = max(E, 1);                       // zero and subnormal rows: exponent of the smallest normal
        sh[row] = YBITS - (E - 126);         // |x| < 2^(E - 126)
    }
}

// Y = rint(x * 2^sh) (round half to even) from the bits of x; |Y| <= 2^YBITS when 2^(YBITS - sh) bounds |x|.
__device__ __forceinline__ long long fixed_point(unsigned b, int sh)
{
    const int E = (int)((b >> 23) & 255u);
    const unsigned M = (E == 255) ? 0u : ((b & 0x7fffffu) | (E ? 0x800000u : 0u));   // Inf / NaN count as 0 (flagged elsewhere)
    const int shift = max(E, 1) - 150 + sh;                  // x = M * 2^(max(E,1) - 150)
    long long y;
    if (shift >= 0) {
        y = (long long)M << min(shift, 39);
    } else {
        const int r = min(-shift, 26);                       // M < 2^24: everything from r = 26 on rounds to 0
        const unsigned q = M >> r, rem = M & ((1u << r) - 1u), half = 1u << (r - 1);
        y = (long long)(q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u));
    }
    return (b >> 31) ? -y : y;
}

// One workgroup: 32 rows x 256 columns (8 k-steps).  Thread (row, k-step) reads its 32 consecutive values
// (a full 128-byte line per lane), turns them into 5 x 32 digits, written to LDS as the 8 x 5 output blocks,
// which leave 16 bytes per thread, 5 KiB contiguous per k-step.
// Digits: with C = 0x8080808080, the bytes of Y + C are the balanced digits plus 128 (adding 128 to every
// digit absorbs the borrows), i.e. the digits are the bytes of (Y + C) ^ C, the least significant first.
constexpr int SL_STEPS = 8;

// The 32 values `in` (bit patterns) of thread (row r of the block, k-step qs of the workgroup's 8) -> digits in
// blk; then the whole workgroup copies blk out.  q0 = first k-step of the workgroup, rb = block of 32 rows.
__device__ __forceinline__ void slice_store(const uint4 (&in)[8], int s_row, int r, int qs, int rb, int64_t q0,
                                            int dpad, int64_t ksteps, signed char (&blk)[SL_STEPS][NS][1024],
                                            signed char* __restrict__ P)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        unsigned w[NS][4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint4 v4 = in[4 * h + g];
            const unsigned vv[4] = {v4.x, v4.y, v4.z, v4.w};
            unsigned lo[4], hi[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned long long z = (unsigned long long)(fixed_point(vv[e], s_row) + 0x8080808080ll);
                lo[e] = (unsigned)z;
                hi[e] = (unsigned)(z >> 32);
            }
            // 4 x 4 byte transpose of lo[0..3]: word k collects byte k of the four values
            const unsigned t0 = __builtin_amdgcn_perm(lo[1], lo[0], 0x05010400u), t1 = __builtin_amdgcn_perm(lo[1], lo[0], 0x07030602u);
            const unsigned t2 = __builtin_amdgcn_perm(lo[3], lo[2], 0x05010400u), t3 = __builtin_amdgcn_perm(lo[3], lo[2], 0x07030602u);
            w[4][g] = __builtin_amdgcn_perm(t2, t0, 0x05040100u) ^ 0x80808080u;
            w[3][g] = __builtin_amdgcn_perm(t2, t0, 0x07060302u) ^ 0x80808080u;
            w[2][g] = __builtin_amdgcn_perm(t3, t1, 0x05040100u) ^ 0x80808080u;
            w[1][g] = __builtin_amdgcn_perm(t3, t1, 0x07060302u) ^ 0x80808080u;
            w[0][g] = ((hi[0] & 255u) | ((hi[1] & 255u) << 8) | ((hi[2] & 255u) << 16) | (hi[3] << 24)) ^ 0x80808080u;
        }
#pragma unroll
        for (int s = 0; s < NS; ++s)
            *reinterpret_cast<uint4*>(&blk[qs][s][(h * 32 + r) * 16]) = make_uint4(w[s][0], w[s][1], w[s][2], w[s][3]);
    }
    __syncthreads();
    // copy out: k-step q0 + qs owns 5 KiB at block index ((q0 + qs) * (dpad / 32) + rb) * NS
    const signed char* __restrict__ src = &blk[0][0][0];
#pragma unroll
    for (int pass = 0; pass < SL_STEPS * NS * 1024 / (256 * 16); ++pass) {
        const int off = (pass * 256 + (int)threadIdx.x) * 16;
        const int q = off / (NS * 1024), within = off % (NS * 1024);
        if (q0 + q < ksteps)
            *reinterpret_cast<uint4*>(P + (((q0 + q) * (dpad / 32) + rb) * NS) * 1024 + within) =
                *reinterpret_cast<const uint4*>(src + off);
    }
}

// X: the columns of this launch start at X[.][0]; n of them; ksteps = ceil(n / 32).
template <bool VEC>
__global__ __launch_bounds__(256) void slice_kernel(const float* __restrict__ X, int64_t ld, int d, int64_t n,
                                                    const int* __restrict__ sh, int dpad, int64_t ksteps,
                                                    signed char* __restrict__ P)
{
    __shared__ __attribute__((aligned(16))) signed char blk[SL_STEPS][NS][1024];
    const int rb = blockIdx.x;                      // block of 32 rows
    const int64_t q0 = (int64_t)blockIdx.y * SL_STEPS;
    const int r = threadIdx.x & 31, qs = threadIdx.x >> 5;
    const int row = rb * 32 + r;
    const int64_t c0 = (q0 + qs) * IK;
    const bool row_ok = row < d;
    const int s_row = row_ok ? sh[row] : 0;
    const float* __restrict__ x = X + (int64_t)(row_ok ? row : 0) * ld + c0;
    uint4 in[8];
    if (VEC && row_ok && c0 + IK <= n) {
#pragma unroll
        for (int g = 0; g < 8; ++g) in[g] = reinterpret_cast<const uint4*>(x)[g];
    } else {
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            unsigned v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (row_ok && c0 + 4 * g + e < n) ? __float_as_uint(x[4 * g + e]) : 0u;
            in[g] = make_uint4(v[0], v[1], v[2], v[3]);
        }
    }
    slice_store(in, s_row, r, qs, rb, q0, dpad, ksteps, blk, P);
}

// ---- convolution input: the digits of the unfolded X, straight from the zero-padded feature maps -------------
// Rows are taken tap-major, row' = (ky * k + kx) * C + c (consecutive rows = consecutive channels, which the maps
// store contiguously; the finalize kernel of the convolution mode puts H back into (c, ky, kx) order).  All k^2
// rows of a channel share the channel's exponent, taken over the whole padded copy.
struct SliceConvP {
    int hp, wp, c, k, stride, ho, wo;
    int64_t zero_origin;     // element offset of the all-zero image
    int64_t npix;            // output pixels of the whole call
};

// amax[c] = max over all pixels of |maps[.][c]| as a bit pattern (integer max: order-free).  blockIdx.x = chunk of
// pixels.  c <= 256: the workgroup walks its chunk T = c * (256 / c) elements at a time, so a thread stays on one
// channel; c > 256: thread = channel (strided), one pixel at a time.
__global__ __launch_bounds__(256) void chan_amax_kernel(const float* __restrict__ padded, int64_t pixels, int c,
                                                        unsigned* __restrict__ amax)
{
    const int64_t per = (pixels + gridDim.x - 1) / gridDim.x;
    const int64_t p0 = (int64_t)blockIdx.x * per, p1 = min(pixels, p0 + per);
    if (p0 >= p1) return;
    if (c <= 256) {
        const int T = c * (256 / c);
        if ((int)threadIdx.x >= T) return;
        unsigned m = 0;
        for (int64_t e = p0 * c + threadIdx.x; e < p1 * c; e += T) m = max(m, __float_as_uint(padded[e]) & 0x7fffffffu);
        atomicMax(&amax[threadIdx.x % c], m);
    } else {
        for (int ch = threadIdx.x; ch < c; ch += 256) {
            unsigned m = 0;
            for (int64_t p = p0; p < p1; ++p) m = max(m, __float_as_uint(padded[p * c + ch]) & 0x7fffffffu);
            atomicMax(&amax[ch], m);
        }
    }
}

__global__ __launch_bounds__(256) void chan_shift_kernel(const unsigned* __restrict__ amax, int c, int d, int* __restrict__ sh,
                                                         int* __restrict__ nonfinite)
{
    const int row = blockIdx.x * 256 + threadIdx.x;      // tap-major row
    if (row >= d) return;
    int E = (int)(amax[row % c] >> 23);
    if (E == 255) { *nonfinite = 1; E = 254; }
    E = max(E, 1);
    sh[row] = YBITS - (E - 126);
}

// The columns of this launch are the output pixels pix0 .. pix0 + n - 1 of the call.
__global__ __launch_bounds__(256) void slice_conv_kernel(const float* __restrict__ padded, SliceConvP cp, int d, int64_t pix0,
                                                         int64_t n, const int* __restrict__ sh, int dpad, int64_t ksteps,
                                                         signed char* __restrict__ P)
{
    __shared__ __attribute__((aligned(16))) signed char blk[SL_STEPS][NS][1024];
    const int rb = blockIdx.x;
    const int64_t q0 = (int64_t)blockIdx.y * SL_STEPS;
    const int r = threadIdx.x & 31, qs = threadIdx.x >> 5;
    const int row = rb * 32 + r;
    const bool row_ok = row < d;
    const int s_row = row_ok ? sh[row] : 0;
    // this row's offset from a window's top-left element in the padded copy
    const int rr = row_ok ? row : 0;
    const int tap = rr / cp.c, ch = rr - tap * cp.c, ky = tap / cp.k, kx = tap - ky * cp.k;
    const int64_t off = ((int64_t)ky * cp.wp + kx) * cp.c + ch;
    // first pixel of this thread's k-step, then stepping
    const int64_t c0 = (q0 + qs) * IK;
    const int64_t pfirst = min(pix0 + c0, cp.npix - 1);
    int64_t img = pfirst / ((int64_t)cp.ho * cp.wo);
    int rem = (int)(pfirst - img * ((int64_t)cp.ho * cp.wo));
    int yo = rem / cp.wo, xo = rem - yo * cp.wo;
    uint4 in[8];
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        unsigned v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t col = c0 + 4 * g + e;
            const bool ok = row_ok && col < n && pix0 + col < cp.npix;
            const int64_t origin = ((img * cp.hp + (int64_t)yo * cp.stride) * cp.wp + (int64_t)xo * cp.stride) * cp.c;
            v[e] = __float_as_uint(padded[(ok ? origin : cp.zero_origin) + off]);
            v[e] = ok ? v[e] : 0u;
            if (++xo == cp.wo) { xo = 0; if (++yo == cp.ho) { yo = 0; ++img; } }
        }
        in[g] = make_uint4(v[0], v[1], v[2], v[3]);
    }
    slice_store(in, s_row, r, qs, rb, q0, dpad, ksteps, blk, P);
}

// ---------------------------------------------------------------------------
// The matrix kernel.  Items are (tile, k-step) pairs, tile-major over the 128 x 128 tiles on and below the
// diagonal; persistent workgroup vb takes items [vb * per_wg, (vb + 1) * per_wg).  The part of a tile done by
// one workgroup is a piece; piece p of a tile goes to slab p of Hpart, and one workgroup owns a given
// (tile, piece), so the fp64 sums do not depend on the order in which workgroups finish.  With ls.full > 0 the
// workgroups go through the tiles in rounds instead (see i8_plan and the comments in the kernel).
// A workgroup is 8 wavefronts (see the kernel); the operands are copied global -> LDS directly
// (global_load_lds_dwordx4: no staging registers), the copy of k-step q + 1 running while the MFMAs of k-step q issue.
// 16 bytes per lane from global memory straight into LDS: lane l's bytes land at dst_block + OFF + 16 l, read
// from src_lane + OFF (the instruction's immediate offset applies to both addresses).
template <int OFF>
__device__ __forceinline__ void lds_copy_block(const signed char* __restrict__ src_lane, signed char* dst_block)
{
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src_lane,
                                     (void __attribute__((address_space(3)))*)dst_block, 16, OFF, 0);
}

// 8 wavefronts, two per SIMD; a wavefront owns 64 rows x 32 columns of the tile = 2 MFMA tiles of 32 x 32 for
// each of the 6 antidiagonals: 192 accumulator registers of the 256 a wavefront has at this occupancy, which
// leaves room for the 5 digits of one operand and 2 fragments of the other, not for a second set of fragments.
// (Tried and slower: 128 x 64 tiles with 4 wavefronts, a ring of three LDS stages and the next k-step's
// fragments prefetched into a second register set -- the compiler shuffles accumulators between the two
// register files in that loop, 1.38 ms against 0.80 on the 2304 x 25088 layer.)
__global__ __launch_bounds__(512) void xxt_i8_kernel(const signed char* __restrict__ P, const int* __restrict__ sh, int d,
                                                        int dpad, int64_t ksteps, double* __restrict__ Hpart, int64_t per_wg,
                                                        int64_t items, int classes, I8Rect rect, I8Lockstep ls)
{
    constexpr int TN = IT, NB = TN / 32;  // row blocks of the B operand
    // [buffer][block of 32 rows][digit]: the 5 digit blocks of a row block are consecutive, as in global memory
    __shared__ __attribute__((aligned(16))) signed char As[2][4][NS][1024];
    __shared__ __attribute__((aligned(16))) signed char Bs[2][NB][NS][1024];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / NB, wn = wave % NB;     // rows 64 wm .., columns 32 wn ..

    // Workgroups are dealt to the 8 XCDs round-robin; vpos = the workgroup's place in an order in which each
    // XCD owns one contiguous run.  Position -> range index vb, class-major: when a tile is cut into `classes`
    // pieces, the ranges vb = c, c + classes, c + 2 classes, ... cover the same part of the calibration
    // dimension of consecutive tiles, and only they can share fetches in the XCD's L2: ordering the ranges
    // by (vb mod classes, vb) puts up to 32 of them on one XCD instead of 32 / classes.
    const int nx = 8, gq = (int)gridDim.x / nx, grem = (int)gridDim.x % nx;
    const int xcd = (int)blockIdx.x % nx;
    const int vpos = xcd * gq + min(xcd, grem) + (int)blockIdx.x / nx;
    int64_t vb = vpos;
    if (classes > 1) {
        int cls = 0, before = 0;
        for (;;) {
            const int cnt = ((int)gridDim.x - cls + classes - 1) / classes;   // ranges with vb mod classes == cls
            if (vpos < before + cnt) break;
            before += cnt;
            ++cls;
        }
        vb = cls + classes * (vpos - before);
    }

    const int64_t g0 = vb * per_wg, g1 = min(items, g0 + per_wg);
    const int64_t step_bytes = (int64_t)(dpad / 32) * NS * 1024;     // one k-step of all rows
    int npieces = 0, t_first = 0, t_last = 0;
    if (ls.full > 0) {
        // In step: `full` rounds of whole tiles, then the tiles left over, each cut into ls.pieces equal parts of
        // the calibration dimension, dealt piece-major.  In every round the workgroup at position vpos takes entry
        // round * gridDim.x + vpos, so all workgroups start a round together at the same k-step and the 32 of an XCD
        // hold 32 consecutive tiles of the blocked order below.
        const int64_t units = (int64_t)ls.rem * ls.pieces;
        npieces = ls.full + (int)(vpos < units ? (units - vpos + gridDim.x - 1) / gridDim.x : 0);
    } else {
        if (g0 >= g1) return;
        t_first = (int)(g0 / ksteps);
        t_last = (int)((g1 - 1) / ksteps);
        npieces = t_last - t_first + 1;
    }

    for (int pi = 0; pi < npieces; ++pi) {
        // Ranges (ls.full == 0).  All workgroups start together and advance one k-step per step, so k-step k is best
        // visited at step k mod per_wg: workgroups on neighbouring tiles (same class, same XCD) then read the same
        // columns at the same time.  A range inside one tile starts at its k-step whose index is a multiple of per_wg
        // and wraps around; a range over two tiles takes the head of the later tile before the tail of the
        // earlier one.  The order of the sum is fixed, so results are reproducible.
        int tile, piece;
        int64_t c_begin, c_end, rot = 0;
        if (ls.full > 0) {
            if (pi < ls.full) {
                tile = pi * (int)gridDim.x + vpos;
                piece = 0;
                c_begin = 0;
                c_end = ksteps;
            } else {
                const int64_t u = (int64_t)(pi - ls.full) * gridDim.x + vpos;
                piece = (int)(u / ls.rem);
                tile = ls.full * (int)gridDim.x + (int)(u - (int64_t)piece * ls.rem);
                c_begin = min(ksteps, piece * ls.piece_len);
                c_end = min(ksteps, c_begin + ls.piece_len);
            }
        } else {
            tile = npieces == 2 ? t_last - pi : t_first + pi;
            const int64_t tile_first = (int64_t)tile * ksteps;
            c_begin = max(g0, tile_first) - tile_first;
            c_end = min(g1, tile_first + ksteps) - tile_first;
            if (npieces == 1) {
                const int64_t aligned = (c_begin + per_wg - 1) / per_wg * per_wg;
                if (aligned < c_end) rot = aligned - c_begin;
            }
            piece = (int)(vb - tile_first / per_wg);            // ranges that reached this tile before this one
        }
        const int64_t len = c_end - c_begin;
        if (len <= 0) continue;                                 // the same for the whole workgroup
        auto kstep_at = [&](int64_t i) {
            int64_t c = i + rot;
            if (c >= len) c -= len;
            return c_begin + c;
        };
        // tile -> (I, J): I >= J, row-major over the lower triangle; or, for a list of tile rows (rect.cb > 0: two
        // groups of rect.cb tile rows, the second starting at tile row rect.gap), all tile columns of those rows;
        // or, in step, the lower triangle in blocks of 8 x 8 tiles (block rows top down, blocks left to right, tiles
        // row-major inside a block): 32 consecutive tiles touch about 12 row blocks of the operands, not 33
        int I, J;
        if (rect.half) {
            I = 0;
            J = tile;
        } else if (rect.cb > 0) {
            const int ntj = dpad / IT, ri = tile / ntj;
            J = tile - ri * ntj;
            I = ri < rect.cb ? ri : ri - rect.cb + rect.gap;
        } else if (ls.full > 0) {
            const int nt = dpad / IT;
            int Ib = 0, before = 0, rows, cnt;
            for (;; ++Ib) {
                rows = min(8, nt - 8 * Ib);
                cnt = rows * 8 * Ib + rows * (rows + 1) / 2;
                if (tile < before + cnt) break;
                before += cnt;
            }
            int w = tile - before;
            if (w < rows * 8 * Ib) {
                const int Jb = w / (rows * 8);
                w -= Jb * rows * 8;
                I = 8 * Ib + w / 8;
                J = 8 * Jb + w % 8;
            } else {
                w -= rows * 8 * Ib;
                int li = 0;
                while ((li + 1) * (li + 2) / 2 <= w) ++li;
                I = 8 * Ib + li;
                J = 8 * Ib + w - li * (li + 1) / 2;
            }
        } else {
            I = (int)((sqrtf(8.0f * (float)tile + 1.0f) - 1.0f) * 0.5f);
            while ((I + 1) * (I + 2) / 2 <= tile) ++I;
            while (I * (I + 1) / 2 > tile) --I;
            J = tile - I * (I + 1) / 2;
        }
        const bool tri = rect.cb == 0;       // only the lower triangle is wanted (and stored)
        const int i0 = I * IT, j0 = J * TN;
        double* __restrict__ out = Hpart + (int64_t)piece * d * d;

        // one wavefront copies one row block of an operand, all 5 digits (5 KiB contiguous in global memory and
        // in LDS); the addresses point at digit 2 so that the five immediates are -2048 .. 2048
        auto copy5 = [&](const signed char* __restrict__ g, signed char* l) {
            lds_copy_block<-2048>(g, l); lds_copy_block<-1024>(g, l); lds_copy_block<0>(g, l);
            lds_copy_block<1024>(g, l);  lds_copy_block<2048>(g, l);
        };
        // A's four blocks of 32 rows: consecutive, or (rect.half) the rows 0 .. 63 and 128 .. 191
        const int ablk = rect.half ? (wave & 1) + 4 * ((wave >> 1) & 1) : i0 / 32 + (wave & 3);
        const signed char* __restrict__ pa = P + ((int64_t)ablk * NS + 2) * 1024 + lane * 16;
        const signed char* __restrict__ pb = P + ((int64_t)(j0 / 32 + (wave % NB)) * NS + 2) * 1024 + lane * 16;
        auto issue = [&](int buf, int64_t q) {      // wavefronts 0..3 take A's row blocks, 4..7 B's
            if (wave < 4) copy5(pa + q * step_bytes, &As[buf][wave][2][0]);
            else copy5(pb + q * step_bytes, &Bs[buf][wave - 4][2][0]);
        };

        for (int64_t ib = 0; ib < len; ib += I8_FOLD_STEPS) {
            const int64_t ie = min(len, ib + I8_FOLD_STEPS);
            i32x16 acc[NM][2];
#pragma unroll
            for (int m = 0; m < NM; ++m)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[m][i][v] = 0;

            __syncthreads();                 // LDS free (the stage before is consumed)
            issue(0, kstep_at(ib));
            __builtin_amdgcn_s_waitcnt(0);   // vmcnt(0): the copies have landed
            __syncthreads();
            // On a diagonal tile only the MFMA tiles on and below the diagonal are formed (10 of the workgroup's 16:
            // row block 2 wm + i against column block wn needs wn <= 2 wm + i); the wavefronts with less to do still
            // copy and meet the others.  The matrix pipes run against a power limit, so what is not multiplied is
            // time for the rest of the chip even where this workgroup's own k-step is no shorter.
            auto ksteps_loop = [&](auto first_block, auto second_block) {
                constexpr bool DO0 = decltype(first_block)::value, DO1 = decltype(second_block)::value;
                int buf = 0;
                for (int64_t it = ib; it < ie; ++it) {
                    if (it + 1 < ie) issue(buf ^ 1, kstep_at(it + 1));
                    if (DO1) {
                        i32x4 fb[NS];
#pragma unroll
                        for (int t = 0; t < NS; ++t)
                            fb[t] = *reinterpret_cast<const i32x4*>(&Bs[buf][wn][t][lane * 16]);
#pragma unroll
                        for (int s = 0; s < NS; ++s) {
                            i32x4 fa[2];
#pragma unroll
                            for (int i = DO0 ? 0 : 1; i < 2; ++i)
                                fa[i] = *reinterpret_cast<const i32x4*>(&As[buf][wm * 2 + i][s][lane * 16]);
#pragma unroll
                            for (int t = 0; t < NS; ++t) {
                                if (s + t < NM) {
#pragma unroll
                                    for (int i = DO0 ? 0 : 1; i < 2; ++i)
                                        acc[s + t][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[t], acc[s + t][i], 0, 0, 0);
                                }
                            }
                        }
                    }
                    __builtin_amdgcn_s_waitcnt(0);
                    __syncthreads();
                    buf ^= 1;
                }
            };
            const bool need0 = !tri || I != J || wn <= 2 * wm, need1 = !tri || I != J || wn <= 2 * wm + 1;
            if (need0) ksteps_loop(std::true_type(), std::true_type());
            else if (need1) ksteps_loop(std::false_type(), std::true_type());
            else ksteps_loop(std::false_type(), std::false_type());

            // fold: sum_m acc_m 256^(8 - m), times 2^-(sh_row + sh_col), added into the fp64 slab (lower triangle)
            const int col = j0 + wn * 32 + (lane & 31);
            const int sc = col < d ? sh[col] : 0;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = i0 + wm * (rect.half ? 128 : 64) + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                    if (row < d && col < d && (!tri || col <= row)) {
                        double sum = 0.0;
#pragma unroll
                        for (int m = NM - 1; m >= 0; --m)
                            sum += (double)acc[m][i][v] * __builtin_ldexp(1.0, 8 * (2 * (NS - 1) - m));
                        out[(int64_t)row * d + col] += ldexp(sum, -(sh[row] + sc));
                    }
                }
            }
        }
    }
}


struct I8Plan { int nt, wgs; int64_t ksteps, items, per_wg; I8Lockstep ls; };

// Digits that fit the 256 MB memory-side cache are served from it however the workgroups walk them; beyond that,
// with at least one tile per workgroup, the ranges below leave every workgroup at a k-step of its own and every
// operand block is fetched from memory again by each tile that uses it (d = 4608, n = 49152: 37 GB for 1.1 GB of
// digits, 5 TB/s, and the kernel waits for it).  Then the tiles are taken in step instead.
constexpr size_t I8_INSTEP_MIN_BYTES = (size_t)256 << 20;
constexpr int I8_MAX_PIECES = 8;

static bool i8_instep_wanted(int d, int64_t n, I8Rect rect)
{
    const int64_t nt = i8_dpad(d) / IT;
    return rect.cb == 0 && nt * (nt + 1) / 2 >= I8_WGS && i8_planes_bytes(d, n) > I8_INSTEP_MIN_BYTES;
}

int xxt_i8_wanted_splits(int d, int64_t n, I8Rect rect)
{
    const int64_t fit = ((int64_t)4 << 30) / ((int64_t)d * d * (int64_t)sizeof(double));     // at most 4 GiB of slabs
    if (rect.cb > 0) {
        // a list of tile rows has fewer tiles than the triangle that the context's count of slabs is made for: enough
        // pieces per tile that every workgroup gets a range
        const int64_t nt = i8_dpad(d) / IT, tiles = rect.half ? nt : 2 * rect.cb * nt;
        const int64_t want = (I8_WGS + tiles - 1) / tiles + 1;
        return (int)(want < fit ? want : (fit < 2 ? 2 : fit));
    }
    if (!i8_instep_wanted(d, n, rect)) return 0;
    return (int)(fit < 2 ? 2 : (fit > I8_MAX_PIECES ? I8_MAX_PIECES : fit));
}

static I8Plan i8_plan(int d, int64_t n, int splits, I8Rect rect)
{
    I8Plan p;
    p.nt = i8_dpad(d) / IT;
    p.ksteps = i8_ksteps(n);
    const int64_t tiles = rect.half ? p.nt : rect.cb > 0 ? (int64_t)2 * rect.cb * p.nt : (int64_t)p.nt * (p.nt + 1) / 2;
    if (i8_instep_wanted(d, n, rect)) {
        // Whole rounds of one tile per workgroup, then the rem tiles left over in `pieces` parts each (part j of a
        // tile goes to slab j): the number of parts that ends soonest, where a slab more is charged what clearing
        // and re-reading it costs -- about d^2 / 2^20 k-steps (a k-step of a workgroup takes 1.8 us).
        const int full = (int)(tiles / I8_WGS), rem = (int)(tiles - (int64_t)full * I8_WGS);
        const int64_t slab_steps = (int64_t)d * d / (1 << 20) + 1;
        int best_p = 0;
        int64_t best_cost = 0, best_len = 0;
        for (int q = 1; rem > 0 && q <= splits && q <= I8_MAX_PIECES; ++q) {
            const int64_t len = (p.ksteps + q - 1) / q;
            const int64_t rounds = ((int64_t)rem * q + I8_WGS - 1) / I8_WGS;
            const int64_t cost = rounds * len + q * slab_steps;
            if (best_p == 0 || cost < best_cost) { best_p = q; best_cost = cost; best_len = len; }
        }
        // in step unless the left-over rounds cost more than 10 % over an even split of all the work
        const int64_t total = (int64_t)full * p.ksteps + (rem > 0 ? best_cost - best_p * slab_steps : 0);
        if ((rem == 0 || best_p > 0) && total * I8_WGS * 10 <= tiles * p.ksteps * 11) {
            p.ls.full = full;
            p.ls.rem = rem;
            p.ls.pieces = best_p;
            p.ls.piece_len = best_len;
            p.items = 0;
            p.per_wg = 1;
            p.wgs = I8_WGS;
            return p;
        }
    }
    p.items = tiles * p.ksteps;
    p.per_wg = (p.items + I8_WGS - 1) / I8_WGS;
    // a tile meets at most ceil(ksteps / per_wg) + 1 ranges; that must not exceed the slabs
    const int64_t min_len = splits > 1 ? (p.ksteps + splits - 2) / (splits - 1) : p.ksteps;
    if (p.per_wg < min_len) p.per_wg = min_len;
    if (p.per_wg < 1) p.per_wg = 1;
    p.wgs = (int)((p.items + p.per_wg - 1) / p.per_wg);
    return p;
}

int xxt_i8_slabs_touched(int d, int64_t n, int splits, I8Rect rect)
{
    const I8Plan pl = i8_plan(d, n, splits, rect);
    if (pl.ls.full > 0) return pl.ls.pieces > 1 ? pl.ls.pieces : 1;
    const int64_t p = (pl.ksteps + pl.per_wg - 1) / pl.per_wg + 1;
    return (int)(p < splits ? p : splits);
}

// Per call: sh (i8_dpad(d) ints) from all n columns of X; *nonfinite is raised when X holds an Inf or NaN.
hipError_t launch_i8_row_shifts(hipStream_t s, const float* X, int64_t ld, int d, int64_t n, int* sh, int* nonfinite)
{
    const bool vec = (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    if (vec) hipLaunchKernelGGL(row_shift_kernel<true>, dim3(d), dim3(256), 0, s, X, ld, d, n, sh, nonfinite);
    else     hipLaunchKernelGGL(row_shift_kernel<false>, dim3(d), dim3(256), 0, s, X, ld, d, n, sh, nonfinite);
    return hipGetLastError();
}

// Digits of the n columns that start at X (planes: i8_planes_bytes(d, n) bytes).
hipError_t launch_i8_slice(hipStream_t s, const float* X, int64_t ld, int d, int64_t n, const int* sh, signed char* planes)
{
    const int dpad = i8_dpad(d);
    const int64_t ksteps = i8_ksteps(n);
    const bool vec = (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    const dim3 grid(dpad / 32, (unsigned)((ksteps + SL_STEPS - 1) / SL_STEPS));
    if (vec) hipLaunchKernelGGL(slice_kernel<true>, grid, dim3(256), 0, s, X, ld, d, n, sh, dpad, ksteps, planes);
    else     hipLaunchKernelGGL(slice_kernel<false>, grid, dim3(256), 0, s, X, ld, d, n, sh, dpad, ksteps, planes);
    return hipGetLastError();
}

// Convolution input, per call: channel maxima over the padded copy ((n_img + 1) x hp x wp x c), then sh for the
// d = c k^2 tap-major rows.  amax: c words of scratch.
hipError_t launch_i8_chan_shifts(hipStream_t s, const float* padded, int64_t pixels, int c, int d, unsigned* amax, int* sh,
                                 int* nonfinite)
{
    hipError_t e = launch_clear_words(s, amax, c, nullptr, 0);
    if (e != hipSuccess) return e;
    const int64_t chunks = (pixels + 63) / 64;           // at least 64 pixels per workgroup
    hipLaunchKernelGGL(chan_amax_kernel, dim3((unsigned)(chunks < 4096 ? (chunks < 1 ? 1 : chunks) : 4096)), dim3(256), 0, s,
                       padded, pixels, c, amax);
    hipLaunchKernelGGL(chan_shift_kernel, dim3((d + 255) / 256), dim3(256), 0, s, amax, c, d, sh, nonfinite);
    return hipGetLastError();
}

// Digits of the unfolded input for the output pixels pix0 .. pix0 + n - 1 (tap-major rows).
hipError_t launch_i8_slice_conv(hipStream_t s, const float* padded, int n_img, int hp, int wp, int c, int k, int stride,
                                int ho, int wo, int64_t npix, int64_t pix0, int64_t n, const int* sh, signed char* planes)
{
    const int d = c * k * k, dpad = i8_dpad(d);
    const int64_t ksteps = i8_ksteps(n);
    SliceConvP cp;
    cp.hp = hp; cp.wp = wp; cp.c = c; cp.k = k; cp.stride = stride; cp.ho = ho; cp.wo = wo;
    cp.zero_origin = (int64_t)n_img * hp * wp * c;
    cp.npix = npix;
    hipLaunchKernelGGL(slice_conv_kernel, dim3(dpad / 32, (unsigned)((ksteps + SL_STEPS - 1) / SL_STEPS)), dim3(256), 0, s,
                       padded, cp, d, pix0, n, sh, dpad, ksteps, planes);
    return hipGetLastError();
}

hipError_t launch_xxt_i8(hipStream_t s, const signed char* planes, const int* sh, int d, int64_t n, double* Hpart,
                         int splits, LaunchEvents ev, I8Rect rect)
{
    const I8Plan pl = i8_plan(d, n, splits, rect);
    // pieces per tile, rounded: the number of classes of ranges (see the kernel)
    int classes = (int)((pl.ksteps + pl.per_wg / 2) / pl.per_wg);
    classes = classes < 1 || pl.ls.full > 0 ? 1 : (classes > pl.wgs ? pl.wgs : classes);
    hipExtLaunchKernelGGL(xxt_i8_kernel, dim3(pl.wgs), dim3(512), 0, s, ev.start, ev.stop, 0, planes, sh, d, i8_dpad(d),
                          pl.ksteps, Hpart, pl.per_wg, pl.items, classes, rect, pl.ls);
    return hipGetLastError();
}

}  // namespace fobq
