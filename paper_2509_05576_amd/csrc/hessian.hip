// Hessian of the layer objective (Section 3, Eq. 2): H = (2/N) X X^T.
//
// xxt_kernel: fp32 X is read from HBM, staged through LDS as fp32, widened to
// fp64 when the MFMA fragments are formed (products of two fp32 values are
// exact in fp64), and accumulated with v_mfma_f64_16x16x4_f64.  Only the 128 x 128
// tiles on or below the diagonal are computed.
//
// Work decomposition ("stream-K"): the work items are (tile, 32-column chunk of
// the calibration dimension) pairs in tile-major order; a fixed number of
// persistent workgroups each take one contiguous, equally long range of items, so
// every workgroup does the same amount of MFMA work whatever d and n are.  A
// range can cross tile boundaries; the part of a tile done by one workgroup is a
// "piece".  Piece p of a tile is added into slab p of Hpart (XXT_SLABS slabs of
// d x d), and exactly one workgroup owns a given (tile, piece) in a launch, so
// the sums do not depend on the order in which workgroups finish.
//
// Convolution mode: the same kernel with a loader that reads the unfolded input of a k x k
// convolution straight from NHWC feature maps (X is never materialised).  Row (c, ky, kx) of
// X, column (image, y, x) is maps[image][y*stride + ky - pad][x*stride + kx - pad][c] or 0
// outside the map.  pad_maps_kernel first writes a zero-padded copy of the maps with one extra
// all-zero image at the end, so that every window lies inside the copy (no per-element test)
// and the columns past the last pixel read zeros from the extra image (no branch).  Inside the
// kernel the rows are taken tap-major (row' = (ky*k + kx)*C + c) so that consecutive rows are
// consecutive channels, which NHWC stores contiguously; the finalize kernel of this mode puts
// H back into the (c, ky, kx) order.
#include <hip/hip_ext.h>

#include "fobq_internal.h"

namespace fobq {

typedef double d4 __attribute__((ext_vector_type(4)));

// n / dv for 0 <= n < 2^32 and a divisor fixed at launch: q = (t + ((n - t) >> s1)) >> s2 with
// t = umulhi(m, n)  (division by an invariant integer through multiplication).
struct FastDiv { uint32_t m; int s1, s2; };

static FastDiv fastdiv_make(uint32_t dv)
{
    FastDiv f;
    int L = 0;
    while ((1ull << L) < dv) ++L;
    f.m = (uint32_t)(((1ull << 32) * ((1ull << L) - dv)) / dv + 1);
    f.s1 = L < 1 ? L : 1;
    f.s2 = L > 1 ? L - 1 : 0;
    return f;
}

__device__ __forceinline__ uint32_t fastdiv(uint32_t n, const FastDiv& f)
{
    const uint32_t t = __umulhi(f.m, n);
    return (t + ((n - t) >> f.s1)) >> f.s2;
}

struct ConvP {
    int hp, wp, c, k, stride, ho, wo;   // hp, wp: height and width of the padded copy
    int64_t zero_origin;                // element offset of the all-zero image
    FastDiv div_img;    // by ho * wo
    FastDiv div_row;    // by wo
    FastDiv div_c;      // by c
    FastDiv div_k;      // by k
};

// out: (n_img + 1) x hp x wp x c, hp = h + 2 pad, wp = w + 2 pad; image n_img is all zeros
__global__ __launch_bounds__(256) void pad_maps_kernel(const float* __restrict__ maps, int n_img, int h, int w, int c,
                                                       int pad, float* __restrict__ out, int64_t total)
{
    const int hp = h + 2 * pad, wp = w + 2 * pad;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int ch = (int)(idx % c);
        int64_t r = idx / c;
        const int x = (int)(r % wp) - pad;
        r /= wp;
        const int y = (int)(r % hp) - pad;
        const int64_t img = r / hp;
        float v = 0.f;
        if (img < n_img && (unsigned)y < (unsigned)h && (unsigned)x < (unsigned)w)
            v = maps[((img * h + y) * w + x) * c + ch];
        out[idx] = v;
    }
}

hipError_t launch_pad_maps(hipStream_t s, const float* maps, int n_img, int h, int w, int c, int pad, float* out)
{
    const int64_t total = (int64_t)(n_img + 1) * (h + 2 * pad) * (w + 2 * pad) * c;
    const int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(pad_maps_kernel, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, s, maps, n_img, h,
                       w, c, pad, out, total);
    return hipGetLastError();
}

// Tile edge XT: 128 (each of the 4 wavefronts owns 64 x 64 = 4 x 4 MFMA tiles) or, for small d where
// 128-wide tiles are mostly padding, 64 (32 x 32 = 2 x 2 MFMA tiles per wavefront; twice the operand
// traffic and conversions per MFMA, but up to 4x less padding).
constexpr int XK = 32;           // calibration columns per LDS stage
constexpr int XLD = XK + 4;      // fp32 row stride in LDS: 16B-aligned rows, conflict-free 16B fragment reads
constexpr int xxt_wgs(int xt) { return xt == 128 ? 512 : 1024; }   // persistent workgroups: 2 or 4 per compute unit

// 64-wide tiles when they cut the padded area (tiles on or below the diagonal) by more than the ~20 % that
// the smaller tile costs in matrix-pipe efficiency.
static int xxt_tile(int d)
{
    const int64_t n128 = (d + 127) / 128, n64 = (d + 63) / 64;
    const int64_t a128 = n128 * (n128 + 1) / 2 * 128 * 128, a64 = n64 * (n64 + 1) / 2 * 64 * 64;
    return a64 * 6 < a128 * 5 ? 64 : 128;
}

// Order of the lower-triangle tiles: tile rows are taken in pairs (2r, 2r + 1) and a pair is walked
// column by column, (2r, J), (2r + 1, J), (2r, J + 1), ...  Consecutive tiles of the order then share a
// panel of X: the column panel J with the tile just before or after, the row panel with the tile two
// places away.  Pair r starts at index 2 r^2 + r and has 4 r + 3 tiles; an odd last row stands alone.
__device__ __forceinline__ void tile_decode(int t, int nt, int& I, int& J)
{
    int r = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.25f);
    while (2 * (r + 1) * (r + 1) + (r + 1) <= t) ++r;
    while (2 * r * r + r > t) --r;
    const int u = t - (2 * r * r + r);
    if (2 * r + 1 >= nt) { I = 2 * r; J = u; }                       // unpaired last row
    else if (u < 4 * r + 2) { I = 2 * r + (u & 1); J = u >> 1; }
    else { I = 2 * r + 1; J = 2 * r + 1; }                           // diagonal tile of the second row
}

// MODE 0: X rows are 16-byte aligned (ld % 4 == 0, base aligned) -> float4 loads.
// MODE 1: any ld / alignment.  MODE 2: X = feature maps, n = images * ho * wo (convolution mode).
template <int MODE, int XT>
__global__ __launch_bounds__(256, XT == 128 ? 2 : 4) void xxt_kernel(const float* __restrict__ X, int64_t ld, int d, int64_t n,
                                                     double* __restrict__ Hpart, int chunks, int64_t per_wg,
                                                     int64_t total_items, int classes, ConvP cp)
{
    constexpr bool FAST = MODE == 0;
    constexpr bool CONV = MODE == 2;
    constexpr int RG = XT / 32;       // groups of 32 rows per operand tile (plain loader: one float4 per group)
    constexpr int WT = XT / 2;        // edge of a wavefront's part of the tile
    constexpr int MT = WT / 16;       // MFMA tiles per edge of that part
    __shared__ float As[2][XT][XLD];
    __shared__ float Bs[2][XT][XLD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = tid >> 3;          // 0..31: row within a group of 32 rows
    const int lk = (tid & 7) * 4;     // 0..28: first of 4 consecutive calibration columns
    const int fr = lane & 15;         // fragment row
    const int fk = (lane >> 4) * 4;   // fragment: 4 consecutive columns, one per k-step (the sum over k is order-free)
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // the same value, known to be wavefront-uniform

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD one contiguous run of ranges, so
    // that the workgroups sharing an L2 work on neighbouring tiles (which share panels of X) at almost
    // the same position of the calibration dimension.
    const int nx = 8, gq = (int)gridDim.x / nx, grem = (int)gridDim.x % nx;
    const int xcd = (int)blockIdx.x % nx;
    const int vpos = xcd * gq + min(xcd, grem) + (int)blockIdx.x / nx;
    // Position vpos in that XCD-contiguous order -> range index vb, class-major: when a tile is cut
    // into `classes` pieces, the ranges vb = c, c + classes, c + 2 classes, ... cover the same part
    // of the calibration dimension of consecutive tiles, and only they can share fetches; ordering
    // the ranges by (vb mod classes, vb) puts up to 64 of them on one XCD instead of 64 / classes.
    int vb = vpos;
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
    const int nt = (d + XT - 1) / XT;

    // This workgroup's range of items [g0, g1) and its pieces (one per tile it touches).  All
    // workgroups start together and advance one chunk per step, so chunk k is best visited at step
    // k mod per_wg: workgroups on neighbouring tiles (which share panels of X and, thanks to the
    // mapping above, an L2) then read the same columns of X at the same time.  A range inside one
    // tile therefore starts at its chunk whose index is a multiple of per_wg and wraps around; a range
    // over two tiles takes the head of the later tile (chunks 0 ...) before the tail of the earlier
    // one.  The order of the sum over chunks is free; it stays fixed, so results are reproducible.
    const int64_t g0 = (int64_t)vb * per_wg;
    const int64_t g1 = min(total_items, g0 + per_wg);
    if (g0 >= g1) return;
    const int t_first = (int)(g0 / chunks), t_last = (int)((g1 - 1) / chunks);
    const int npieces = t_last - t_first + 1;

    for (int pi = 0; pi < npieces; ++pi) {
        const int tile = npieces == 2 ? t_last - pi : t_first + pi;
        const int64_t tile_first = (int64_t)tile * chunks;
        const int c_begin = (int)(max(g0, tile_first) - tile_first);
        const int c_end = (int)(min(g1, tile_first + chunks) - tile_first);
        const int len = c_end - c_begin;
        int rot = 0;
        if (npieces == 1) {
            const int64_t aligned = (c_begin + per_wg - 1) / per_wg * per_wg;
            if (aligned < c_end) rot = (int)(aligned - c_begin);
        }
        auto chunk_at = [&](int i) {
            int c = i + rot;
            if (c >= len) c -= len;
            return c_begin + c;
        };
        // piece index of this range inside its tile: number of workgroup boundaries before it
        const int piece = (int)(vb - tile_first / per_wg);    // 0 for the workgroup whose range reaches the tile first
        int I, J;
        tile_decode(tile, nt, I, J);
        const int i0 = I * XT, j0 = J * XT;

        // plain modes: clamped row pointers (rows past d produce outputs that are never stored);
        // thread = (row lr + 32 u, 4 consecutive columns)
        const float* __restrict__ arow[RG];
        const float* __restrict__ brow[RG];
        // convolution mode: thread = (rows lane + 64 q, pixels 8 wave + j): a load covers 64
        // consecutive channels (256 contiguous bytes) of ONE pixel, so the pixel's decoding and its
        // window origin are wavefront-uniform (scalar unit).  Per tile: the offset of this thread's
        // two rows (ky, kx, channel) of each operand from the window's top-left element in the
        // padded copy.  Rows past d stand in as row d - 1.
        constexpr int QN = XT / 64;    // rows per operand and thread in convolution mode
        uint32_t offA[QN], offB[QN];
        if (CONV) {
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                const int ra = min(i0 + lane + 64 * q, d - 1), rb = min(j0 + lane + 64 * q, d - 1);
                const uint32_t ta = fastdiv((uint32_t)ra, cp.div_c), tb = fastdiv((uint32_t)rb, cp.div_c);
                const uint32_t kya = fastdiv(ta, cp.div_k), kyb = fastdiv(tb, cp.div_k);
                offA[q] = (kya * cp.wp + (ta - kya * cp.k)) * cp.c + ((uint32_t)ra - ta * cp.c);
                offB[q] = (kyb * cp.wp + (tb - kyb * cp.k)) * cp.c + ((uint32_t)rb - tb * cp.c);
            }
        } else {
#pragma unroll
            for (int u = 0; u < RG; ++u) {
                arow[u] = X + (int64_t)min(i0 + lr + 32 * u, d - 1) * ld;
                brow[u] = X + (int64_t)min(j0 + lr + 32 * u, d - 1) * ld;
            }
        }
        float4 pa[RG], pb[RG];
        // Convolution mode: the loads of pixel j (0..7) of chunk c for this thread's rows; called
        // with j = 0, 1, ..., 7 in this order.  Pixel 0 is decoded in full (two divisions by
        // invariant integers), the others by stepping (image, y, x) one pixel on; a pixel past the
        // last one takes the all-zero image.  All of it is wavefront-uniform, i.e. scalar-unit
        // work with no branch: arithmetic on the vector unit takes cycles from the fp64 matrix
        // instructions (the kernel slows down by what the vector instructions add).
        int px_img = 0, px_yo = 0, px_xo = 0;
        auto gload_px = [&](int c, int j) {
            float* fa = reinterpret_cast<float*>(pa);
            float* fb = reinterpret_cast<float*>(pb);
            const int p = c * XK + 8 * wave_s + j;               // < 2^31 (checked by the caller)
            const bool pv = p < (int)n;
            if (j == 0) {
                const uint32_t pc = (uint32_t)min(p, (int)n - 1);
                const uint32_t img = fastdiv(pc, cp.div_img);
                const uint32_t rem = pc - img * (uint32_t)(cp.ho * cp.wo);
                const uint32_t yo = fastdiv(rem, cp.div_row);
                px_img = (int)img;
                px_yo = (int)yo;
                px_xo = (int)(rem - yo * (uint32_t)cp.wo);
            } else {
                ++px_xo;
                const bool wx = px_xo == cp.wo;
                px_xo = wx ? 0 : px_xo;
                px_yo += wx ? 1 : 0;
                const bool wy = px_yo == cp.ho;
                px_yo = wy ? 0 : px_yo;
                px_img += wy ? 1 : 0;
            }
            const int64_t origin = (((int64_t)px_img * cp.hp + px_yo * cp.stride) * cp.wp + px_xo * cp.stride) * cp.c;
            const float* __restrict__ win = X + (pv ? origin : cp.zero_origin);
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                fa[q * 8 + j] = win[offA[q]];
                fb[q * 8 + j] = win[offB[q]];
            }
        };
        auto gload = [&](int c) {
            if (CONV) {
#pragma unroll
                for (int j = 0; j < 8; ++j) gload_px(c, j);
                return;
            }
            const int64_t k = (int64_t)c * XK + lk;
            if (FAST && k + 3 < n) {
#pragma unroll
                for (int u = 0; u < RG; ++u) {
                    pa[u] = *reinterpret_cast<const float4*>(arow[u] + k);
                    pb[u] = *reinterpret_cast<const float4*>(brow[u] + k);
                }
            } else {
#pragma unroll
                for (int u = 0; u < RG; ++u) {
                    float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va;
                    if (k + 0 < n) { va.x = arow[u][k + 0]; vb.x = brow[u][k + 0]; }
                    if (k + 1 < n) { va.y = arow[u][k + 1]; vb.y = brow[u][k + 1]; }
                    if (k + 2 < n) { va.z = arow[u][k + 2]; vb.z = brow[u][k + 2]; }
                    if (k + 3 < n) { va.w = arow[u][k + 3]; vb.w = brow[u][k + 3]; }
                    pa[u] = va;
                    pb[u] = vb;
                }
            }
        };
        auto sstore = [&](int buf) {
            if (CONV) {
                // 8 consecutive pixels of a row: two 16-byte stores per row
#pragma unroll
                for (int q = 0; q < QN; ++q) {
                    *reinterpret_cast<float4*>(&As[buf][lane + 64 * q][8 * wave]) = pa[2 * q];
                    *reinterpret_cast<float4*>(&As[buf][lane + 64 * q][8 * wave + 4]) = pa[2 * q + 1];
                    *reinterpret_cast<float4*>(&Bs[buf][lane + 64 * q][8 * wave]) = pb[2 * q];
                    *reinterpret_cast<float4*>(&Bs[buf][lane + 64 * q][8 * wave + 4]) = pb[2 * q + 1];
                }
                return;
            }
#pragma unroll
            for (int u = 0; u < RG; ++u) {
                *reinterpret_cast<float4*>(&As[buf][lr + 32 * u][lk]) = pa[u];
                *reinterpret_cast<float4*>(&Bs[buf][lr + 32 * u][lk]) = pb[u];
            }
        };

        d4 acc[MT][MT];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < MT; ++j) acc[i][j] = d4{0.0, 0.0, 0.0, 0.0};

        __syncthreads();              // LDS free (previous tile's last stage consumed)
        gload(chunk_at(0));
        sstore(0);
        __syncthreads();
        int cur = 0;
        for (int ci = 0; ci < len; ++ci) {
            const bool more = ci + 1 < len;
            // plain modes: 8 wide loads, issued up front.  Convolution mode: one pixel's loads per
            // group of 16 MFMAs (after the last chunk of a range the same chunk is simply loaded
            // again and not stored).
            const int cn = chunk_at(more ? ci + 1 : ci);
            if (!CONV && more) gload(cn);
#pragma unroll
            for (int g = 0; g < XK / 16; ++g) {
                float4 fa[MT], fb[MT];
#pragma unroll
                for (int i = 0; i < MT; ++i)
                    fa[i] = *reinterpret_cast<const float4*>(&As[cur][wm * WT + i * 16 + fr][g * 16 + fk]);
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    fb[j] = *reinterpret_cast<const float4*>(&Bs[cur][wn * WT + j * 16 + fr][g * 16 + fk]);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    double a[MT], b[MT];
#pragma unroll
                    for (int i = 0; i < MT; ++i)
                        a[i] = (double)(ks == 0 ? fa[i].x : ks == 1 ? fa[i].y : ks == 2 ? fa[i].z : fa[i].w);
#pragma unroll
                    for (int j = 0; j < MT; ++j)
                        b[j] = (double)(ks == 0 ? fb[j].x : ks == 1 ? fb[j].y : ks == 2 ? fb[j].z : fb[j].w);
#pragma unroll
                    for (int i = 0; i < MT; ++i)
#pragma unroll
                        for (int j = 0; j < MT; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
                    if (CONV) gload_px(cn, g * 4 + ks);
                }
            }
            if (more) sstore(cur ^ 1);
            __syncthreads();
            cur ^= 1;
        }

        double* __restrict__ out = Hpart + (int64_t)piece * d * d;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < MT; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int gr = i0 + wm * WT + i * 16 + 4 * v + (lane >> 4);
                    const int gc = j0 + wn * WT + j * 16 + (lane & 15);
                    if (gr < d && gc < d) out[(int64_t)gr * d + gc] += acc[i][j][v];
                }
    }
}

// Number of d x d slabs of partial sums = the most pieces a tile can be cut into:
// with W equal ranges over tiles * chunks items, a tile spans at most ceil(W / tiles) ranges,
// plus one when it starts inside a range.
int xxt_pick_splits(int d)
{
    const int xt = xxt_tile(d);
    const int nt = (d + xt - 1) / xt;
    const int64_t tiles = (int64_t)nt * (nt + 1) / 2;
    return (int)((xxt_wgs(xt) + tiles - 1) / tiles) + 1;
}

// length of one workgroup's range of (tile, chunk) items
static int64_t xxt_range(int d, int64_t n, int splits, int* chunks_out)
{
    const int xt = xxt_tile(d);
    const int nt = (d + xt - 1) / xt;
    const int64_t tiles = (int64_t)nt * (nt + 1) / 2;
    const int chunks = (int)((n + XK - 1) / XK);
    const int64_t total = tiles * chunks;
    // each workgroup's range must be long enough that no tile is cut into more than `splits` pieces
    int64_t per_wg = (total + xxt_wgs(xt) - 1) / xxt_wgs(xt);
    const int64_t min_per = splits > 1 ? (chunks + splits - 2) / (splits - 1) : chunks;
    if (per_wg < min_per) per_wg = min_per;
    *chunks_out = chunks;
    return per_wg;
}

// Slabs a launch over n calibration columns can write to (the rest of Hpart is not touched):
// a tile of `chunks` items meets at most ceil(chunks / range) + 1 ranges.
int xxt_slabs_touched(int d, int64_t n, int splits)
{
    int chunks;
    const int64_t per_wg = xxt_range(d, n, splits, &chunks);
    const int64_t p = (chunks + per_wg - 1) / per_wg + 1;
    return (int)(p < splits ? p : splits);
}

// Zero the part of the slabs [first, first + count) that xxt_kernel adds into and the finalize kernels read:
// the tiles on and below the diagonal, i.e. in row a the columns up to the end of its diagonal tile.
__global__ __launch_bounds__(256) void clear_slabs_kernel(double* __restrict__ Hpart, int d, int xt, int first)
{
    const int a = blockIdx.x;
    const int lim = min(d, (a / xt + 1) * xt);
    double* __restrict__ row = Hpart + ((int64_t)(first + blockIdx.y) * d + a) * d;
    for (int c = threadIdx.x; c < lim; c += 256) row[c] = 0.0;
}

hipError_t launch_clear_slabs(hipStream_t s, double* Hpart, int d, int first, int count)
{
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(clear_slabs_kernel, dim3(d, count), dim3(256), 0, s, Hpart, d, xxt_tile(d), first);
    return hipGetLastError();
}

template <int MODE>
static void xxt_launch(hipStream_t s, int xt, int wgs, const float* X, int64_t ld, int d, int64_t n, double* Hpart,
                       int chunks, int64_t per_wg, int64_t total, const ConvP& cp, LaunchEvents ev)
{
    // pieces per tile, rounded: the number of classes of ranges (see the kernel)
    int classes = (int)((chunks + per_wg / 2) / per_wg);
    classes = classes < 1 ? 1 : (classes > wgs ? wgs : classes);
    if (xt == 128)
        hipExtLaunchKernelGGL((xxt_kernel<MODE, 128>), dim3(wgs), dim3(256), 0, s, ev.start, ev.stop, 0, X, ld, d, n, Hpart,
                              chunks, per_wg, total, classes, cp);
    else
        hipExtLaunchKernelGGL((xxt_kernel<MODE, 64>), dim3(wgs), dim3(256), 0, s, ev.start, ev.stop, 0, X, ld, d, n, Hpart,
                              chunks, per_wg, total, classes, cp);
}

hipError_t launch_xxt(hipStream_t s, const float* X, int64_t ld, int d, int64_t n, double* Hpart, int splits,
                      LaunchEvents ev)
{
    const int xt = xxt_tile(d);
    const int nt = (d + xt - 1) / xt;
    const int64_t tiles = (int64_t)nt * (nt + 1) / 2;
    int chunks;
    const int64_t per_wg = xxt_range(d, n, splits, &chunks);
    const int64_t total = tiles * chunks;
    const int wgs = (int)((total + per_wg - 1) / per_wg);
    const bool fast = (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    ConvP none{};
    if (fast) xxt_launch<0>(s, xt, wgs, X, ld, d, n, Hpart, chunks, per_wg, total, none, ev);
    else      xxt_launch<1>(s, xt, wgs, X, ld, d, n, Hpart, chunks, per_wg, total, none, ev);
    return hipGetLastError();
}

// Convolution mode: padded = the copy written by launch_pad_maps ((n_img + 1) x hp x wp x c),
// d = c k^2, one calibration column per output pixel; npix = n_img * ho * wo < 2^31 - 64.
hipError_t launch_xxt_conv(hipStream_t s, const float* padded, int n_img, int hp, int wp, int c, int k, int stride,
                           int ho, int wo, int64_t npix, double* Hpart, int splits,
                           LaunchEvents ev)
{
    const int d = c * k * k;
    const int xt = xxt_tile(d);
    const int nt = (d + xt - 1) / xt;
    const int64_t tiles = (int64_t)nt * (nt + 1) / 2;
    int chunks;
    const int64_t per_wg = xxt_range(d, npix, splits, &chunks);
    const int64_t total = tiles * chunks;
    const int wgs = (int)((total + per_wg - 1) / per_wg);
    ConvP cp;
    cp.hp = hp; cp.wp = wp; cp.c = c; cp.k = k; cp.stride = stride; cp.ho = ho; cp.wo = wo;
    cp.zero_origin = (int64_t)n_img * hp * wp * c;
    cp.div_img = fastdiv_make((uint32_t)(ho * wo));
    cp.div_row = fastdiv_make((uint32_t)wo);
    cp.div_c = fastdiv_make((uint32_t)c);
    cp.div_k = fastdiv_make((uint32_t)k);
    xxt_launch<2>(s, xt, wgs, padded, 0, d, npix, Hpart, chunks, per_wg, total, cp, ev);
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

// Convolution mode: the slabs are in tap-major row order; H is written in (c, ky, kx) order.
__global__ __launch_bounds__(256) void hessian_finalize_conv_kernel(const double* __restrict__ Hpart, int splits, int d,
                                                                    double factor, double* __restrict__ H, int c,
                                                                    int kk)
{
    const int b = blockIdx.x * 16 + (threadIdx.x & 15);
    const int a = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (a >= d || b >= d || b > a) return;
    const int ai = (a % kk) * c + a / kk, bi = (b % kk) * c + b / kk;
    const int hi = max(ai, bi), lo = min(ai, bi);
    double s = 0.0;
    for (int k = 0; k < splits; ++k) s += Hpart[(int64_t)k * d * d + (int64_t)hi * d + lo];
    s *= factor;
    H[(int64_t)a * d + b] = s;
    H[(int64_t)b * d + a] = s;
}

// conv_c > 0: the slabs were accumulated in convolution mode with conv_c channels and conv_kk taps
hipError_t launch_hessian_finalize(hipStream_t s, const double* Hpart, int splits, int d, double factor, double* H,
                                   int conv_c, int conv_kk)
{
    dim3 grid((d + 15) / 16, (d + 15) / 16), block(256);
    if (conv_c > 0)
        hipLaunchKernelGGL(hessian_finalize_conv_kernel, grid, block, 0, s, Hpart, splits, d, factor, H, conv_c, conv_kk);
    else
        hipLaunchKernelGGL(hessian_finalize_kernel, grid, block, 0, s, Hpart, splits, d, factor, H);
    return hipGetLastError();
}

// Hd = H + lambda I on the tiles on and below the diagonal (all the factorization reads), with
// lambda = damp * mean(diag H) + damp_abs   (Section 6.1: damping added to the diagonal).
// Four workgroups per 64 x 64 tile.  OWN_SUM: every workgroup sums the diagonal itself, in the same order,
// so all of them add the same lambda without a launch of its own for it -- d cache lines read per
// workgroup against 4096 elements copied, which pays for small d only; otherwise workgroup-uniform
// lambda comes from lam_io, written by damp_lambda_kernel.
__device__ __forceinline__ double diag_sum(const double* __restrict__ H, int d, double* part)
{
    double s = 0.0;
    for (int a = threadIdx.x; a < d; a += 256) s += H[(int64_t)a * d + a];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    return part[0];
}

__global__ __launch_bounds__(256) void damp_lambda_kernel(const double* __restrict__ H, int d, double damp,
                                                          double damp_abs, double* __restrict__ lam)
{
    __shared__ double part[256];
    const double tr = diag_sum(H, d, part);
    if (threadIdx.x == 0) *lam = damp * (tr / (double)d) + damp_abs;
}

template <bool OWN_SUM>
__global__ __launch_bounds__(256) void damp_kernel(const double* __restrict__ H, int d, double damp, double damp_abs,
                                                   double* __restrict__ Hd, double* __restrict__ lam_io)
{
    __shared__ double part[256];
    double lam;
    if (OWN_SUM) {
        lam = damp * (diag_sum(H, d, part) / (double)d) + damp_abs;
        if (blockIdx.x == 0 && threadIdx.x == 0) *lam_io = lam;
    } else {
        lam = *lam_io;
    }
    // tile (ti, tj), ti >= tj, of index blockIdx.x = ti (ti + 1) / 2 + tj
    int ti = (int)((sqrtf(8.0f * (float)blockIdx.x + 1.0f) - 1.0f) * 0.5f);
    while ((ti + 1) * (ti + 2) / 2 <= (int)blockIdx.x) ++ti;
    while (ti * (ti + 1) / 2 > (int)blockIdx.x) --ti;
    const int tj = (int)blockIdx.x - ti * (ti + 1) / 2;
    // blockIdx.y: which 16 rows of the tile; 4 elements per thread, all loads before the stores
    double v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = (int)blockIdx.y * 1024 + threadIdx.x + 256 * i;
        const int a = min(ti * 64 + (e >> 6), d - 1), b = min(tj * 64 + (e & 63), d - 1);
        v[i] = H[(int64_t)a * d + b];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = (int)blockIdx.y * 1024 + threadIdx.x + 256 * i;
        const int a = ti * 64 + (e >> 6), b = tj * 64 + (e & 63);
        if (a < d && b < d) Hd[(int64_t)a * d + b] = (a == b) ? v[i] + lam : v[i];
    }
}

hipError_t launch_damp(hipStream_t s, const double* H, int d, double damp, double damp_abs, double* Hd, double* lam_out)
{
    const int nt = (d + 63) / 64;
    const dim3 grid((unsigned)(nt * (nt + 1) / 2), 4);
    if (d <= 512) {
        hipLaunchKernelGGL(damp_kernel<true>, grid, dim3(256), 0, s, H, d, damp, damp_abs, Hd, lam_out);
    } else {
        hipLaunchKernelGGL(damp_lambda_kernel, dim3(1), dim3(256), 0, s, H, d, damp, damp_abs, lam_out);
        hipLaunchKernelGGL(damp_kernel<false>, grid, dim3(256), 0, s, H, d, damp, damp_abs, Hd, lam_out);
    }
    return hipGetLastError();
}

}  // namespace fobq
