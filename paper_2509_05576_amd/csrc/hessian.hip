// Hessian of the layer objective (Section 3, Eq. 2): H = (2/N) X X^T.
//
// xxt_kernel: fp32 X is read from HBM, staged through LDS as fp32, widened to
// fp64 when the MFMA fragments are formed (products of two fp32 values are
// exact in fp64), and accumulated with v_mfma_f64_16x16x4_f64.  Only the 128 x 128
// tiles on or below the diagonal are computed, and of a diagonal tile only the
// 16 x 16 MFMA tiles on or below its diagonal (36 of 64).
//
// Work decomposition ("stream-K"): the work items are (tile, 32-column chunk of
// the calibration dimension) pairs in tile-major order, diagonal tiles first; a
// fixed number of persistent workgroups each take one contiguous range of items,
// all ranges equally expensive (an item of a diagonal tile is priced below one of
// another tile), so every workgroup does the same amount of work whatever d and n are.  A
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

#include <type_traits>

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

// Price of one chunk of a diagonal tile in units of 1/16 of another tile's chunk.  A 128 x 128 diagonal tile
// is 8 x 8 MFMA tiles of which the 36 on and below its diagonal are needed: 9 per wavefront (diag_mma), and one
// operand panel instead of two.  By MFMA count that is 9/16; the loads, LDS stores and barriers per chunk stay,
// and the ranges come out equally long in time at 10/16 (plain loader) and 12/16 (convolution loader: more
// address arithmetic per chunk) -- measured: with 9 the workgroups on the diagonal tiles finish last.
// A 64 x 64 tile has 4 x 4 MFMA tiles, 10 needed: no split over 4 wavefronts beats the 4 each of the full tile.
constexpr int XXT_WD_PLAIN = 10, XXT_WD_CONV = 12;
constexpr int xxt_diag_cost(int xt, bool conv) { return xt == 128 ? (conv ? XXT_WD_CONV : XXT_WD_PLAIN) : 16; }
constexpr int xxt_diag_cost_min(int xt) { return xt == 128 ? (XXT_WD_CONV < XXT_WD_PLAIN ? XXT_WD_CONV : XXT_WD_PLAIN) : 16; }

// One group of 16 calibration columns of a diagonal 128 x 128 tile for wavefront W (0..3): the MFMA tiles
// (W, 0..W) and (7 - W, 0..7 - W) of the 8 x 8 grid -- rows W and 7 - W of its lower triangle, 9 tiles for
// every W.  acc[0..W] are row W's, acc[W+1..8] row 7 - W's.  Both operands come from the one panel At.
template <int W, class F>
__device__ __forceinline__ void diag_mma(const float (*At)[XLD], int g, int fr, int fk, d4 (&acc)[9], F after_step)
{
    constexpr int RS = W, RL = 7 - W;
    float4 fb[RL + 1];
#pragma unroll
    for (int j = 0; j <= RL; ++j) fb[j] = *reinterpret_cast<const float4*>(&At[j * 16 + fr][g * 16 + fk]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        double b[RL + 1];
#pragma unroll
        for (int j = 0; j <= RL; ++j)
            b[j] = (double)(ks == 0 ? fb[j].x : ks == 1 ? fb[j].y : ks == 2 ? fb[j].z : fb[j].w);
#pragma unroll
        for (int j = 0; j <= RS; ++j) acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(b[RS], b[j], acc[j], 0, 0, 0);
#pragma unroll
        for (int j = 0; j <= RL; ++j)
            acc[RS + 1 + j] = __builtin_amdgcn_mfma_f64_16x16x4f64(b[RL], b[j], acc[RS + 1 + j], 0, 0, 0);
        after_step(ks);     // the convolution loader's share of this k-step
    }
}

// Order of the tiles.  The nt diagonal tiles come first, in order; the tiles below the diagonal follow as the
// lower triangle (with its diagonal) of an (nt - 1) x (nt - 1) grid whose row r stands for tile row r + 1, in
// this order of such a triangle: tile rows are taken in pairs (2r, 2r + 1) and a pair is walked
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
                                                     double* __restrict__ Hpart, int chunks, int64_t range_cost,
                                                     int64_t total_items, int classes, int splits, ConvP cp)
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
    // Items are laid out with the nt diagonal tiles first, then the tiles below the diagonal.  A chunk of
    // a diagonal tile costs WD units of work (36 of the 64 MFMA tiles, see diag_mma), any other 16; the
    // ranges are equally long in cost, and both ends of a range are rounded down to an item in the same way.
    constexpr int WD = xxt_diag_cost(XT, CONV);
    const int64_t diag_items = (int64_t)nt * chunks, diag_cost = diag_items * WD;
    auto item_at = [&](int64_t x) { return x < diag_cost ? x / WD : diag_items + (x - diag_cost) / 16; };
    const int64_t g0 = min(total_items, item_at((int64_t)vb * range_cost));
    const int64_t g1 = min(total_items, item_at((int64_t)(vb + 1) * range_cost));
    if (g0 >= g1) return;
    const int t_first = (int)(g0 / chunks), t_last = (int)((g1 - 1) / chunks);
    const int npieces = t_last - t_first + 1;

    for (int pi = 0; pi < npieces; ++pi) {
        const int tile = npieces == 2 ? t_last - pi : t_first + pi;
        const int64_t tile_first = (int64_t)tile * chunks;
        const int c_begin = (int)(max(g0, tile_first) - tile_first);
        const int c_end = (int)(min(g1, tile_first + chunks) - tile_first);
        const int len = c_end - c_begin;
        const bool diag = tile < nt;
        const int64_t per_wg = max((int64_t)1, range_cost / (diag ? WD : 16));   // nominal range length in this tile's chunks
        const bool load_b = !(XT == 128 && diag);     // a diagonal tile's two operand panels are one: only As is filled
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
        // 0 for the workgroup whose range reaches the tile first
        int64_t first_range = (diag ? tile_first * WD : diag_cost + (tile_first - diag_items) * 16) / range_cost;
        while (first_range < vb && item_at((first_range + 1) * range_cost) <= tile_first) ++first_range;
        const int piece = min((int)(vb - first_range), splits - 1);   // (the host sizes the ranges so that it is < splits)
        int I, J;
        if (diag) { I = tile; J = tile; }
        else { tile_decode(tile - nt, nt - 1, I, J); ++I; }
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
                if (load_b) fb[q * 8 + j] = win[offB[q]];
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
                    if (load_b) pb[u] = *reinterpret_cast<const float4*>(brow[u] + k);
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
                    if (load_b) {
                        *reinterpret_cast<float4*>(&Bs[buf][lane + 64 * q][8 * wave]) = pb[2 * q];
                        *reinterpret_cast<float4*>(&Bs[buf][lane + 64 * q][8 * wave + 4]) = pb[2 * q + 1];
                    }
                }
                return;
            }
#pragma unroll
            for (int u = 0; u < RG; ++u) {
                *reinterpret_cast<float4*>(&As[buf][lr + 32 * u][lk]) = pa[u];
                if (load_b) *reinterpret_cast<float4*>(&Bs[buf][lr + 32 * u][lk]) = pb[u];
            }
        };

        double* __restrict__ out = Hpart + (int64_t)piece * d * d;
        // The pipeline over the piece's chunks; DG: diagonal tile of XT = 128 (only the MFMA tiles on and
        // below its diagonal are formed, 9 per wavefront instead of 16).
        auto run_piece = [&](auto dg_tag) {
            constexpr bool DG = decltype(dg_tag)::value;
            d4 acc[MT][MT];
            d4 accd[DG ? 9 : 1];
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < MT; ++j) acc[i][j] = d4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int i = 0; i < (DG ? 9 : 1); ++i) accd[i] = d4{0.0, 0.0, 0.0, 0.0};

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
                    if constexpr (DG) {
                        auto after = [&](int ks) { if (CONV) gload_px(cn, g * 4 + ks); };
                        if (wave_s == 0) diag_mma<0>(As[cur], g, fr, fk, accd, after);
                        else if (wave_s == 1) diag_mma<1>(As[cur], g, fr, fk, accd, after);
                        else if (wave_s == 2) diag_mma<2>(As[cur], g, fr, fk, accd, after);
                        else diag_mma<3>(As[cur], g, fr, fk, accd, after);
                    } else {
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
                }
                if (more) sstore(cur ^ 1);
                __syncthreads();
                cur ^= 1;
            }

            if constexpr (DG) {
                // wavefront w holds the MFMA tiles (w, 0..w) and (7 - w, 0..7 - w): see diag_mma
#pragma unroll
                for (int q = 0; q < 9; ++q) {
                    const int sr = q <= wave_s ? wave_s : 7 - wave_s;
                    const int sc = q <= wave_s ? q : q - wave_s - 1;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int gr = i0 + sr * 16 + 4 * v + (lane >> 4);
                        const int gc = j0 + sc * 16 + (lane & 15);
                        if (gr < d && gc < d) out[(int64_t)gr * d + gc] += accd[q][v];
                    }
                }
            } else {
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
        };
        if constexpr (XT == 128) {
            if (diag) run_piece(std::true_type{});
            else run_piece(std::false_type{});
        } else {
            run_piece(std::false_type{});
        }
    }
}

// The split of a launch over n calibration columns: W ranges of equal cost over the items (tile, chunk),
// diagonal tiles first.  Cost units: 1/16 of a chunk of a tile below the diagonal (xxt_diag_cost for a
// diagonal tile's).
struct XxtPlan {
    int xt, nt, chunks, wgs;
    int64_t items;        // (tile, chunk) pairs
    int64_t range_cost;   // cost of one workgroup's range
};

static int64_t xxt_cost_per_chunk_column(int xt, int nt, int wd)     // cost of one chunk of every tile
{
    return (int64_t)wd * nt + 16 * ((int64_t)nt * (nt - 1) / 2);
}

// Number of d x d slabs of partial sums = the most pieces a tile can be cut into: a tile below the
// diagonal (the most expensive kind) spans at most ceil(its cost / range cost) ranges, plus one when it
// starts inside a range; the range cost is at least the total cost / W.
int xxt_pick_splits(int d)
{
    const int xt = xxt_tile(d);
    const int nt = (d + xt - 1) / xt;
    const int64_t per_column = xxt_cost_per_chunk_column(xt, nt, xxt_diag_cost_min(xt));   // either mode fits
    return (int)((16 * (int64_t)xxt_wgs(xt) + per_column - 1) / per_column) + 1;
}

static XxtPlan xxt_plan(int d, int64_t n, int splits, bool conv)
{
    XxtPlan p;
    p.xt = xxt_tile(d);
    p.nt = (d + p.xt - 1) / p.xt;
    p.chunks = (int)((n + XK - 1) / XK);
    p.items = ((int64_t)p.nt * (p.nt + 1) / 2) * p.chunks;
    const int64_t total_cost = xxt_cost_per_chunk_column(p.xt, p.nt, xxt_diag_cost(p.xt, conv)) * p.chunks;
    p.range_cost = (total_cost + xxt_wgs(p.xt) - 1) / xxt_wgs(p.xt);
    // a range must cost enough that no tile is cut into more than `splits` pieces
    const int64_t tile_cost = 16 * (int64_t)p.chunks;
    const int64_t min_cost = splits > 1 ? (tile_cost + splits - 2) / (splits - 1) : tile_cost;
    if (p.range_cost < min_cost) p.range_cost = min_cost;
    if (p.range_cost < 16) p.range_cost = 16;      // at least one whole chunk per range
    p.wgs = (int)((total_cost + p.range_cost - 1) / p.range_cost);
    return p;
}

// Slabs a launch over n calibration columns can write to (the rest of Hpart is not touched):
// a tile meets at most ceil(its cost / range cost) + 1 ranges.
int xxt_slabs_touched(int d, int64_t n, int splits, bool conv)
{
    const XxtPlan pl = xxt_plan(d, n, splits, conv);
    const int64_t p = (16 * (int64_t)pl.chunks + pl.range_cost - 1) / pl.range_cost + 1;
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
static void xxt_launch(hipStream_t s, const XxtPlan& pl, const float* X, int64_t ld, int d, int64_t n, double* Hpart,
                       int splits, const ConvP& cp, LaunchEvents ev)
{
    // pieces per tile (below the diagonal), rounded: the number of classes of ranges (see the kernel)
    const int64_t tile_cost = 16 * (int64_t)pl.chunks;
    int classes = (int)((tile_cost + pl.range_cost / 2) / pl.range_cost);
    classes = classes < 1 ? 1 : (classes > pl.wgs ? pl.wgs : classes);
    if (pl.xt == 128)
        hipExtLaunchKernelGGL((xxt_kernel<MODE, 128>), dim3(pl.wgs), dim3(256), 0, s, ev.start, ev.stop, 0, X, ld, d, n,
                              Hpart, pl.chunks, pl.range_cost, pl.items, classes, splits, cp);
    else
        hipExtLaunchKernelGGL((xxt_kernel<MODE, 64>), dim3(pl.wgs), dim3(256), 0, s, ev.start, ev.stop, 0, X, ld, d, n,
                              Hpart, pl.chunks, pl.range_cost, pl.items, classes, splits, cp);
}

hipError_t launch_xxt(hipStream_t s, const float* X, int64_t ld, int d, int64_t n, double* Hpart, int splits,
                      LaunchEvents ev)
{
    const XxtPlan pl = xxt_plan(d, n, splits, false);
    const bool fast = (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    ConvP none{};
    if (fast) xxt_launch<0>(s, pl, X, ld, d, n, Hpart, splits, none, ev);
    else      xxt_launch<1>(s, pl, X, ld, d, n, Hpart, splits, none, ev);
    return hipGetLastError();
}

// Convolution mode: padded = the copy written by launch_pad_maps ((n_img + 1) x hp x wp x c),
// d = c k^2, one calibration column per output pixel; npix = n_img * ho * wo < 2^31 - 64.
hipError_t launch_xxt_conv(hipStream_t s, const float* padded, int n_img, int hp, int wp, int c, int k, int stride,
                           int ho, int wo, int64_t npix, double* Hpart, int splits,
                           LaunchEvents ev)
{
    const int d = c * k * k;
    const XxtPlan pl = xxt_plan(d, npix, splits, true);
    ConvP cp;
    cp.hp = hp; cp.wp = wp; cp.c = c; cp.k = k; cp.stride = stride; cp.ho = ho; cp.wo = wo;
    cp.zero_origin = (int64_t)n_img * hp * wp * c;
    cp.div_img = fastdiv_make((uint32_t)(ho * wo));
    cp.div_row = fastdiv_make((uint32_t)wo);
    cp.div_c = fastdiv_make((uint32_t)c);
    cp.div_k = fastdiv_make((uint32_t)k);
    xxt_launch<2>(s, pl, padded, 0, d, npix, Hpart, splits, cp, ev);
    return hipGetLastError();
}

// H[a][b] = H[b][a] = factor * sum_s Hpart[s][a][b]   for b <= a (lower slabs hold the sums)
// poison (may be null): a word that is non-zero when an input of the integer-slice path held an Inf or NaN;
// H then becomes NaN throughout, as the floating-point sum would have made the rows concerned.
__global__ __launch_bounds__(256) void hessian_finalize_kernel(const double* __restrict__ Hpart, int splits, int sstride, int d,
                                                               double factor, double* __restrict__ H,
                                                               const int* __restrict__ poison)
{
    const int b = blockIdx.x * 16 + (threadIdx.x & 15);
    const int a = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (a >= d || b >= d || b > a) return;
    double s = 0.0;
    for (int k = 0; k < splits; ++k) s += Hpart[(int64_t)k * sstride * d * d + (int64_t)a * d + b];
    s *= factor;
    if (poison && *poison) s = __builtin_nan("");
    H[(int64_t)a * d + b] = s;
    H[(int64_t)b * d + a] = s;
}

// Convolution mode: the slabs are in tap-major row order; H is written in (c, ky, kx) order.
__global__ __launch_bounds__(256) void hessian_finalize_conv_kernel(const double* __restrict__ Hpart, int splits, int sstride, int d,
                                                                    double factor, double* __restrict__ H, int c,
                                                                    int kk, const int* __restrict__ poison)
{
    const int b = blockIdx.x * 16 + (threadIdx.x & 15);
    const int a = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (a >= d || b >= d || b > a) return;
    const int ai = (a % kk) * c + a / kk, bi = (b % kk) * c + b / kk;
    const int hi = max(ai, bi), lo = min(ai, bi);
    double s = 0.0;
    for (int k = 0; k < splits; ++k) s += Hpart[(int64_t)k * sstride * d * d + (int64_t)hi * d + lo];
    s *= factor;
    if (poison && *poison) s = __builtin_nan("");
    H[(int64_t)a * d + b] = s;
    H[(int64_t)b * d + a] = s;
}

// conv_c > 0: the slabs were accumulated in convolution mode with conv_c channels and conv_kk taps
// Small d, many slabs (a tile of a 64-column layer is cut into up to 1024 pieces): the lower triangles of groups of
// SLAB_GROUP consecutive slabs are first added into the first slab of each group, one workgroup per (16 x 16 entries,
// group), so that the finalize kernel -- one thread per entry, the slabs one after the other -- has SLAB_GROUP times
// fewer to walk through.  The order of the sum is fixed either way.
constexpr int SLAB_GROUP = 32;
__global__ __launch_bounds__(256) void hessian_group_slabs_kernel(double* __restrict__ Hpart, int splits, int d)
{
    const int b = blockIdx.x * 16 + (threadIdx.x & 15);
    const int a = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (a >= d || b >= d || b > a) return;
    const int k0 = blockIdx.z * SLAB_GROUP, k1 = min(splits, k0 + SLAB_GROUP);
    const int64_t at = (int64_t)a * d + b;
    double s = 0.0;
    for (int k = k0; k < k1; ++k) s += Hpart[(int64_t)k * d * d + at];
    Hpart[(int64_t)k0 * d * d + at] = s;
}

hipError_t launch_hessian_finalize(hipStream_t s, double* Hpart, int splits, int d, double factor, double* H,
                                   int conv_c, int conv_kk, const int* poison)
{
    dim3 grid((d + 15) / 16, (d + 15) / 16), block(256);
    int sstride = 1;
    if (splits > 2 * SLAB_GROUP) {
        const int groups = (splits + SLAB_GROUP - 1) / SLAB_GROUP;
        hipLaunchKernelGGL(hessian_group_slabs_kernel, dim3(grid.x, grid.y, groups), block, 0, s, Hpart, splits, d);
        splits = groups;
        sstride = SLAB_GROUP;
    }
    if (conv_c > 0)
        hipLaunchKernelGGL(hessian_finalize_conv_kernel, grid, block, 0, s, Hpart, splits, sstride, d, factor, H, conv_c, conv_kk,
                           poison);
    else
        hipLaunchKernelGGL(hessian_finalize_kernel, grid, block, 0, s, Hpart, splits, sstride, d, factor, H, poison);
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
