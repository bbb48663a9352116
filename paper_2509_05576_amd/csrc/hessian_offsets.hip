// Hessian of a stride-1 k x k convolution from its input maps by tap offsets (Section 3, Eq. 2: H = 2 X X^T / N
// with X the unfolded input).  With M the zero-padded maps, a = (a_y, a_x) and b two taps and W_a the window of
// padded positions that tap a visits (rows a_y .. a_y + ho - 1, columns a_x .. a_x + wo - 1),
//     H[(a, c), (b, c')] = sum over images and q in W_a of  M[q, c] * M[q + (b - a), c'],
// i.e. a block depends on its taps through the offset b - a and the window only.  Every offset occurs in one of two
// block rows, those of the taps (0, 0) and (0, k - 1); they are formed exactly by the digit-product kernel (a list
// of tile rows instead of the lower triangle).  Any other block is one of those plus and minus the same summand over
// the rows and columns by which the two windows differ: a few correlations over single rows or columns of the
// padded maps per pair of taps ("strips"), formed here in fp64 and added into a correction matrix per accumulate
// call; the finalize kernel puts blocks and corrections together.
#include <hip/hip_ext.h>

#include <map>
#include <tuple>

#include "fobq_internal.h"

namespace fobq {

typedef double od4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Host: the strips and the signed terms of every pair of taps for one geometry (stride 1).
//   pair (a, b) in canonical orientation (the offset b - a points down, or right within a row); base tap
//   a0 = (0, 0) for offsets pointing right or straight down, (0, k - 1) for offsets pointing left; b0 = a0 + offset.
//   sum over W_a minus sum over W_a0: first move the window down by a_y (rows ho .. ho + a_y - 1 enter, rows
//   0 .. a_y - 1 leave, columns of W_a), then sideways from a0_x to a_x (columns enter and leave, rows 0 .. ho - 1).
// A strip whose row or column lies in the zero border -- or whose partner row or column does -- is dropped.
// Returns false when the tables do not hold the geometry (the caller then takes the general path).
bool offset_tables_build(int k, int pad, int h, int w, OffsetTables* tab)
{
    const int hp = h + 2 * pad, wp = w + 2 * pad, ho = hp - k + 1, wo = wp - k + 1;
    if (k < 2 || k * k > OFFSET_MAX_TAPS || ho < 1 || wo < 1) return false;
    std::map<std::tuple<int, int, int, int, int, int>, int> ids;
    tab->njobs = 0;
    tab->npairs = 0;
    tab->nterms = 0;
    auto zero_row = [&](int y) { return y < pad || y >= pad + h; };
    auto zero_col = [&](int x) { return x < pad || x >= pad + w; };
    bool ok = true;
    auto add_term = [&](int kind, int coord, int start, int len, int dy, int dx, int sign) {
        if (len <= 0) return;
        if (kind == 0 ? (zero_row(coord) || zero_row(coord + dy)) : (zero_col(coord) || zero_col(coord + dx))) return;
        const auto key = std::make_tuple(kind, coord, start, len, dy, dx);
        auto it = ids.find(key);
        int id;
        if (it == ids.end()) {
            if (tab->njobs >= OFFSET_MAX_JOBS) { ok = false; return; }
            id = tab->njobs++;
            ids[key] = id;
            tab->jobs[id] = OffsetJob{coord, start, len, (signed char)kind, (signed char)dy, (signed char)dx, 0};
        } else {
            id = it->second;
        }
        if (tab->nterms >= OFFSET_MAX_TERMS) { ok = false; return; }
        tab->term_job[tab->nterms] = (unsigned char)id;
        tab->term_sign[tab->nterms] = (signed char)sign;
        ++tab->nterms;
    };
    for (int ta = 0; ta < k * k; ++ta)
        for (int tb = 0; tb < k * k; ++tb) {
            const int ay = ta / k, ax = ta % k, by = tb / k, bx = tb % k;
            const int dy = by - ay, dx = bx - ax;
            if (!(dy > 0 || (dy == 0 && dx >= 0))) continue;         // the other orientation is the transpose
            const int a0x = dx >= 0 ? 0 : k - 1;
            if (ay == 0 && ax == a0x) continue;                      // a base block: nothing to correct
            const int p = tab->npairs++;
            tab->pair_ta[p] = (unsigned char)ta;
            tab->pair_tb[p] = (unsigned char)tb;
            tab->pair_begin[p] = (short)tab->nterms;
            for (int y = ho; y < ho + ay; ++y) add_term(0, y, ax, wo, dy, dx, +1);
            for (int y = 0; y < ay; ++y) add_term(0, y, ax, wo, dy, dx, -1);
            if (ax > a0x) {
                for (int x = a0x + wo; x < ax + wo; ++x) add_term(1, x, 0, ho, dy, dx, +1);
                for (int x = a0x; x < ax; ++x) add_term(1, x, 0, ho, dy, dx, -1);
            } else {
                for (int x = ax; x < a0x; ++x) add_term(1, x, 0, ho, dy, dx, +1);
                for (int x = ax + wo; x < a0x + wo; ++x) add_term(1, x, 0, ho, dy, dx, -1);
            }
        }
    tab->pair_begin[tab->npairs] = (short)tab->nterms;
    return ok;
}

// ---------------------------------------------------------------------------
// strips[half][job][c][c'] = sum over images and the job's positions q of M[q, c] * M[q + (dy, dx), c']  (fp64 MFMA on
// exactly widened fp32 inputs), the positions cut into `parts` contiguous parts whose sums are added later in a
// fixed order (offset_parts: enough of them that a layer with few channels still fills the chip).  One workgroup of 8 wavefronts (16 x 32 of the tile each: two per SIMD, as the fp64 matrix pipe
// wants) per (64 x 64 tile of channels, job, part); positions in chunks of 32 (a position is 64 contiguous floats per
// operand), the loads of a chunk in flight while the chunk before is multiplied.
constexpr int OFFSET_MIN_PARTS = 2, OFFSET_MAX_PARTS = 16;

static int offset_parts(int njobs, int c)
{
    const int tiles = (c / 64) * (c / 64) * (njobs > 0 ? njobs : 1);
    const int want = (512 + tiles - 1) / tiles;              // about two workgroups per compute unit
    return want < OFFSET_MIN_PARTS ? OFFSET_MIN_PARTS : (want > OFFSET_MAX_PARTS ? OFFSET_MAX_PARTS : want);
}

__global__ __launch_bounds__(512) void offset_strip_kernel(const float* __restrict__ padded, int n_img, int hp, int wp, int c,
                                                           OffsetTables tab, int parts, double* __restrict__ strips)
{
    constexpr int PC = 32, LDW = 64 + 16;      // row stride 80 doubles: conflict-free 8-byte fragment reads per half-wave
    __shared__ double As[PC][LDW];
    __shared__ double Bs[PC][LDW];
    const int jid = blockIdx.z / parts, part = blockIdx.z % parts;
    const OffsetJob job = tab.jobs[jid];
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wi = wave >> 1, wj = wave & 1;                 // rows 16 wi .., columns 32 wj ..
    const int64_t npos = (int64_t)n_img * job.len;
    const int64_t per = ((npos + parts - 1) / parts + PC - 1) / PC * PC;
    const int64_t p_lo = part * per, p_hi = min(npos, p_lo + per);
    od4 acc[2];
    acc[0] = od4{0.0, 0.0, 0.0, 0.0};
    acc[1] = od4{0.0, 0.0, 0.0, 0.0};
    const int lp = tid >> 4, lc = (tid & 15) * 4;            // this thread's position in the chunk, its 4 channels
    float4 va, vb;
    auto gload = [&](int64_t p0) {
        const int64_t p = p0 + lp;
        va = make_float4(0.f, 0.f, 0.f, 0.f);
        vb = va;
        if (p < p_hi) {
            const int img = (int)(p / job.len), t = (int)(p - (int64_t)img * job.len);
            const int qy = job.kind == 0 ? job.coord : job.start + t;
            const int qx = job.kind == 0 ? job.start + t : job.coord;
            const int64_t oa = (((int64_t)img * hp + qy) * wp + qx) * c;
            const int64_t ob = (((int64_t)img * hp + qy + job.dy) * wp + qx + job.dx) * c;
            va = *reinterpret_cast<const float4*>(padded + oa + i0 + lc);
            vb = *reinterpret_cast<const float4*>(padded + ob + j0 + lc);
        }
    };
    if (p_lo < p_hi) gload(p_lo);
    for (int64_t p0 = p_lo; p0 < p_hi; p0 += PC) {
        __syncthreads();                                      // the chunk before is consumed
        As[lp][lc + 0] = (double)va.x; As[lp][lc + 1] = (double)va.y; As[lp][lc + 2] = (double)va.z; As[lp][lc + 3] = (double)va.w;
        Bs[lp][lc + 0] = (double)vb.x; Bs[lp][lc + 1] = (double)vb.y; Bs[lp][lc + 2] = (double)vb.z; Bs[lp][lc + 3] = (double)vb.w;
        __syncthreads();
        if (p0 + PC < p_hi) gload(p0 + PC);
#pragma unroll
        for (int ks = 0; ks < PC / 4; ++ks) {
            const double a = As[ks * 4 + (lane >> 4)][wi * 16 + (lane & 15)];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, Bs[ks * 4 + (lane >> 4)][wj * 32 + j * 16 + (lane & 15)], acc[j], 0, 0, 0);
        }
    }
    double* __restrict__ out = strips + ((int64_t)part * tab.njobs + jid) * c * c;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gi = i0 + wi * 16 + 4 * v + (lane >> 4), gj = j0 + wj * 32 + j * 16 + (lane & 15);
            out[(int64_t)gi * c + gj] = acc[j][v];
        }
}

// corr[(ta c + ch), (tb c + ch')] += sum over the pair's terms of sign * strips[job][ch][ch'], tap-major d x d
__global__ __launch_bounds__(256) void offset_apply_kernel(OffsetTables tab, const double* __restrict__ strips, int parts, int c,
                                                           int d, double* __restrict__ corr)
{
    const int p = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= c * c) return;
    const int t0 = tab.pair_begin[p], t1 = tab.pair_begin[p + 1];
    if (t0 == t1) return;
    double s = 0.0;
    for (int t = t0; t < t1; ++t) {
        double v = 0.0;
        for (int part = 0; part < parts; ++part) v += strips[((int64_t)part * tab.njobs + tab.term_job[t]) * c * c + e];
        s += (double)tab.term_sign[t] * v;
    }
    const int ch = e / c, ch2 = e - ch * c;
    corr[(int64_t)((int)tab.pair_ta[p] * c + ch) * d + (int)tab.pair_tb[p] * c + ch2] += s;
}

// H in (c, ky, kx) order from the base blocks (slabs, tap-major rows of the taps (0, 0) and (0, k - 1)) and the
// corrections.  Every entry is taken in its canonical orientation (offset pointing down, or right within a row;
// for the zero offset the lower triangle of the block), so H comes out exactly symmetric.
__global__ __launch_bounds__(256) void hessian_finalize_offsets_kernel(const double* __restrict__ Hpart, int splits, int d,
                                                                       double factor, double* __restrict__ H, int c, int k,
                                                                       const double* __restrict__ corr,
                                                                       const int* __restrict__ poison)
{
    const int col = blockIdx.x * 16 + (threadIdx.x & 15);
    const int row = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (row >= d || col >= d || col > row) return;
    const int kk = k * k;
    int ta = row % kk, ch = row / kk, tb = col % kk, ch2 = col / kk;       // H's order: index = channel * k^2 + tap
    int dy = tb / k - ta / k, dx = tb % k - ta % k;
    const bool canonical = dy > 0 || (dy == 0 && dx > 0) || (dy == 0 && dx == 0 && ch2 <= ch);
    if (!canonical) {
        int t = ta; ta = tb; tb = t;
        t = ch; ch = ch2; ch2 = t;
        dy = -dy; dx = -dx;
    }
    const int a0x = dx >= 0 ? 0 : k - 1;
    const int t0 = a0x, t1 = dy * k + a0x + dx;                             // the base taps a0 = (0, a0x), b0 = a0 + offset
    const int64_t at = (int64_t)(t0 * c + ch) * d + t1 * c + ch2;
    double s = 0.0;
    for (int q = 0; q < splits; ++q) s += Hpart[(int64_t)q * d * d + at];
    if (!(ta / k == 0 && ta % k == a0x)) s += corr[(int64_t)(ta * c + ch) * d + tb * c + ch2];
    s *= factor;
    if (poison && *poison) s = __builtin_nan("");
    H[(int64_t)row * d + col] = s;
    H[(int64_t)col * d + row] = s;
}

// full rows [row0, row0 + n0) and [row1, row1 + n1) of `count` slabs from slab `first` on
__global__ __launch_bounds__(256) void clear_slab_rows_kernel(double* __restrict__ Hpart, int d, int first, int row0, int n0,
                                                              int row1)
{
    const int r = (int)blockIdx.x < n0 ? row0 + (int)blockIdx.x : row1 + (int)blockIdx.x - n0;
    double* __restrict__ row = Hpart + ((int64_t)(first + blockIdx.y) * d + r) * d;
    for (int x = threadIdx.x; x < d; x += 256) row[x] = 0.0;
}

hipError_t launch_clear_slab_rows(hipStream_t s, double* Hpart, int d, int first, int count, int row0, int n0, int row1, int n1)
{
    if (count <= 0 || n0 + n1 <= 0) return hipSuccess;
    hipLaunchKernelGGL(clear_slab_rows_kernel, dim3(n0 + n1, count), dim3(256), 0, s, Hpart, d, first, row0, n0, row1);
    return hipGetLastError();
}

// the strips of one call (overwritten; offset_strips_bytes of scratch), then their signed sums into the correction matrix
size_t offset_strips_bytes(int njobs, int c) { return (size_t)offset_parts(njobs, c) * (njobs > 0 ? njobs : 1) * c * c * sizeof(double); }

hipError_t launch_offset_corrections(hipStream_t s, const float* padded, int n_img, int hp, int wp, int c, int d,
                                     const OffsetTables& tab, double* strips, double* corr)
{
    if (tab.njobs == 0) return hipSuccess;
    const int parts = offset_parts(tab.njobs, c);
    hipLaunchKernelGGL(offset_strip_kernel, dim3(c / 64, c / 64, tab.njobs * parts), dim3(512), 0, s, padded, n_img, hp, wp, c,
                       tab, parts, strips);
    hipLaunchKernelGGL(offset_apply_kernel, dim3((c * c + 255) / 256, tab.npairs), dim3(256), 0, s, tab, strips, parts, c, d, corr);
    return hipGetLastError();
}

hipError_t launch_hessian_finalize_offsets(hipStream_t s, const double* Hpart, int splits, int d, double factor, double* H, int c,
                                           int k, const double* corr, const int* poison)
{
    hipLaunchKernelGGL(hessian_finalize_offsets_kernel, dim3((d + 15) / 16, (d + 15) / 16), dim3(256), 0, s, Hpart, splits, d,
                       factor, H, c, k, corr, poison);
    return hipGetLastError();
}

}  // namespace fobq
