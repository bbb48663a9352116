// What the int8 matrix cores sustain: the inner loop of the X X^T digit-product kernel (19 products per k-step
// on v_mfma_i32_32x32x32_i8, two A fragments per digit read from LDS, the B digits in registers, 8 wavefronts per
// compute unit, 12 accumulator tiles each) with its operands fixed in LDS -- no global traffic, no barrier.  The
// rate of this loop depends on the operand BYTES (all equal: near the nominal peak; random: about two thirds of
// it, the chip holds its power by slowing the matrix pipes), so it is the yardstick that tells whether the real
// kernel loses time to its memory system and synchronisation or is held by the pipes themselves.
#include <hip/hip_ext.h>

#include <cmath>
#include <vector>

#include "fobq_internal.h"

namespace fobq {

typedef int pi32x4 __attribute__((ext_vector_type(4)));
typedef int pi32x16 __attribute__((ext_vector_type(16)));

constexpr int PROBE_NS = 5, PROBE_NM = 6;
constexpr int PROBE_BLOCKS = 3 * PROBE_NS;      // A row block 0, A row block 1, B: 5 digit blocks of 1 KiB each

__global__ __launch_bounds__(512) void probe_i8_kernel(const signed char* __restrict__ blocks, int ksteps, int* __restrict__ out)
{
    __shared__ __attribute__((aligned(16))) signed char L[PROBE_BLOCKS][1024];
    for (int i = threadIdx.x; i < PROBE_BLOCKS * 1024 / 16; i += 512)
        reinterpret_cast<pi32x4*>(&L[0][0])[i] = reinterpret_cast<const pi32x4*>(blocks)[i];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    pi32x16 acc[PROBE_NM][2];
#pragma unroll
    for (int m = 0; m < PROBE_NM; ++m)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[m][i][v] = 0;
    pi32x4 fb[PROBE_NS];
#pragma unroll
    for (int t = 0; t < PROBE_NS; ++t) fb[t] = *reinterpret_cast<const pi32x4*>(&L[2 * PROBE_NS + t][lane * 16]);
    for (int q = 0; q < ksteps; ++q) {
#pragma unroll
        for (int s = 0; s < PROBE_NS; ++s) {
            pi32x4 fa[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const pi32x4*>(&L[i * PROBE_NS + s][lane * 16]);
#pragma unroll
            for (int t = 0; t < PROBE_NS; ++t) {
                if (s + t < PROBE_NM) {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        acc[s + t][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[t], acc[s + t][i], 0, 0, 0);
                }
            }
        }
        // keeps the compiler from hoisting the LDS reads out of the loop
        __asm__ volatile("" ::: "memory");
    }
    int sum = 0;
#pragma unroll
    for (int m = 0; m < PROBE_NM; ++m)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[m][i][v];
    out[(int64_t)blockIdx.x * 512 + threadIdx.x] = sum;
}

// 64-bit mix (SplitMix64 finalizer) of a counter: the probe's own operand bytes, nothing of the method
static uint64_t probe_mix(uint64_t z)
{
    z += 0x9e3779b97f4a7c15ull;
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

// operand blocks in MFMA lane order: block (operand o, digit s), slot l = row + 32 (col / 16), byte col % 16
static void probe_operands(int kind, std::vector<signed char>& bytes)
{
    bytes.assign((size_t)PROBE_BLOCKS * 1024, 1);
    if (kind == FOBQ_PROBE_EQUAL_BYTES) return;
    uint64_t ctr = 0;
    for (int o = 0; o < 3; ++o)
        for (int r = 0; r < 32; ++r)
            for (int c = 0; c < 32; ++c) {
                int64_t y;
                if (kind == FOBQ_PROBE_RANDOM_BYTES) {
                    y = (int64_t)(probe_mix(ctr++) >> 24);          // 40 random bits: every digit uniform
                } else {
                    // ReLU of a standard normal, in fixed point with 35 fraction bits (largest value below 8)
                    const double u1 = ((double)(probe_mix(ctr++) >> 11) + 1.0) * 0x1p-53;
                    const double u2 = (double)(probe_mix(ctr++) >> 11) * 0x1p-53;
                    const double g = std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586 * u2);
                    y = g > 0.0 ? (int64_t)std::llrint(std::fmin(g, 7.9) * 0x1p35) : 0;
                }
                // balanced base-256 digits: the bytes of y + 0x8080808080, each less 128
                const uint64_t biased = (uint64_t)y + 0x8080808080ull;
                for (int s = 0; s < PROBE_NS; ++s)
                    bytes[((size_t)(o * PROBE_NS + s) * 64 + r + 32 * (c / 16)) * 16 + c % 16] =
                        (signed char)((int)((biased >> (8 * s)) & 0xff) - 128);
            }
}

}  // namespace fobq

using namespace fobq;

extern "C" int fobq_probe_int8_matrix_rate(fobq_ctx* ctx, int operand_kind, double* tera_ops_per_second)
{
    if (!ctx || !tera_ops_per_second) return FOBQ_EINVAL;
    if (operand_kind < FOBQ_PROBE_EQUAL_BYTES || operand_kind > FOBQ_PROBE_RELU_DIGITS)
        return set_err(ctx, FOBQ_EINVAL, "unknown operand kind %d", operand_kind);
    int prev = -1;
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    if (prev != ctx->device && hipSetDevice(ctx->device) != hipSuccess) return set_err(ctx, FOBQ_EHIP, "cannot select the device");
    int cus = 0;
    hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device);
    signed char* blocks = nullptr;
    int* out = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    float ms = 0.0f;
    const int ksteps = 4000;
    std::vector<signed char> host;
    probe_operands(operand_kind, host);
    if (e == hipSuccess) e = hipMalloc((void**)&blocks, host.size());
    if (e == hipSuccess) e = hipMalloc((void**)&out, (size_t)cus * 512 * sizeof(int));
    if (e == hipSuccess) e = hipMemcpy(blocks, host.data(), host.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipEventCreate(&ev0);
    if (e == hipSuccess) e = hipEventCreate(&ev1);
    if (e == hipSuccess) {
        // one short launch first (clocks, code load), then the timed one, its own start and stop events
        hipLaunchKernelGGL(probe_i8_kernel, dim3(cus), dim3(512), 0, ctx->stream, blocks, 200, out);
        hipExtLaunchKernelGGL(probe_i8_kernel, dim3(cus), dim3(512), 0, ctx->stream, ev0, ev1, 0, blocks, ksteps, out);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventSynchronize(ev1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev0, ev1);
    if (ev0) (void)hipEventDestroy(ev0);
    if (ev1) (void)hipEventDestroy(ev1);
    if (blocks) (void)hipFree(blocks);
    if (out) (void)hipFree(out);
    if (prev >= 0 && prev != ctx->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) return hip_err(ctx, e, "int8 matrix rate probe");
    // 38 MFMAs of 32 x 32 x 32 multiply-adds per wavefront and k-step, 8 wavefronts per workgroup
    const double ops = (double)cus * 8.0 * (double)ksteps * 38.0 * 65536.0;
    *tera_ops_per_second = ops / ((double)ms * 1e-3) / 1e12;
    return FOBQ_OK;
}
