// Measurement helpers (no part of the method): the rates this chip reaches on the two resources
// that bound the kernels of this library, measured with the same access pattern / instruction the
// kernels use, so that their results can be stated against a measured ceiling as well as against
// the published one.
//   stream read : every byte of a buffer read once with 16-byte non-temporal loads, 1 KiB
//                 contiguous per wavefront instruction (the pattern of the filter pass);
//   fp32 MFMA   : back-to-back independent V_MFMA_F32_16X16X4_F32 (the instruction of the Gram
//                 kernels) on all SIMDs, operands in registers.
#include "../../include/detox.h"
#include "rows.h"

namespace detox {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kBlock) void probe_stream_read_kernel(const u32x4_t *p, int64_t vecs,
                                                                   uint32_t *sink)
{
    // a workgroup takes runs of four neighbouring 4 KiB pieces, its four loads in flight together
    u32x4_t acc = {0u, 0u, 0u, 0u};
    const int64_t stride = (int64_t)gridDim.x * kBlock * 4;
    int64_t i = (int64_t)blockIdx.x * kBlock * 4 + threadIdx.x;
    for (; i + 3 * kBlock < vecs; i += stride) {
        const u32x4_t a = __builtin_nontemporal_load(p + i);
        const u32x4_t b = __builtin_nontemporal_load(p + i + kBlock);
        const u32x4_t c = __builtin_nontemporal_load(p + i + 2 * kBlock);
        const u32x4_t e = __builtin_nontemporal_load(p + i + 3 * kBlock);
        acc ^= a ^ b ^ c ^ e;
    }
    for (int u = 0; u < 4; ++u)   // the ragged end of the buffer
        if (i + u * kBlock < vecs && i < vecs) acc ^= __builtin_nontemporal_load(p + i + u * kBlock);
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9e3779b9u) sink[0] = x;   // keeps the loads alive; practically never taken
}

__global__ __launch_bounds__(kBlock) void probe_mfma_f32_kernel(int iters, float seed, float *sink)
{
    constexpr int kChains = 8;   // independent accumulators: no instruction waits for another
    f32x4 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) acc[c] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    const float a = seed + (float)(threadIdx.x & 15) * 1.0e-3f, b = seed - (float)(threadIdx.x >> 4) * 1.0e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < kChains; ++c)
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kChains; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
    if (s == 12345.678f) sink[0] = s;
}

}  // namespace
}  // namespace detox

using namespace detox;

extern "C" {

int detox_probe_stream_read(const void *buf, size_t bytes, void *sink, void *stream)
{
    if (buf == nullptr || sink == nullptr || bytes < 16 || reinterpret_cast<uintptr_t>(buf) % 16 != 0)
        return DETOX_EINVAL;
    const int64_t vecs = (int64_t)(bytes / 16);
    int64_t grid = (int64_t)num_compute_units() * 32;
    const int64_t need = (vecs + 4 * kBlock - 1) / (4 * kBlock);
    if (grid > need) grid = need;
    probe_stream_read_kernel<<<(unsigned)grid, kBlock, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const u32x4_t *>(buf), vecs, static_cast<uint32_t *>(sink));
    return hipGetLastError() == hipSuccess ? DETOX_OK : DETOX_EDEVICE;
}

int detox_probe_mfma_f32(int iters, void *sink, double *flop, void *stream)
{
    if (sink == nullptr || iters < 1) return DETOX_EINVAL;
    const int grid = num_compute_units() * 2;   // two wavefronts per SIMD
    probe_mfma_f32_kernel<<<grid, kBlock, 0, static_cast<hipStream_t>(stream)>>>(iters, 1.0f,
                                                                                 static_cast<float *>(sink));
    // 16 x 16 x 4 multiply-adds per instruction, 32 instructions per iteration and wavefront
    if (flop) *flop = 2.0 * 16 * 16 * 4 * 32.0 * iters * (double)grid * (kBlock / kWave);
    return hipGetLastError() == hipSuccess ? DETOX_OK : DETOX_EDEVICE;
}

}  // extern "C"
