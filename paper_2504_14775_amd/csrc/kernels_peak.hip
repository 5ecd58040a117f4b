// Ceiling probes: what this GPU sustains on a bare MFMA loop and on a bare streaming read.  They give
// the benchmark a measured reference next to the published peaks (clocks drop under matrix-core load).
#include "common.h"

namespace {

// Every wave issues `iters` rounds of 16 independent 32x32x16 bf16 MFMAs (no memory traffic in the loop).
// Operands come from `sink` (whatever bits the caller put there: random data draws more power than
// constants) and alternate between two sets so that the operand buses toggle as in a real GEMM.
__global__ __launch_bounds__(256) void peak_mfma_kernel(float* __restrict__ sink, int iters) {
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const u32x4* data = reinterpret_cast<const u32x4*>(sink) + (threadIdx.x & 63) * 4;
    bf16x8 a0 = __builtin_bit_cast(bf16x8, data[0]), b0 = __builtin_bit_cast(bf16x8, data[1]);
    bf16x8 a1 = __builtin_bit_cast(bf16x8, data[2]), b1 = __builtin_bit_cast(bf16x8, data[3]);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[i], 0, 0, 0);
            acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[i + 1], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0];
    if (s == 12345.678f) sink[0] = s;  // keeps the loop alive
}

// Grid-stride read of `count16` 16-byte words; one partial sum per thread is kept live.  NT: with the non-temporal hint.
template <bool NT>
__global__ __launch_bounds__(256) void peak_read_kernel(const u32x4* __restrict__ src, int64_t count16,
                                                         uint32_t* __restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    uint32_t s = 0;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    auto ld = [&](int64_t j) { return NT ? __builtin_nontemporal_load(src + j) : src[j]; };
    for (; i + 3 * stride < count16; i += 4 * stride) {
        u32x4 a = ld(i), b = ld(i + stride), c = ld(i + 2 * stride), d = ld(i + 3 * stride);
        s += a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3] ^ c[0] ^ c[1] ^ c[2] ^ c[3] ^ d[0] ^ d[1] ^ d[2] ^ d[3];
    }
    for (; i < count16; i += stride) {
        u32x4 a = ld(i);
        s += a[0] ^ a[1] ^ a[2] ^ a[3];
    }
    if (s == 0x9E3779B9u) sink[0] = s;
}

}  // namespace

hipError_t launch_peak_mfma(float* sink, int workgroups, int iters, hipStream_t stream) {
    peak_mfma_kernel<<<workgroups, 256, 0, stream>>>(sink, iters);
    return hipGetLastError();
}

hipError_t launch_peak_read(const void* src, int64_t bytes, void* sink, int workgroups, hipStream_t stream, bool non_temporal) {
    if (non_temporal) peak_read_kernel<true><<<workgroups, 256, 0, stream>>>((const u32x4*)src, bytes / 16, (uint32_t*)sink);
    else peak_read_kernel<false><<<workgroups, 256, 0, stream>>>((const u32x4*)src, bytes / 16, (uint32_t*)sink);
    return hipGetLastError();
}
