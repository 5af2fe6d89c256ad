// On-box ceilings for the roofline report (measurement only, no part of the method): what a plain streaming
// kernel and a register-resident matrix-core loop reach on this GPU, to be printed beside the datasheet peaks.
#include "gm_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// dst[i] = src[i], 16 bytes per lane and step, grid-stride
__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// reads n16 16-byte words, four loads in flight per lane; the sum keeps the loads alive
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, int64_t n16, u32* sink) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    u32 acc = 0;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc += a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = src[i];
        acc += a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;
}

// v_mfma_f32_32x32x16_bf16 with operands and accumulators in registers: four independent accumulators per wave
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
    for (int v = 0; v < 8; ++v) {
        a[v] = (__bf16)(1.0f + 0.125f * (float)((lane + v) & 7));
        b[v] = (__bf16)(0.5f + 0.0625f * (float)((lane * 3 + v) & 7));
    }
    f32x16 acc[4];
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    if (s == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = s;
}

void launch_stream_copy(hipStream_t st, const void* src, void* dst, int64_t bytes) {
    hipLaunchKernelGGL(stream_copy_kernel, dim3(256 * 16), dim3(256), 0, st, reinterpret_cast<const uint4*>(src),
                       reinterpret_cast<uint4*>(dst), bytes / 16);
}
void launch_stream_read(hipStream_t st, const void* src, int64_t bytes, u32* sink) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(256 * 16), dim3(256), 0, st, reinterpret_cast<const uint4*>(src), bytes / 16, sink);
}
// 256 compute units x 8 workgroups of 4 waves; returns the flops of the launch
double launch_mfma_loop(hipStream_t st, int iters, float* sink) {
    const int blocks = 256 * 8;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(256), 0, st, iters, sink);
    return 2.0 * 32 * 32 * 16 * 4.0 * iters * 4.0 * blocks;
}
