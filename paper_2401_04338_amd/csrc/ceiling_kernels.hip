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

// The same loop with operands that change from one MFMA to the next (eight register sets of pseudo-random values in
// (-1, 1) and (-0.05, 0.05), the magnitudes of activations and weights): the rate the matrix cores sustain on data
// that toggles their inputs, which is the one a GEMM on real operands can be held against.  With constant operands the
// chip holds its full clock; with these it settles lower.
__global__ __launch_bounds__(256) void mfma_loop_random_kernel(int iters, float* sink) {
    bf16x8 a[8], b[8];
    u32 z = (blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
    for (int s = 0; s < 8; ++s)
        for (int v = 0; v < 8; ++v) {
            z = z * 1664525u + 1013904223u;
            a[s][v] = (__bf16)((float)((z >> 8) & 0xffff) / 32768.f - 1.f);
            z = z * 1664525u + 1013904223u;
            b[s][v] = (__bf16)(((float)((z >> 8) & 0xffff) / 32768.f - 1.f) * 0.05f);
        }
    f32x16 acc[4];
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(s + j) & 7], b[(s * 3 + j) & 7], acc[j], 0, 0, 0);
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
// one workgroup of four waves per compute unit (one wave per SIMD, as the widest GEMM tiles run)
double launch_mfma_loop_random(hipStream_t st, int iters, float* sink) {
    const int blocks = 256;
    hipLaunchKernelGGL(mfma_loop_random_kernel, dim3(blocks), dim3(256), 0, st, iters, sink);
    return 2.0 * 32 * 32 * 16 * 32.0 * iters * 4.0 * blocks;
}
