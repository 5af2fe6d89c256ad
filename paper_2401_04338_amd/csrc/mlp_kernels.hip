// Dense side of the MAML step (G-Meta Alg. 1): inner forward / local back-propagation on theta, outer
// forward with the task's adapted theta', and the tangent passes of the second-order term.  Every
// product is a GROUPED GEMM: one group per task, each group with its own rows and (when theta has been
// adapted) its own weights.
#include <algorithm>

#include "gm_internal.h"

// ------------------------------------------------------------------------------------------------
// fp32 grouped GEMM (vector FMA), C = A1*B1 (+ A2*B2) with generic strides and a fused epilogue
// ------------------------------------------------------------------------------------------------
#define GB_M 64
#define GB_N 64
#define GB_K 16

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs a, int n_ntiles, int mt_per_group) {
    __shared__ float As[GB_K][GB_M + 4];
    __shared__ float Bs[GB_K][GB_N + 4];
    const int ntile = blockIdx.x % n_ntiles;
    const int mtile = blockIdx.x / n_ntiles;
    int g, m0;
    if (a.tile_group) {
        g = a.tile_group[mtile];
        m0 = a.tile_m0[mtile];
    } else {
        g = mtile / mt_per_group;
        m0 = (mtile % mt_per_group) * GB_M;
    }
    const int64_t r0 = a.row_offsets ? a.row_offsets[g] : 0;
    const int rows_g = a.row_offsets ? (int)(a.row_offsets[g + 1] - r0) : 0;
    const int M = a.M < 0 ? rows_g : a.M;
    const int K = a.K < 0 ? rows_g : a.K;
    const int N = a.N;
    const int n0 = ntile * GB_N;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int pr = 0; pr < a.n_pairs; ++pr) {
        const float* A = a.A[pr] + (int64_t)g * a.gA[pr] + r0 * a.rA[pr];
        const float* B = a.B[pr] + (int64_t)g * a.gB[pr] + r0 * a.rB[pr];
        const int64_t sAm = a.sAm[pr], sAk = a.sAk[pr], sBk = a.sBk[pr], sBn = a.sBn[pr];
        for (int k0 = 0; k0 < K; k0 += GB_K) {
#pragma unroll
            for (int e = threadIdx.x; e < GB_M * GB_K; e += 256) {
                int m, k;
                if (sAk == 1) { m = e / GB_K; k = e % GB_K; } else { m = e % GB_M; k = e / GB_M; }
                const int gm = m0 + m, gk = k0 + k;
                As[k][m] = (gm < M && gk < K) ? A[gm * sAm + gk * sAk] : 0.f;
            }
#pragma unroll
            for (int e = threadIdx.x; e < GB_N * GB_K; e += 256) {
                int n, k;
                if (sBk == 1) { n = e / GB_K; k = e % GB_K; } else { n = e % GB_N; k = e / GB_N; }
                const int gn = n0 + n, gk = k0 + k;
                Bs[k][n] = (gn < N && gk < K) ? B[gk * sBk + gn * sBn] : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < GB_K; ++k) {
                float av[4], bv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) av[i] = As[k][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) bv[j] = Bs[k][tx * 4 + j];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
            }
            __syncthreads();
        }
    }

    float* C = a.C + (int64_t)g * a.gC + r0 * a.rC;
    const float* bias = a.bias ? a.bias + (int64_t)g * a.gBias : nullptr;
    const float* mask = a.mask ? a.mask + r0 * a.ld_mask : nullptr;
    const float* Cin = a.Cin ? a.Cin + (int64_t)g * a.gCin : nullptr;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc[i][j];
            switch (a.epi) {
                case EPI_BIAS_RELU: v = fmaxf(v + bias[n], 0.f); break;
                case EPI_BIAS_MASK: v = (mask[(int64_t)m * a.ld_mask + n] > 0.f) ? v + bias[n] : 0.f; break;
                case EPI_MASK: v = (mask[(int64_t)m * a.ld_mask + n] > 0.f) ? v : 0.f; break;
                case EPI_AXPBY: v = a.c1 * v + (Cin ? a.c0 * Cin[(int64_t)m * a.ldc + n] : 0.f); break;
                default: break;
            }
            C[(int64_t)m * a.ldc + n] = v;
        }
    }
}

void launch_gemm_f32(hipStream_t st, const GemmArgs& a) {
    const int n_ntiles = (a.N + GB_N - 1) / GB_N;
    int64_t n_mtiles;
    int mt_per_group = 1;
    if (a.tile_group) {
        n_mtiles = a.n_mtiles;
    } else {
        mt_per_group = (a.M + GB_M - 1) / GB_M;
        n_mtiles = (int64_t)mt_per_group * a.G;
    }
    if (n_mtiles <= 0 || n_ntiles <= 0) return;
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((unsigned)(n_mtiles * n_ntiles)), dim3(256), 0, st, a, n_ntiles,
                       mt_per_group);
}

// ------------------------------------------------------------------------------------------------
// element access in either activation type
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float ldf(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16_t* p, int64_t i) { return bf2f(p[i]); }
__device__ __forceinline__ void stf(float* p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(bf16_t* p, int64_t i, float v) { p[i] = f2bf(v); }

// ------------------------------------------------------------------------------------------------
// per-task column sums (bias gradients, last-layer weight gradient, per-task mean loss)
// out[g,n] = c0*in[g,n] + c1 * sum_{s in g} ( X1[s,n]*w1[s] + X2[s,n]*w2[s] ), rows summed in a fixed order
// ------------------------------------------------------------------------------------------------
// One workgroup of 4 waves per (task, block of columns): a lane owns 16 bytes of columns (8 bf16 or 4 fp32), the
// waves take the task's rows round-robin in batches of 8 independent loads, and the four partial sums are
// added in wave order.  The partition depends only on the shapes: results are reproducible.
template <typename T>
struct ColVec;
template <>
struct ColVec<float> {
    static constexpr int N = 4;
    __device__ static void load(const float* p, float (&v)[4]) {
        const float4 x = *reinterpret_cast<const float4*>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
};
template <>
struct ColVec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void load(const bf16_t* p, float (&v)[8]) {
        const uint4 x = *reinterpret_cast<const uint4*>(p);
        const u32 w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] = __builtin_bit_cast(float, w[k] << 16);
            v[2 * k + 1] = __builtin_bit_cast(float, w[k] & 0xFFFF0000u);
        }
    }
};

template <typename T, bool VEC>
__global__ __launch_bounds__(256) void task_colsum_kernel(const int32_t* __restrict__ row_offsets, int N,
                                                          const T* __restrict__ X1, const float* __restrict__ w1,
                                                          const T* __restrict__ X2, const float* __restrict__ w2,
                                                          int64_t ldx, float* out, int64_t g_out, const float* in,
                                                          int64_t g_in, float c0, float c1) {
    constexpr int V = VEC ? ColVec<T>::N : 1;
    __shared__ float part[3][64 * V];
    const int g = blockIdx.y;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int n = (blockIdx.x * 64 + lane) * V;
    const int64_t r0 = row_offsets[g], r1 = row_offsets[g + 1];
    float acc[V];
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = 0.f;
    if (n < N) {
        constexpr int UB = 8;
        for (int64_t s0 = r0 + wv * UB; s0 < r1; s0 += 4 * UB) {
            float x1[UB][V], x2[UB][V], f1[UB], f2[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int64_t s = s0 + u;
                const bool ok = s < r1;
                const int64_t sc = ok ? s : r0;
                if constexpr (VEC) ColVec<T>::load(X1 + sc * ldx + n, x1[u]);
                else x1[u][0] = ldf(X1, sc * ldx + n);
                f1[u] = ok ? (w1 ? w1[sc] : 1.f) : 0.f;
                if (X2) {
                    if constexpr (VEC) ColVec<T>::load(X2 + sc * ldx + n, x2[u]);
                    else x2[u][0] = ldf(X2, sc * ldx + n);
                    f2[u] = ok ? (w2 ? w2[sc] : 1.f) : 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < UB; ++u)
#pragma unroll
                for (int k = 0; k < V; ++k) {
                    float v = x1[u][k] * f1[u];
                    if (X2) v += x2[u][k] * f2[u];
                    acc[k] += v;
                }
        }
    }
    if (wv > 0) {
#pragma unroll
        for (int k = 0; k < V; ++k) part[wv - 1][lane * V + k] = acc[k];
    }
    __syncthreads();
    if (wv == 0 && n < N) {
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const float sum = ((acc[k] + part[0][lane * V + k]) + part[1][lane * V + k]) + part[2][lane * V + k];
            if (n + k < N) out[(int64_t)g * g_out + n + k] = c1 * sum + (in ? c0 * in[(int64_t)g * g_in + n + k] : 0.f);
        }
    }
}

template <typename T>
static void task_colsum_t(hipStream_t st, int G, const int32_t* row_offsets, int N, const T* X1, const float* w1,
                          const T* X2, const float* w2, int64_t ldx, float* out, int64_t g_out, const float* in,
                          int64_t g_in, float c0, float c1) {
    if (G <= 0 || N <= 0) return;
    // 16-byte loads need aligned rows and whole vectors inside the row
    constexpr int V = ColVec<T>::N;
    const bool vec = N >= 64 && ldx % V == 0 && (reinterpret_cast<uintptr_t>(X1) % 16 == 0) &&
                     (!X2 || reinterpret_cast<uintptr_t>(X2) % 16 == 0) && ((N + V - 1) / V * V <= ldx);
    const int cols = 64 * (vec ? V : 1);
    for (int g0 = 0; g0 < G; g0 += 32768) {
        const int gc = (G - g0) < 32768 ? (G - g0) : 32768;
        const dim3 grid((N + cols - 1) / cols, gc);
        if (vec)
            hipLaunchKernelGGL((task_colsum_kernel<T, true>), grid, dim3(256), 0, st, row_offsets + g0, N, X1, w1, X2, w2, ldx,
                               out + (int64_t)g0 * g_out, g_out, in ? in + (int64_t)g0 * g_in : nullptr, g_in, c0, c1);
        else
            hipLaunchKernelGGL((task_colsum_kernel<T, false>), grid, dim3(256), 0, st, row_offsets + g0, N, X1, w1, X2, w2, ldx,
                               out + (int64_t)g0 * g_out, g_out, in ? in + (int64_t)g0 * g_in : nullptr, g_in, c0, c1);
    }
}
void launch_task_colsum(hipStream_t st, int G, const int32_t* row_offsets, int N, const float* X1, const float* w1,
                        const float* X2, const float* w2, int64_t ldx, float* out, int64_t g_out, const float* in,
                        int64_t g_in, float c0, float c1) {
    task_colsum_t<float>(st, G, row_offsets, N, X1, w1, X2, w2, ldx, out, g_out, in, g_in, c0, c1);
}
void launch_task_colsum_bf(hipStream_t st, int G, const int32_t* row_offsets, int N, const bf16_t* X1, const float* w1,
                           const bf16_t* X2, const float* w2, int64_t ldx, float* out, int64_t g_out, const float* in,
                           int64_t g_in, float c0, float c1) {
    task_colsum_t<bf16_t>(st, G, row_offsets, N, X1, w1, X2, w2, ldx, out, g_out, in, g_in, c0, c1);
}

// ------------------------------------------------------------------------------------------------
// last layer (d_L = 1) fused with the sigmoid / binary cross-entropy: one wavefront per row.
// Rows may be padded per task: row r of task g is sample real_offsets[g] + (r - row_offsets[g]) when that
// is below real_offsets[g+1]; pad rows get delta = 0 and loss = 0.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
    const uint4 x = *reinterpret_cast<const uint4*>(p);
    const u32 w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        v[2 * k] = __builtin_bit_cast(float, w[k] << 16);
        v[2 * k + 1] = __builtin_bit_cast(float, w[k] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// lpr: lanes per row, a power of two (64: one row per wave; fewer when 8 columns per lane cover the row with less,
// so that a wave takes 64 / lpr rows at once)
template <typename T>
__global__ void last_fwd_kernel(LastFwdArgs a, int lpr) {
    const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t s = gt / lpr;
    const int lane = (int)(gt % lpr);
    if (s >= a.n) return;
    const int g = a.row_task[s];
    const int r_in = (int)(s - a.row_offsets[g]);
    const int n_real = a.real_offsets[g + 1] - a.real_offsets[g];
    if (r_in >= n_real) {  // pad row
        if (lane == 0) {
            a.delta_out[s] = 0.f;
            if (a.z_out) a.z_out[s] = 0.f;
            if (a.loss_out) a.loss_out[s] = 0.f;
        }
        return;
    }
    const float* w = a.w + (int64_t)g * a.gW;
    const T* x = reinterpret_cast<const T*>(a.a) + s * a.ld;
    float acc = 0.f;
    // bf16 rows whose width and stride are multiples of 8: 16-byte loads (pad columns hold zeros on both sides)
    const bool vec = sizeof(T) == 2 && (a.N % 8 == 0) && (a.ld % 8 == 0) && (a.gW % 4 == 0) && (!a.ta || a.gTW % 4 == 0) &&
                     reinterpret_cast<uintptr_t>(a.w) % 16 == 0 && (!a.ta || reinterpret_cast<uintptr_t>(a.tw) % 16 == 0);
    if (vec) {
        const bf16_t* xb = reinterpret_cast<const bf16_t*>(x);
        const bf16_t* txb = a.ta ? reinterpret_cast<const bf16_t*>(a.ta) + s * a.ld : nullptr;
        const float* tw = a.ta ? a.tw + (int64_t)g * a.gTW : nullptr;
        for (int n = lane * 8; n < a.N; n += lpr * 8) {
            float xv[8], wv[8];
            load8(xb + n, xv);
            load8(w + n, wv);
            if (!a.ta) {
#pragma unroll
                for (int k = 0; k < 8; ++k) acc = fmaf(xv[k], wv[k], acc);
            } else {
                float tv[8], twv[8];
                load8(txb + n, tv);
                load8(tw + n, twv);
#pragma unroll
                for (int k = 0; k < 8; ++k) acc += tv[k] * wv[k] + xv[k] * twv[k];
            }
        }
    } else if (!a.ta) {
        for (int n = lane; n < a.N; n += 64) acc = fmaf(ldf(x, n), w[n], acc);
    } else {
        const T* tx = reinterpret_cast<const T*>(a.ta) + s * a.ld;
        const float* tw = a.tw + (int64_t)g * a.gTW;
        for (int n = lane; n < a.N; n += 64) acc += ldf(tx, n) * w[n] + ldf(x, n) * tw[n];
    }
    for (int d = lpr >> 1; d > 0; d >>= 1) acc += __shfl_xor(acc, d, 64);   // within the row's lanes
    if (lane != 0) return;
    const float inv_n = 1.f / (float)n_real;
    if (!a.ta) {
        const float z = acc + a.b[(int64_t)g * a.gW];
        const float y = a.labels[a.real_offsets[g] + r_in];
        const float e = __expf(-fabsf(z));
        const float sig = z >= 0.f ? 1.f / (1.f + e) : e / (1.f + e);
        if (a.z_out) a.z_out[s] = z;
        a.delta_out[s] = (sig - y) * inv_n;
        if (a.loss_out) a.loss_out[s] = (fmaxf(z, 0.f) - y * z + log1pf(e)) * inv_n;
    } else {
        const float tz = acc + a.tb[(int64_t)g * a.gTW];
        const float z = a.z_in[s];
        const float e = __expf(-fabsf(z));
        const float sig = z >= 0.f ? 1.f / (1.f + e) : e / (1.f + e);
        a.delta_out[s] = sig * (1.f - sig) * tz * inv_n;
    }
}

void launch_last_fwd(hipStream_t st, const LastFwdArgs& a) {
    if (a.n <= 0) return;
    int lpr = 64;
    // the 16-byte path of the kernel (same conditions) reads 8 columns per lane: narrow rows need fewer lanes
    if (a.bf16 && a.N % 8 == 0 && a.ld % 8 == 0 && a.gW % 4 == 0 && (!a.ta || a.gTW % 4 == 0) &&
        reinterpret_cast<uintptr_t>(a.w) % 16 == 0 && (!a.ta || reinterpret_cast<uintptr_t>(a.tw) % 16 == 0)) {
        while (lpr > 8 && (lpr / 2) * 8 >= a.N) lpr /= 2;
    }
    const dim3 grid((unsigned)((a.n * lpr + 255) / 256));
    if (a.bf16) hipLaunchKernelGGL(last_fwd_kernel<bf16_t>, grid, dim3(256), 0, st, a, lpr);
    else hipLaunchKernelGGL(last_fwd_kernel<float>, grid, dim3(256), 0, st, a, lpr);
}

template <typename T>
__global__ void last_bwd_kernel(int64_t n, int N, int64_t ld_a, int64_t ld_d, const int32_t* __restrict__ row_task,
                                const float* __restrict__ dl, const float* __restrict__ w, int64_t gW,
                                const float* __restrict__ dl2, const float* __restrict__ w2, int64_t gW2,
                                const T* __restrict__ act, T* d, float* d_f32) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * N) return;
    const int64_t s = i / N;
    const int c = (int)(i - s * N);
    const int g = row_task[s];
    float v = dl[s] * w[(int64_t)g * gW + c];
    if (dl2) v += dl2[s] * w2[(int64_t)g * gW2 + c];
    if (act && !(ldf(act, s * ld_a + c) > 0.f)) v = 0.f;
    if (d) stf(d, s * ld_d + c, v);
    if (d_f32) d_f32[s * ld_d + c] = v;
}

// bf16 rows, 8 columns per thread (N, strides and the weight strides allow 16-byte accesses)
__global__ void last_bwd_vec_kernel(int64_t n, int N, int64_t ld_a, int64_t ld_d, const int32_t* __restrict__ row_task,
                                    const float* __restrict__ dl, const float* __restrict__ w, int64_t gW,
                                    const float* __restrict__ dl2, const float* __restrict__ w2, int64_t gW2,
                                    const bf16_t* __restrict__ act, bf16_t* d, float* d_f32) {
    const int per_row = N / 8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * per_row) return;
    const int64_t s = i / per_row;
    const int c = (int)(i - s * per_row) * 8;
    const int g = row_task[s];
    float wv[8], v[8];
    load8(w + (int64_t)g * gW + c, wv);
    const float a1 = dl[s];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = a1 * wv[k];
    if (dl2) {
        load8(w2 + (int64_t)g * gW2 + c, wv);
        const float a2 = dl2[s];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] += a2 * wv[k];
    }
    if (act) {
        float av[8];
        load8(act + s * ld_a + c, av);
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (!(av[k] > 0.f)) v[k] = 0.f;
    }
    if (d) *reinterpret_cast<uint4*>(d + s * ld_d + c) = make_uint4(f2bf2(v[0], v[1]), f2bf2(v[2], v[3]), f2bf2(v[4], v[5]), f2bf2(v[6], v[7]));
    if (d_f32) {
        *reinterpret_cast<float4*>(d_f32 + s * ld_d + c) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(d_f32 + s * ld_d + c + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// d[s,n] = (dl[s]*w_g[n] (+ dl2[s]*w2_g[n])) * (act[s,n] > 0); act null: no mask.  Output in the
// activation type (d) and/or fp32 (d_f32).
void launch_last_bwd(hipStream_t st, int bf16, int64_t n, int N, int64_t ld_a, int64_t ld_d, const int32_t* row_task,
                     const float* dl, const float* w, int64_t gW, const float* dl2, const float* w2, int64_t gW2,
                     const void* act, void* d, float* d_f32) {
    if (n <= 0 || N <= 0) return;
    const dim3 grid((unsigned)((n * N + 255) / 256));
    if (bf16 && N % 8 == 0 && ld_a % 8 == 0 && ld_d % 8 == 0 && gW % 4 == 0 && (!dl2 || gW2 % 4 == 0) &&
        reinterpret_cast<uintptr_t>(w) % 16 == 0 && (!w2 || reinterpret_cast<uintptr_t>(w2) % 16 == 0))
        hipLaunchKernelGGL(last_bwd_vec_kernel, dim3((unsigned)((n * (N / 8) + 255) / 256)), dim3(256), 0, st, n, N, ld_a, ld_d,
                           row_task, dl, w, gW, dl2, w2, gW2, (const bf16_t*)act, (bf16_t*)d, d_f32);
    else if (bf16)
        hipLaunchKernelGGL(last_bwd_kernel<bf16_t>, grid, dim3(256), 0, st, n, N, ld_a, ld_d, row_task, dl, w, gW, dl2,
                           w2, gW2, (const bf16_t*)act, (bf16_t*)d, d_f32);
    else
        hipLaunchKernelGGL(last_bwd_kernel<float>, grid, dim3(256), 0, st, n, N, ld_a, ld_d, row_task, dl, w, gW, dl2, w2,
                           gW2, (const float*)act, (float*)d, d_f32);
}

// ------------------------------------------------------------------------------------------------
// cross-task reduction of the dense meta-gradient (Alg. 1, global back-propagation on theta; Sec. 2.1.3):
// out[j] (+)= sum_g v[g, j], tasks added in task order; with a scale other than 1: out[j] (+)= scale * (sum_g v[g, j])
// ------------------------------------------------------------------------------------------------
__global__ void reduce_tasks_kernel(const float* __restrict__ v, int64_t ld, int G, int64_t n, float* out,
                                    int accumulate, float scale) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n) return;
    // eight tasks' values are requested before the first is added (the order of the sum stays the task order)
    float acc = (accumulate && scale == 1.f) ? out[j] : 0.f;
    int g = 0;
    for (; g + 8 <= G; g += 8) {
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = v[(int64_t)(g + u) * ld + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += x[u];
    }
    for (; g < G; ++g) acc += v[(int64_t)g * ld + j];
    out[j] = scale == 1.f ? acc : (accumulate ? out[j] : 0.f) + scale * acc;
}

void launch_reduce_tasks(hipStream_t st, const float* v, int64_t ld, int G, int64_t n, float* out, int accumulate,
                         float scale) {
    if (n <= 0) return;
    hipLaunchKernelGGL(reduce_tasks_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, v, ld, G, n, out,
                       accumulate, scale);
}

__global__ void fill_sample_task_kernel(const int32_t* row_offsets, int32_t* sample_task) {
    const int g = blockIdx.x;
    for (int s = row_offsets[g] + threadIdx.x; s < row_offsets[g + 1]; s += blockDim.x) sample_task[s] = g;
}
void launch_fill_sample_task(hipStream_t st, const int32_t* row_offsets, int G, int32_t* sample_task) {
    if (G <= 0) return;
    hipLaunchKernelGGL(fill_sample_task_kernel, dim3(G), dim3(256), 0, st, row_offsets, sample_task);
}

// W [din, dout] row-major  <->  padded [ld_in, ld_out] (pad rows / columns zero)
__global__ void pack_weights_kernel(const float* W, int din, int dout, int ld_in, int ld_out, float* dst) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)ld_in * ld_out) return;
    const int r = (int)(i / ld_out), c = (int)(i % ld_out);
    dst[i] = (r < din && c < dout) ? W[(int64_t)r * dout + c] : 0.f;
}
void launch_pack_weights(hipStream_t st, const float* W, int din, int dout, int ld_in, int ld_out, float* dst) {
    const int64_t n = (int64_t)ld_in * ld_out;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, W, din, dout, ld_in,
                       ld_out, dst);
}
__global__ void unpack_weights_kernel(const float* src, int din, int dout, int ld_out, float* W) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)din * dout) return;
    const int r = (int)(i / dout), c = (int)(i % dout);
    W[i] = src[(int64_t)r * ld_out + c];
}
void launch_unpack_weights(hipStream_t st, const float* src, int din, int dout, int ld_out, float* W) {
    const int64_t n = (int64_t)din * dout;
    if (n <= 0) return;
    hipLaunchKernelGGL(unpack_weights_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src, din, dout,
                       ld_out, W);
}

__global__ void axpy_kernel(int64_t n, float a, const float* __restrict__ x, float* y) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        y[i] += a * x[i];
}
// y += a * x and x = 0 in one pass (the table-shaped sparse meta-gradient applied to the tables and cleared for the next
// iteration); 16 bytes per lane
__global__ void axpy_clear_kernel(int64_t n4, float a, float4* x, float4* y) {
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
        const float4 g = x[i];
        if (g.x == 0.f && g.y == 0.f && g.z == 0.f && g.w == 0.f) continue;   // (rows nobody looked up: nothing to read or write)
        float4 v = y[i];
        v.x += a * g.x; v.y += a * g.y; v.z += a * g.z; v.w += a * g.w;
        y[i] = v;
        x[i] = zero;
    }
}
void launch_axpy_clear(hipStream_t st, int64_t n, float a, float* x, float* y) {   // n a multiple of 4, both 16-byte aligned
    if (n <= 0) return;
    const int64_t n4 = n / 4;
    const unsigned grid = (unsigned)std::min<int64_t>((n4 + 255) / 256, 256 * 64);
    hipLaunchKernelGGL(axpy_clear_kernel, dim3(grid), dim3(256), 0, st, n4, a, reinterpret_cast<float4*>(x), reinterpret_cast<float4*>(y));
}
void launch_axpy(hipStream_t st, int64_t n, float a, const float* x, float* y) {
    if (n <= 0) return;
    int64_t nb = (n + 255) / 256;
    if (nb > 65536) nb = 65536;
    hipLaunchKernelGGL(axpy_kernel, dim3((unsigned)nb), dim3(256), 0, st, n, a, x, y);
}

__global__ void sum_to_scalar_kernel(const float* x, int n, float* out, int accumulate) {
    // one wavefront, fixed order: lanes stride the array, then a butterfly
    float acc = 0.f;
    for (int i = threadIdx.x; i < n; i += 64) acc += x[i];
    acc = wave_sum(acc);
    if (threadIdx.x == 0) *out = accumulate ? *out + acc : acc;
}
void launch_sum_to_scalar(hipStream_t st, const float* x, int n, float* out, int accumulate) {
    hipLaunchKernelGGL(sum_to_scalar_kernel, dim3(1), dim3(64), 0, st, x, n, out, accumulate);
}
