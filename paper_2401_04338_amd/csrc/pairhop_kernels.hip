// Task-local embedding-row arithmetic as a dense contraction on the matrix cores.
//
// Every row-space operation of the inner loop and of the second-order chain (G-Meta Alg. 1: local
// back-propagation on xi^Sup, the overlap update of Sec. 2.1.2, and their tangents) is, for one
// (task, field),
//     Y[i, :] = Y_in[i, :] + c * sum_j M[i][j] * Z[j, :],      M = P_out * P_in^T,
// where P_set[bag][row] counts how often the bag looks the row up, restricted to the rows of the
// task's support set.  M[i][j] is therefore the number of (lookup of out-bag i, lookup of in-bag j)
// pairs that hit the same row: a small integer that depends on the indices only.  It is the same for
// every inner step and for the whole second-order chain, so it is counted ONCE per call
// (pair_count_kernel, integer atomics in LDS: exact and order-free) and stored as bytes; each of the
// hops is then a [n_out, n_in] x [n_in, D] product on MFMA (pair_hop_kernel).
//
// fp32 accuracy on bf16 matrix cores: an fp32 value splits EXACTLY into three bf16 pieces (its 24
// significand bits cut 8+8+8 by truncation, every remainder exact), counts up to 255 are exact in
// bf16, and every product count*piece is exact in the fp32 accumulator; only the accumulation rounds,
// as it would in an fp32 loop.
//
// Counts above 255 or tasks too large for this path are handled by the sparse two-hop kernel instead.
#include "gm_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 ph_short8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float ph_float16;

__device__ __forceinline__ int pad64(int n) { return (n + 63) & ~63; }

// ------------------------------------------------------------------------------------------------
// counting: M[i][j] for one (task, field) and one pair of sets, in LDS tiles of out-rows
// ------------------------------------------------------------------------------------------------
#define PC_NT 512

__global__ __launch_bounds__(PC_NT) void pair_count_kernel(PairCountArgs a) {
    extern __shared__ u32 pc_lds[];
    const int f = blockIdx.x, t = blockIdx.y;
    const bool qs = blockIdx.z == 1;   // 0: support x support, 1: query x support (and its transpose)
    if (!qs && !a.want_ss) return;
    const size_t tf = (size_t)t * a.F + f;
    const int ns = a.real_off_s[t + 1] - a.real_off_s[t], nq = a.real_off_q[t + 1] - a.real_off_q[t];
    const int n_out = qs ? nq : ns;
    const int colsP = pad64(ns), rowsP = pad64(n_out);
    if (colsP == 0 || rowsP == 0) return;
    const u32 B = a.base_s[tf], Bq = a.base_q[tf];
    const int nu = (int)a.n_slots[tf];
    const int n_in_entries = a.slot_start[B + tf + nu] - (int)B;
    const int n_out_entries = qs ? (int)a.cnt_q[tf] : n_in_entries;
    const int2* in_list = a.sup_sorted + B;
    const int2* out_list = qs ? a.qry_sorted + Bq : a.sup_sorted + B;
    const int in_row0 = a.row_off_s[t], out_row0 = qs ? a.row_off_q[t] : a.row_off_s[t];
    const int lds_ld = colsP + 2;                       // u16 elements per tile row (odd number of words)
    int R = (a.tile_bytes / (lds_ld * 2)) & ~63;        // out-rows per tile
    if (R > rowsP) R = rowsP;
    uint16_t* out_rows = reinterpret_cast<uint16_t*>(pc_lds + a.tile_bytes / 4);
    for (int e = threadIdx.x; e < n_out_entries; e += PC_NT) out_rows[e] = (uint16_t)(out_list[e].x - out_row0);
    uint8_t* M = a.mat + (qs ? a.off_qs[t] : a.off_ss[t]) + (size_t)f * rowsP * colsP;
    uint8_t* Mt = (qs && a.want_sq) ? a.mat + a.off_sq[t] + (size_t)f * colsP * rowsP : nullptr;  // [colsP rows][rowsP cols]
    bool ovf = false;
    for (int i0 = 0; i0 < rowsP; i0 += R) {
        const int rows_here = min(R, rowsP - i0);
        for (int i = threadIdx.x; i < rows_here * lds_ld / 2; i += PC_NT) pc_lds[i] = 0;
        __syncthreads();
        for (int p = threadIdx.x; p < n_in_entries; p += PC_NT) {
            const int2 e = in_list[p];
            const int j = e.x - in_row0, u = e.y;
            int lo, hi;
            if (qs) { lo = a.qseg_lo[B + u] - (int)Bq; hi = a.qseg_hi[B + u] - (int)Bq; }
            else { lo = a.slot_start[B + tf + u] - (int)B; hi = a.slot_start[B + tf + u + 1] - (int)B; }
            const u32 inc = 1u << (16 * (j & 1));
            for (int x = lo; x < hi; ++x) {
                const int i = (int)out_rows[x] - i0;
                if ((unsigned)i < (unsigned)rows_here) atomicAdd(&pc_lds[(i * lds_ld + j) >> 1], inc);
            }
        }
        __syncthreads();
        const uint16_t* tile = reinterpret_cast<const uint16_t*>(pc_lds);
        // rows [i0, i0 + rows_here) of M, four counts per store
        const int wpr = colsP / 4;
        for (int w = threadIdx.x; w < rows_here * wpr; w += PC_NT) {
            const int i = w / wpr, j4 = (w - i * wpr) * 4;
            const u32 lo2 = *reinterpret_cast<const u32*>(tile + i * lds_ld + j4);
            const u32 hi2 = *reinterpret_cast<const u32*>(tile + i * lds_ld + j4 + 2);
            const u32 c0 = lo2 & 0xFFFFu, c1 = lo2 >> 16, c2 = hi2 & 0xFFFFu, c3 = hi2 >> 16;
            ovf |= (c0 | c1 | c2 | c3) > 255u;
            *reinterpret_cast<u32*>(M + (size_t)(i0 + i) * colsP + j4) = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
        }
        if (Mt) {  // the transpose: row j of it holds columns [i0, i0 + rows_here)
            const int gpr = rows_here / 4;
            for (int w = threadIdx.x; w < colsP * gpr; w += PC_NT) {
                const int j = w / gpr, i4 = (w - j * gpr) * 4;
                const u32 c0 = tile[(i4 + 0) * lds_ld + j], c1 = tile[(i4 + 1) * lds_ld + j];
                const u32 c2 = tile[(i4 + 2) * lds_ld + j], c3 = tile[(i4 + 3) * lds_ld + j];
                *reinterpret_cast<u32*>(Mt + (size_t)j * rowsP + i0 + i4) = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
            }
        }
        __syncthreads();
    }
    if (ovf) a.status[ST_PAIR_OVF] = 1u;
}

size_t pair_count_lds_bytes(int cap) { return (size_t)PAIR_TILE_BYTES + (size_t)cap * 2; }

void launch_pair_count(hipStream_t st, PairCountArgs a, int Tw, int cap) {
    if (Tw <= 0 || a.F <= 0) return;
    a.tile_bytes = PAIR_TILE_BYTES;
    const size_t shmem = pair_count_lds_bytes(cap);
    (void)hipFuncSetAttribute((const void*)pair_count_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    hipLaunchKernelGGL(pair_count_kernel, dim3(a.F, Tw, 2), dim3(PC_NT), shmem, st, a);
}

// ------------------------------------------------------------------------------------------------
// the hop: Y = Y_in + c * M * Z on MFMA 32x32x16 (bf16 operands, fp32 accumulation)
//
// One workgroup of 4 waves owns (task, field, DS columns, 256 out-rows); each wave owns 64 of the rows
// (two 32-row strips).  Z is staged 64 rows at a time: split into its three bf16 pieces and stored
// contraction-contiguous per column, so that a B fragment is one 16-byte LDS read.  M is read
// straight from memory: within a 64-wide chunk the lane half h contracts columns [32h, 32h+32) of the
// chunk (the contraction index may be enumerated in any order as long as A and B agree), which makes
// a lane's share of a strip 32 contiguous bytes of one row of M.
// ------------------------------------------------------------------------------------------------
#define PH_KC 64
#define PH_LDK (PH_KC + 8)

__device__ __forceinline__ u32 ph_pack_hi(u32 e0, u32 e1) {  // {e1[31:16], e0[31:16]}
    return __builtin_amdgcn_perm(e1, e0, 0x07060302u);
}

// four counts (bytes of x) -> four bf16 (exact for 0..255)
__device__ __forceinline__ void ph_cvt4(u32 x, u32& lo, u32& hi) {
    const float f0 = (float)(x & 0xFFu), f1 = (float)((x >> 8) & 0xFFu), f2 = (float)((x >> 16) & 0xFFu), f3 = (float)(x >> 24);
    lo = ph_pack_hi(__builtin_bit_cast(u32, f0), __builtin_bit_cast(u32, f1));
    hi = ph_pack_hi(__builtin_bit_cast(u32, f2), __builtin_bit_cast(u32, f3));
}

template <int DS>
__global__ __launch_bounds__(256) void pair_hop_kernel(PairHopArgs a) {
    constexpr int NCT = DS / 32;      // 32-column tiles
    constexpr int CG = DS / 4;        // float4 column groups of a row of Z
    constexpr int RPT = CG / 4;       // rows of the 64-row chunk staged per thread (256 threads)
    __shared__ __attribute__((aligned(16))) bf16_t zs[3][DS][PH_LDK];
    const int nsl = a.D / DS;
    const int f = blockIdx.x / nsl, sl = blockIdx.x - f * nsl, t = blockIdx.y;
    const int o = blockIdx.z / a.row_blocks, rb = blockIdx.z - o * a.row_blocks;
    const PairHopOut& out = a.out[o];
    const int n_in = a.in_real_off[t + 1] - a.in_real_off[t];
    const int n_out = out.real_off[t + 1] - out.real_off[t];
    if (rb * 256 >= n_out) return;
    const int colsP = pad64(n_in), rowsP = pad64(n_out);
    const uint8_t* M = a.mat + out.mat_off[t] + (size_t)f * rowsP * colsP;
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63, ln = lane & 31, h = lane >> 5;
    const int row_w = rb * 256 + wv * 64;             // first out-row of this wave
    const bool wave_on = row_w < n_out;               // both strips then lie inside the padded matrix
    const int cg = threadIdx.x % CG, rg = threadIdx.x / CG;
    const int64_t colz = (int64_t)f * a.D + (int64_t)sl * DS;
    const float* Zt = a.Z + (int64_t)a.in_row_off[t] * a.ldz + colz + cg * 4;

    ph_float16 acc[2][NCT];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][ct][v] = 0.f;

    for (int kc = 0; kc < colsP; kc += PH_KC) {
        float4 z[RPT];
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int row = kc + rg * RPT + r;
            z[r] = row < n_in ? *reinterpret_cast<const float4*>(Zt + (int64_t)row * a.ldz) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        uint4 araw[2][2];
        if (wave_on) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const uint4* src = reinterpret_cast<const uint4*>(M + (size_t)(row_w + s * 32 + ln) * colsP + kc + h * 32);
                araw[s][0] = src[0];
                araw[s][1] = src[1];
            }
        }
        __syncthreads();  // the previous chunk's fragments have been read
        {
            u32 p0[4][RPT], p1[4][RPT], p2[4][RPT];  // [column][row]: the three pieces as fp32 bit patterns
#pragma unroll
            for (int r = 0; r < RPT; ++r) {
                const float zz[4] = {z[r].x, z[r].y, z[r].z, z[r].w};
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    const u32 u0 = __builtin_bit_cast(u32, zz[cc]);
                    const float r1 = zz[cc] - __builtin_bit_cast(float, u0 & 0xFFFF0000u);
                    const u32 u1 = __builtin_bit_cast(u32, r1);
                    const float r2 = r1 - __builtin_bit_cast(float, u1 & 0xFFFF0000u);
                    p0[cc][r] = u0; p1[cc][r] = u1; p2[cc][r] = __builtin_bit_cast(u32, r2);
                }
            }
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                bf16_t* d0 = &zs[0][cg * 4 + cc][rg * RPT];
                bf16_t* d1 = &zs[1][cg * 4 + cc][rg * RPT];
                bf16_t* d2 = &zs[2][cg * 4 + cc][rg * RPT];
                if constexpr (RPT == 4) {
                    *reinterpret_cast<uint2*>(d0) = make_uint2(ph_pack_hi(p0[cc][0], p0[cc][1]), ph_pack_hi(p0[cc][2], p0[cc][3]));
                    *reinterpret_cast<uint2*>(d1) = make_uint2(ph_pack_hi(p1[cc][0], p1[cc][1]), ph_pack_hi(p1[cc][2], p1[cc][3]));
                    *reinterpret_cast<uint2*>(d2) = make_uint2(ph_pack_hi(p2[cc][0], p2[cc][1]), ph_pack_hi(p2[cc][2], p2[cc][3]));
                } else {
                    *reinterpret_cast<u32*>(d0) = ph_pack_hi(p0[cc][0], p0[cc][1]);
                    *reinterpret_cast<u32*>(d1) = ph_pack_hi(p1[cc][0], p1[cc][1]);
                    *reinterpret_cast<u32*>(d2) = ph_pack_hi(p2[cc][0], p2[cc][1]);
                }
            }
        }
        __syncthreads();
        if (wave_on) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                ph_short8 af[2];
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const uint4 q = araw[s][ks >> 1];
                    const u32 b0 = (ks & 1) ? q.z : q.x, b1 = (ks & 1) ? q.w : q.y;
                    u32 w0, w1, w2, w3;
                    ph_cvt4(b0, w0, w1);
                    ph_cvt4(b1, w2, w3);
                    const uint4 packed = make_uint4(w0, w1, w2, w3);
                    af[s] = __builtin_bit_cast(ph_short8, packed);
                }
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
                    for (int sp = 2; sp >= 0; --sp) {  // smallest pieces first
                        const ph_short8 bfrag = *reinterpret_cast<const ph_short8*>(&zs[sp][ct * 32 + ln][h * 32 + ks * 8]);
#pragma unroll
                        for (int s = 0; s < 2; ++s)
                            acc[s][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s], bfrag, acc[s][ct], 0, 0, 0);
                    }
            }
        }
    }
    if (!wave_on) return;
    // D layout of the 32x32 tile: register v of lane (ln, h) is row 8*(v/4) + 4*h + v%4, column ln
    const int64_t orow0 = out.row_off[t];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row_w + s * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (row >= n_out) continue;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const int64_t off = (orow0 + row) * out.ld + colz + ct * 32 + ln;
                const float y = (out.y_in ? out.y_in[off] : 0.f) + out.c * acc[s][ct][v];
                if (out.y_out) out.y_out[off] = y;
                if (out.y_bf) out.y_bf[off] = f2bf(y);
            }
        }
}

void launch_pair_hop(hipStream_t st, PairHopArgs a, int Tw, int max_out_rows) {
    if (Tw <= 0 || a.F <= 0 || max_out_rows <= 0) return;
    int n_out = 0;
    PairHopOut packed[2];
    for (int o = 0; o < 2; ++o)
        if (a.out[o].enabled) packed[n_out++] = a.out[o];
    if (n_out == 0) return;
    for (int o = 0; o < n_out; ++o) a.out[o] = packed[o];
    a.row_blocks = (max_out_rows + 255) / 256;
    if (a.D % 64 == 0)
        hipLaunchKernelGGL(pair_hop_kernel<64>, dim3(a.F * (a.D / 64), Tw, n_out * a.row_blocks), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(pair_hop_kernel<32>, dim3(a.F * (a.D / 32), Tw, n_out * a.row_blocks), dim3(256), 0, st, a);
}
