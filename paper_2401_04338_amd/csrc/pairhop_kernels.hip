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
// counting: M[i][j] for one (task, field) and one pair of sets, in tiles of out-rows held in LDS
//
// M = sum over the rows u of the task's support set of  c_out(:, u) (x) c_in(:, u),  with c_set(b, u) the
// number of times bag b looks row u up.  Under a skewed row distribution a few hot rows carry nearly all
// of the pairs (a row looked up a times by one set and b times by the other adds a*b of them), and LDS
// atomics retire only about one lane per cycle, so the hot rows do not go through atomics: sixteen hot
// rows at a time, their count vectors are laid out densely ([bags, 16], a few thousand atomics) and
// multiplied on the matrix cores (counts up to 255 are exact in bf16, sums exact in fp32).  Only the
// remaining rows (fewer than PC_HOT lookups from either set, at most 9 pairs each) are counted pair by
// pair with atomics on 16-bit cells, on top of the stored hot part.  Everything is integer arithmetic:
// the result does not depend on any order.
// ------------------------------------------------------------------------------------------------
#define PC_NT 1024
#define PC_TPW (64 / (PC_NT / 64))   // MFMA tiles per wave: at most 64 tiles per row tile
#define PC_HB 16     // hot rows per matrix-core batch (the contraction length of one MFMA)
#define PC_HOT 4     // a row is hot when one of the two sets looks it up at least this often
#define PC_CLAMP 60000.f

__device__ __forceinline__ ph_short8 pc_counts_to_bf16(uint4 q) {  // eight 16-bit counts -> eight bf16 (exact up to 256)
    u32 w[4];
    const u32 x[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float lo = (float)(x[k] & 0xFFFFu), hi = (float)(x[k] >> 16);
        w[k] = __builtin_amdgcn_perm(__builtin_bit_cast(u32, hi), __builtin_bit_cast(u32, lo), 0x07060302u);
    }
    return __builtin_bit_cast(ph_short8, make_uint4(w[0], w[1], w[2], w[3]));
}

__global__ __launch_bounds__(PC_NT) void pair_count_kernel(PairCountArgs a) {
    extern __shared__ __attribute__((aligned(16))) u32 pc_lds[];
    __shared__ int sh_nhot;
    const int f = blockIdx.x, t = blockIdx.y;
    const bool qs = blockIdx.z == 1;   // 0: support x support, 1: query x support (and its transpose)
    if (!qs && !a.want_ss) return;
    const size_t tf = (size_t)t * a.F + f;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, ln = lane & 31, h = lane >> 5;
    const int ns = a.real_off_s[t + 1] - a.real_off_s[t], nq = a.real_off_q[t + 1] - a.real_off_q[t];
    const int n_out = qs ? nq : ns;
    const int colsP = pad64(ns), rowsP = pad64(n_out);
    if (colsP == 0 || rowsP == 0) return;
    const u32 B = a.base_s[tf], Bq = a.base_q[tf];
    const int nu = (int)a.n_slots[tf];
    const int n_in_entries = a.slot_start[B + tf + nu] - (int)B;
    const int2* in_list = a.sup_sorted + B;                           // {row, slot}, slot-sorted
    const int2* out_list = qs ? a.qry_sorted + Bq : a.sup_sorted + B;
    const int in_row0 = a.row_off_s[t], out_row0 = qs ? a.row_off_q[t] : a.row_off_s[t];
    // positions [lo, hi) of row u's lookups in the in / out list
    auto in_seg = [&](int u, int& lo, int& hi) { lo = a.slot_start[B + tf + u] - (int)B; hi = a.slot_start[B + tf + u + 1] - (int)B; };
    auto out_seg = [&](int u, int& lo, int& hi) {
        if (qs) { lo = a.qseg_lo[B + u] - (int)Bq; hi = a.qseg_hi[B + u] - (int)Bq; }
        else in_seg(u, lo, hi);
    };
    // LDS: tile of R out-rows, 16-bit cells, row stride colsP + 2 (an odd number of words); then the two dense
    // count blocks of a batch, [R][16] and [colsP][16] 16-bit counts.  At most 64 MFMA tiles per row tile.
    const int lds_ld = colsP + 2;
    int R = rowsP;
    while (R > 32 && ((size_t)R * lds_ld * 2 + (size_t)(R + colsP) * PC_HB * 2 > (size_t)a.tile_bytes || R * colsP > 65536)) R -= 32;
    uint16_t* tile = reinterpret_cast<uint16_t*>(pc_lds);
    u32* c_out = pc_lds + (R * lds_ld) / 2;            // R * lds_ld * 2 bytes is a multiple of 16
    u32* c_in = c_out + R * PC_HB / 2;
    u32* hot_list = pc_lds;                            // lives in the tile area until the hot part is stored
    uint8_t* M = a.mat + (qs ? a.off_qs[t] : a.off_ss[t]) + (size_t)f * rowsP * colsP;
    uint8_t* Mt = (qs && a.want_sq) ? a.mat + a.off_sq[t] + (size_t)f * colsP * rowsP : nullptr;  // [colsP rows][rowsP cols]
    const int tiles_c = colsP / 32;
    bool ovf = false;
    for (int i0 = 0; i0 < rowsP; i0 += R) {
        const int rows_here = min(R, rowsP - i0);
        const int n_tiles = (rows_here / 32) * tiles_c;
        // ---- the hot rows of this (task, field)
        if (threadIdx.x == 0) sh_nhot = 0;
        __syncthreads();
        for (int u = threadIdx.x; u < nu; u += PC_NT) {
            int lo, hi, lo2, hi2;
            in_seg(u, lo, hi);
            out_seg(u, lo2, hi2);
            if (hi - lo >= PC_HOT || hi2 - lo2 >= PC_HOT) hot_list[atomicAdd(&sh_nhot, 1)] = (u32)u;
        }
        __syncthreads();
        const int nhot = sh_nhot;
        ph_float16 acc[PC_TPW];
#pragma unroll
        for (int q = 0; q < PC_TPW; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
        for (int hb = 0; hb < nhot; hb += PC_HB) {
            for (int i = threadIdx.x; i < (R + colsP) * PC_HB / 8; i += PC_NT)   // both count blocks, contiguous
                reinterpret_cast<uint4*>(c_out)[i] = make_uint4(0u, 0u, 0u, 0u);
            __syncthreads();
            for (int hx = wv; hx < PC_HB && hb + hx < nhot; hx += PC_NT / 64) {
                const int u = (int)hot_list[hb + hx];
                const u32 inc = 1u << (16 * (hx & 1));
                int lo, hi;
                in_seg(u, lo, hi);
                for (int e = lo + lane; e < hi; e += 64) {
                    const int j = in_list[e].x - in_row0;
                    atomicAdd(&c_in[(j * PC_HB + hx) >> 1], inc);
                }
                out_seg(u, lo, hi);
                for (int e = lo + lane; e < hi; e += 64) {
                    const int i = out_list[e].x - out_row0 - i0;
                    if ((unsigned)i < (unsigned)rows_here) atomicAdd(&c_out[(i * PC_HB + hx) >> 1], inc);
                }
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < PC_TPW; ++q) {
                const int tt = wv * PC_TPW + q;
                if (tt < n_tiles) {
                    const int tr = tt / tiles_c, tc = tt - tr * tiles_c;
                    const uint4 qa = *reinterpret_cast<const uint4*>(c_out + ((tr * 32 + ln) * PC_HB + h * 8) / 2);
                    const uint4 qb = *reinterpret_cast<const uint4*>(c_in + ((tc * 32 + ln) * PC_HB + h * 8) / 2);
                    acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pc_counts_to_bf16(qa), pc_counts_to_bf16(qb), acc[q], 0, 0, 0);
                }
            }
            __syncthreads();
        }
        // ---- the hot part becomes the tile's initial content (every cell of the tile's rows is written)
#pragma unroll
        for (int q = 0; q < PC_TPW; ++q) {
            const int tt = wv * PC_TPW + q;
            if (tt < n_tiles) {
                const int tr = tt / tiles_c, tc = tt - tr * tiles_c;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = tr * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                    tile[i * lds_ld + tc * 32 + ln] = (uint16_t)fminf(acc[q][v], PC_CLAMP);
                }
            }
        }
        __syncthreads();
        // ---- the other rows, pair by pair (a lookup of the in-set walks the row's few lookups of the out-set)
        for (int p = threadIdx.x; p < n_in_entries; p += PC_NT) {
            const int2 e = in_list[p];
            const int u = e.y, j = e.x - in_row0;
            int lo, hi, lo2, hi2;
            in_seg(u, lo, hi);
            out_seg(u, lo2, hi2);
            if (hi - lo >= PC_HOT || hi2 - lo2 >= PC_HOT) continue;
            const u32 inc = 1u << (16 * (j & 1));
            for (int x = lo2; x < hi2; ++x) {
                const int i = out_list[x].x - out_row0 - i0;
                if ((unsigned)i < (unsigned)rows_here) atomicAdd(&pc_lds[(i * lds_ld + j) >> 1], inc);
            }
        }
        __syncthreads();
        // ---- rows [i0, i0 + rows_here) of M, four counts per store
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

void launch_pair_count(hipStream_t st, PairCountArgs a, int Tw) {
    if (Tw <= 0 || a.F <= 0) return;
    a.tile_bytes = PAIR_LDS_BYTES;
    (void)hipFuncSetAttribute((const void*)pair_count_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, PAIR_LDS_BYTES);
    hipLaunchKernelGGL(pair_count_kernel, dim3(a.F, Tw, 2), dim3(PC_NT), PAIR_LDS_BYTES, st, a);
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

__device__ __forceinline__ u32 ph_pack_hi(u32 e0, u32 e1) {  // {e1[31:16], e0[31:16]}
    return __builtin_amdgcn_perm(e1, e0, 0x07060302u);
}

// four counts (bytes of x) -> four bf16 (exact for 0..255)
__device__ __forceinline__ void ph_cvt4(u32 x, u32& lo, u32& hi) {
    const float f0 = (float)(x & 0xFFu), f1 = (float)((x >> 8) & 0xFFu), f2 = (float)((x >> 16) & 0xFFu), f3 = (float)(x >> 24);
    lo = ph_pack_hi(__builtin_bit_cast(u32, f0), __builtin_bit_cast(u32, f1));
    hi = ph_pack_hi(__builtin_bit_cast(u32, f2), __builtin_bit_cast(u32, f3));
}

// LDS layout of the staged chunk: per (piece, column) 64 contraction values = eight 16-byte groups; group g of
// column c sits at position g ^ key(c).  With this key both the 16-byte fragment reads (32 consecutive columns,
// one group) and the staging writes (every fourth column, one group) spread over all banks.
__device__ __forceinline__ int ph_key(int col) { return ((col >> 1) + (col >> 4)) & 7; }

template <int DS>
__global__ __launch_bounds__(256) void pair_hop_kernel(PairHopArgs a) {
    constexpr int NCT = DS / 32;      // 32-column tiles
    constexpr int CG = DS / 4;        // float4 column groups of a row of Z
    constexpr int RPT = CG / 4;       // rows of the 64-row chunk staged per thread (256 threads)
    __shared__ __attribute__((aligned(16))) bf16_t zs[3 * DS * PH_KC];
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
    // a wave without rows multiplies rows 0..63 (valid memory) and stores nothing: the loop stays free of branches
    const uint8_t* Mw = M + (size_t)((wave_on ? row_w : 0) + ln) * colsP + h * 32;

    int wr_off[4];   // element offsets of this thread's staging writes, per column of its float4
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        const int col = cg * 4 + cc, k0 = rg * RPT;
        wr_off[cc] = col * PH_KC + (((k0 >> 3) ^ ph_key(col)) << 3) + (k0 & 7);
    }
    int rd_key[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) rd_key[ct] = ph_key(ct * 32 + ln);

    ph_float16 acc[2][NCT];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][ct][v] = 0.f;

    float4 z[RPT];
    uint4 araw[2][2], anext[2][2];
    auto load_z = [&](int kc) {
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int row = kc + rg * RPT + r;
            z[r] = row < n_in ? *reinterpret_cast<const float4*>(Zt + (int64_t)row * a.ldz) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto load_a = [&](int kc, uint4 (&dst)[2][2]) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const uint4* src = reinterpret_cast<const uint4*>(Mw + (size_t)(s * 32) * colsP + kc);
            dst[s][0] = src[0];
            dst[s][1] = src[1];
        }
    };
    if (colsP > 0) {
        load_z(0);
        load_a(0, araw);
    }
    for (int kc = 0; kc < colsP; kc += PH_KC) {
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
                bf16_t* d0 = zs + wr_off[cc];
                bf16_t* d1 = d0 + DS * PH_KC;
                bf16_t* d2 = d1 + DS * PH_KC;
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
        // the next chunk's loads fly while this one is multiplied (the last chunk loads itself again)
        const int kn = kc + PH_KC < colsP ? kc + PH_KC : kc;
        load_z(kn);
        load_a(kn, anext);
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
            for (int ct = 0; ct < NCT; ++ct) {
                const bf16_t* src = zs + (ct * 32 + ln) * PH_KC + (((h * 4 + ks) ^ rd_key[ct]) << 3);
#pragma unroll
                for (int sp = 2; sp >= 0; --sp) {  // smallest pieces first
                    const ph_short8 bfrag = *reinterpret_cast<const ph_short8*>(src + sp * DS * PH_KC);
#pragma unroll
                    for (int s = 0; s < 2; ++s)
                        acc[s][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s], bfrag, acc[s][ct], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) { araw[s][0] = anext[s][0]; araw[s][1] = anext[s][1]; }
    }
    if (!wave_on) return;
    // D layout of the 32x32 tile: register v of lane (ln, h) is row 8*(v/4) + 4*h + v%4, column ln
    const int64_t base = ((int64_t)out.row_off[t] + row_w) * out.ld + colz + ln;
    const float* yin = out.y_in ? out.y_in + base : nullptr;
    float* yout = out.y_out ? out.y_out + base : nullptr;
    bf16_t* ybf = out.y_bf ? out.y_bf + base : nullptr;
    const int ldo = (int)out.ld;
    const float cc = out.c;
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = s * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (row_w + rl >= n_out) continue;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const int idx = rl * ldo + ct * 32;
                const float y = (yin ? yin[idx] : 0.f) + cc * acc[s][ct][v];
                if (yout) yout[idx] = y;
                if (ybf) ybf[idx] = f2bf(y);
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
