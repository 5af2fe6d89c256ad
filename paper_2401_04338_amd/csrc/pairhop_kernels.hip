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

__host__ __device__ __forceinline__ int pad64(int n) { return (n + 63) & ~63; }

// ------------------------------------------------------------------------------------------------
// counting: M[i][j] for one (task, field) and one pair of sets, in tiles of out-rows held in LDS
//
// M = sum over the rows u of the task's support set of  c_out(:, u) (x) c_in(:, u),  with c_set(b, u) the
// number of times bag b looks row u up.  Under a skewed row distribution a few hot rows carry nearly all
// of the pairs (a row looked up a times by one set and b times by the other adds a*b of them), and LDS
// atomics retire only about one lane per cycle, so the hot rows do not go through pair-by-pair atomics:
// PC_HB hot rows at a time, their count vectors are laid out densely ([bags, PC_HB] bytes, one atomic per
// lookup) and multiplied on the matrix cores as 8-bit integers (v_mfma_i32_32x32x32_i8: a count is at
// most the bag's length, which this path limits to 127; sums are exact in 32 bits).
// Only the remaining rows (fewer than PC_HOT lookups from either set, at most 9 pairs each) are counted
// pair by pair with atomics on the byte cells, on top of the stored hot part.  Everything is integer
// arithmetic: the result does not depend on any order.
//
// The kernel is bound by latency, not by arithmetic, so everything it walks more than once is staged in
// LDS when the workgroup starts: the bag of every lookup of both lists (16 bits each) and one record per
// row with pairs (hot: the bounds of its two lookup ranges; cold: packed starts and sizes).  After that
// only LDS is read until the matrix is written out.
// ------------------------------------------------------------------------------------------------
#define PC_TPW 4          // MFMA tiles per wave: a workgroup of NT threads covers NT / 16 tiles per row tile
#define PC_SMALL_ROWS 128 // samples per set of a 'small' task: 16 tiles, four waves
#define PC_SMALL_N 1984   // lookups per set of a 'small' (task, field)
#define PC_HB 32     // hot rows per matrix-core batch (one MFMA contraction step)
#define PC_HBS 48    // bytes per bag in a count block (16-byte fragment reads; 12 words spread them over the banks)
#define PC_HOT 4     // a row is hot when one of the two sets looks it up at least this often

typedef int pc_int4 __attribute__((ext_vector_type(4)));
typedef int pc_int16 __attribute__((ext_vector_type(16)));

template <int NT>
__global__ __launch_bounds__(NT) void pair_count_kernel(PairCountArgs a) {
    extern __shared__ __attribute__((aligned(16))) u32 pc_lds[];
    __shared__ int sh_nhot, sh_ncold;
    const int f = blockIdx.x, t = blockIdx.y;
    const bool qs = blockIdx.z == 1;   // 0: support x support, 1: query x support (and its transpose)
    if (!qs && !a.want_ss) return;
    if (!a.task_path[t]) return;
    const size_t tf = (size_t)t * a.F + f;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, ln = lane & 31, h = lane >> 5;
    const int ns = a.real_off_s[t + 1] - a.real_off_s[t], nq = a.real_off_q[t + 1] - a.real_off_q[t];
    const int n_out = qs ? nq : ns;
    const int colsP = pad64(ns), rowsP = pad64(n_out);
    if (colsP == 0 || rowsP == 0) return;
    const u32 B = a.base_s[tf], Bq = a.base_q[tf];
    const int nu = (int)a.n_slots[tf];
    const int n_in_entries = a.slot_start[B + tf + nu] - (int)B;
    const int n_out_entries = qs ? (int)a.cnt_q[tf] : n_in_entries;
    if (a.cls) {   // uneven tasks: the small (task, field)s have a launch of their own, with small workgroups
        const bool small = max(ns, nq) <= PC_SMALL_ROWS && max(n_in_entries, n_out_entries) <= a.small_n;
        if (small != (a.cls == 1)) return;
    }
    // LDS, from the end (6 * n_max bytes): the bag of every out lookup and of every in lookup (16 bits each, in the
    // order of the row-sorted lists; one array when both sets are the support set), then the records: hot rows
    // from the front (two words: in range, out range), cold rows with pairs from the back (one word).
    // From the start: the tile of R out-rows, TRANSPOSED, one byte per cell: cell (i, j) at j * ldT + i with
    // ldT = R + 4 (an odd number of words: the MFMA result, the transposed read-out and the atomics all spread
    // over the banks); then the two dense count blocks of a batch, [R] and [colsP] bags of PC_HBS bytes.
    const int nmax = a.n_max;                                  // a multiple of 8
    uint16_t* out_rows = reinterpret_cast<uint16_t*>(pc_lds) + (a.lds_bytes / 2 - nmax);
    uint16_t* in_rows = qs ? out_rows - nmax : out_rows;
    const int RW = qs ? nmax / 2 : nmax;                       // record words
    u32* recs = reinterpret_cast<u32*>(in_rows) - RW;
    if (threadIdx.x == 0) { sh_nhot = 0; sh_ncold = 0; }
    __syncthreads();
    {
        // eight loads in flight per thread and list: the workgroup has the compute unit to itself, so nothing else hides
        // the latency of these first reads
        auto stage_rows = [&](const int2* list, int n_entries, int row0, uint16_t* dst) {
            for (int e0 = threadIdx.x; e0 < n_entries; e0 += 8 * NT) {
                int r[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) r[q] = list[min(e0 + q * NT, n_entries - 1)].x;
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (e0 + q * NT < n_entries) dst[e0 + q * NT] = (uint16_t)(r[q] - row0);
            }
        };
        stage_rows(a.sup_sorted + B, n_in_entries, a.row_off_s[t], in_rows);   // {row, slot}, slot-sorted
        if (qs) stage_rows(a.qry_sorted + Bq, n_out_entries, a.row_off_q[t], out_rows);
    }
    for (int u0 = threadIdx.x; u0 < nu; u0 += 4 * NT) {   // (the loads of four rows in flight per thread)
        int lo_[4], hi_[4], lo2_[4], hi2_[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int u = min(u0 + q * NT, nu - 1);
            lo_[q] = a.slot_start[B + tf + u] - (int)B;
            hi_[q] = a.slot_start[B + tf + u + 1] - (int)B;
            lo2_[q] = lo_[q]; hi2_[q] = hi_[q];
            if (qs) { lo2_[q] = a.qseg_lo[B + u] - (int)Bq; hi2_[q] = a.qseg_hi[B + u] - (int)Bq; }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (u0 + q * NT >= nu) continue;
            const int lo = lo_[q], hi = hi_[q], lo2 = lo2_[q], hi2 = hi2_[q];
            const int na = hi - lo, nb = hi2 - lo2;
            if (na <= 0 || nb <= 0) continue;
            if (na >= PC_HOT || nb >= PC_HOT) {
                const int k = atomicAdd(&sh_nhot, 1);
                if (2 * k + 1 < RW) {
                    recs[2 * k] = (u32)lo | ((u32)hi << 16);
                    recs[2 * k + 1] = (u32)lo2 | ((u32)hi2 << 16);
                }
            } else {
                const int k = atomicAdd(&sh_ncold, 1);
                if (k < RW) recs[RW - 1 - k] = (u32)lo | ((u32)lo2 << 14) | ((u32)na << 28) | ((u32)nb << 30);
            }
        }
    }
    __syncthreads();
    const int nhot = sh_nhot, ncold = sh_ncold;
    if (2 * nhot + ncold > RW) {   // the records do not fit (they may have overwritten each other): sparse kernel
        if (threadIdx.x == 0) {
            a.task_path[t] = 0u;
            a.status[ST_PAIR_OVF] = 1u;
        }
        return;
    }
    const size_t budget = (size_t)a.lds_bytes - 6 * (size_t)nmax;
    int R = min(rowsP, a.max_tile_rows);   // at most 64 MFMA tiles per row tile
    while (R > 32 && ((size_t)colsP * (R + 4) + (size_t)(R + colsP) * PC_HBS > budget || R * colsP > NT * 64)) R -= 32;
    if ((size_t)colsP * (R + 4) + (size_t)(R + colsP) * PC_HBS > budget) {   // not even 32 rows fit: sparse kernel
        if (threadIdx.x == 0) {
            a.task_path[t] = 0u;
            a.status[ST_PAIR_OVF] = 1u;
        }
        return;
    }
    const int ldT = R + 4;
    uint8_t* tile = reinterpret_cast<uint8_t*>(pc_lds);
    uint8_t* c_out = tile + (size_t)colsP * ldT;   // colsP * ldT is a multiple of 16
    uint8_t* c_in = c_out + R * PC_HBS;
    uint8_t* M = a.mat + (qs ? a.off_qs[t] : a.off_ss[t]) + (size_t)f * rowsP * colsP;
    uint8_t* Mt = (qs && a.want_sq) ? a.mat + a.off_sq[t] + (size_t)f * colsP * rowsP : nullptr;  // [colsP rows][rowsP cols]
    const int tiles_c = colsP / 32;
    bool ovf = false;
    for (int i0 = 0; i0 < rowsP; i0 += R) {
        const int rows_here = min(R, rowsP - i0);
        const int n_tiles = (rows_here / 32) * tiles_c;
        int my_tr[PC_TPW], my_tc[PC_TPW];
#pragma unroll
        for (int q = 0; q < PC_TPW; ++q) {
            const int tt = wv * PC_TPW + q;
            my_tr[q] = tt < n_tiles ? tt / tiles_c : -1;
            my_tc[q] = tt - (tt / tiles_c) * tiles_c;
        }
        pc_int16 acc[PC_TPW];
#pragma unroll
        for (int q = 0; q < PC_TPW; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[q][v] = 0;
        for (int hb = 0; hb < nhot; hb += PC_HB) {
            __syncthreads();   // the previous batch's fragments (or the previous tile) have been read
            for (int i = threadIdx.x; i < (R + colsP) * PC_HBS / 16; i += NT)   // both count blocks, contiguous
                reinterpret_cast<uint4*>(c_out)[i] = make_uint4(0u, 0u, 0u, 0u);
            __syncthreads();
            // one atomic per lookup (a count is at most the bag's length); a wave per hot row
            for (int hx = wv; hx < PC_HB && hb + hx < nhot; hx += NT / 64) {
                const u32 r0 = recs[2 * (hb + hx)], r1 = recs[2 * (hb + hx) + 1];
                const u32 inc = 1u << (8 * (hx & 3));
                for (int e = (int)(r0 & 0xFFFFu) + lane; e < (int)(r0 >> 16); e += 64)
                    atomicAdd(reinterpret_cast<u32*>(c_in) + (((int)in_rows[e] * PC_HBS + hx) >> 2), inc);
                for (int e = (int)(r1 & 0xFFFFu) + lane; e < (int)(r1 >> 16); e += 64) {
                    const int i = (int)out_rows[e] - i0;
                    if ((unsigned)i < (unsigned)rows_here) atomicAdd(reinterpret_cast<u32*>(c_out) + ((i * PC_HBS + hx) >> 2), inc);
                }
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < PC_TPW; ++q) {
                if (my_tr[q] >= 0) {
                    const pc_int4 qa = *reinterpret_cast<const pc_int4*>(c_out + (my_tr[q] * 32 + ln) * PC_HBS + h * 16);
                    const pc_int4 qb = *reinterpret_cast<const pc_int4*>(c_in + (my_tc[q] * 32 + ln) * PC_HBS + h * 16);
                    acc[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(qa, qb, acc[q], 0, 0, 0);
                }
            }
        }
        // ---- the hot part becomes the tile's initial content (every cell of the tile's rows is written); a lane
        //      holds four consecutive rows of one column: one word of the transposed tile.  255 stands for
        //      "255 or more" and is reported when the tile is read out.
        __syncthreads();   // the previous tile has been read out
#pragma unroll
        for (int q = 0; q < PC_TPW; ++q) {
            if (my_tr[q] >= 0) {
                uint8_t* col = tile + (size_t)(my_tc[q] * 32 + ln) * ldT + my_tr[q] * 32 + 4 * h;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const u32 b0 = min((u32)acc[q][4 * g + 0], 255u), b1 = min((u32)acc[q][4 * g + 1], 255u);
                    const u32 b2 = min((u32)acc[q][4 * g + 2], 255u), b3 = min((u32)acc[q][4 * g + 3], 255u);
                    *reinterpret_cast<u32*>(col + 8 * g) = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
                }
            }
        }
        __syncthreads();
        // ---- the other rows, pair by pair; a cell that was at 254 or more before an increment may have
        //      wrapped: reported
        for (int k = threadIdx.x; k < ncold; k += NT) {
            const u32 r = recs[RW - 1 - k];
            const int lo = (int)(r & 0x3FFFu), lo2 = (int)((r >> 14) & 0x3FFFu), na = (int)((r >> 28) & 3u), nb = (int)(r >> 30);
            for (int y = 0; y < nb; ++y) {
                const int i = (int)out_rows[lo2 + y] - i0;
                if ((unsigned)i >= (unsigned)rows_here) continue;
                const int sh = 8 * (i & 3);
                for (int x = 0; x < na; ++x) {
                    const int j = (int)in_rows[lo + x];
                    const u32 old = atomicAdd(&pc_lds[(j * ldT + i) >> 2], 1u << sh);
                    ovf |= ((old >> sh) & 0xFFu) >= 254u;
                }
            }
        }
        __syncthreads();
        // ---- rows [i0, i0 + rows_here) of M.  A thread takes a 4 x 4 block of cells: four words of the transposed tile
        //      (four rows of one column each), turned in registers into four words of M (four columns of one row each).
        //      Of a wave, 16 lanes lie along the columns and 4 along the rows: the tile reads then spread over all
        //      banks (a column step moves 4 banks, a row step 1), and every row gets 64 contiguous bytes per store.
        {
            const int jl = lane & 15, il = lane >> 4;
            const int pj_n = colsP / 64, n_patches = pj_n * (rows_here / 16);
            for (int wq = wv; wq < n_patches; wq += NT / 64) {
                const int pj = wq % pj_n, pi = wq / pj_n;
                const int j4 = (pj * 16 + jl) * 4, i4 = (pi * 4 + il) * 4;
                const u32 ca = *reinterpret_cast<const u32*>(tile + (j4 + 0) * ldT + i4), cb = *reinterpret_cast<const u32*>(tile + (j4 + 1) * ldT + i4);
                const u32 cc = *reinterpret_cast<const u32*>(tile + (j4 + 2) * ldT + i4), cd = *reinterpret_cast<const u32*>(tile + (j4 + 3) * ldT + i4);
                // a byte of 255: some byte of the complement is zero
                const u32 na_ = ~ca, nb_ = ~cb, nc_ = ~cc, nd_ = ~cd;
                ovf |= (((na_ - 0x01010101u) & ca & 0x80808080u) | ((nb_ - 0x01010101u) & cb & 0x80808080u) |
                        ((nc_ - 0x01010101u) & cc & 0x80808080u) | ((nd_ - 0x01010101u) & cd & 0x80808080u)) != 0u;
                const u32 t0 = __builtin_amdgcn_perm(cb, ca, 0x05010400u), t1 = __builtin_amdgcn_perm(cb, ca, 0x07030602u);
                const u32 u0 = __builtin_amdgcn_perm(cd, cc, 0x05010400u), u1 = __builtin_amdgcn_perm(cd, cc, 0x07030602u);
                u32* dst = reinterpret_cast<u32*>(M + (size_t)(i0 + i4) * colsP + j4);
                const size_t rw = (size_t)colsP / 4;
                dst[0] = __builtin_amdgcn_perm(u0, t0, 0x05040100u);
                dst[rw] = __builtin_amdgcn_perm(u0, t0, 0x07060302u);
                dst[2 * rw] = __builtin_amdgcn_perm(u1, t1, 0x05040100u);
                dst[3 * rw] = __builtin_amdgcn_perm(u1, t1, 0x07060302u);
            }
        }
        if (Mt) {  // the transpose is the tile as it lies: row j holds columns [i0, i0 + rows_here)
            const int gpr = rows_here / 4;
            for (int w = threadIdx.x; w < colsP * gpr; w += NT) {
                const int j = w / gpr, i4 = (w - j * gpr) * 4;
                *reinterpret_cast<u32*>(Mt + (size_t)j * rowsP + i0 + i4) = *reinterpret_cast<const u32*>(tile + j * ldT + i4);
            }
        }
    }
    if (ovf) {   // this task goes to the sparse kernel
        a.task_path[t] = 0u;
        a.status[ST_PAIR_OVF] = 1u;
    }
}

// max_tf: the most lookups any (task, field) of the wave has in one set; max_rows: the most samples any
// counted task has in one set
template <int NT>
static void launch_pair_count_nt(hipStream_t st, PairCountArgs a, int Tw, int max_tf, int max_rows) {
    a.n_max = (max_tf + 7) / 8 * 8 + 8;
    // LDS: what the largest (task, field) needs for one tile of all its rows, or all there is
    const size_t P = (size_t)pad64(max_rows > 0 ? max_rows : 1);
    const size_t R = P < (size_t)a.max_tile_rows ? P : (size_t)a.max_tile_rows;
    size_t need = 6 * (size_t)a.n_max + P * (R + 4) + (R + P) * PC_HBS + 64;
    if (need > PAIR_LDS_BYTES) need = PAIR_LDS_BYTES;
    a.lds_bytes = (int)(need / 16 * 16);
    (void)hipFuncSetAttribute((const void*)pair_count_kernel<NT>, hipFuncAttributeMaxDynamicSharedMemorySize, PAIR_LDS_BYTES);
    hipLaunchKernelGGL(pair_count_kernel<NT>, dim3(a.F, Tw, 2), dim3(NT), (size_t)a.lds_bytes, st, a);
}

// max_rows / min_rows: the most / fewest samples any counted task has in one set (the larger of its two sets)
void launch_pair_count(hipStream_t st, PairCountArgs a, int Tw, int max_tf, int max_rows, int min_rows, int max_tile_rows) {
    if (Tw <= 0 || a.F <= 0) return;
    a.max_tile_rows = max_tile_rows > 0 ? (max_tile_rows + 31) / 32 * 32 : 1 << 20;
    a.small_n = PC_SMALL_N;
    if (max_rows <= PC_SMALL_ROWS && max_tf <= PC_SMALL_N) {   // every task is small
        a.cls = 0;
        launch_pair_count_nt<256>(st, a, Tw, max_tf, max_rows);
    } else if (max_rows > 2 * PC_SMALL_ROWS && min_rows <= PC_SMALL_ROWS && (int64_t)Tw * a.F >= 32) {   // uneven: two launches, each workgroup checks its class
        a.cls = 1;
        launch_pair_count_nt<256>(st, a, Tw, max_tf < PC_SMALL_N ? max_tf : PC_SMALL_N, PC_SMALL_ROWS);
        a.cls = 2;
        launch_pair_count_nt<1024>(st, a, Tw, max_tf, max_rows);
    } else {
        a.cls = 0;
        launch_pair_count_nt<1024>(st, a, Tw, max_tf, max_rows);
    }
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
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void pair_hop_kernel(PairHopArgs a) {
    constexpr int NCT = DS / 32;      // 32-column tiles
    constexpr int CG = DS / 4;        // float4 column groups of a row of Z
    constexpr int RPT = CG / 4;       // rows of the 64-row chunk staged per thread (256 threads)
    __shared__ __attribute__((aligned(16))) bf16_t zs[2 * 3 * DS * PH_KC];
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): re-number them so that the
    // workgroups of one (task, field, column slice) -- both out sets, all row blocks: they read the same rows of
    // Z -- are consecutive on one XCD.
    const int nsl = a.D / DS;
    const int per_xcd = gridDim.x >> 3;
    const int wid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (wid >= a.n_work) return;
    const int nz = a.n_out * a.row_blocks, fx = a.F * nsl;
    const int zi = wid % nz, rest = wid / nz;
    const int fs = rest % fx, t = rest / fx;
    const int f = fs / nsl, sl = fs - f * nsl;
    const int o = zi / a.row_blocks, rb = zi - o * a.row_blocks;
    const PairHopOut& out = a.out[o];
    const int n_in = a.in_real_off[t + 1] - a.in_real_off[t];
    const int n_out = out.real_off[t + 1] - out.real_off[t];
    if (rb * 256 >= n_out || !a.task_path[t]) return;
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
        for (int r = 0; r < RPT; ++r) {   // branch-free: a row beyond the task reads the task's last row and is zeroed
            const int row = kc + rg * RPT + r;
            z[r] = *reinterpret_cast<const float4*>(Zt + (int64_t)min(row, n_in - 1) * a.ldz);
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
    // splits the staged rows into their three bf16 pieces and writes them into one LDS buffer
    auto stage = [&](bf16_t* buf, int kc) {
        u32 p0[4][RPT], p1[4][RPT], p2[4][RPT];  // [column][row]: the three pieces as fp32 bit patterns
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const float keep = kc + rg * RPT + r < n_in ? 1.f : 0.f;
            const float zz[4] = {z[r].x * keep, z[r].y * keep, z[r].z * keep, z[r].w * keep};
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
            bf16_t* d0 = buf + wr_off[cc];
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
    };
    // Two LDS buffers: while chunk c is multiplied out of one, chunk c+1 (loaded during the multiplication) is
    // split into the other; one barrier per chunk.
    if (colsP > 0) {
        load_z(0);
        load_a(0, araw);
        stage(zs, 0);
    }
    __syncthreads();
    int cur = 0;
    for (int kc = 0; kc < colsP; kc += PH_KC) {
        const int kn = kc + PH_KC < colsP ? kc + PH_KC : kc;   // the last chunk loads itself again: no branches
        load_z(kn);
        load_a(kn, anext);
        __builtin_amdgcn_sched_barrier(0);   // the loads above are consumed only after the multiplication below
        const bf16_t* zb = zs + cur * (3 * DS * PH_KC);
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
            ph_short8 bfrag[NCT][3];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const bf16_t* src = zb + (ct * 32 + ln) * PH_KC + (((h * 4 + ks) ^ rd_key[ct]) << 3);
#pragma unroll
                for (int sp = 0; sp < 3; ++sp) bfrag[ct][sp] = *reinterpret_cast<const ph_short8*>(src + sp * DS * PH_KC);
            }
#pragma unroll
            for (int sp = 2; sp >= 0; --sp)  // smallest pieces first
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
                    for (int s = 0; s < 2; ++s)
                        acc[s][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s], bfrag[ct][sp], acc[s][ct], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        cur ^= 1;
        stage(zs + cur * (3 * DS * PH_KC), kn);
#pragma unroll
        for (int s = 0; s < 2; ++s) { araw[s][0] = anext[s][0]; araw[s][1] = anext[s][1]; }
        __syncthreads();
    }
    if (!wave_on) return;
    // D layout of the 32x32 tile: register v of lane (ln, h) is row 8*(v/4) + 4*h + v%4, column ln
    const int64_t base = ((int64_t)out.row_off[t] + row_w) * out.ld + colz + ln;
    const float* yin = out.y_in ? out.y_in + base : nullptr;
    float* yout = out.y_out ? out.y_out + base : nullptr;
    bf16_t* ybf = out.y_bf ? out.y_bf + base : nullptr;
    const int ldo = (int)out.ld;
    const float cc = out.c;
    // y_in may be y_out: the loads of a 32x32 tile are issued together, ahead of its stores
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            float yv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rl = s * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                yv[v] = (yin && row_w + rl < n_out) ? yin[rl * ldo + ct * 32] : 0.f;
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rl = s * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row_w + rl >= n_out) continue;
                const int idx = rl * ldo + ct * 32;
                const float y = yv[v] + cc * acc[s][ct][v];
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
    a.n_out = n_out;
    const int ds = a.D % 64 == 0 ? 64 : 32;
    const int64_t n_work = (int64_t)a.F * (a.D / ds) * Tw * n_out * a.row_blocks;
    if (n_work >= ((int64_t)1 << 31) - 8) return;   // cannot happen within the library's own limits on a call
    a.n_work = (int)n_work;
    const unsigned grid = (unsigned)((n_work + 7) / 8 * 8);
    if (ds == 64) hipLaunchKernelGGL(pair_hop_kernel<64>, dim3(grid), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(pair_hop_kernel<32>, dim3(grid), dim3(256), 0, st, a);
}
