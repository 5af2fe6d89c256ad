// Task-local embedding-row arithmetic of the MAML step without a row table in HBM.
//
// Every row-space operation of the inner loop and of the second-order chain (G-Meta Alg. 1: local
// back-propagation on xi^Sup, the overlap update of Sec. 2.1.2, and their tangents) has the form
//     Y[bag] (+)= c * sum over the bag's lookups of  G[slot of the lookup],
//     G[slot]  =      sum over the lookups of that slot of  Z[row of the lookup's sample, field]
// for one (task, field) at a time, where a slot is a distinct row of the task's support set.  One
// workgroup owns one (task, field).  For one range of slots at a time it
//   hop 1: cuts the range's lookups (contiguous in the slot-sorted list) into equal position chunks,
//          one lane group per chunk; a run of equal slots inside a chunk goes straight to G in LDS,
//          the first and last run of every chunk become records that a join adds in chunk order
//          (so a hot row's run is summed by many groups, yet always in the same order);
//   hop 2: adds G into the pooled vectors of the task's support and/or query bags, which live in
//          registers across the slot ranges (the bag's lookups left to right).
// HBM sees one read of Z and one read/write of Y per (sample, field) plus a few bytes per lookup; the
// per-lookup 4*D bytes stay in LDS.  Every order of summation is fixed: results are bit-reproducible.
// The work of a (task, field) is latency-bound (short dependent chains of loads between barriers), so
// it is also split by COLUMN SLICES of the embedding dimension (blockIdx.z): small workgroups with a
// small LDS footprint, several of which share a compute unit and hide each other's stalls.
#include "gm_internal.h"

__device__ __forceinline__ float4 th_add(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

template <int MAXB, int DC, int NT, bool STAGE_Z>
__global__ __launch_bounds__(NT) void two_hop_kernel(TwoHopArgs a) {
    extern __shared__ __attribute__((aligned(16))) float th_lds[];
    constexpr int D = DC, LG = DC / 4;   // D: columns of this slice (DC of the a.D embedding columns)
    constexpr int NIDS = LG >= 16 ? 2 : 32 / LG;  // slot ids of the first NIDS*LG lookups of a bag stay in registers
    const int F = a.F;
    const int groups = blockDim.x / LG;
    float* G = th_lds;                                        // [range][D]
    float* rec_vec = th_lds + (size_t)a.range * D;            // [groups*2][D]
    int* rec_slot = reinterpret_cast<int*>(rec_vec + (size_t)groups * 2 * D);  // [groups*2]
    float* Zs = reinterpret_cast<float*>(rec_slot + groups * 2);               // [rows of the task][D]: this slice of Z
    const int f = blockIdx.x, t = blockIdx.y;
    if (a.task_path && a.task_path[t]) return;   // the pair-count kernels own this task
    const int tf = t * F + f;
    const int g = threadIdx.x / LG, l = threadIdx.x % LG;
    const int lane = threadIdx.x & 63, gbase = lane & ~(LG - 1);
    const bool active = g < groups;
    const int nu = (int)a.n_slots[tf];
    const int64_t B = a.tf_base[tf];
    const int64_t sb = B + (int64_t)tf * a.in_seg_tf_stride;
    const int64_t colz = (int64_t)f * a.D + (int64_t)blockIdx.z * DC + l * 4;

    // this column slice of the task's rows of Z, staged once: hop 1 then reads LDS only
    const int zrow0 = STAGE_Z ? a.in_row_offsets[t] : 0, zrows = STAGE_Z ? a.in_row_offsets[t + 1] - zrow0 : 0;
    for (int i = threadIdx.x; i < zrows * LG; i += blockDim.x) {
        const int r = i / LG, cq = i - r * LG;
        reinterpret_cast<float4*>(Zs)[i] =
            *reinterpret_cast<const float4*>(a.Z + (int64_t)(zrow0 + r) * a.ldz + (int64_t)f * a.D + (int64_t)blockIdx.z * DC + cq * 4);
    }

    // the bags this group owns in each output set: lookup range and (cached) slot ids
    int nb[2] = {0, 0};
    int64_t s_lo[2] = {0, 0};
    int32_t p0[2][MAXB], plen[2][MAXB], ids[2][MAXB][NIDS];
    float4 acc[2][MAXB];
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        const TwoHopOut& out = a.out[o];
        if (!out.enabled) continue;
        s_lo[o] = out.real_offsets[t];
        nb[o] = out.real_offsets[t + 1] - out.real_offsets[t];
#pragma unroll
        for (int i = 0; i < MAXB; ++i) {
            acc[o][i] = make_float4(0.f, 0.f, 0.f, 0.f);
            const int j = a.bag0 + g + i * groups;
            p0[o][i] = 0;
            plen[o][i] = 0;
            if (active && j < nb[o]) {
                const int64_t bag = (out.sample0 + s_lo[o] + j) * F + f;
                const int64_t q0 = out.bag_offsets[bag];
                p0[o][i] = (int32_t)(q0 - out.lookup0);
                plen[o][i] = (int32_t)(out.bag_offsets[bag + 1] - q0);
            }
        }
#pragma unroll
        for (int i = 0; i < MAXB; ++i)
#pragma unroll
            for (int k = 0; k < NIDS; ++k)
                ids[o][i][k] = k * LG + l < plen[o][i] ? out.slot_of_lookup[p0[o][i] + k * LG + l] : -1;
    }

    for (int u0 = 0; u0 < nu; u0 += a.range) {
        const int u1 = min(nu, u0 + a.range);
        // ---- hop 1
        for (int i = threadIdx.x; i < (u1 - u0) * LG; i += blockDim.x)
            reinterpret_cast<float4*>(G)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        const int P0 = a.in_seg_lo[sb + u0], P1 = a.in_seg_hi[sb + u1 - 1];
        const int C = (P1 - P0 + groups - 1) / groups;
        int first_slot = -1, last_slot = -1;
        float4 first_vec = make_float4(0.f, 0.f, 0.f, 0.f), last_vec = first_vec;
        __syncthreads();
        if (active && C > 0) {
            const int ca = P0 + g * C, cb = min(P1, ca + C);
            int cur = -1;
            bool is_first = true;
            float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
            auto close_run = [&]() {
                if (cur < 0) return;
                if (is_first) { first_slot = cur; first_vec = s; is_first = false; }
                else *reinterpret_cast<float4*>(G + (size_t)(cur - u0) * D + l * 4) = s;
            };
            constexpr int NE = LG >= 16 ? 1 : (LG >= 8 ? 2 : 4);  // entries per lane and batch, fetched with independent loads
            constexpr int EB = LG < 4 ? LG : 4;                      // rows of Z in flight per lane
            for (int i0 = ca; i0 < cb; i0 += NE * LG) {
                int2 mine[NE];
#pragma unroll
                for (int k = 0; k < NE; ++k)
                    mine[k] = (i0 + k * LG + l < cb) ? a.in_sorted[i0 + k * LG + l] : make_int2(0, -1);
#pragma unroll
                for (int k = 0; k < NE; ++k) {
                    const int cnt = min(LG, cb - (i0 + k * LG));
                    for (int e0 = 0; e0 < cnt; e0 += EB) {
                        int rw[EB], sl[EB];
                        float4 z[EB];
#pragma unroll
                        for (int e = 0; e < EB; ++e) {
                            rw[e] = __shfl(mine[k].x, gbase + ((e0 + e) & (LG - 1)), 64);
                            sl[e] = __shfl(mine[k].y, gbase + ((e0 + e) & (LG - 1)), 64);   // -1 beyond the chunk's end
                            if (e0 + e >= cnt) sl[e] = -1;
                        }
#pragma unroll
                        for (int e = 0; e < EB; ++e)
                            if (sl[e] >= 0)
                                z[e] = STAGE_Z ? *reinterpret_cast<const float4*>(Zs + (size_t)(rw[e] - zrow0) * D + l * 4)
                                               : *reinterpret_cast<const float4*>(a.Z + (int64_t)rw[e] * a.ldz + colz);
#pragma unroll
                        for (int e = 0; e < EB; ++e) {
                            if (sl[e] < 0) continue;   // a query lookup of a row the support set does not hold, or padding
                            if (sl[e] != cur) {
                                close_run();
                                cur = sl[e];
                                s = z[e];
                            } else {
                                s = th_add(s, z[e]);
                            }
                        }
                    }
                }
            }
            // the last run of the chunk (if it is also the first, it stays the only record)
            if (cur >= 0) {
                if (is_first) { first_slot = cur; first_vec = s; }
                else { last_slot = cur; last_vec = s; }
            }
        }
        if (active) {
            *reinterpret_cast<float4*>(rec_vec + (size_t)(g * 2) * D + l * 4) = first_vec;
            *reinterpret_cast<float4*>(rec_vec + (size_t)(g * 2 + 1) * D + l * 4) = last_vec;
            if (l == 0) {
                rec_slot[g * 2] = first_slot;
                rec_slot[g * 2 + 1] = last_slot;
            }
        }
        __syncthreads();
        // join: the records are in position order; the first record of every slot adds the later ones of that slot
        if (active) {
            for (int r = g * 2; r < g * 2 + 2; ++r) {
                const int slot = rec_slot[r];
                if (slot < 0) continue;
                int prev = r - 1;
                while (prev >= 0 && rec_slot[prev] < 0) --prev;
                if (prev >= 0 && rec_slot[prev] == slot) continue;  // not the first record of its slot
                float4 s = *reinterpret_cast<const float4*>(rec_vec + (size_t)r * D + l * 4);
                for (int r2 = r + 1; r2 < groups * 2; ++r2) {
                    const int s2 = rec_slot[r2];
                    if (s2 < 0) continue;
                    if (s2 != slot) break;
                    s = th_add(s, *reinterpret_cast<const float4*>(rec_vec + (size_t)r2 * D + l * 4));
                }
                *reinterpret_cast<float4*>(G + (size_t)(slot - u0) * D + l * 4) = s;
            }
        }
        __syncthreads();
        // ---- hop 2: add G into the pooled vectors of the bags
        if (active) {
#pragma unroll
            for (int o = 0; o < 2; ++o) {
                const TwoHopOut& out = a.out[o];
                if (!out.enabled) continue;
#pragma unroll
                for (int i = 0; i < MAXB; ++i) {
                    const int len = plen[o][i];
#pragma unroll
                    for (int k = 0; k < NIDS; ++k) {
                        const int cnt = min(LG, len - k * LG);
                        for (int e = 0; e < cnt; ++e) {
                            // lookups beyond the bag's end carry id -1 and fail the range test
                            const int u = __shfl(ids[o][i][k], gbase + e, 64);
                            if ((unsigned)(u - u0) < (unsigned)(u1 - u0))
                                acc[o][i] = th_add(acc[o][i], *reinterpret_cast<const float4*>(G + (size_t)(u - u0) * D + l * 4));
                        }
                    }
                    for (int q0 = NIDS * LG; q0 < len; q0 += LG) {  // long bags: ids beyond the cached ones
                        const int q = q0 + l;
                        const int my = q < len ? out.slot_of_lookup[p0[o][i] + q] : -1;
                        const int cnt = min(LG, len - q0);
                        for (int e = 0; e < cnt; ++e) {
                            const int u = __shfl(my, gbase + e, 64);
                            if ((unsigned)(u - u0) < (unsigned)(u1 - u0))
                                acc[o][i] = th_add(acc[o][i], *reinterpret_cast<const float4*>(G + (size_t)(u - u0) * D + l * 4));
                        }
                    }
                }
            }
        }
        __syncthreads();
    }

    // ---- outputs: Y_out = Y_in + c * acc  (fp32 and/or bf16)
    if (!active) return;
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        const TwoHopOut& out = a.out[o];
        if (!out.enabled) continue;
#pragma unroll
        for (int i = 0; i < MAXB; ++i) {
            const int j = a.bag0 + g + i * groups;
            if (j >= nb[o]) continue;
            const int64_t row = out.row_map[s_lo[o] + j] - out.row_base;
            const int64_t off = row * out.ld + colz;
            float4 y = out.y_in ? *reinterpret_cast<const float4*>(out.y_in + off) : make_float4(0.f, 0.f, 0.f, 0.f);
            const float4 s = acc[o][i];
            y = make_float4(y.x + out.c * s.x, y.y + out.c * s.y, y.z + out.c * s.z, y.w + out.c * s.w);
            if (out.y_out) *reinterpret_cast<float4*>(out.y_out + off) = y;
            if (out.y_bf) {
                uint2 pk;
                pk.x = f2bf2(y.x, y.y);
                pk.y = f2bf2(y.z, y.w);
                *reinterpret_cast<uint2*>(out.y_bf + off) = pk;
            }
        }
    }
}

template <int DC, int NT, bool STAGE_Z>
static void launch_two_hop_dc(hipStream_t st, TwoHopArgs a, int n_tasks, int max_bags, size_t lds_budget) {
    constexpr int LG = DC / 4;
    const int groups = NT / LG;
    a.dc = DC;
    const size_t fixed = (size_t)groups * 2 * DC * sizeof(float) + (size_t)groups * 2 * sizeof(int) +
                         (STAGE_Z ? (size_t)a.max_in_rows * DC * sizeof(float) : 0);
    int range = fixed + 64 * DC * sizeof(float) < lds_budget ? (int)((lds_budget - fixed) / ((size_t)DC * sizeof(float))) : 64;
    if (range > 8192) range = 8192;
    a.range = range;
    const size_t shmem = (size_t)range * DC * sizeof(float) + fixed;
    // bags per group held in registers; larger tasks are covered by several launches over bag ranges
    auto launch = [&](auto kern, int maxb) {
        if (shmem > 48 * 1024)
            (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
        for (int b0 = 0; b0 < max_bags; b0 += groups * maxb) {
            a.bag0 = b0;
            hipLaunchKernelGGL(kern, dim3(a.F, n_tasks, a.D / DC), dim3(NT), shmem, st, a);
        }
    };
    if (max_bags <= groups * 2) launch(two_hop_kernel<2, DC, NT, STAGE_Z>, 2);
    else launch(two_hop_kernel<4, DC, NT, STAGE_Z>, 4);
}

void launch_two_hop(hipStream_t st, TwoHopArgs a, int n_tasks, int max_bags) {
    if (n_tasks <= 0 || a.F <= 0) return;
    // wide rows: one workgroup of 1024 lanes per (task, field, 64 columns), a full row per 16-lane group
    if (a.D >= 64) launch_two_hop_dc<64, 1024, false>(st, a, n_tasks, max_bags, 144 * 1024);
    else if (a.D == 32) launch_two_hop_dc<32, 512, false>(st, a, n_tasks, max_bags, 72 * 1024);
    else if (a.D == 16) launch_two_hop_dc<16, 256, true>(st, a, n_tasks, max_bags, 50 * 1024);
    else if (a.D == 8) launch_two_hop_dc<8, 256, true>(st, a, n_tasks, max_bags, 50 * 1024);
    else launch_two_hop_dc<4, 256, true>(st, a, n_tasks, max_bags, 50 * 1024);
}
