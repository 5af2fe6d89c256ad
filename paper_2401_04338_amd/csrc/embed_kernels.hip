// Embedding side of the MAML step (G-Meta Alg. 1): the one-pass prefetch of support and query rows
// with sum pooling (prefetch step, Sec. 2.1.1), the task-local row updates and the overlap update
// (their dense and pad columns; the row arithmetic itself is in twohop_kernels.hip), and the segment reduction that coalesces the sparse
// meta-gradient (global back-propagation on xi).  All HBM-bound: rows are read as float4 by groups of
// D/4 lanes so that one wavefront keeps several independent row reads in flight.
#include "gm_internal.h"

__device__ __forceinline__ void store_bf4(bf16_t* dst, float4 v) {
    uint2 o;
    o.x = f2bf2(v.x, v.y);
    o.y = f2bf2(v.z, v.w);
    *reinterpret_cast<uint2*>(dst) = o;
}

__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// ------------------------------------------------------------------------------------------------
// prefetch + sum pooling: x[s, f*D:(f+1)*D] = sum over bag(s,f) of emb[field_base[f] + index]
// ------------------------------------------------------------------------------------------------
__global__ void gather_pool_kernel(int F, int D, int LG, const int64_t* __restrict__ field_base,
                                   const int64_t* __restrict__ bag_offsets, const int32_t* __restrict__ indices,
                                   const float* __restrict__ emb, int64_t sample0, int64_t n_bags,
                                   const int32_t* __restrict__ row_map, int32_t row_base, float* x, int ldx,
                                   bf16_t* x_bf) {
    const int groups_per_block = blockDim.x / LG;
    const int g_in_block = threadIdx.x / LG, l = threadIdx.x % LG;
    if (g_in_block >= groups_per_block) return;
    const int64_t n_groups = (int64_t)gridDim.x * groups_per_block;
    const float4* emb4 = reinterpret_cast<const float4*>(emb);
    for (int64_t bag = (int64_t)blockIdx.x * groups_per_block + g_in_block; bag < n_bags; bag += n_groups) {
        const int64_t s = bag / F;
        const int f = (int)(bag - s * F);
        const int64_t gb = sample0 * F + bag;
        const int64_t p0 = bag_offsets[gb], p1 = bag_offsets[gb + 1];
        const int64_t fb = field_base[f];
        // the order of the sums is gather_pool_xcd_kernel's, bit for bit: eight lookups at a time, the first four into
        // one chain and the next four into the other (one chain when a lane group is narrower than eight lanes)
        float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f), acc1 = acc0;
        const float4 zero = acc0;
        for (int64_t p = p0; p < p1; p += 8) {
            float4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = p + j < p1 ? emb4[(fb + indices[p + j]) * LG + l] : zero;
            acc0 = add4(add4(add4(add4(acc0, v[0]), v[1]), v[2]), v[3]);
            if (LG >= 8) acc1 = add4(add4(add4(add4(acc1, v[4]), v[5]), v[6]), v[7]);
            else acc0 = add4(add4(add4(add4(acc0, v[4]), v[5]), v[6]), v[7]);
        }
        const float4 acc = add4(acc0, acc1);
        const int64_t o = (int64_t)(row_map[s] - row_base) * ldx + (int64_t)f * D + l * 4;
        if (x) *reinterpret_cast<float4*>(x + o) = acc;
        if (x_bf) store_bf4(x_bf + o, acc);
    }
}

// The same pooling with the fields dealt to the 8 XCDs: workgroup b runs on XCD b % 8 and pools one eighth of the
// (field, sample) pairs in field-major order, i.e. about F / 8 consecutive fields (a field may be shared by two
// neighbours, so that the shares are equal whatever F is).  Under Zipf skew most lookups of a field hit a few thousand
// hot rows; with an eighth of the fields per XCD the hot rows of "its" fields fit that XCD's L2 (8 fields x 1000 rows
// x 256 B = 2 MB of 4 MB), so they stop travelling over the fabric for every lookup -- the fabric, not HBM, is what
// this kernel is bound by.  (The lookups of a bag are summed in two interleaved chains of four, a fixed order.)  Indices
// and the fp32 outputs stream past once: they are read and written with the non-temporal hint, which leaves L2 to the
// rows (measured: 2-3 %; whether all XCDs sweep one field range together or each its own eighth makes no difference).
__global__ void gather_pool_xcd_kernel(int F, int D, int LG, const int64_t* __restrict__ field_base,
                                       const int64_t* __restrict__ bag_offsets, const int32_t* __restrict__ indices,
                                       const float* __restrict__ emb, int64_t sample0, int64_t n_samples,
                                       const int32_t* __restrict__ row_map, int32_t row_base, float* x, int ldx,
                                       bf16_t* x_bf) {
    const int groups_per_block = blockDim.x / LG;
    const int g_in_block = threadIdx.x / LG, l = threadIdx.x % LG;
    if (g_in_block >= groups_per_block) return;
    const int xcd = blockIdx.x & 7, bi = blockIdx.x >> 3, nbx = gridDim.x >> 3;
    const float4* emb4 = reinterpret_cast<const float4*>(emb);
    // work items of this XCD: pairs [lo, hi) of the field-major list (pair = field * n_samples + sample)
    const int64_t n_pairs = n_samples * F;
    const int64_t lo = n_pairs * xcd / 8, hi = n_pairs * (xcd + 1) / 8;
    const int64_t stride = (int64_t)nbx * groups_per_block;
    // A bag is a chain of dependent reads (offsets -> indices -> rows).  The chain of the NEXT bag is started before
    // the rows of this one are summed: its offsets and its first LG indices (one per lane of the group, handed round
    // by lane shuffles) are in registers when its turn comes, and up to 8 row reads are in flight per lane.
    int64_t it = lo + (int64_t)bi * groups_per_block + g_in_block;
    int64_t p0 = 0, p1 = 0;
    int32_t idx_l = 0;
    if (it < hi) {
        const int f = (int)(it / n_samples);
        const int64_t gb = (sample0 + (it - (int64_t)f * n_samples)) * F + f;
        p0 = bag_offsets[gb]; p1 = bag_offsets[gb + 1];
        if (p0 + l < p1) idx_l = __builtin_nontemporal_load(indices + p0 + l);
    }
    for (; it < hi; it += stride) {
        const int f = (int)(it / n_samples);
        const int64_t s = it - (int64_t)f * n_samples;
        const int64_t fb = field_base[f];
        const int64_t c0 = p0, c1 = p1;
        int32_t cur_idx = idx_l;
        // next bag's offsets and first indices
        const int64_t itn = it + stride;
        if (itn < hi) {
            const int fn = (int)(itn / n_samples);
            const int64_t gbn = (sample0 + (itn - (int64_t)fn * n_samples)) * F + fn;
            p0 = bag_offsets[gbn]; p1 = bag_offsets[gbn + 1];
            idx_l = (p0 + l < p1) ? __builtin_nontemporal_load(indices + p0 + l) : 0;
        }
        float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f), acc1 = acc0;
        for (int64_t base = c0; base < c1; base += LG) {
            if (base > c0) cur_idx = (base + l < c1) ? __builtin_nontemporal_load(indices + base + l) : 0;
            const int m = (int)min<int64_t>(LG, c1 - base);
            for (int j0 = 0; j0 < m; j0 += 8) {
                float4 v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int jj = j0 + j;
                    const int32_t r = __shfl(cur_idx, jj < LG ? jj : 0, LG);
                    v[j] = jj < m ? emb4[(fb + r) * LG + l] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
                acc0 = add4(add4(add4(add4(acc0, v[0]), v[1]), v[2]), v[3]);
                acc1 = add4(add4(add4(add4(acc1, v[4]), v[5]), v[6]), v[7]);
            }
        }
        const float4 acc = add4(acc0, acc1);
        const int64_t o = (int64_t)(row_map[s] - row_base) * ldx + (int64_t)f * D + l * 4;
        if (x) {
            __builtin_nontemporal_store(acc.x, x + o); __builtin_nontemporal_store(acc.y, x + o + 1);
            __builtin_nontemporal_store(acc.z, x + o + 2); __builtin_nontemporal_store(acc.w, x + o + 3);
        }
        if (x_bf) store_bf4(x_bf + o, acc);
    }
}

// dense features and zero padding behind the pooled fields
__global__ void dense_tail_kernel(int FD, int n_dense, const float* __restrict__ dense, int64_t sample0,
                                  int64_t n_samples, const int32_t* __restrict__ row_map, int32_t row_base, float* x,
                                  int ldx, bf16_t* x_bf) {
    const int tail = ldx - FD;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_samples * tail) return;
    const int64_t s = i / tail;
    const int c = (int)(i - s * tail);
    const float v = (dense && c < n_dense) ? dense[(sample0 + s) * n_dense + c] : 0.f;
    const int64_t o = (int64_t)(row_map[s] - row_base) * ldx + FD + c;
    if (x) x[o] = v;
    if (x_bf) x_bf[o] = f2bf(v);
}

static inline unsigned pool_grid(int64_t n_bags, int groups_per_block) {
    int64_t nb = (n_bags + groups_per_block - 1) / groups_per_block;
    const int64_t cap = 256 * 32;  // grid-stride beyond 32 blocks per CU
    if (nb > cap) nb = cap;
    if (nb < 1) nb = 1;
    return (unsigned)nb;
}

void launch_gather_pool(hipStream_t st, int F, int D, int n_dense, const int64_t* field_base,
                        const int64_t* bag_offsets, const int32_t* indices, const float* dense, const float* emb,
                        int64_t sample0, int64_t n_samples, const int32_t* row_map, int32_t row_base, float* x, int ldx,
                        bf16_t* x_bf) {
    if (n_samples <= 0) return;
    const int LG = D / 4;
    const int64_t n_bags = n_samples * F;
    if (n_bags > 0 && F >= 8 && n_bags >= (1 << 14)) {
        const unsigned grid = pool_grid(n_bags, 256 / LG) / 8 * 8;
        hipLaunchKernelGGL(gather_pool_xcd_kernel, dim3(grid), dim3(256), 0, st, F, D, LG, field_base, bag_offsets,
                           indices, emb, sample0, n_samples, row_map, row_base, x, ldx, x_bf);
    } else if (n_bags > 0)
        hipLaunchKernelGGL(gather_pool_kernel, dim3(pool_grid(n_bags, 256 / LG)), dim3(256), 0, st, F, D, LG, field_base,
                           bag_offsets, indices, emb, sample0, n_bags, row_map, row_base, x, ldx, x_bf);
    const int64_t nt = n_samples * (ldx - F * D);
    if (nt > 0)
        hipLaunchKernelGGL(dense_tail_kernel, dim3((unsigned)((nt + 255) / 256)), dim3(256), 0, st, F * D, n_dense, dense,
                           sample0, n_samples, row_map, row_base, x, ldx, x_bf);
}

// dense and pad columns of every (padded) row: copied from x_base, or zero
__global__ void copy_tail_kernel(int FD, const float* x_base, int64_t n_rows, float* x_out, int ldx, bf16_t* x_bf) {
    const int tail = ldx - FD;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows * tail) return;
    const int64_t s = i / tail;
    const int c = (int)(i - s * tail);
    const float v = x_base ? x_base[s * ldx + FD + c] : 0.f;
    if (x_out) x_out[s * ldx + FD + c] = v;
    if (x_bf) x_bf[s * ldx + FD + c] = f2bf(v);
}

void launch_copy_tail(hipStream_t st, int FD, const float* x_base, int64_t n_rows, float* x_out, int ldx, bf16_t* x_bf) {
    const int64_t nt = n_rows * (ldx - FD);
    if (nt > 0)
        hipLaunchKernelGGL(copy_tail_kernel, dim3((unsigned)((nt + 255) / 256)), dim3(256), 0, st, FD, x_base, n_rows,
                           x_out, ldx, x_bf);
}

// ------------------------------------------------------------------------------------------------
// global segment reduction: emb_grad[seg] = sum over the segment's lookups (stable (field,row) order) of
// gx[(row of the sample, field)], gx laid out [rows (support then query), F, D].
//
// Under Zipf skew a hot row's segment holds a large share of all lookups, so segments are not the unit
// of work: the sorted lookup list is cut into fixed chunks of SEG_CH positions, one lane group walks one
// chunk, a segment that lies inside one chunk is written directly, and a segment that crosses chunk
// borders leaves one partial sum per chunk that a second pass adds in chunk order.  The cutting depends
// only on positions, so the order of every sum is fixed.
// ------------------------------------------------------------------------------------------------
#define SEG_CH 64

// One lane group (LG = D/4 lanes, a float4 of the row each) walks one chunk.  The chunk's metadata is read LG positions
// at a time, one position per lane (coalesced), and handed round the group by lane shuffles; the head flags of
// the LG positions come back as one ballot word.  Whether a run began before the chunk or continues past it
// follows from the head flags at the chunk's two borders, so no segment table is read here.
template <int LG>
__global__ void __launch_bounds__(256)
seg_reduce_chunks_kernel(int D, int F, ValEnc enc, const u32* __restrict__ keys, const u32* __restrict__ scan,
                         const int64_t* __restrict__ n_rows, int64_t capacity, int64_t n,
                         const u32* __restrict__ sorted_vals, const float* __restrict__ gx, float* emb_grad,
                         float* partial, float* table) {
    constexpr int GPB = 256 / LG;            // lane groups per workgroup
    constexpr int U = LG < 8 ? LG : 8;       // row loads in flight per lane
    const int g_in_block = threadIdx.x / LG, l = threadIdx.x % LG;
    const int group_lane0 = (threadIdx.x % 64) / LG * LG;   // the group's first lane inside its wave
    const int64_t n_valid = table ? 0 : min(*n_rows, capacity);
    const int64_t n_chunks = (n + SEG_CH - 1) / SEG_CH;
    const int64_t n_groups = (int64_t)gridDim.x * GPB;
    const float4* gx4 = reinterpret_cast<const float4*>(gx);
    for (int64_t c = (int64_t)blockIdx.x * GPB + g_in_block; c < n_chunks; c += n_groups) {
        const int64_t cb = c * SEG_CH;
        const int cnt = (int)min((int64_t)SEG_CH, n - cb);
        // borders: does the chunk's last run go on in the next chunk; which segment does position cb lie in
        const bool goes_on = (cb + cnt < n) && keys[cb + cnt] == keys[cb + cnt - 1];
        int64_t seg = table ? 0 : (int64_t)scan[cb] - 1;     // + 1 at every head, the one at cb included
        u32 v_next = 0, k_next = 0;
        bool h_next = false;
        auto load_meta = [&](int p0) {       // positions cb + p0 + l of the chunk
            const int p = p0 + l;
            v_next = 0, k_next = 0, h_next = false;
            if (p < cnt) {
                const int64_t i = cb + p;
                v_next = sorted_vals[i];
                // (bit-field values: the bag's place in the gradient buffer is row * F + field)
                if (enc.rshift) v_next = (v_next >> enc.rshift) * (u32)F + ((v_next >> enc.pshift) & enc.fmask);
                k_next = keys[i];
                h_next = (i == 0) || keys[i - 1] != k_next;
            }
        };
        load_meta(0);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        bool began_before = false;           // the current run began in an earlier chunk
        u32 run_key = 0;
        auto flush = [&](bool continues) {
            float* dst;
            if (began_before) dst = partial + (c * 2 + 0) * D;
            else if (continues) dst = partial + (c * 2 + 1) * D;
            else if (table) {  // table-shaped output: added to the segment's row (rows of one call are distinct)
                float4* tp = reinterpret_cast<float4*>(table + (int64_t)run_key * D + l * 4);
                *tp = add4(*tp, acc);
                return;
            } else {
                if (seg >= n_valid) return;
                dst = emb_grad + seg * D;
            }
            *reinterpret_cast<float4*>(dst + l * 4) = acc;
        };
        for (int p0 = 0; p0 < cnt; p0 += LG) {
            const u32 v = v_next, k = k_next;
            const unsigned long long heads = (__ballot(h_next) >> group_lane0);
            if (p0 + LG < cnt) load_meta(p0 + LG);
            const int m = min(LG, cnt - p0);
            for (int s0 = 0; s0 < m; s0 += U) {
                u32 vv[U], kk[U];
                float4 x[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    vv[u] = __shfl(v, s0 + u, LG);          // lanes past cnt hold row 0: a valid, unused read
                    kk[u] = __shfl(k, s0 + u, LG);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) x[u] = gx4[(int64_t)vv[u] * LG + l];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int s = s0 + u;
                    if (s >= m) break;
                    const bool head = (heads >> s) & 1;
                    if (p0 + s == 0) {
                        began_before = !head;
                        seg += head ? 1 : 0;
                        run_key = kk[u];
                        acc = x[u];
                    } else if (head) {
                        flush(false);
                        began_before = false;
                        seg += 1;
                        run_key = kk[u];
                        acc = x[u];
                    } else {
                        acc = add4(acc, x[u]);
                    }
                }
            }
        }
        flush(goes_on);
    }
}

// One lane group per CHUNK: if the chunk's last run begins inside the chunk and goes on past it, this group adds
// the pieces the following chunks left (each of them starts with the same key) in chunk order.  Every such
// segment is the last one of exactly one chunk.
__global__ void seg_reduce_join_kernel(int D, int LG, const u32* __restrict__ keys, const u32* __restrict__ scan,
                                       const int64_t* __restrict__ n_rows, int64_t capacity, int64_t n,
                                       const float* __restrict__ partial, float* emb_grad, float* table) {
    const int groups_per_block = blockDim.x / LG;
    const int g_in_block = threadIdx.x / LG, l = threadIdx.x % LG;
    if (g_in_block >= groups_per_block) return;
    const int64_t n_valid = table ? 0 : min(*n_rows, capacity);
    const int64_t n_chunks = (n + SEG_CH - 1) / SEG_CH;
    const int64_t n_groups = (int64_t)gridDim.x * groups_per_block;
    for (int64_t c = (int64_t)blockIdx.x * groups_per_block + g_in_block; c + 1 < n_chunks; c += n_groups) {
        const int64_t cb = c * SEG_CH, ce = cb + SEG_CH;   // not the last chunk, so it is full and ce < n
        const u32 key = keys[ce - 1];
        if (keys[ce] != key) continue;                     // the run ends with the chunk
        if (cb > 0 && keys[cb - 1] == key) continue;       // began in an earlier chunk, which adds it up
        int64_t seg = 0;
        if (!table) {
            seg = (int64_t)scan[ce - 1] + (keys[ce - 2] != key ? 1 : 0) - 1;
            if (seg >= n_valid) continue;
        }
        // c1: the last chunk that starts with the key.  Most segments end in chunk c + 1, a hot row's spans
        // thousands: gallop forward in doubling steps, then bisect (the keys are sorted).
        auto starts_with_key = [&](int64_t cc) { return cc < n_chunks && keys[cc * SEG_CH] == key; };
        int64_t c1 = c + 1, step = 1;
        while (starts_with_key(c1 + step)) {
            c1 += step;
            step *= 2;
        }
        for (int64_t hi = c1 + step; hi - c1 > 1;) {       // chunk c1 starts with the key, chunk hi does not
            const int64_t mid = c1 + (hi - c1) / 2;
            if (starts_with_key(mid)) c1 = mid;
            else hi = mid;
        }
        float4 acc = *reinterpret_cast<const float4*>(partial + (c * 2 + 1) * D + l * 4);
        int64_t cc = c + 1;
        for (; cc + 8 <= c1 + 1; cc += 8) {       // 8 independent loads in flight, added in chunk order
            float4 x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = *reinterpret_cast<const float4*>(partial + ((cc + u) * 2 + 0) * D + l * 4);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = add4(acc, x[u]);
        }
        for (; cc <= c1; ++cc)
            acc = add4(acc, *reinterpret_cast<const float4*>(partial + (cc * 2 + 0) * D + l * 4));
        if (table) {
            float4* tp = reinterpret_cast<float4*>(table + (int64_t)key * D + l * 4);
            *tp = add4(*tp, acc);
        } else {
            *reinterpret_cast<float4*>(emb_grad + seg * D + l * 4) = acc;
        }
    }
}

size_t seg_reduce_partial_floats(int64_t n, int D) { return (size_t)((n + SEG_CH - 1) / SEG_CH) * 2 * D + 16; }

void launch_seg_reduce(hipStream_t st, int D, int F, ValEnc enc, const u32* keys, const u32* scan, const int64_t* n_rows, int64_t capacity, int64_t n, const u32* sorted_vals, const float* gx,
                       float* emb_grad, float* partial, float* table) {
    if (n <= 0 || capacity <= 0) return;
    const int LG = D / 4;
    const int64_t n_chunks = (n + SEG_CH - 1) / SEG_CH;
    const dim3 grid(pool_grid(n_chunks, 256 / LG));
#define SEG_CHUNKS(LG_)                                                                                              \
    case LG_:                                                                                                        \
        hipLaunchKernelGGL(seg_reduce_chunks_kernel<LG_>, grid, dim3(256), 0, st, D, F, enc, keys, scan, n_rows, capacity, n, \
                           sorted_vals, gx, emb_grad, partial, table);                                               \
        break;
    switch (LG) {
        SEG_CHUNKS(1) SEG_CHUNKS(2) SEG_CHUNKS(4) SEG_CHUNKS(8) SEG_CHUNKS(16) SEG_CHUNKS(32) SEG_CHUNKS(64)
        default: return;   // emb_dim is a power of two in 4..256 (checked when the context is made)
    }
#undef SEG_CHUNKS
    hipLaunchKernelGGL(seg_reduce_join_kernel, dim3(pool_grid(n_chunks, 256 / LG)), dim3(256), 0, st, D, LG, keys, scan,
                       n_rows, capacity, n, partial, emb_grad, table);
}

__global__ void scatter_add_kernel(int D, int LG, float* table, const int64_t* __restrict__ rows,
                                   const float* __restrict__ grad, int64_t n_rows, float scale) {
    const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = gt / LG;
    const int l = (int)(gt % LG);
    if (i >= n_rows) return;
    float4* dst = reinterpret_cast<float4*>(table + rows[i] * D + l * 4);
    const float4 g = *reinterpret_cast<const float4*>(grad + i * D + l * 4);
    float4 o = *dst;
    o.x += scale * g.x; o.y += scale * g.y; o.z += scale * g.z; o.w += scale * g.w;
    *dst = o;
}

void launch_scatter_add(hipStream_t st, int D, float* table, const int64_t* rows, const float* grad, int64_t n_rows,
                        float scale) {
    if (n_rows <= 0) return;
    const int LG = D / 4;
    const int64_t nt = n_rows * LG;
    hipLaunchKernelGGL(scatter_add_kernel, dim3((unsigned)((nt + 255) / 256)), dim3(256), 0, st, D, LG, table, rows, grad,
                       n_rows, scale);
}
