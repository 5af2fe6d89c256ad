// Integer side of the MAML step (G-Meta Alg. 1): the per-(task, field) row dictionaries behind the
// inner-loop row update and the overlap join of Sec. 2.1.2, and the global (field,row) ordering that
// routes the sparse meta-gradient (Alg. 1, global back-propagation on xi).  Everything here has exactly
// one correct answer and is compared bit-exactly with the CPU oracle.
#include "gm_internal.h"

#define WAVE 64

// ------------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int wave_incl_scan(int v) {
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        int o = __shfl_up(v, d, WAVE);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan of one int per thread over the block; `sh` holds >= blockDim/64 + 1 ints.
__device__ __forceinline__ int block_excl_scan(int v, int* sh, int* total) {
    const int lane = threadIdx.x & (WAVE - 1), wid = threadIdx.x / WAVE, nw = blockDim.x / WAVE;
    int incl = wave_incl_scan(v);
    __syncthreads();
    if (lane == WAVE - 1) sh[wid] = incl;
    __syncthreads();
    if (wid == 0) {
        int x = lane < nw ? sh[lane] : 0;
        int xi = wave_incl_scan(x);
        if (lane < nw) sh[lane] = xi - x;
        if (lane == nw - 1) sh[nw] = xi;
    }
    __syncthreads();
    int r = sh[wid] + incl - v;
    *total = sh[nw];
    return r;
}

// ------------------------------------------------------------------------------------------------
// validation + per-(task, field) lookup counts
// ------------------------------------------------------------------------------------------------
// One task per blockIdx.x, its bags dealt to gridDim.y workgroups; cnt_sup / cnt_qry must be zero on entry.
// A well-formed input that exceeds a size limit of the index kernels (a bag of more than 65,535 lookups, a task of more
// than 65,536 samples in one set) raises ST_TOO_LARGE, not ST_BAD_INDEX.
// uniform_rows >= 0: every table has that many rows, so an index is checked without knowing its field: the task's
// lookups, one contiguous range, are then read by all lanes in order instead of bag by bag.
__global__ void tf_count_kernel(int F, int t0, SetView sup, SetView qry, const int64_t* field_base,
                                int64_t nnz_sup, int64_t nnz_qry, int64_t uniform_rows, u32* cnt_sup, u32* cnt_qry, u32* status) {
    extern __shared__ u32 sh_cnt[];  // [2F]
    const int t = blockIdx.x;
    for (int i = threadIdx.x; i < 2 * F; i += blockDim.x) sh_cnt[i] = 0;
    __syncthreads();
    bool bad = false, too_large = false;
    u32 longest = 0;
    for (int set = 0; set < 2; ++set) {
        const SetView& v = set ? qry : sup;
        const int64_t nnz = set ? nnz_qry : nnz_sup;
        const int64_t s_lo = v.task_offsets[t0 + t], s_hi = v.task_offsets[t0 + t + 1];
        if (s_hi - s_lo > 65536) too_large = true;
        const int64_t n = (s_hi - s_lo) * F;
        for (int64_t i = (int64_t)blockIdx.y * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.y * blockDim.x) {
            const int64_t bag = s_lo * F + i;
            const int f = (int)(i % F);
            const int64_t p0 = v.bag_offsets[bag], p1 = v.bag_offsets[bag + 1];
            if (p0 < 0 || p1 < p0 || p1 > nnz) {
                bad = true;
                continue;
            }
            if (p1 - p0 > 65535) {
                too_large = true;
                continue;
            }
            if (uniform_rows < 0) {
                const int64_t R = field_base[f + 1] - field_base[f];
                for (int64_t p = p0; p < p1; ++p) {
                    const int32_t r = v.indices[p];
                    if (r < 0 || r >= R) bad = true;
                }
            }
            atomicAdd(&sh_cnt[set * F + f], (u32)(p1 - p0));
            longest = max(longest, (u32)(p1 - p0));
        }
        if (uniform_rows >= 0 && n > 0) {   // (offsets outside [0, nnz] are flagged above; the range read here is clamped)
            const int64_t q0 = min(max(v.bag_offsets[s_lo * F], (int64_t)0), nnz), q1 = min(max(v.bag_offsets[s_hi * F], q0), nnz);
            for (int64_t p = q0 + (int64_t)blockIdx.y * blockDim.x + threadIdx.x; p < q1; p += (int64_t)gridDim.y * blockDim.x) {
                const int32_t r = v.indices[p];
                if (r < 0 || r >= uniform_rows) bad = true;
            }
        }
    }
    if (t == 0 && blockIdx.y == 0 && threadIdx.x == 0) {  // the ends of both offset arrays
        if (sup.bag_offsets[0] != 0 || sup.bag_offsets[sup.n_samples * F] != nnz_sup) bad = true;
        if (qry.bag_offsets[0] != 0 || qry.bag_offsets[qry.n_samples * F] != nnz_qry) bad = true;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * F; i += blockDim.x) {
        const u32 c = sh_cnt[i];
        if (!c) continue;
        u32* dst = i < F ? &cnt_sup[(size_t)t * F + i] : &cnt_qry[(size_t)t * F + (i - F)];
        const u32 whole = atomicAdd(dst, c) + c;     // the (task, field)'s count so far: the last adder sees the total
        atomicMax(&status[ST_MAX_TF], whole);
    }
    if (longest) atomicMax(&status[ST_MAX_BAG], longest);
    if (bad) atomicOr(&status[ST_BAD_INDEX], 1u);
    if (too_large) atomicOr(&status[ST_TOO_LARGE], 1u);
}

void launch_tf_count(hipStream_t st, int F, int t0, int Tw, SetView sup, SetView qry, const int64_t* field_base,
                     int64_t nnz_sup, int64_t nnz_qry, int64_t uniform_rows, u32* cnt_sup, u32* cnt_qry, u32* status) {
    if (Tw <= 0) return;
    launch_fill_u32(st, cnt_sup, (int64_t)Tw * F, 0u);
    if (cnt_qry != cnt_sup) launch_fill_u32(st, cnt_qry, (int64_t)Tw * F, 0u);
    // enough workgroups to fill the chip whatever the number of tasks in the wave
    const int split = Tw >= 2048 ? 1 : (Tw >= 512 ? 4 : 8);
    hipLaunchKernelGGL(tf_count_kernel, dim3(Tw, split), dim3(256), 2 * F * sizeof(u32), st, F, t0, sup, qry, field_base,
                       nnz_sup, nnz_qry, uniform_rows, cnt_sup, cnt_qry, status);
}

// ------------------------------------------------------------------------------------------------
// device-wide exclusive scan of u32 (three-phase, recursive on the block sums)
// ------------------------------------------------------------------------------------------------
#define SCAN_NT 256
#define SCAN_ITEMS 8
#define SCAN_TILE (SCAN_NT * SCAN_ITEMS)

// (a thread's 8 items are 32 contiguous bytes: two 16-byte accesses when the pointers allow and the items are all inside)
__global__ void scan_block_kernel(const u32* in, u32* out, int64_t n, u32* block_sums) {
    __shared__ int sh[SCAN_NT / WAVE + 2];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    const bool wide = base + SCAN_ITEMS <= n && ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
    u32 v[SCAN_ITEMS];
    u32 sum = 0;
    if (wide) {
        const uint4 a = *reinterpret_cast<const uint4*>(in + base), b = *reinterpret_cast<const uint4*>(in + base + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
        for (int i = 0; i < SCAN_ITEMS; ++i) v[i] = (base + i < n) ? in[base + i] : 0u;
    }
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) sum += v[i];
    int total;
    u32 run = (u32)block_excl_scan((int)sum, sh, &total);
    u32 o[SCAN_ITEMS];
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        o[i] = run;
        run += v[i];
    }
    if (wide) {
        *reinterpret_cast<uint4*>(out + base) = make_uint4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<uint4*>(out + base + 4) = make_uint4(o[4], o[5], o[6], o[7]);
    } else {
#pragma unroll
        for (int i = 0; i < SCAN_ITEMS; ++i)
            if (base + i < n) out[base + i] = o[i];
    }
    if (threadIdx.x == 0) block_sums[blockIdx.x] = (u32)total;
}

// first level of the scan of segment-head flags: the flag of key i (1 where a new row starts) is taken from the sorted
// keys themselves, so no flag array is written and read back
__global__ void scan_heads_block_kernel(const u32* __restrict__ keys, u32* out, int64_t n, u32* block_sums) {
    __shared__ int sh[SCAN_NT / WAVE + 2];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    u32 k[SCAN_ITEMS + 1];
    k[0] = (base > 0 && base < n) ? keys[base - 1] : 0u;
    if (base + SCAN_ITEMS <= n) {   // (the buffers are 16-byte aligned and base is a multiple of 8)
        const uint4 a = *reinterpret_cast<const uint4*>(keys + base), b = *reinterpret_cast<const uint4*>(keys + base + 4);
        k[1] = a.x; k[2] = a.y; k[3] = a.z; k[4] = a.w; k[5] = b.x; k[6] = b.y; k[7] = b.z; k[8] = b.w;
    } else {
#pragma unroll
        for (int i = 0; i < SCAN_ITEMS; ++i) k[i + 1] = (base + i < n) ? keys[base + i] : 0u;
    }
    u32 v[SCAN_ITEMS];
    u32 sum = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        v[i] = (base + i < n && (base + i == 0 || k[i + 1] != k[i])) ? 1u : 0u;
        sum += v[i];
    }
    int total;
    u32 run = (u32)block_excl_scan((int)sum, sh, &total);
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        if (base + i < n) out[base + i] = run;
        run += v[i];
    }
    if (threadIdx.x == 0) block_sums[blockIdx.x] = (u32)total;
}

__global__ void scan_add_kernel(u32* out, int64_t n, const u32* block_offsets) {
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    const u32 o = block_offsets[blockIdx.x];
    if (base + SCAN_ITEMS <= n && (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
        uint4* p = reinterpret_cast<uint4*>(out + base);
        uint4 a = p[0], b = p[1];
        a.x += o; a.y += o; a.z += o; a.w += o; b.x += o; b.y += o; b.z += o; b.w += o;
        p[0] = a;
        p[1] = b;
        return;
    }
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i)
        if (base + i < n) out[base + i] += o;
}

__global__ void copy_u32_kernel(const u32* src, u32* dst) { *dst = *src; }

size_t scan_tmp_words(int64_t n) {
    size_t w = 0;
    while (true) {
        int64_t nb = (n + SCAN_TILE - 1) / SCAN_TILE;
        if (nb < 1) nb = 1;
        w += (size_t)((nb + 63) / 64 * 64);
        if (nb <= 1) break;
        n = nb;
    }
    return w + 64;
}

void launch_scan_u32(hipStream_t st, const u32* in, u32* out, int64_t n, u32* tmp, u32* total) {
    if (n <= 0) {
        if (total) launch_fill_u32(st, total, 1, 0);
        return;
    }
    const int64_t nb = (n + SCAN_TILE - 1) / SCAN_TILE;
    hipLaunchKernelGGL(scan_block_kernel, dim3((unsigned)nb), dim3(SCAN_NT), 0, st, in, out, n, tmp);
    if (nb == 1) {
        if (total) hipLaunchKernelGGL(copy_u32_kernel, dim3(1), dim3(1), 0, st, tmp, total);
        return;
    }
    u32* next = tmp + (nb + 63) / 64 * 64;
    launch_scan_u32(st, tmp, tmp, nb, next, total);
    hipLaunchKernelGGL(scan_add_kernel, dim3((unsigned)nb), dim3(SCAN_NT), 0, st, out, n, tmp);
}

// ------------------------------------------------------------------------------------------------
// per-(task, field) dictionaries: LDS sort of the support lookups, then the query join
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void bitonic_sort_lds(u64* keys, int n2) {
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int p = threadIdx.x; p < (n2 >> 1); p += blockDim.x) {
                const int i = ((p & ~(j - 1)) << 1) | (p & (j - 1));
                const int ixj = i + j;
                const bool asc = (i & k) == 0;
                const u64 a = keys[i], b = keys[ixj];
                if ((a > b) == asc) {
                    keys[i] = b;
                    keys[ixj] = a;
                }
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ int load_tf_keys(u64* keys, int* sh_fill, const SetView& v, int F, int f, int64_t s_lo,
                                            int64_t s_hi, u32 fb) {
    if (threadIdx.x == 0) *sh_fill = 0;
    __syncthreads();
    const int ns = (int)(s_hi - s_lo);
    for (int s = threadIdx.x; s < ns; s += blockDim.x) {
        const int64_t bag = (s_lo + s) * F + f;
        const int64_t p0 = v.bag_offsets[bag];
        const int len = (int)(v.bag_offsets[bag + 1] - p0);
        if (len > 0) {
            const int base = atomicAdd(sh_fill, len);
            for (int j = 0; j < len; ++j)
                keys[base + j] = ((u64)(fb + (u32)v.indices[p0 + j]) << 32) | ((u64)s << 16) | (u64)j;
        }
    }
    __syncthreads();
    return *sh_fill;
}

// The same keys in (row, sample, position) order by a stable LSD radix sort inside LDS: the keys are written in
// (sample, position) order first (an exclusive scan of the bag lengths places every bag), so only the row bits
// have to be sorted, in passes of at most 8 bits.  Per pass every wave ranks a contiguous share of the keys, 64 at
// a time, with ballot matching (equal digits keep their order), and the per-(digit, wave) counts are turned into
// positions.  Returns the buffer (one of the two) that holds the result.  At most TFR_ROUNDS * 64 keys per wave
// and TFR_MAXS bags per task and set.
#define TFR_ROUNDS 16
#define TF_SMALL_N 1984    // lookups per set of a 'small' (task, field): its key buffer is 2048 + 64 keys
#define TF_SMALL_MS 512    // samples per set of a 'small' task
#define TFR_MAXS 2048
struct TfRadixLds {
    u64* buf;               // [cap]: every pass holds all keys in registers between its read and its write
    u32 *sbase, *sp0;       // [ms + 1], [ms]: first key / first lookup (relative to the wave's) of every bag
    uint16_t* cnt;          // [waves][256]
    u32* digstart;          // [256]
    int* sh_scan;
};
__device__ __forceinline__ u64* tf_radix_sorted(const TfRadixLds& L, const SetView& v, int F, int f, int64_t s_lo,
                                                int64_t s_hi, u32 fb, int bits, int n) {
    const int NT = blockDim.x, W = NT / WAVE, lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
    const int ns = (int)(s_hi - s_lo);
    // bag lengths -> first key of every bag
    {
        const int per = (ns + NT - 1) / NT;
        const int b0 = min(ns, (int)threadIdx.x * per), b1 = min(ns, b0 + per);
        int sum = 0;
        for (int sidx = b0; sidx < b1; ++sidx) {
            const int64_t bag = (s_lo + sidx) * F + f;
            sum += (int)(v.bag_offsets[bag + 1] - v.bag_offsets[bag]);
        }
        int total;
        int run = block_excl_scan(sum, L.sh_scan, &total);
        for (int sidx = b0; sidx < b1; ++sidx) {
            const int64_t bag = (s_lo + sidx) * F + f;
            const int64_t p0 = v.bag_offsets[bag];
            L.sbase[sidx] = (u32)run;
            L.sp0[sidx] = (u32)(p0 - v.lookup0);
            run += (int)(v.bag_offsets[bag + 1] - p0);
        }
        if (threadIdx.x == 0) L.sbase[ns] = (u32)n;
    }
    __syncthreads();
    // Every thread builds a run of consecutive keys: one bisection for the bag of its first key, then a walk along the
    // bag table; the index loads of the run are all requested before the first key is assembled.
    {
        const int C = (n + NT - 1) / NT;   // at most TFR_ROUNDS + 1
        const int e0 = min(n, (int)threadIdx.x * C), e1 = min(n, e0 + C);
        int lo = 0;
        if (e0 < e1) {
            int hi = ns;   // last bag whose first key is <= e0 (empty bags share their successor's first key)
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (L.sbase[mid] <= (u32)e0) lo = mid;
                else hi = mid;
            }
        }
        u32 meta[TFR_ROUNDS + 1], idx[TFR_ROUNDS + 1];
#pragma unroll
        for (int q = 0; q < TFR_ROUNDS + 1; ++q) {
            const int e = e0 + q;
            if (e < e1) {
                while (L.sbase[lo + 1] <= (u32)e) ++lo;   // (the table ends with n: the walk stops)
                const u32 j = (u32)e - L.sbase[lo];
                meta[q] = ((u32)lo << 16) | j;
                idx[q] = (u32)v.indices[v.lookup0 + L.sp0[lo] + j];
            }
        }
#pragma unroll
        for (int q = 0; q < TFR_ROUNDS + 1; ++q)
            if (e0 + q < e1) L.buf[e0 + q] = ((u64)(fb + idx[q]) << 32) | (u64)meta[q];
    }
    const int passes = (bits + 7) / 8 > 0 ? (bits + 7) / 8 : 1;
    const int width = (bits + passes - 1) / passes > 0 ? (bits + passes - 1) / passes : 1;
    const int NB = 1 << width;
    const int chunk = ((n + W * WAVE - 1) / (W * WAVE)) * WAVE;   // keys per wave, a multiple of 64
    const int rounds = chunk / WAVE;
    const u64 lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    u64* const in = L.buf;
    u64* const out = L.buf;   // in place: the barriers between ranking and placing separate the last read from the first write
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = pass * width;
        for (int i = threadIdx.x; i < W * NB; i += NT) L.cnt[i] = 0;
        __syncthreads();   // also: the keys of the previous step are in place
        u64 key[TFR_ROUNDS];
        u32 rank[TFR_ROUNDS];
        const int w_end = min(n, (wv + 1) * chunk);
#pragma unroll
        for (int r = 0; r < TFR_ROUNDS; ++r) {
            if (r < rounds) {
                const int i = wv * chunk + r * WAVE + lane;
                const bool valid = i < w_end;
                key[r] = valid ? in[i] : ~0ull;
                const u32 d = (((u32)(key[r] >> 32) - fb) >> shift) & (u32)(NB - 1);
                u64 peers = __ballot(valid);
                for (int b = 0; b < width; ++b) {
                    const bool bit = (d >> b) & 1u;
                    const u64 m = __ballot(bit);
                    peers &= bit ? m : ~m;
                }
                const int leader = valid ? (__ffsll((unsigned long long)peers) - 1) : lane;
                u32 old = 0;
                if (valid && lane == leader) {
                    old = L.cnt[wv * NB + d];
                    L.cnt[wv * NB + d] = (uint16_t)(old + (u32)__popcll(peers));
                }
                old = __shfl(old, leader, WAVE);
                rank[r] = old + (u32)__popcll(peers & lt_mask);
            }
        }
        __syncthreads();
        u32 total = 0;
        if ((int)threadIdx.x < NB) {
            for (int ww = 0; ww < W; ++ww) {
                const u32 cc = L.cnt[ww * NB + threadIdx.x];
                L.cnt[ww * NB + threadIdx.x] = (uint16_t)total;
                total += cc;
            }
        }
        int tile_count;
        const int ds = block_excl_scan((int)total, L.sh_scan, &tile_count);
        if ((int)threadIdx.x < NB) L.digstart[threadIdx.x] = (u32)ds;
        __syncthreads();
#pragma unroll
        for (int r = 0; r < TFR_ROUNDS; ++r) {
            if (r < rounds) {
                const int i = wv * chunk + r * WAVE + lane;
                if (i < w_end) {
                    const u32 d = (((u32)(key[r] >> 32) - fb) >> shift) & (u32)(NB - 1);
                    out[L.digstart[d] + L.cnt[wv * NB + d] + rank[r]] = key[r];
                }
            }
        }
        __syncthreads();   // every wave has placed its keys and is done with the counters
    }
    return L.buf;
}

// cap: key capacity of an LDS buffer (bitonic: a power of two); ms: most samples a task has in one set (radix)
// cls: 0 = every (task, field); 1 = only the small ones (at most small_n lookups and small_ms samples per set);
// 2 = only the others.  A launch is sized for its largest (task, field): with very uneven tasks the small ones get a
// launch of their own, with workgroups and LDS that let several share a compute unit.
template <bool LDS_UNIQ, bool RADIX>
__global__ void tf_sort_kernel(TfSortArgs a, int cap, int ms, int cls, int small_n, int small_ms) {
    extern __shared__ u64 sh_dyn[];  // bitonic: keys [cap] (+ u32 uniq[cap]); radix: two key buffers, uniq, bag tables, counters
    __shared__ int sh_scan[20];
    __shared__ int sh_fill;
    __shared__ u32 sh_digstart[256];
    u64* sh_keys = sh_dyn;
    TfRadixLds L;
    if (RADIX) {
        L.buf = sh_dyn;
        u32* w32 = reinterpret_cast<u32*>(sh_dyn + cap) + (LDS_UNIQ ? cap : 0);
        L.sbase = w32;
        L.sp0 = w32 + (ms + 1);
        L.cnt = reinterpret_cast<uint16_t*>(w32 + 2 * ms + 2);
        L.digstart = sh_digstart;
        L.sh_scan = sh_scan;
    }
    const int f = blockIdx.x, t = blockIdx.y;
    const size_t tf = (size_t)t * a.F + f;
    const u32 fb = (u32)a.field_base[f];
    const u32 n = a.cnt_sup[tf], B = a.base_sup[tf];
    const u32 nq = a.cnt_qry[tf], Bq = a.base_qry[tf];
    if (cls) {
        const int64_t ns_ = a.sup.task_offsets[a.t0 + t + 1] - a.sup.task_offsets[a.t0 + t];
        const int64_t nq_ = a.qry.task_offsets[a.t0 + t + 1] - a.qry.task_offsets[a.t0 + t];
        const bool small = (int)max(n, nq) <= small_n && max(ns_, nq_) <= (int64_t)small_ms;
        if (small != (cls == 1)) return;
    }
    u32* uniq = LDS_UNIQ ? (u32*)(sh_dyn + cap) : (a.slot_rows + B);
    int bits = 1;
    while (((int64_t)1 << bits) < a.field_base[f + 1] - a.field_base[f]) ++bits;
    int n_unique = 0;

    // ---- phase A: support lookups sorted by (row, sample, position in bag)
    const int64_t s_lo = a.sup.task_offsets[a.t0 + t], s_hi = a.sup.task_offsets[a.t0 + t + 1];
    if (n > 0) {
        if (RADIX) {
            sh_keys = tf_radix_sorted(L, a.sup, a.F, f, s_lo, s_hi, fb, bits, (int)n);
        } else {
            load_tf_keys(sh_keys, &sh_fill, a.sup, a.F, f, s_lo, s_hi, fb);
            int n2 = 1;
            while (n2 < (int)n) n2 <<= 1;
            for (int i = n + threadIdx.x; i < n2; i += blockDim.x) sh_keys[i] = ~0ull;
            __syncthreads();
            bitonic_sort_lds(sh_keys, n2);
        }
        const int chunk = ((int)n + blockDim.x - 1) / blockDim.x;
        const int i0 = min((int)n, (int)threadIdx.x * chunk), i1 = min((int)n, i0 + chunk);
        int c = 0;
        // row of the key before this thread's range, read before any key is rewritten below
        const u32 row_before = i0 > 0 && i0 < (int)n ? (u32)(sh_keys[i0 - 1] >> 32) : ~0u;
        for (int i = i0; i < i1; ++i) c += (i == 0) || ((sh_keys[i] >> 32) != (sh_keys[i - 1] >> 32));
        int slot = block_excl_scan(c, sh_scan, &n_unique) - 1;
        // radix: the slot of every key replaces its row first, so that the second sweep below has independent
        // iterations and reads only LDS (the bag tables of the sort give every lookup's position)
        u32 prev = row_before;
        for (int i = i0; i < i1; ++i) {
            const u64 key = sh_keys[i];
            const u32 row = (u32)(key >> 32);
            const bool head = RADIX ? (i == 0 || row != prev) : ((i == 0) || (row != (u32)(sh_keys[i - 1] >> 32)));
            prev = row;
            if (head) {
                ++slot;
                a.slot_start[B + tf + slot] = (int32_t)(B + i);
                a.slot_rows[B + slot] = row;
                if (LDS_UNIQ) uniq[slot] = row;
            }
            if (RADIX) {
                sh_keys[i] = ((u64)(u32)slot << 32) | (key & 0xFFFFFFFFull);
            } else {
                const int s = (int)((key >> 16) & 0xFFFF), j = (int)(key & 0xFFFF);
                const int64_t p = a.sup.bag_offsets[(s_lo + s) * a.F + f] + j;
                a.sup_slot[p - a.sup.lookup0] = slot;
                a.sup_sorted[B + i] = make_int2(a.sup_rows[s_lo + s] - a.sup_row_base, slot);
            }
        }
        if (RADIX) {
            __syncthreads();
            const int prow0 = a.sup_rows[s_lo] - a.sup_row_base;   // rows of a task are consecutive
            for (int i = threadIdx.x; i < (int)n; i += blockDim.x) {
                const u64 key = sh_keys[i];
                const int s = (int)((key >> 16) & 0xFFFF), j = (int)(key & 0xFFFF);
                const int sl = (int)(key >> 32);
                a.sup_slot[L.sp0[s] + j] = sl;
                a.sup_sorted[B + i] = make_int2(prow0 + s, sl);
            }
        }
    }
    if (threadIdx.x == 0) {
        a.slot_start[B + tf + n_unique] = (int32_t)(B + n);
        a.n_slots[tf] = (u32)n_unique;
    }
    __threadfence_block();
    __syncthreads();

    // ---- phase B: query lookups sorted the same way, joined against the support rows
    if (nq == 0) {
        for (int u = threadIdx.x; u < n_unique; u += blockDim.x) {
            a.qseg_lo[B + u] = (int32_t)Bq;
            a.qseg_hi[B + u] = (int32_t)Bq;
        }
        return;
    }
    const int64_t q_lo = a.qry.task_offsets[a.t0 + t], q_hi = a.qry.task_offsets[a.t0 + t + 1];
    if (RADIX) {
        sh_keys = tf_radix_sorted(L, a.qry, a.F, f, q_lo, q_hi, fb, bits, (int)nq);
    } else {
        sh_keys = sh_dyn;
        load_tf_keys(sh_keys, &sh_fill, a.qry, a.F, f, q_lo, q_hi, fb);
        int n2 = 1;
        while (n2 < (int)nq) n2 <<= 1;
        for (int i = nq + threadIdx.x; i < n2; i += blockDim.x) sh_keys[i] = ~0ull;
        __syncthreads();
        bitonic_sort_lds(sh_keys, n2);
    }
    const int qprow0 = a.qry_rows[q_lo] - a.qry_row_base;
    for (int i = threadIdx.x; i < (int)nq; i += blockDim.x) {
        const u64 key = sh_keys[i];
        const u32 row = (u32)(key >> 32);
        int lo = 0, hi = n_unique;  // first slot with uniq >= row
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (uniq[mid] < row) lo = mid + 1;
            else hi = mid;
        }
        const int slot = (lo < n_unique && uniq[lo] == row) ? lo : -1;
        const int s = (int)((key >> 16) & 0xFFFF), j = (int)(key & 0xFFFF);
        if (RADIX) {
            a.qry_slot[L.sp0[s] + j] = slot;
            a.qry_sorted[Bq + i] = make_int2(qprow0 + s, slot);
        } else {
            const int64_t p = a.qry.bag_offsets[(q_lo + s) * a.F + f] + j;
            a.qry_slot[p - a.qry.lookup0] = slot;
            a.qry_sorted[Bq + i] = make_int2(a.qry_rows[q_lo + s] - a.qry_row_base, slot);
        }
    }
    for (int u = threadIdx.x; u < n_unique; u += blockDim.x) {
        const u64 klo = (u64)uniq[u] << 32, khi = ((u64)uniq[u] + 1) << 32;
        int lo = 0, hi = (int)nq;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (sh_keys[mid] < klo) lo = mid + 1;
            else hi = mid;
        }
        int lo2 = lo, hi2 = (int)nq;
        while (lo2 < hi2) {
            const int mid = (lo2 + hi2) >> 1;
            if (sh_keys[mid] < khi) lo2 = mid + 1;
            else hi2 = mid;
        }
        a.qseg_lo[B + u] = (int32_t)(Bq + lo);
        a.qseg_hi[B + u] = (int32_t)(Bq + lo2);
    }
}

int tf_sort_max_cap() { return 16384; }

// max_tf: the largest number of lookups any (task, field) of the wave has in one set; max_set_rows: the largest
// number of samples any task of the wave has in one set
void launch_tf_sort(hipStream_t st, const TfSortArgs& a, int max_tf, int max_set_rows) {
    if (a.Tw <= 0 || a.F <= 0) return;
    dim3 grid(a.F, a.Tw);
    int cap = 1024;
    while (cap < max_tf) cap <<= 1;
    if (max_set_rows <= TFR_MAXS) {   // radix sort in LDS
        auto launch = [&](int mtf, int mrows, int cls, int small_n, int small_ms) {
            int cp = 1024;
            while (cp < mtf) cp <<= 1;
            const int kcap = (mtf + 63) / 64 * 64 + 64;                   // keys in the buffer
            const int ms = mrows > 0 ? mrows : 1;
            int nt = cp / 8;                                              // at most 8 rounds of 64 keys per wave while the block
            nt = nt < 256 ? 256 : (nt > 1024 ? 1024 : nt);                // allows (TFR_ROUNDS = 16 at the largest capacity)
            const size_t fixed = (size_t)(2 * ms + 2) * 4 + (size_t)(nt / WAVE) * 256 * 2;
            // the row list in LDS while two workgroups still fit a compute unit -- or when only one fits anyway
            const bool lds_uniq = (size_t)kcap * 12 + fixed <= 80 * 1024 ||
                                  ((size_t)kcap * 8 + fixed > 80 * 1024 && (size_t)kcap * 12 + fixed <= 158 * 1024);
            const size_t shmem = (size_t)kcap * 8 + (lds_uniq ? (size_t)kcap * 4 : 0) + fixed;
            if (lds_uniq) {
                hipFuncSetAttribute((const void*)tf_sort_kernel<true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
                hipLaunchKernelGGL((tf_sort_kernel<true, true>), grid, dim3(nt), shmem, st, a, kcap, ms, cls, small_n, small_ms);
            } else {
                hipFuncSetAttribute((const void*)tf_sort_kernel<false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
                hipLaunchKernelGGL((tf_sort_kernel<false, true>), grid, dim3(nt), shmem, st, a, kcap, ms, cls, small_n, small_ms);
            }
        };
        // uneven tasks: the (task, field)s of at most TF_SMALL_N lookups and TF_SMALL_MS samples per set run in a launch
        // of their own (every workgroup of either launch checks its class first)
        if (max_tf > 2 * TF_SMALL_N && (int64_t)a.Tw * a.F >= 32) {
            launch(TF_SMALL_N, max_set_rows < TF_SMALL_MS ? max_set_rows : TF_SMALL_MS, 1, TF_SMALL_N, TF_SMALL_MS);
            launch(max_tf, max_set_rows, 2, TF_SMALL_N, TF_SMALL_MS);
        } else {
            launch(max_tf, max_set_rows, 0, 0, 0);
        }
        return;
    }
    const bool lds_uniq = cap <= 8192;
    const size_t shmem = (size_t)cap * (lds_uniq ? 12 : 8);
    const int nt = cap <= 1024 ? 256 : (cap <= 4096 ? 512 : 1024);
    if (lds_uniq) {
        hipFuncSetAttribute((const void*)tf_sort_kernel<true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
        hipLaunchKernelGGL((tf_sort_kernel<true, false>), grid, dim3(nt), shmem, st, a, cap, 0, 0, 0, 0);
    } else {
        hipFuncSetAttribute((const void*)tf_sort_kernel<false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
        hipLaunchKernelGGL((tf_sort_kernel<false, false>), grid, dim3(nt), shmem, st, a, cap, 0, 0, 0, 0);
    }
}

// ------------------------------------------------------------------------------------------------
// global (field,row) ordering of all lookups: keys, stable LSD radix sort, segments
// ------------------------------------------------------------------------------------------------
// One workgroup per 256 consecutive bags: their lookups are one contiguous range, walked by all lanes with
// coalesced reads and writes; the bag of a lookup is found by bisection of the 257 staged offsets.
// The value of a lookup names its bag in the gradient buffer: (row of the sample) * F + field when enc.rshift is 0, else
// the bit fields row << rshift | field << pshift | position of the lookup in its bag (ValEnc).
__global__ __launch_bounds__(256) void build_keys_kernel(int F, const int64_t* field_base, const int64_t* bag_offsets,
                                                         const int32_t* indices, int64_t n_bags, int64_t lookup0,
                                                         const int32_t* __restrict__ row_map, u32 row0, ValEnc enc, u32* keys,
                                                         u32* vals) {
    __shared__ int64_t offs[257];
    const int64_t b0 = (int64_t)blockIdx.x * 256;
    const int nb = (int)min<int64_t>(256, n_bags - b0);
    for (int i = threadIdx.x; i <= nb; i += 256) offs[i] = bag_offsets[b0 + i];
    __syncthreads();
    const int64_t p0 = offs[0], p1 = offs[nb];
    for (int64_t p = p0 + threadIdx.x; p < p1; p += 256) {
        int lo = 0, hi = nb;   // last bag with offs[bag] <= p
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (offs[mid] <= p) lo = mid;
            else hi = mid;
        }
        const int64_t b = b0 + lo;
        const int f = (int)(b % F);
        const u32 row = row0 + (u32)row_map[b / F];   // row of the sample in the gradient buffer
        keys[p - lookup0] = (u32)field_base[f] + (u32)indices[p];
        vals[p - lookup0] = enc.rshift ? (row << enc.rshift) | ((u32)f << enc.pshift) | (u32)(p - offs[lo]) : row * (u32)F + (u32)f;
    }
}

// bag_offsets / row_map point at the first bag / sample of the range (a multiple of F bags); lookup0 is the range's first
// lookup: keys and vals are numbered from it
void launch_build_keys(hipStream_t st, int F, const int64_t* field_base, const int64_t* bag_offsets,
                       const int32_t* indices, int64_t n_bags, int64_t lookup0, const int32_t* row_map, u32 row0, ValEnc enc,
                       u32* keys, u32* vals) {
    if (n_bags <= 0) return;
    hipLaunchKernelGGL(build_keys_kernel, dim3((unsigned)((n_bags + 255) / 256)), dim3(256), 0, st, F, field_base,
                       bag_offsets, indices, n_bags, lookup0, row_map, row0, enc, keys, vals);
}

// ------------------------------------------------------------------------------------------------
// the same keys laid out field after field (support lookups of a field first, then its query lookups, each in input
// order): the field needs no sorting then -- every field's range is sorted by row alone, in fewer radix passes
// ------------------------------------------------------------------------------------------------
// One workgroup per field: fm_off_*[t * F + f] = lookups of field f in the tasks before t (per set), tot[f] / tot[F + f]
// = the field's support / query lookups in the wave.
__global__ __launch_bounds__(256) void field_offsets_kernel(int F, int Tw, const u32* cnt_s, const u32* cnt_q, u32* fm_off_s,
                                                            u32* fm_off_q, u32* tot) {
    __shared__ int sh[8];
    const int f = blockIdx.x;
    for (int set = 0; set < 2; ++set) {
        const u32* cnt = set ? cnt_q : cnt_s;
        u32* off = set ? fm_off_q : fm_off_s;
        u32 run = 0;
        for (int t0 = 0; t0 < Tw; t0 += 256) {
            const int t = t0 + threadIdx.x;
            const u32 c = t < Tw ? cnt[(size_t)t * F + f] : 0u;
            int total;
            const u32 ex = (u32)block_excl_scan((int)c, sh, &total);
            if (t < Tw) off[(size_t)t * F + f] = run + ex;
            run += (u32)total;
            __syncthreads();
        }
        if (threadIdx.x == 0) tot[set * F + f] = run;
    }
}

// first key and first tile of every field's range, and what a key of the field has in front of its row number
__global__ void field_table_kernel(int F, const u32* tot, const int64_t* field_base, int tile_keys, u32* key_pos, u32* tile_base,
                                   u32* key_sub) {
    if (threadIdx.x || blockIdx.x) return;
    u32 k = 0, tl = 0;
    for (int f = 0; f < F; ++f) {
        key_pos[f] = k;
        tile_base[f] = tl;
        key_sub[f] = (u32)field_base[f];
        const u32 nf = tot[f] + tot[F + f];
        k += nf;
        tl += (nf + (u32)tile_keys - 1) / (u32)tile_keys;
    }
    key_pos[F] = k;
    tile_base[F] = tl;
    key_sub[F] = 0u;
}

#define BKF_CH 1024   // bags of a task staged at a time
// One workgroup per (field, task, set): the bags (sample, field) of the task, BKF_CH at a time -- their lengths are
// scanned into LDS, then every lane takes lookups of the piece in order (coalesced writes), finding a lookup's bag
// by bisection of the staged table.
__global__ __launch_bounds__(256) void build_keys_fm_kernel(FieldKeysArgs a) {
    __shared__ u32 sbase[BKF_CH + 1];
    __shared__ u32 sp0[BKF_CH];
    __shared__ int sh[8];
    const int f = blockIdx.x, t = blockIdx.y, set = blockIdx.z;
    const SetView& v = set ? a.qry : a.sup;
    const size_t tf = (size_t)t * a.F + f;
    const u32 n_tf = (set ? a.cnt_q : a.cnt_s)[tf];
    if (n_tf == 0) return;
    const int64_t s_lo = v.task_offsets[a.t0 + t], s_hi = v.task_offsets[a.t0 + t + 1];
    const int32_t* prow = set ? a.prow_q : a.prow_s;
    const u32 row0 = set ? a.row0_q : a.row0_s;
    const u32 fb = (u32)a.field_base[f];
    size_t dest = (size_t)a.key_pos[f] + (set ? a.tot[f] : 0u) + (set ? a.fm_off_q : a.fm_off_s)[tf];
    for (int64_t c0 = s_lo; c0 < s_hi; c0 += BKF_CH) {
        const int nb = (int)min<int64_t>(BKF_CH, s_hi - c0);
        __syncthreads();   // the table of the piece before has been read
        {
            const int b0 = (int)threadIdx.x * 4;   // four consecutive bags per thread
            u32 len[4], p0r[4];
            u32 sum = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                len[q] = 0; p0r[q] = 0;
                if (b0 + q < nb) {
                    const int64_t bag = (c0 + b0 + q) * a.F + f;
                    const int64_t p0 = v.bag_offsets[bag];
                    len[q] = (u32)(v.bag_offsets[bag + 1] - p0);
                    p0r[q] = (u32)(p0 - v.lookup0);
                }
                sum += len[q];
            }
            int total;
            u32 run = (u32)block_excl_scan((int)sum, sh, &total);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (b0 + q < nb) {
                    sbase[b0 + q] = run;
                    sp0[b0 + q] = p0r[q];
                    run += len[q];
                }
            if (threadIdx.x == 0) sbase[nb] = (u32)total;
        }
        __syncthreads();
        const u32 total = sbase[nb];
        for (u32 e0 = threadIdx.x; e0 < total; e0 += 4 * 256) {
            int bag[4];
            u32 j[4], idx[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32 e = e0 + q * 256;
                bag[q] = 0; j[q] = 0; idx[q] = 0;
                if (e < total) {
                    int lo = 0, hi = nb;   // last bag whose first lookup is <= e (empty bags share their successor's)
                    while (hi - lo > 1) {
                        const int mid = (lo + hi) >> 1;
                        if (sbase[mid] <= e) lo = mid;
                        else hi = mid;
                    }
                    bag[q] = lo;
                    j[q] = e - sbase[lo];
                    idx[q] = (u32)v.indices[v.lookup0 + sp0[lo] + j[q]];
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32 e = e0 + q * 256;
                if (e < total) {
                    const u32 row = row0 + (u32)prow[c0 + bag[q]];
                    a.keys[dest + e] = fb + idx[q];
                    a.vals[dest + e] = (row << a.enc.rshift) | ((u32)f << a.enc.pshift) | j[q];
                }
            }
        }
        dest += total;
    }
}

// tables: 3 (F + 1) words (key_pos, tile_base, key_sub), then 2 F words of totals
void launch_build_keys_by_field(hipStream_t st, FieldKeysArgs a, u32* tables) {
    if (a.F <= 0 || a.Tw <= 0) return;
    u32* key_pos = tables;
    u32* tile_base = key_pos + (a.F + 1);
    u32* key_sub = tile_base + (a.F + 1);
    u32* tot = key_sub + (a.F + 1);
    hipLaunchKernelGGL(field_offsets_kernel, dim3(a.F), dim3(256), 0, st, a.F, a.Tw, a.cnt_s, a.cnt_q, a.fm_off_s, a.fm_off_q, tot);
    hipLaunchKernelGGL(field_table_kernel, dim3(1), dim3(64), 0, st, a.F, tot, a.field_base, RS_TILE_KEYS, key_pos, tile_base, key_sub);
    a.key_pos = key_pos;
    a.tot = tot;
    hipLaunchKernelGGL(build_keys_fm_kernel, dim3(a.F, a.Tw, 2), dim3(256), 0, st, a);
}
SegTab field_seg_tab(int F, u32* tables) { return SegTab{F, tables + (F + 1), tables, tables + 2 * (F + 1)}; }
size_t field_table_words(int F) { return (size_t)5 * (F + 1); }

#define RS_NT 256
#define RS_ITEMS 8
#define RS_TILE (RS_NT * RS_ITEMS)
static_assert(RS_TILE == RS_TILE_KEYS, "tile size");
#define RS_WAVES (RS_NT / WAVE)

// Digits are BITS wide (8 or 9): 25-bit row keys sort in three 9-bit passes instead of four 8-bit ones.
// Tiles are dealt to workgroups so that every XCD (workgroups are spread over the 8 XCDs round-robin) walks one
// contiguous range of tiles: the pieces that neighbouring tiles write into a digit's output range then meet in one L2.
__device__ __forceinline__ int rs_tile_of_block(int nblk) {
    const int per = (nblk + 7) >> 3;
    return (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
}

// What a pass sorts by: a digit of the key, or (BYTASK) a digit of the task that the value's sample belongs to --
// the stable pass that turns the (field, row) order of a wave's lookups into (task, field, row) order.
__device__ __forceinline__ u32 rs_task_of(const TaskOf& m, u32 val) {
    const u32 r = min(val >> m.rshift, m.n_rows - 1u);   // (every value names a row of the wave; the bound keeps any other inside the tables)
    // tasks of one size (a power of two of padded rows in both sets): the task is a shift of the row, no table read
    if (m.uniform_shift >= 0) return (r < m.n_sup_rows ? r : r - m.n_sup_rows) >> m.uniform_shift;
    return (u32)(r < m.n_sup_rows ? m.row_task_s[r] : m.row_task_q[r - m.n_sup_rows]);
}

// A pass may sort several independent ranges of the list at once (SegTab: the fields of a wave's lookups, each range
// holding one field's keys).  Tiles then never straddle two ranges: tile numbers run range after range, a range's
// share of the digit-count table is laid out [digit][tile of the range] behind the shares of the ranges before it, so
// that ONE exclusive scan over the whole table still yields every (range, digit, tile)'s place in the output; the
// digit is taken from the key minus the range's key base.  seg.n_seg == 0: one range, the whole list.
struct RsTile {
    int64_t k0, k1;      // keys of the tile
    u32 key_base;        // subtracted from a key before its digit is taken
    size_t h0;           // count-table index of (digit 0, this tile)
    size_t hstride;      // ... and the distance between digits
    bool any;
};
__device__ __forceinline__ RsTile rs_tile(const SegTab& seg, int tile, int nblk, int64_t n, int nb) {
    RsTile t;
    if (seg.n_seg == 0) {
        t.k0 = (int64_t)tile * RS_TILE;
        t.k1 = min(n, t.k0 + RS_TILE);
        t.key_base = 0u;
        t.h0 = (size_t)tile;
        t.hstride = (size_t)nblk;
        t.any = tile < nblk;
        return t;
    }
    int lo = 0, hi = seg.n_seg;   // last range whose first tile is <= tile
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (seg.tile_base[mid] <= (u32)tile) lo = mid;
        else hi = mid;
    }
    const u32 tb = seg.tile_base[lo], te = seg.tile_base[lo + 1];
    t.any = (u32)tile < te;       // (tiles past the last range's: nothing to do)
    t.k0 = (int64_t)seg.key_base_pos[lo] + (int64_t)((u32)tile - tb) * RS_TILE;
    t.k1 = min((int64_t)seg.key_base_pos[lo + 1], t.k0 + RS_TILE);
    t.key_base = seg.key_sub[lo];
    t.hstride = (size_t)(te - tb);
    t.h0 = (size_t)nb * tb + ((u32)tile - tb);
    return t;
}

template <int BITS, bool BYTASK>
__global__ void radix_hist_kernel(const u32* src, int64_t n, int shift, u32* hist, int nblk, TaskOf tk, SegTab seg) {
    constexpr int NB = 1 << BITS;
    __shared__ u32 h[NB];
    const int tile = rs_tile_of_block(nblk);
    if (tile >= nblk) return;
    const RsTile T = rs_tile(seg, tile, nblk, n, NB);
    if (!T.any) return;
    for (int i = threadIdx.x; i < NB; i += RS_NT) h[i] = 0;
    __syncthreads();
    const int64_t base = T.k0;
    const int64_t n_end = T.k1;
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int i = 0; i < RS_ITEMS; ++i) {
        const int64_t idx = base + i * RS_NT + threadIdx.x;
        // One atomic per run of equal digits in the wave instead of one per lane.  By task: inside a row the lookups
        // are in input order, i.e. by task, so a hot row gives long runs of one digit, which as one atomic per lane
        // would all queue on one counter.  By key: from the second pass on the keys of a hot row lie next to each
        // other (they share every digit sorted so far), and LDS atomics retire about one lane per cycle.
        const bool valid = idx < n_end;
        u32 d = 0xFFFFFFFFu;
        if (valid) d = ((BYTASK ? rs_task_of(tk, src[idx]) : src[idx] - T.key_base) >> shift) & (NB - 1);
        const u32 dp = __shfl_up(d, 1, WAVE);
        const u64 heads = __ballot(lane == 0 || d != dp);
        if (valid && (lane == 0 || d != dp)) {
            const u64 later = lane == 63 ? 0ull : (heads >> (lane + 1));   // heads after this lane
            const int run = later ? __ffsll((unsigned long long)later) : 64 - lane;
            atomicAdd(&h[d], (u32)run);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < NB; i += RS_NT) hist[T.h0 + (size_t)i * T.hstride] = h[i];
}

// Stable scatter: every wave owns a contiguous 1/4 of the tile and ranks its keys round by round (64
// consecutive keys per round) with ballot matching, so equal digits keep their input order.
template <int BITS, bool BYTASK>
__global__ void radix_scatter_kernel(const u32* kin, const u32* vin, u32* kout, u32* vout, const u32* gofs,
                                     int64_t n_all, int shift, int nblk, TaskOf tk, SegTab seg) {
    constexpr int NB = 1 << BITS, DPT = NB / RS_NT;   // digits per thread in the per-digit phase
    __shared__ u32 cnt[RS_WAVES][NB];
    __shared__ u32 digstart[NB];
    __shared__ u32 skeys[RS_TILE];
    __shared__ u32 svals[RS_TILE];
    __shared__ uint16_t sdig[BYTASK ? RS_TILE : 1];   // the digit of every staged pair (a key names its own)
    __shared__ int sh_scan[RS_WAVES + 2];
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    const int tile = rs_tile_of_block(nblk);
    if (tile >= nblk) return;
    const RsTile T = rs_tile(seg, tile, nblk, n_all, NB);
    if (!T.any) return;
    for (int i = threadIdx.x; i < RS_WAVES * NB; i += RS_NT) (&cnt[0][0])[i] = 0;
    __syncthreads();
    const int64_t tile0 = T.k0, n = T.k1;
    u32 key[RS_ITEMS], val[RS_ITEMS], rank[RS_ITEMS], dig[RS_ITEMS];
    const u64 lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int r = 0; r < RS_ITEMS; ++r) {
        const int64_t idx = tile0 + (int64_t)w * (WAVE * RS_ITEMS) + r * WAVE + lane;
        const bool valid = idx < n;
        key[r] = valid ? kin[idx] : 0xFFFFFFFFu;
        val[r] = valid ? vin[idx] : 0u;
        const u32 d = ((BYTASK ? (valid ? rs_task_of(tk, val[r]) : 0u) : key[r] - T.key_base) >> shift) & (NB - 1);
        dig[r] = d;
        u64 peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < BITS; ++b) {
            const bool bit = (d >> b) & 1u;
            const u64 m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const int leader = valid ? (__ffsll((unsigned long long)peers) - 1) : lane;
        u32 old = 0;
        if (valid && lane == leader) {
            old = cnt[w][d];
            cnt[w][d] = old + (u32)__popcll(peers);
        }
        old = __shfl(old, leader, WAVE);
        rank[r] = old + (u32)__popcll(peers & lt_mask);   // (a wave's counters are its own: no barrier between rounds)
    }
    __syncthreads();
    // per digit: exclusive prefix over the waves, block total, start of each digit inside the tile
    u32 total[DPT];
    u32 mine = 0;
#pragma unroll
    for (int k = 0; k < DPT; ++k) {
        const int d = threadIdx.x * DPT + k;
        u32 t = 0;
#pragma unroll
        for (int ww = 0; ww < RS_WAVES; ++ww) {
            const u32 c = cnt[ww][d];
            cnt[ww][d] = t;
            t += c;
        }
        total[k] = t;
        mine += t;
    }
    int tile_count;
    u32 ds = (u32)block_excl_scan((int)mine, sh_scan, &tile_count);
#pragma unroll
    for (int k = 0; k < DPT; ++k) {
        digstart[threadIdx.x * DPT + k] = ds;
        ds += total[k];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RS_ITEMS; ++r) {
        const int64_t idx = tile0 + (int64_t)w * (WAVE * RS_ITEMS) + r * WAVE + lane;
        if (idx < n) {
            const u32 d = dig[r];
            const u32 pos = digstart[d] + cnt[w][d] + rank[r];
            skeys[pos] = key[r];
            svals[pos] = val[r];
            if (BYTASK) sdig[pos] = (uint16_t)d;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RS_ITEMS; ++i) {
        const int pos = i * RS_NT + threadIdx.x;
        if (pos < tile_count) {
            const u32 k = skeys[pos];
            const u32 d = BYTASK ? (u32)sdig[pos] : ((k - T.key_base) >> shift) & (NB - 1);
            const size_t dst = (size_t)gofs[T.h0 + (size_t)d * T.hstride] + (pos - digstart[d]);
            kout[dst] = k;
            vout[dst] = svals[pos];
        }
    }
}

// extra_tiles: tiles beyond ceil(n / tile) that a pass over several ranges may need (one per range)
size_t radix_hist_words(int64_t n, int extra_tiles) {
    const int64_t nblk = (n + RS_TILE - 1) / RS_TILE + extra_tiles;
    return (size_t)(512 * nblk + 64) + scan_tmp_words(512 * nblk);
}

template <int BITS, bool BYTASK>
static void radix_pass(hipStream_t st, const u32* ki, const u32* vi, u32* ko, u32* vo, int64_t n, int shift, u32* hist,
                       const TaskOf& tk, const SegTab& seg) {
    // ranges: at most one partly filled tile per range beyond the tiles of the whole list; the count table is cleared
    // first, since the tiles past the last range's write nothing into it
    const int nblk = (int)((n + RS_TILE - 1) / RS_TILE) + seg.n_seg;
    u32* scan_tmp = hist + ((size_t)512 * nblk + 63) / 64 * 64;
    const dim3 grid((nblk + 7) / 8 * 8);
    if (seg.n_seg) launch_fill_u32(st, hist, (int64_t)(1 << BITS) * nblk, 0u);
    hipLaunchKernelGGL((radix_hist_kernel<BITS, BYTASK>), grid, dim3(RS_NT), 0, st, BYTASK ? vi : ki, n, shift, hist, nblk, tk, seg);
    launch_scan_u32(st, hist, hist, (int64_t)(1 << BITS) * nblk, scan_tmp, nullptr);
    hipLaunchKernelGGL((radix_scatter_kernel<BITS, BYTASK>), grid, dim3(RS_NT), 0, st, ki, vi, ko, vo, hist, n, shift, nblk, tk, seg);
}

// Returns the number of passes made: after an odd number the result is in (keys_tmp, vals_tmp).
int launch_radix_sort(hipStream_t st, u32* keys, u32* vals, u32* keys_tmp, u32* vals_tmp, int64_t n, int bits,
                      u32* hist, const SegTab* seg_in) {
    if (n <= 0) return 0;
    const SegTab seg = seg_in ? *seg_in : SegTab{0, nullptr, nullptr, nullptr};
    if (bits < 1) bits = 1;
    if (bits > 32) bits = 32;
    const int p8 = (bits + 7) / 8, p9 = (bits + 8) / 9;
    const int width = p9 < p8 ? 9 : 8, passes = p9 < p8 ? p9 : p8;
    const TaskOf none{nullptr, nullptr, 0u, 0u, 0, -1};
    u32 *ki = keys, *vi = vals, *ko = keys_tmp, *vo = vals_tmp;
    for (int p = 0; p < passes; ++p) {
        if (width == 9) radix_pass<9, false>(st, ki, vi, ko, vo, n, width * p, hist, none, seg);
        else radix_pass<8, false>(st, ki, vi, ko, vo, n, width * p, hist, none, seg);
        u32* t = ki; ki = ko; ko = t;
        t = vi; vi = vo; vo = t;
    }
    return passes;
}

// The pairs of (keys, vals), which are in (field, row) order, stably re-ordered by the task of their sample: the result
// is in (task, field, row) order, support lookups before query lookups inside a row, each in input order.  One pass
// for up to 512 tasks into (out_keys, out_vals); two passes of at most 8 bits beyond that, the first into
// (mid_keys, mid_vals).  The input is left as it is.
void launch_task_sort(hipStream_t st, const u32* keys, const u32* vals, u32* mid_keys, u32* mid_vals, u32* out_keys,
                      u32* out_vals, int64_t n, int n_tasks, const TaskOf& tk, u32* hist) {
    if (n <= 0) return;
    int bits = 1;
    while ((1 << bits) < n_tasks) ++bits;
    const SegTab one{0, nullptr, nullptr, nullptr};
    if (bits <= 8) {
        radix_pass<8, true>(st, keys, vals, out_keys, out_vals, n, 0, hist, tk, one);
    } else if (bits == 9) {
        radix_pass<9, true>(st, keys, vals, out_keys, out_vals, n, 0, hist, tk, one);
    } else {   // (the second pass masks with 8 bits: bits <= 16)
        radix_pass<8, true>(st, keys, vals, mid_keys, mid_vals, n, 0, hist, tk, one);
        radix_pass<8, true>(st, mid_keys, mid_vals, out_keys, out_vals, n, 8, hist, tk, one);
    }
}
int task_sort_passes(int n_tasks) { return n_tasks > 512 ? 2 : 1; }

// ------------------------------------------------------------------------------------------------
// per-(task, field) dictionaries and overlap join read off the (task, field, row) order of the wave's lookups
// ------------------------------------------------------------------------------------------------
// One workgroup per (task, field): its lookups are one contiguous run of the ordered list, support lookups before
// query lookups inside every row.  The run is walked 1024 entries at a time (four consecutive entries per thread);
// what the entries need from before them -- how many support lookups, how many distinct support rows, and the slot of
// the row they belong to (none when the support set does not look the row up) -- comes from one block-wide sum scan of
// two packed counters and one segmented copy scan, carried from one 1024-entry piece to the next.  Writes exactly what
// tf_sort_kernel writes, for (task, field)s of any size.
template <bool SLOTS>
__global__ __launch_bounds__(256) void tf_join_kernel(TfJoinArgs a) {
    __shared__ int sh_scan[8];
    __shared__ u32 sh_wstate[4];
    const int f = blockIdx.x, t = blockIdx.y;
    const size_t tf = (size_t)t * a.F + f;
    const u32 ns = a.cnt_s[tf], nq = a.cnt_q[tf], B = a.base_s[tf], Bq = a.base_q[tf];
    const u32 n = ns + nq;
    // The run is read four entries per thread as 16-byte words, from the 16-byte boundary at or before its start: the
    // `mis` entries in front belong to the (task, field) before and count as absent.
    const size_t S = (size_t)B + Bq;
    const u32 mis = (u32)(S & 3);
    const u32* K = a.keys + (S - mis);
    const u32* V = a.vals + (S - mis);
    const u32 n_al = n + mis;
    const int64_t readable = (a.n_lookups_s + a.n_lookups_q) - (int64_t)(S - mis);   // entries of the list from K on
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const u32 FLAG = 0x80000000u;
    const u32 posmask = (1u << a.pshift) - 1u;
    u32 a_carry = 0, u_carry = 0, st_carry = 0;   // the same on every thread
    for (u32 c0 = 0; c0 < n_al; c0 += 1024) {
        const u32 j0 = c0 + threadIdx.x * 4;   // position in the aligned run; entry i of the (task, field) is position i + mis
        u32 k[6], v[5];   // k[0]: the entry before the thread's four, k[5] / v[4]: the one after
        if ((int64_t)j0 + 4 <= readable) {
            const uint4 kq = *reinterpret_cast<const uint4*>(K + j0), vq = *reinterpret_cast<const uint4*>(V + j0);
            k[1] = kq.x; k[2] = kq.y; k[3] = kq.z; k[4] = kq.w;
            v[0] = vq.x; v[1] = vq.y; v[2] = vq.z; v[3] = vq.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                k[e + 1] = (int64_t)j0 + e < readable ? K[j0 + e] : 0u;
                v[e] = (int64_t)j0 + e < readable ? V[j0 + e] : 0u;
            }
        }
        // neighbours across threads by lane shuffles; the wave's first and last lanes read theirs
        k[0] = __shfl_up(k[4], 1, 64);
        k[5] = __shfl_down(k[1], 1, 64);
        v[4] = __shfl_down(v[0], 1, 64);
        if (lane == 0) k[0] = (j0 > 0 && j0 <= n_al) ? K[j0 - 1] : 0u;
        if (lane == 63) {
            k[5] = j0 + 4 < n_al ? K[j0 + 4] : 0u;
            v[4] = j0 + 4 < n_al ? V[j0 + 4] : 0u;
        }
        const u32 i0 = j0 - mis;   // (wraps for positions in front of the run: `in` below is false for them)
        bool in[5];
#pragma unroll
        for (int e = 0; e < 5; ++e) in[e] = j0 + e >= mis && j0 + e < n_al;
        bool sup[5], head[4];
        int n_sup = 0, n_sh = 0;
#pragma unroll
        for (int e = 0; e < 5; ++e) sup[e] = in[e] && (v[e] >> a.rshift) < a.n_sup_rows;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            head[e] = in[e] && (i0 + e == 0 || k[e + 1] != k[e]);
            n_sup += sup[e] ? 1 : 0;
            n_sh += (head[e] && sup[e]) ? 1 : 0;
        }
        int total;
        const int excl = block_excl_scan(n_sup | (n_sh << 16), sh_scan, &total);
        u32 aex = a_carry + ((u32)excl & 0xFFFFu);        // support lookups before the thread's first entry
        u32 uex = u_carry + ((u32)excl >> 16);            // distinct support rows before it
        // state of an entry: slot + 1 of its row, 0 when the support set does not look the row up; set at the head of a
        // run of equal keys and copied along the run
        u32 stt[4];
        u32 cur = 0;
        bool any_head = false;
        {
            u32 u = uex;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (head[e]) {
                    any_head = true;
                    cur = sup[e] ? u + 1u : 0u;
                    u += sup[e] ? 1u : 0u;
                }
                stt[e] = cur;   // valid from the thread's first head on; before it the incoming state applies
            }
        }
        u32 x = any_head ? (FLAG | cur) : 0u;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const u32 y = __shfl_up(x, d, 64);
            if (lane >= d && !(x & FLAG)) x = y;
        }
        if (lane == 63) sh_wstate[wv] = x;
        u32 inc = __shfl_up(x, 1, 64);
        if (lane == 0) inc = 0u;
        __syncthreads();
        u32 wave_in = FLAG | st_carry, all = FLAG | st_carry;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) {
            const u32 s = sh_wstate[ww];
            if (s & FLAG) {
                all = s;
                if (ww < wv) wave_in = s;
            }
        }
        if (!(inc & FLAG)) inc = wave_in;
        inc &= ~FLAG;
        {
            bool seen = false;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                seen = seen || head[e];
                if (!seen) stt[e] = inc;
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const u32 i = i0 + e;
            if (in[e]) {
                const u32 key = k[e + 1], val = v[e];
                const u32 row = val >> a.rshift;
                const bool next_same = in[e + 1] && k[e + 2] == key;
                const int32_t slot = (int32_t)stt[e] - 1;
                // (every index below is in range when the list is in the stated order; the checks keep a list that is
                //  not -- a defect elsewhere -- from writing outside the (task, field)'s own ranges)
                if (sup[e]) {
                    if (slot >= 0 && (u32)slot < ns && aex < ns) {
                        a.sup_sorted[B + aex] = make_int2((int)row, slot);
                        if (head[e]) {
                            a.slot_rows[B + slot] = key;
                            a.slot_start[B + tf + slot] = (int32_t)(B + aex);
                        }
                        if (!(next_same && sup[e + 1])) a.qseg_lo[B + slot] = (int32_t)(Bq + (i - aex));
                        if (SLOTS) {
                            const int rel = (int)row - a.row_off_s[t];
                            if (rel >= 0 && rel < a.real_off_s[t + 1] - a.real_off_s[t]) {
                                const int64_t lk = a.bag_s[(a.sample0_s + a.real_off_s[t] + rel) * a.F + f] - a.lookup0_s + (val & posmask);
                                if (lk >= 0 && lk < a.n_lookups_s) a.sup_slot[lk] = slot;
                            }
                        }
                    }
                } else if (i - aex < nq) {
                    const u32 rq = row - a.n_sup_rows;
                    a.qry_sorted[Bq + (i - aex)] = make_int2((int)rq, slot);
                    if (SLOTS) {
                        const int rel = (int)rq - a.row_off_q[t];
                        if (rel >= 0 && rel < a.real_off_q[t + 1] - a.real_off_q[t]) {
                            const int64_t lk = a.bag_q[(a.sample0_q + a.real_off_q[t] + rel) * a.F + f] - a.lookup0_q + (val & posmask);
                            if (lk >= 0 && lk < a.n_lookups_q) a.qry_slot[lk] = slot;
                        }
                    }
                }
                if (!next_same && slot >= 0 && (u32)slot < ns) a.qseg_hi[B + slot] = (int32_t)(Bq + (i + 1) - (aex + (sup[e] ? 1u : 0u)));
                aex += sup[e] ? 1u : 0u;
            }
        }
        a_carry += (u32)total & 0xFFFFu;
        u_carry += (u32)total >> 16;
        st_carry = all & ~FLAG;
    }
    if (threadIdx.x == 0) {
        const u32 nu = min(u_carry, ns);
        a.n_slots[tf] = nu;
        a.slot_start[B + tf + nu] = (int32_t)(B + ns);
    }
}

void launch_tf_join(hipStream_t st, const TfJoinArgs& a) {
    if (a.Tw <= 0 || a.F <= 0) return;
    if (a.sup_slot) hipLaunchKernelGGL(tf_join_kernel<true>, dim3(a.F, a.Tw), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(tf_join_kernel<false>, dim3(a.F, a.Tw), dim3(256), 0, st, a);
}

__global__ void seg_emit_kernel(const u32* keys, int64_t n, const u32* scan, int64_t* emb_rows, u32* seg_start,
                                int64_t capacity, int64_t* n_rows_out, u32* status) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const bool head = (i == 0 || keys[i] != keys[i - 1]);
    const u32 seg = scan[i];
    if (head && (int64_t)seg < capacity) {
        if (emb_rows) emb_rows[seg] = (int64_t)keys[i];
        seg_start[seg] = (u32)i;
    }
    if (i == n - 1) {
        const int64_t total = (int64_t)seg + (head ? 1 : 0);
        *n_rows_out = total;
        status[ST_NROWS] = (u32)total;
        if (total > capacity) atomicOr(&status[ST_CAPACITY], 1u);
        else seg_start[total] = (u32)n;
    }
}

__global__ void seg_counts_kernel(const u32* seg_start, const int64_t* n_rows, int64_t capacity, int64_t* counts) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n = min(*n_rows, capacity);
    if (i < n) counts[i] = (int64_t)seg_start[i + 1] - (int64_t)seg_start[i];
}

__global__ void zero_rows_kernel(int64_t* n_rows_out, u32* status) {
    *n_rows_out = 0;
    status[ST_NROWS] = 0;
}

void launch_segments(hipStream_t st, const u32* sorted_keys, int64_t n, u32* flags_scan, u32* scan_tmp,
                     int64_t* emb_rows, u32* seg_start, int64_t* seg_counts, int64_t capacity,
                     int64_t* n_rows_out, u32* status) {
    if (n <= 0) {
        hipLaunchKernelGGL(zero_rows_kernel, dim3(1), dim3(1), 0, st, n_rows_out, status);
        return;
    }
    const unsigned nb = (unsigned)((n + 255) / 256);
    {   // exclusive scan of the segment-head flags (launch_scan_u32 with its first level reading the keys)
        const int64_t nblk = (n + SCAN_TILE - 1) / SCAN_TILE;
        hipLaunchKernelGGL(scan_heads_block_kernel, dim3((unsigned)nblk), dim3(SCAN_NT), 0, st, sorted_keys, flags_scan, n, scan_tmp);
        if (nblk > 1) {
            u32* next = scan_tmp + (nblk + 63) / 64 * 64;
            launch_scan_u32(st, scan_tmp, scan_tmp, nblk, next, nullptr);
            hipLaunchKernelGGL(scan_add_kernel, dim3((unsigned)nblk), dim3(SCAN_NT), 0, st, flags_scan, n, scan_tmp);
        }
    }
    hipLaunchKernelGGL(seg_emit_kernel, dim3(nb), dim3(256), 0, st, sorted_keys, n, flags_scan, emb_rows, seg_start,
                       capacity, n_rows_out, status);
    if (seg_counts) {
        const int64_t m = capacity < n ? capacity : n;
        hipLaunchKernelGGL(seg_counts_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st, seg_start,
                           n_rows_out, capacity, seg_counts);
    }
}

// ------------------------------------------------------------------------------------------------
__global__ void fill_u32_kernel(u32* p, int64_t n, u32 v) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}
void launch_fill_u32(hipStream_t st, u32* p, int64_t n, u32 v) {
    if (n <= 0) return;
    int64_t nb = (n + 255) / 256;
    if (nb > 65536) nb = 65536;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)nb), dim3(256), 0, st, p, n, v);
}
void launch_fill_f32(hipStream_t st, float* p, int64_t n, float v) {
    launch_fill_u32(st, (u32*)p, n, __builtin_bit_cast(u32, v));
}
