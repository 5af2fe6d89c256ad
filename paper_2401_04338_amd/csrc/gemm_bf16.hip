// Grouped bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// One kernel serves every dense product of the MAML step (G-Meta Alg. 1: inner forward, local
// back-propagation, outer forward, and the tangent passes of the second-order term):
//     C_g[M, N] = sum_p  A_p,g[M, K] * B_p,g[K, N]          (p = 1 or 2 products)
// A lane's MFMA fragment is 8 consecutive contraction values.  An operand stored contraction-contiguous
// delivers them as one 16-byte LDS read; an operand stored with the contraction index slowest (template
// flags KA / KB) goes to LDS row by row as it lies in memory and the lane collects its 8 values with two
// transposing LDS reads (ds_read_b64_tr_b16).  Every matrix therefore exists once, in the orientation it
// was produced in:
//   forward      A = activations [rows, d_in]  (contiguous),  B = W [d_in, d_out]          (KB)
//   backward dA  A = deltas      [rows, d_out] (contiguous),  B = W [d_in, d_out] read as [n][k] (contiguous)
//   weight grad  A = activations [rows, d_in]  (KA),          B = deltas [rows, d_out]     (KB), K = rows of the task
// A group is a task: its rows are [row_offsets[g], row_offsets[g+1]) and, once theta has been adapted,
// its weights are its own (group stride != 0).
#include "gm_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define GK 64          // k extent of one LDS tile
#define GLD (GK + 8)   // LDS row stride in elements: 144 bytes, an odd number of 16-byte units
#define GPADK 32       // pad of a contraction-slowest tile's rows: four consecutive rows start 16 banks apart

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// Waves: 2 along m, BN / 128 * 2 along n -- 4 waves for 128-wide tiles, 8 for 256-wide ones, so that a wave's share
// is at most 128 x 64 (128 accumulator registers) whatever the block tile.
template <int BM, int BN, bool DB, bool KA, bool KB>
__global__ __launch_bounds__(BN > 128 ? 2 * (BN / 64) * 64 : 256) void gemm_bf16_kernel(GemmBArgs a, int n_ntiles, int mt_per_group, int n_tiles) {
    constexpr int WN = BN > 128 ? BN / 64 : 2;   // waves along n
    constexpr int NT = 2 * WN * 64;              // threads
    constexpr int MI = BM / 64, NI = BN / (32 * WN);  // 32x32 blocks per wave in each direction
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    constexpr int LDA_K = BM + GPADK, LDB_K = BN + GPADK;  // KM: LDS row strides of the [GK][BM] and [GK][BN] tiles
    constexpr int TILE = (KA ? GK * LDA_K : BM * GLD) + (KB ? GK * LDB_K : BN * GLD);  // elements of one operand stage

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Re-number them so that
    // consecutive tiles -- the n-tiles of one row block, then the next row block of the same task, which
    // read the same rows and the same weights -- run on the same XCD.
    const int per_xcd = gridDim.x >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= n_tiles) return;
    const int ntile = tile % n_ntiles;
    const int mtile = tile / n_ntiles;
    int g, m0;
    if (a.tile_group) {
        g = a.tile_group[mtile];
        m0 = a.tile_m0[mtile];
    } else {
        g = mtile / mt_per_group;
        m0 = (mtile % mt_per_group) * BM;
    }
    const int64_t r0 = a.row_offsets[g];
    const int rows_g = (int)(a.row_offsets[g + 1] - r0);
    const int M = a.M < 0 ? rows_g : a.M;
    const int K = a.K < 0 ? rows_g : a.K;
    const int N = a.N;
    const int n0 = ntile * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WN) * (BM / 2), wn0 = (wave % WN) * (BN / WN);
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // global -> register staging: 16-byte chunks, 8 chunks per tile row
    constexpr int CA = BM * 8 / NT, CB = BN * 8 / NT;  // chunks per thread
    constexpr int CR = NT / 8;                          // tile rows covered by one chunk round
    uint4 ra[CA], rb[CB];
    const int crow = tid >> 3, ccol = (tid & 7) * 8;     // chunk c = tid + NT*i: row = crow + CR*i, k = ccol

    const int kt_per_pair = (K + GK - 1) / GK;
    const int n_kt = kt_per_pair * a.n_pairs;

    constexpr int A_ELEMS = KA ? GK * LDA_K : BM * GLD;   // LDS elements of the A tile; the B tile follows
    auto load_tile = [&](int kt) {
        const int pr = kt / kt_per_pair;
        const int k0 = (kt - pr * kt_per_pair) * GK;
        const bf16_t* A = a.A[pr] + (int64_t)g * a.gA[pr] + r0 * a.rA[pr];
        const bf16_t* B = a.B[pr] + (int64_t)g * a.gB[pr] + r0 * a.rB[pr];
        const int64_t lda = a.lda[pr], ldb = a.ldb[pr];
        const bool kok = k0 + ccol < K;
        if constexpr (KA) {  // contraction slowest: 16-byte chunks along m, chunk c = tid + NT*i of row c / (BM/8)
#pragma unroll
            for (int i = 0; i < CA; ++i) {
                const int ch = tid + NT * i, kr = ch / (BM / 8), mc = (ch % (BM / 8)) * 8;
                ra[i] = (k0 + kr < K && m0 + mc < M) ? *reinterpret_cast<const uint4*>(A + (int64_t)(k0 + kr) * lda + m0 + mc)
                                                     : make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < CA; ++i) {
                const int m = m0 + crow + CR * i;
                ra[i] = (kok && m < M) ? *reinterpret_cast<const uint4*>(A + (int64_t)m * lda + k0 + ccol) : make_uint4(0, 0, 0, 0);
            }
        }
        if constexpr (KB) {
#pragma unroll
            for (int i = 0; i < CB; ++i) {
                const int ch = tid + NT * i, kr = ch / (BN / 8), nc = (ch % (BN / 8)) * 8;
                rb[i] = (k0 + kr < K && n0 + nc < N) ? *reinterpret_cast<const uint4*>(B + (int64_t)(k0 + kr) * ldb + n0 + nc)
                                                     : make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < CB; ++i) {
                const int n = n0 + crow + CR * i;
                rb[i] = (kok && n < N) ? *reinterpret_cast<const uint4*>(B + (int64_t)n * ldb + k0 + ccol) : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_tile = [&](bf16_t* stage) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int ch = tid + NT * i;
            if constexpr (KA) *reinterpret_cast<uint4*>(stage + (ch / (BM / 8)) * LDA_K + (ch % (BM / 8)) * 8) = ra[i];
            else *reinterpret_cast<uint4*>(stage + (crow + CR * i) * GLD + ccol) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const int ch = tid + NT * i;
            if constexpr (KB) *reinterpret_cast<uint4*>(stage + A_ELEMS + (ch / (BN / 8)) * LDB_K + (ch % (BN / 8)) * 8) = rb[i];
            else *reinterpret_cast<uint4*>(stage + A_ELEMS + (crow + CR * i) * GLD + ccol) = rb[i];
        }
    };
    // 8 contraction values of one column of a contraction-slowest tile: two transposing LDS reads
    // (ds_read_b64_tr_b16).  Such a read serves 16 lanes at a time: lane s of the 16 points at 4 consecutive
    // columns (s % 4) * 4.. of row s / 4, and lane i receives column i of those 4 rows.
    const int tr_off_row = lhi * 8 + ((lane & 15) >> 2), tr_off_col = (lane & 16) + (lane & 3) * 4;
    auto frag = [&](const bf16_t* tile, int ld, int c0, int k) {
        const bf16_t* p = tile + (k + tr_off_row) * ld + c0 + tr_off_col;
        typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * ld));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto compute = [&](const bf16_t* stage) {
        const bf16_t* As = stage;
        const bf16_t* Bs = stage + A_ELEMS;
#pragma unroll
        for (int kk = 0; kk < GK / 16; ++kk) {
            bf16x8 af[MI], bfr[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                if constexpr (KA) af[i] = frag(As, LDA_K, wm0 + i * 32, kk * 16);
                else af[i] = *reinterpret_cast<const bf16x8*>(As + (wm0 + i * 32 + l32) * GLD + kk * 16 + lhi * 8);
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                if constexpr (KB) bfr[j] = frag(Bs, LDB_K, wn0 + j * 32, kk * 16);
                else bfr[j] = *reinterpret_cast<const bf16x8*>(Bs + (wn0 + j * 32 + l32) * GLD + kk * 16 + lhi * 8);
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    };

    if (DB) {
        // two LDS stages: the next tile is fetched to registers while this one feeds the MFMAs and is parked in the
        // other stage afterwards; one barrier per tile
        if (n_kt > 0) {
            load_tile(0);
            store_tile(smem);
        }
        __syncthreads();
        for (int kt = 0; kt < n_kt; ++kt) {
            const bool more = kt + 1 < n_kt;
            if (more) load_tile(kt + 1);
            compute(smem + (kt & 1) * TILE);
            if (more) store_tile(smem + ((kt + 1) & 1) * TILE);
            __syncthreads();
        }
    } else {
        if (n_kt > 0) load_tile(0);
        for (int kt = 0; kt < n_kt; ++kt) {
            __syncthreads();  // previous tile fully consumed
            store_tile(smem);
            __syncthreads();
            if (kt + 1 < n_kt) load_tile(kt + 1);  // overlaps with the MFMAs below
            compute(smem);
        }
        __syncthreads();  // every wave is done with the operand tiles
    }

    // epilogue.  A lane holds column l32 of each 32x32 block and rows 8*(v/4) + 4*lhi + v%4, which would give
    // 2-byte scattered stores; instead every wave passes its accumulators through LDS one 32-row strip at a
    // time, applies the fused operation on 4 consecutive columns per lane and writes whole row segments.
    const float* bias = a.bias ? a.bias + (int64_t)g * a.gBias : nullptr;
    const bf16_t* mask = a.mask ? a.mask + r0 * a.ld_mask : nullptr;
    const float* Cin = a.Cin ? a.Cin + (int64_t)g * a.gCin : nullptr;
    float* Cf = a.Cf ? a.Cf + (int64_t)g * a.gCf + r0 * a.rCf : nullptr;
    float* Cacc = a.Cacc ? a.Cacc + r0 * a.rCacc : nullptr;
    bf16_t* Cb = a.Cb ? a.Cb + (int64_t)g * a.gCb + r0 * a.rCb : nullptr;
    constexpr int SW = NI * 32, ELD = SW + 4;      // strip width, LDS row stride (floats)
    constexpr int LPR = SW / 4, RPI = 64 / LPR;    // lanes per strip row, rows per pass
    float* E = reinterpret_cast<float*>(smem) + wave * (32 * ELD);
    const int er = lane / LPR, ec = (lane % LPR) * 4;
    const int n = n0 + wn0 + ec;
    const bool nok = n < N;
    float4 bn = make_float4(0.f, 0.f, 0.f, 0.f);
    if (bias && nok) bn = *reinterpret_cast<const float4*>(bias + n);
    const bool has_mask = a.epi == EPI_BIAS_MASK || a.epi == EPI_MASK;
    const bool has_cin = a.epi == EPI_AXPBY && Cin;
    const bool has_acc = Cacc && !has_cin;   // the accumulate-into output shares the registers of Cin
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        // What the strip reads from memory is requested before anything of it is stored: the outputs may alias
        // the inputs (an in-place update), which would otherwise chain every load behind the previous store.
        uint2 mk_all[32 / RPI];
        float4 ci_all[32 / RPI];
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
            const int m = m0 + wm0 + i * 32 + it * RPI + er;
            const bool ok = nok && m < M;
            mk_all[it] = make_uint2(0u, 0u);
            ci_all[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ok && has_mask) mk_all[it] = *reinterpret_cast<const uint2*>(mask + (int64_t)m * a.ld_mask + n);
            if (ok && has_cin) ci_all[it] = *reinterpret_cast<const float4*>(Cin + (int64_t)m * a.ldcin + n);
            if (ok && has_acc && !a.cacc_init) ci_all[it] = *reinterpret_cast<const float4*>(Cacc + (int64_t)m * a.ldcacc + n);
        }
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) E[(8 * (v >> 2) + 4 * lhi + (v & 3)) * ELD + j * 32 + l32] = acc[i][j][v];
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
            const int rr = it * RPI + er;
            const int m = m0 + wm0 + i * 32 + rr;
            if (!nok || m >= M) continue;
            float4 x = *reinterpret_cast<const float4*>(E + rr * ELD + ec);
            if (a.epi == EPI_BIAS_RELU) {
                x = make_float4(fmaxf(x.x + bn.x, 0.f), fmaxf(x.y + bn.y, 0.f), fmaxf(x.z + bn.z, 0.f), fmaxf(x.w + bn.w, 0.f));
            } else if (has_mask) {
                const uint2 mk = mk_all[it];
                if (a.epi == EPI_BIAS_MASK) x = make_float4(x.x + bn.x, x.y + bn.y, x.z + bn.z, x.w + bn.w);
                // a bf16 is positive iff it is neither zero nor has its sign bit set
                const u32 h0 = mk.x & 0xffffu, h1 = mk.x >> 16, h2 = mk.y & 0xffffu, h3 = mk.y >> 16;
                x.x = (h0 != 0 && h0 < 0x8000u) ? x.x : 0.f;
                x.y = (h1 != 0 && h1 < 0x8000u) ? x.y : 0.f;
                x.z = (h2 != 0 && h2 < 0x8000u) ? x.z : 0.f;
                x.w = (h3 != 0 && h3 < 0x8000u) ? x.w : 0.f;
            } else if (a.epi == EPI_AXPBY) {
                x = make_float4(a.c1 * x.x, a.c1 * x.y, a.c1 * x.z, a.c1 * x.w);
                if (Cin) {
                    const float4 ci = ci_all[it];
                    x = make_float4(x.x + a.c0 * ci.x, x.y + a.c0 * ci.y, x.z + a.c0 * ci.z, x.w + a.c0 * ci.w);
                }
            }
            if (Cf) *reinterpret_cast<float4*>(Cf + (int64_t)m * a.ldcf + n) = x;
            if (has_acc) {
                const float4 ci = ci_all[it];
                *reinterpret_cast<float4*>(Cacc + (int64_t)m * a.ldcacc + n) =
                    make_float4(ci.x + a.cacc * x.x, ci.y + a.cacc * x.y, ci.z + a.cacc * x.z, ci.w + a.cacc * x.w);
            }
            if (Cb) {
                uint2 pk;
                pk.x = f2bf2(x.x, x.y);
                pk.y = f2bf2(x.z, x.w);
                *reinterpret_cast<uint2*>(Cb + (int64_t)m * a.ldcb + n) = pk;
            }
        }
        __syncthreads();
    }
}

template <int BM, int BN, bool DB, bool KA = false, bool KB = false>
static void launch_variant(hipStream_t st, const GemmBArgs& a) {
    const int n_ntiles = (a.N + BN - 1) / BN;
    int64_t n_mtiles;
    int mt_per_group = 1;
    if (a.tile_group) {
        n_mtiles = a.n_mtiles;
    } else {
        mt_per_group = (a.M + BM - 1) / BM;
        n_mtiles = (int64_t)mt_per_group * a.G;
    }
    if (n_mtiles <= 0 || n_ntiles <= 0) return;
    const int64_t n_tiles = n_mtiles * n_ntiles;
    size_t shmem = ((KA ? (size_t)GK * (BM + GPADK) : (size_t)BM * GLD) + (KB ? (size_t)GK * (BN + GPADK) : (size_t)BN * GLD)) * sizeof(bf16_t) * (DB ? 2 : 1);
    constexpr int WN = BN > 128 ? BN / 64 : 2, NT = 2 * WN * 64;
    const size_t epi = (size_t)(2 * WN) * 32 * (BN / WN + 4) * sizeof(float);  // the epilogue's strips, one per wave
    if (shmem < epi) shmem = epi;
    auto kern = gemm_bf16_kernel<BM, BN, DB, KA, KB>;
    if (shmem > 48 * 1024) (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    const unsigned grid = (unsigned)((n_tiles + 7) / 8 * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), shmem, st, a, n_ntiles, mt_per_group, (int)n_tiles);
}

// bm: row tile the caller built its (tile_group, tile_m0) lists for (64, 128 or 256).  Measured on the
// benchmark shapes: one LDS stage with register prefetch beats two stages (occupancy), and 256x128 beats
// 128x128 and 256x256 when a task has enough rows; the weight-gradient set-up (fixed M, K = rows of a
// task) is bound by the theta' it writes and keeps 128x128.
// bn: 128 or 256 (256 only with bm = 256: eight waves, for products that are bound by the matrix cores)
void launch_gemm_bf16(hipStream_t st, const GemmBArgs& a, int bm, int bn) {
    if (bm == 64) launch_variant<64, 128, false>(st, a);
    else if (bm == 256 && bn == 256) launch_variant<256, 256, false>(st, a);
    else if (bm == 256) launch_variant<256, 128, false>(st, a);
    else launch_variant<128, 128, false>(st, a);
}

// Weight-gradient form: both operands stored with the contraction index slowest (A [K, M], B [K, N]).
void launch_gemm_bf16_kmajor(hipStream_t st, const GemmBArgs& a) { launch_variant<128, 128, false, true, true>(st, a); }

// Forward form with the weights as they are stored (B [K, N] = W [d_in, d_out]): no transposed copy of theta.
void launch_gemm_bf16_bkmajor(hipStream_t st, const GemmBArgs& a, int bm, int bn) {
    if (bm == 64) launch_variant<64, 128, false, false, true>(st, a);
    else if (bm == 256 && bn == 256) launch_variant<256, 256, false, false, true>(st, a);
    else if (bm == 256) launch_variant<256, 128, false, false, true>(st, a);
    else launch_variant<128, 128, false, false, true>(st, a);
}

// fp32 padded weights [rows, cols] -> bf16 W [rows, cols] and W^T [cols, rows], per group
__global__ void convert_weights_kernel(const float* __restrict__ src, int64_t g_src, int rows, int cols, bf16_t* w,
                                       bf16_t* wT, int64_t g_dst) {
    __shared__ float tile[32][33];
    const int g = blockIdx.z;
    const float* s = src + (int64_t)g * g_src;
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 256 threads: 8 rows at a time
    for (int i = ty; i < 32; i += 8) {
        const int r = r0 + i, c = c0 + tx;
        const float v = (r < rows && c < cols) ? s[(int64_t)r * cols + c] : 0.f;
        tile[i][tx] = v;
        if (w && r < rows && c < cols) w[(int64_t)g * g_dst + (int64_t)r * cols + c] = f2bf(v);
    }
    __syncthreads();
    if (!wT) return;
    for (int i = ty; i < 32; i += 8) {
        const int c = c0 + i, r = r0 + tx;
        if (c < cols && r < rows) wT[(int64_t)g * g_dst + (int64_t)c * rows + r] = f2bf(tile[tx][i]);
    }
}

void launch_convert_weights(hipStream_t st, const float* src, int64_t g_src, int G, int rows, int cols, bf16_t* w,
                            bf16_t* wT, int64_t g_dst) {
    if (G <= 0 || rows <= 0 || cols <= 0) return;
    for (int g0 = 0; g0 < G; g0 += 32768) {
        const int gc = (G - g0) < 32768 ? (G - g0) : 32768;
        hipLaunchKernelGGL(convert_weights_kernel, dim3((cols + 31) / 32, (rows + 31) / 32, gc), dim3(256), 0, st,
                           src + (int64_t)g0 * g_src, g_src, rows, cols, w ? w + (int64_t)g0 * g_dst : nullptr,
                           wT ? wT + (int64_t)g0 * g_dst : nullptr, g_dst);
    }
}
