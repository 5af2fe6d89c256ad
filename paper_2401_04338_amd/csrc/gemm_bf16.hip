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
#include <algorithm>

#include "gm_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define GK 64          // k extent of one LDS tile
#define GLD (GK + 8)   // LDS row stride in elements: 144 bytes, an odd number of 16-byte units
#define GPADK 32       // pad of a contraction-slowest tile's rows: four consecutive rows start 16 banks apart

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// What an epilogue does is fixed at compile time for the launches the step makes (EP >= 0: bits 0-2 the fused
// operation, then whether the fp32 output, the bf16 output, the accumulate-into output and the added input exist), so
// that the per-element code is straight-line; EP < 0 reads the same facts from the arguments at run time (any other
// combination).  With everything decided per element at run time the epilogue of a 256 x 256 tile ran to some 14,000
// instructions -- as long as twelve k-tiles of its main loop.
enum { EP_CF = 8, EP_CB = 16, EP_CACC = 32, EP_CIN = 64, EP_RUNTIME = -1 };
static int ep_of(const GemmBArgs& a) {
    const bool cin = a.epi == EPI_AXPBY && a.Cin;
    return a.epi | (a.Cf ? EP_CF : 0) | (a.Cb ? EP_CB : 0) | ((a.Cacc && !cin) ? EP_CACC : 0) | (cin ? EP_CIN : 0);
}
template <int EP>
struct EpiFlags {
    int epi;
    bool cf, cb, cacc, cin;
    __device__ __forceinline__ explicit EpiFlags(const GemmBArgs& a) {
        if constexpr (EP >= 0) {
            epi = EP & 7; cf = (EP & EP_CF) != 0; cb = (EP & EP_CB) != 0; cacc = (EP & EP_CACC) != 0; cin = (EP & EP_CIN) != 0;
        } else {
            epi = a.epi; cf = a.Cf != nullptr; cb = a.Cb != nullptr;
            cin = a.epi == EPI_AXPBY && a.Cin != nullptr; cacc = a.Cacc != nullptr && !cin;
        }
    }
};

// Epilogue shared by the GEMM kernels.  A lane holds column l32 of each 32x32 block and rows 8*(v/4) + 4*lhi + v%4,
// which would give 2-byte scattered stores; instead every wave passes its accumulators through LDS one 32-row strip at
// a time, applies the fused operation on 4 consecutive columns per lane and writes whole row segments.  TRANSPOSED: the
// accumulators were computed with the operand roles swapped (first MFMA operand = B fragment), so a lane holds ROW l32
// and four consecutive columns per group of four registers; stored straight from the registers that is 16 bytes per
// lane in 32 different rows per instruction, which the memory pipeline takes several times longer over than whole
// row segments (measured on the 256 x 256 tiles: epilogue 32 -> 26 thousand cycles forward, 56 -> 33 backward).
template <int BM, int BN, int MI, int NI, int EP, bool TRANSPOSED = false>
__device__ __forceinline__ void gemm_epilogue(const GemmBArgs& a, f32x16 (&acc)[MI][NI], bf16_t* smem, int g, int64_t r0, int m0,
                                              int n0, int M, int N, int wm0, int wn0, int lane, int wave) {
    const EpiFlags<EP> fl(a);
    const int l32 = lane & 31, lhi = lane >> 5;
    const bool has_bias = (fl.epi == EPI_BIAS_RELU || fl.epi == EPI_BIAS_MASK) && a.bias;
    const bool has_mask = fl.epi == EPI_BIAS_MASK || fl.epi == EPI_MASK;
    const bool has_cin = fl.cin, has_acc = fl.cacc;
    const float* bias = has_bias ? a.bias + (int64_t)g * a.gBias : nullptr;
    const bf16_t* mask = has_mask ? a.mask + r0 * a.ld_mask : nullptr;
    const float* Cin = has_cin ? a.Cin + (int64_t)g * a.gCin : nullptr;
    float* Cf = fl.cf ? a.Cf + (int64_t)g * a.gCf + r0 * a.rCf : nullptr;
    float* Cacc = has_acc ? a.Cacc + r0 * a.rCacc : nullptr;
    bf16_t* Cb = fl.cb ? a.Cb + (int64_t)g * a.gCb + r0 * a.rCb : nullptr;
    constexpr int SW = NI * 32, ELD = SW + 4;      // strip width, LDS row stride (floats)
    constexpr int LPR = SW / 4, RPI = 64 / LPR;    // lanes per strip row, rows per pass
    float* E = reinterpret_cast<float*>(smem) + wave * (32 * ELD);
    const int er = lane / LPR, ec = (lane % LPR) * 4;
    const int n = n0 + wn0 + ec;
    const bool nok = n < N;
    float4 bn = make_float4(0.f, 0.f, 0.f, 0.f);
    if (has_bias && nok) bn = *reinterpret_cast<const float4*>(bias + n);
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
        if constexpr (TRANSPOSED) {   // (operand roles swapped in the MFMA: the lane holds row l32, four consecutive columns per q)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<float4*>(E + l32 * ELD + j * 32 + 8 * q + 4 * lhi) =
                        make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        } else {
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) E[(8 * (v >> 2) + 4 * lhi + (v & 3)) * ELD + j * 32 + l32] = acc[i][j][v];
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the strip is this wave's own: LDS order within the wave suffices
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
            const int rr = it * RPI + er;
            const int m = m0 + wm0 + i * 32 + rr;
            if (!nok || m >= M) continue;
            float4 x = *reinterpret_cast<const float4*>(E + rr * ELD + ec);
            if (fl.epi == EPI_BIAS_RELU) {
                x = make_float4(fmaxf(x.x + bn.x, 0.f), fmaxf(x.y + bn.y, 0.f), fmaxf(x.z + bn.z, 0.f), fmaxf(x.w + bn.w, 0.f));
            } else if (has_mask) {
                const uint2 mk = mk_all[it];
                if (fl.epi == EPI_BIAS_MASK) x = make_float4(x.x + bn.x, x.y + bn.y, x.z + bn.z, x.w + bn.w);
                // a bf16 is positive iff it is neither zero nor has its sign bit set
                const u32 h0 = mk.x & 0xffffu, h1 = mk.x >> 16, h2 = mk.y & 0xffffu, h3 = mk.y >> 16;
                x.x = (h0 != 0 && h0 < 0x8000u) ? x.x : 0.f;
                x.y = (h1 != 0 && h1 < 0x8000u) ? x.y : 0.f;
                x.z = (h2 != 0 && h2 < 0x8000u) ? x.z : 0.f;
                x.w = (h3 != 0 && h3 < 0x8000u) ? x.w : 0.f;
            } else if (fl.epi == EPI_AXPBY) {
                x = make_float4(a.c1 * x.x, a.c1 * x.y, a.c1 * x.z, a.c1 * x.w);
                if (has_cin) {
                    const float4 ci = ci_all[it];
                    x = make_float4(x.x + a.c0 * ci.x, x.y + a.c0 * ci.y, x.z + a.c0 * ci.z, x.w + a.c0 * ci.w);
                }
            }
            if (fl.cf) *reinterpret_cast<float4*>(Cf + (int64_t)m * a.ldcf + n) = x;
            if (has_acc) {
                const float4 ci = ci_all[it];
                *reinterpret_cast<float4*>(Cacc + (int64_t)m * a.ldcacc + n) =
                    make_float4(ci.x + a.cacc * x.x, ci.y + a.cacc * x.y, ci.z + a.cacc * x.z, ci.w + a.cacc * x.w);
            }
            if (fl.cb) {
                uint2 pk;
                pk.x = f2bf2(x.x, x.y);
                pk.y = f2bf2(x.z, x.w);
                *reinterpret_cast<uint2*>(Cb + (int64_t)m * a.ldcb + n) = pk;
            }
        }
        asm volatile("" ::: "memory");   // (no block barrier: it would also wait for the strip's global stores to land)
    }
}

// Four waves, 2 along m and 2 along n: a wave's share of a BM x BN tile is BM / 2 x BN / 2.
template <int BM, int BN, bool DB, bool KA, bool KB, int EP>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmBArgs a, int n_ntiles, int mt_per_group, int n_tiles) {
    constexpr int WN = 2;   // waves along n
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

    gemm_epilogue<BM, BN, MI, NI, EP>(a, acc, smem, g, r0, m0, n0, M, N, wm0, wn0, lane, wave);
}

// ------------------------------------------------------------------------------------------------
// 256 x 256 tiles for products that are bound by the matrix cores (forward and backward products of tasks with
// hundreds of rows).  Four waves, each owning a 128 x 128 block of the tile (16 accumulator blocks = 256 registers):
// per contraction step a wave reads 8 operand fragments from LDS for 16 MFMAs, half the LDS traffic per flop of a
// 128 x 64 block, which is what the smaller tiles are bound by.  One wave per SIMD, so nothing but the instruction
// order hides latencies: two LDS stages, fragments double-buffered in registers, and within each k-tile
//   step 0: fragments of step 1 requested, first half of the NEXT tile parked in the other stage, first half of the
//           tile after it requested from memory, MFMAs of step 0
//   step 1: the same with the second halves
//   step 2: fragments of step 3 requested, MFMAs of step 2
//   step 3: barrier (everyone has read this stage and written the other), fragments of the next tile's step 0
//           requested, MFMAs of step 3
// Operand tiles come through buffer loads: a row, column or whole tile outside the operand reads as zero without a
// branch, so the loop body is straight-line code.  A is stored contraction-contiguous; B either way (KB).
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

#ifdef GEMM_TIMING
__device__ unsigned long long g_gemm_ts[4 * 16384];
void gemm_timing_fetch(unsigned long long* host, int n) { (void)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_gemm_ts), sizeof(unsigned long long) * n); }
#endif
template <bool KA, bool KB, int EP, bool TIMED = false>
__global__ __launch_bounds__(256) void gemm_bf16_pipe_kernel(GemmBArgs a, int n_ntiles, int mt_per_group, int n_tiles) {
    constexpr int BM = 256, BN = 256, MI = 4, NI = 4, NT = 256;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    constexpr int LDB_K = BN + GPADK;   // (also the row stride of a contraction-slowest A tile: BM = BN)
    constexpr int A_ELEMS = KA ? GK * LDB_K : BM * GLD;
    constexpr int TILE = A_ELEMS + (KB ? GK * LDB_K : BN * GLD);

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
    const int wm0 = (wave >> 1) * 128, wn0 = (wave & 1) * 128;
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int kt_per_pair = (K + GK - 1) / GK;
    const int n_kt = kt_per_pair * a.n_pairs;

    // operands of the (up to two) products as buffer resources: an access past the group's matrix returns zero
    const u32 OOB = 0x7ffffff0u;
    __amdgpu_buffer_rsrc_t rsA[2], rsB[2];
    u32 ldA2[2], ldB2[2];
#pragma unroll
    for (int p2 = 0; p2 < 2; ++p2) {
        const int pr = p2 < a.n_pairs ? p2 : 0;
        const bf16_t* A = a.A[pr] + (int64_t)g * a.gA[pr] + r0 * a.rA[pr];
        const bf16_t* B = a.B[pr] + (int64_t)g * a.gB[pr] + r0 * a.rB[pr];
        ldA2[p2] = (u32)a.lda[pr] * 2u;
        ldB2[p2] = (u32)a.ldb[pr] * 2u;
        rsA[p2] = __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, (int)((u32)(KA ? K : M) * ldA2[p2]), 0x00020000);
        rsB[p2] = __builtin_amdgcn_make_buffer_rsrc((void*)B, 0, (int)((u32)(KB ? K : N) * ldB2[p2]), 0x00020000);
    }
    // chunk c = tid + 256 i of a tile: A (and B stored like A): row c / 8, 16 bytes at k = (c % 8) * 8;
    // B stored contraction-slowest: k-row c / 32, 16 bytes at n = (c % 32) * 8
    const int crow = tid >> 3, ccol = (tid & 7) * 8;
    const int kbrow = tid >> 5, kbcol = (tid & 31) * 8;
    u32x4 ra[8], rb[8];
    auto gload_half = [&](int h, int lt) {   // chunks 4h .. 4h+3 of tile lt (a tile past the end reads as zero)
        const int pr = (lt >= kt_per_pair && a.n_pairs > 1) ? 1 : 0;
        const int k0 = (lt - pr * kt_per_pair) * GK;
        const __amdgpu_buffer_rsrc_t rA = pr ? rsA[1] : rsA[0];
        const __amdgpu_buffer_rsrc_t rB = pr ? rsB[1] : rsB[0];
        const u32 la = pr ? ldA2[1] : ldA2[0], lb = pr ? ldB2[1] : ldB2[0];
        const bool kok = k0 + ccol < K;
        if constexpr (KA) {   // (a column past M would read on into the next row: such a chunk is sent out of bounds)
            const bool mok = m0 + kbcol < M;
            const u32 a0 = mok ? (u32)(k0 + kbrow) * la + (u32)(m0 + kbcol) * 2u : OOB;
#pragma unroll
            for (int i = 4 * h; i < 4 * h + 4; ++i) ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rA, (int)(a0 + (mok ? (u32)(8 * i) * la : 0u)), 0, 0);
        } else {
            const u32 a0 = kok ? (u32)(m0 + crow) * la + (u32)(k0 + ccol) * 2u : OOB;
#pragma unroll
            for (int i = 4 * h; i < 4 * h + 4; ++i) ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rA, (int)(a0 + (kok ? (u32)(32 * i) * la : 0u)), 0, 0);
        }
        if constexpr (KB) {
            const u32 b0 = (u32)(k0 + kbrow) * lb + (u32)(n0 + kbcol) * 2u;
#pragma unroll
            for (int i = 4 * h; i < 4 * h + 4; ++i) rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rB, (int)(b0 + (u32)(8 * i) * lb), 0, 0);
        } else {
            const u32 b0 = kok ? (u32)(n0 + crow) * lb + (u32)(k0 + ccol) * 2u : OOB;
#pragma unroll
            for (int i = 4 * h; i < 4 * h + 4; ++i) rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rB, (int)(b0 + (kok ? (u32)(32 * i) * lb : 0u)), 0, 0);
        }
    };
    auto store_half = [&](bf16_t* stage, int h) {
#pragma unroll
        for (int i = 4 * h; i < 4 * h + 4; ++i) {
            if constexpr (KA) *reinterpret_cast<u32x4*>(stage + (kbrow + 8 * i) * LDB_K + kbcol) = ra[i];
            else *reinterpret_cast<u32x4*>(stage + (crow + 32 * i) * GLD + ccol) = ra[i];
        }
#pragma unroll
        for (int i = 4 * h; i < 4 * h + 4; ++i) {
            if constexpr (KB) *reinterpret_cast<u32x4*>(stage + A_ELEMS + (kbrow + 8 * i) * LDB_K + kbcol) = rb[i];
            else *reinterpret_cast<u32x4*>(stage + A_ELEMS + (crow + 32 * i) * GLD + ccol) = rb[i];
        }
    };
    const int tr_off_row = lhi * 8 + ((lane & 15) >> 2), tr_off_col = (lane & 16) + (lane & 3) * 4;
    auto frag_tr = [&](const bf16_t* tile_, int c0, int k) {
        const bf16_t* p = tile_ + (k + tr_off_row) * LDB_K + c0 + tr_off_col;
        typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * LDB_K));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto read_frags = [&](const bf16_t* stage, int kk, bf16x8 (&af)[MI], bf16x8 (&bfr)[NI]) {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            if constexpr (KA) af[i] = frag_tr(stage, wm0 + i * 32, kk * 16);
            else af[i] = *reinterpret_cast<const bf16x8*>(stage + (wm0 + i * 32 + l32) * GLD + kk * 16 + lhi * 8);
        }
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            if constexpr (KB) bfr[j] = frag_tr(stage + A_ELEMS, wn0 + j * 32, kk * 16);
            else bfr[j] = *reinterpret_cast<const bf16x8*>(stage + A_ELEMS + (wn0 + j * 32 + l32) * GLD + kk * 16 + lhi * 8);
        }
    };
    auto mfmas = [&](const bf16x8 (&af)[MI], const bf16x8 (&bfr)[NI]) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);   // transposed block
    };

    bf16x8 fa0[MI], fb0[NI], fa1[MI], fb1[NI];
#ifdef GEMM_TIMING
    unsigned long long ts0 = 0, ts1 = 0, ts2 = 0;
    if (TIMED) ts0 = __builtin_readcyclecounter();
#endif
    gload_half(0, 0);
    gload_half(1, 0);
    store_half(smem, 0);
    store_half(smem, 1);
    gload_half(0, 1);
    gload_half(1, 1);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    read_frags(smem, 0, fa0, fb0);
#ifdef GEMM_TIMING
    if (TIMED) ts1 = __builtin_readcyclecounter();
#endif
    for (int kt = 0; kt < n_kt; ++kt) {
        bf16_t* cur = smem + (kt & 1) * TILE;
        bf16_t* nxt = smem + ((kt + 1) & 1) * TILE;
        // instruction order of a step: the fragment reads first, then one LDS write or one memory request in the
        // shadow of every MFMA (0x100 LDS read, 0x200 LDS write, 0x020 memory read, 0x008 MFMA)
        constexpr int NR = 8 + (KA ? 4 : 0) + (KB ? 4 : 0);   // LDS reads of one set of fragments
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 1, fa1, fb1);
        mfmas(fa0, fb0);
        store_half(nxt, 0);
        gload_half(0, kt + 2);
        __builtin_amdgcn_sched_group_barrier(0x100, NR, 0);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 2, fa0, fb0);
        mfmas(fa1, fb1);
        store_half(nxt, 1);
        gload_half(1, kt + 2);
        __builtin_amdgcn_sched_group_barrier(0x100, NR, 1);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 1);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 3, fa1, fb1);
        mfmas(fa0, fb0);
        __builtin_amdgcn_sched_group_barrier(0x100, NR, 2);
        __builtin_amdgcn_sched_group_barrier(0x008, 16, 2);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        read_frags(nxt, 0, fa0, fb0);
        mfmas(fa1, fb1);
        __builtin_amdgcn_sched_group_barrier(0x100, NR, 3);
        __builtin_amdgcn_sched_group_barrier(0x008, 16, 3);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();   // every wave is done with the operand stages (the epilogue reuses them)
#ifdef GEMM_TIMING
    if (TIMED) ts2 = __builtin_readcyclecounter();
#endif
    gemm_epilogue<BM, BN, MI, NI, EP, true>(a, acc, smem, g, r0, m0, n0, M, N, wm0, wn0, lane, wave);
#ifdef GEMM_TIMING
    if (TIMED && tid == 0 && tile < 16384) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        g_gemm_ts[4 * tile] = ts0; g_gemm_ts[4 * tile + 1] = ts1; g_gemm_ts[4 * tile + 2] = ts2;
        g_gemm_ts[4 * tile + 3] = __builtin_readcyclecounter();
    }
#endif
}

static void tile_counts(const GemmBArgs& a, int BM, int BN, int& n_ntiles, int& mt_per_group, int64_t& n_tiles) {
    n_ntiles = (a.N + BN - 1) / BN;
    int64_t n_mtiles;
    mt_per_group = 1;
    if (a.tile_group) {
        n_mtiles = a.n_mtiles;
    } else {
        mt_per_group = (a.M + BM - 1) / BM;
        n_mtiles = (int64_t)mt_per_group * a.G;
    }
    n_tiles = (n_mtiles <= 0 || n_ntiles <= 0) ? 0 : n_mtiles * n_ntiles;
}

template <bool KA, bool KB, int EP, bool TIMED = false>
static void launch_pipe(hipStream_t st, const GemmBArgs& a) {
    constexpr int BM = 256, BN = 256;
    int n_ntiles, mt_per_group;
    int64_t n_tiles;
    tile_counts(a, BM, BN, n_ntiles, mt_per_group, n_tiles);
    if (n_tiles <= 0) return;
    const size_t shmem = ((KA ? (size_t)GK * (BM + GPADK) : (size_t)BM * GLD) + (KB ? (size_t)GK * (BN + GPADK) : (size_t)BN * GLD)) * sizeof(bf16_t) * 2;
    auto kern = gemm_bf16_pipe_kernel<KA, KB, EP, TIMED>;
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    const unsigned grid = (unsigned)((n_tiles + 7) / 8 * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), shmem, st, a, n_ntiles, mt_per_group, (int)n_tiles);
}

template <int BM, int BN, bool KA, bool KB, int EP>
static void launch_variant(hipStream_t st, const GemmBArgs& a) {
    int n_ntiles, mt_per_group;
    int64_t n_tiles;
    tile_counts(a, BM, BN, n_ntiles, mt_per_group, n_tiles);
    if (n_tiles <= 0) return;
    size_t shmem = ((KA ? (size_t)GK * (BM + GPADK) : (size_t)BM * GLD) + (KB ? (size_t)GK * (BN + GPADK) : (size_t)BN * GLD)) * sizeof(bf16_t);
    const size_t epi = (size_t)4 * 32 * (BN / 2 + 4) * sizeof(float);  // the epilogue's strips, one per wave
    if (shmem < epi) shmem = epi;
    auto kern = gemm_bf16_kernel<BM, BN, false, KA, KB, EP>;
    if (shmem > 48 * 1024) (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    const unsigned grid = (unsigned)((n_tiles + 7) / 8 * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), shmem, st, a, n_ntiles, mt_per_group, (int)n_tiles);
}

// Tile shapes of one operand form.  bm: row tile the caller built its (tile_group, tile_m0) lists for (64, 128 or
// 256); bn: 128, or 256 (with bm = 256: the pipelined 256 x 256 kernel).  Measured on the benchmark shapes: one LDS
// stage with register prefetch beats two stages for the smaller tiles (occupancy).
template <bool KB, int EP>
static void launch_rows_form(hipStream_t st, const GemmBArgs& a, int bm, int bn) {
    if (bm == 256 && bn == 256) launch_pipe<false, KB, EP>(st, a);
    else if (bm == 256) launch_variant<256, 128, false, KB, EP>(st, a);
    else if (bm == 128) launch_variant<128, 128, false, KB, EP>(st, a);
    else launch_variant<64, 128, false, KB, EP_RUNTIME>(st, a);
}

// backward form: both operands contraction-contiguous
void launch_gemm_bf16(hipStream_t st, const GemmBArgs& a, int bm, int bn) {
    switch (ep_of(a)) {
        case EPI_MASK | EP_CB: launch_rows_form<false, EPI_MASK | EP_CB>(st, a, bm, bn); break;
        case EPI_NONE | EP_CF: launch_rows_form<false, EPI_NONE | EP_CF>(st, a, bm, bn); break;
        case EPI_NONE | EP_CF | EP_CACC: launch_rows_form<false, EPI_NONE | EP_CF | EP_CACC>(st, a, bm, bn); break;
        case EPI_NONE | EP_CACC: launch_rows_form<false, EPI_NONE | EP_CACC>(st, a, bm, bn); break;
        default: launch_rows_form<false, EP_RUNTIME>(st, a, bm, bn); break;
    }
}

// Weight-gradient form: both operands stored with the contraction index slowest (A [K, M], B [K, N]).  tile: 128, or 256
// (the pipelined 256 x 256 kernel; N a multiple of 256): worth it when the contraction is thousands of rows long -- per
// task (K = a task's rows, every task writing its own [M, N]) the product is bound by what it writes, and more
// workgroups per compute unit hide that better than wider tiles.
template <int EP>
static void launch_kmajor_tile(hipStream_t st, const GemmBArgs& a, int tile) {
    if (tile == 256) launch_pipe<true, true, EP>(st, a);
    else launch_variant<128, 128, true, true, EP>(st, a);
}
void launch_gemm_bf16_kmajor(hipStream_t st, const GemmBArgs& a, int tile) {
    if (a.n_pairs > 2) tile = 128;   // (the pipelined kernel keeps two operand descriptors)
    switch (ep_of(a)) {
        case EPI_AXPBY | EP_CF: launch_kmajor_tile<EPI_AXPBY | EP_CF>(st, a, tile); break;
        case EPI_AXPBY | EP_CF | EP_CB: launch_kmajor_tile<EPI_AXPBY | EP_CF | EP_CB>(st, a, tile); break;
        case EPI_AXPBY | EP_CF | EP_CIN: launch_kmajor_tile<EPI_AXPBY | EP_CF | EP_CIN>(st, a, tile); break;
        case EPI_AXPBY | EP_CF | EP_CB | EP_CIN: launch_kmajor_tile<EPI_AXPBY | EP_CF | EP_CB | EP_CIN>(st, a, tile); break;
        case EPI_AXPBY | EP_CB | EP_CIN: launch_kmajor_tile<EPI_AXPBY | EP_CB | EP_CIN>(st, a, tile); break;
        default: launch_variant<128, 128, true, true, EP_RUNTIME>(st, a); break;
    }
}

// Forward form with the weights as they are stored (B [K, N] = W [d_in, d_out]): no transposed copy of theta.
void launch_gemm_bf16_bkmajor(hipStream_t st, const GemmBArgs& a, int bm, int bn) {
    switch (ep_of(a)) {
        case EPI_BIAS_RELU | EP_CB: launch_rows_form<true, EPI_BIAS_RELU | EP_CB>(st, a, bm, bn); break;
        case EPI_BIAS_MASK | EP_CB: launch_rows_form<true, EPI_BIAS_MASK | EP_CB>(st, a, bm, bn); break;
        default: launch_rows_form<true, EP_RUNTIME>(st, a, bm, bn); break;
    }
}

#ifdef GEMM_TIMING
void launch_gemm_bf16_timed(hipStream_t st, const GemmBArgs& a, bool kb) {   // development: per-phase cycle counts of the pipelined kernel
    if (kb) launch_pipe<false, true, EPI_BIAS_RELU | EP_CB, true>(st, a);
    else launch_pipe<false, false, EPI_MASK | EP_CB, true>(st, a);
}
#endif

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
