// Internal declarations shared by the kernel files and the host orchestration.
// Nothing here is visible across the C ABI (see include/gmeta.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32;
typedef uint64_t u64;
typedef uint16_t bf16_t;  // raw bfloat16 bits

#ifdef __HIPCC__
// fp32 -> bf16, round to nearest even: the gfx950 conversion instruction (two values per instruction)
__device__ __forceinline__ bf16_t f2bf(float x) { return __builtin_bit_cast(bf16_t, (__bf16)x); }
__device__ __forceinline__ u32 f2bf2(float lo, float hi) {  // {bf16(hi), bf16(lo)}
    typedef float gm_f2 __attribute__((ext_vector_type(2)));
    typedef __bf16 gm_b2 __attribute__((ext_vector_type(2)));
    const gm_f2 v = {lo, hi};
    return __builtin_bit_cast(u32, __builtin_convertvector(v, gm_b2));
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __builtin_bit_cast(float, (u32)h << 16); }
#endif

// Device-side status word indices (ctx->d_status).
enum { ST_BAD_INDEX = 0, ST_CAPACITY = 1, ST_MAX_TF = 2, ST_NROWS = 3, ST_MAX_BAG = 4, ST_PAIR_OVF = 5, ST_TOO_LARGE = 6, ST_WORDS = 8 };

// ------------------------------------------------------------------ index kernels
// Per-wave geometry handed to the index kernels (all device pointers).
struct SetView {
    const int64_t* bag_offsets;  // whole set
    const int32_t* indices;      // whole set
    const int64_t* task_offsets; // device copy, whole set
    int64_t sample0;             // first sample of the wave in the set
    int64_t lookup0;             // first lookup of the wave in the set
    int64_t n_samples;           // samples of the whole set
};

// uniform_rows: the number of rows every table has, or -1 when the tables differ in size
void launch_tf_count(hipStream_t st, int F, int t0, int Tw, SetView sup, SetView qry, const int64_t* field_base,
                     int64_t nnz_sup, int64_t nnz_qry, int64_t uniform_rows, u32* cnt_sup, u32* cnt_qry, u32* status);
void launch_scan_u32(hipStream_t st, const u32* in, u32* out, int64_t n, u32* tmp /* >= n/1024+2048 */,
                     u32* total /* may be null */);
size_t scan_tmp_words(int64_t n);

struct TfSortArgs {
    int F, t0, Tw;
    SetView sup, qry;
    const int64_t* field_base;      // [F+1] device
    const u32* cnt_sup;             // [Tw*F]
    const u32* base_sup;            // exclusive scan of cnt_sup
    const u32* cnt_qry;
    const u32* base_qry;
    // outputs (wave-local lookup numbering)
    u32* n_slots;                   // [Tw*F]
    u32* slot_rows;                 // [nnz_sup_w]       at base_sup[tf] + slot
    int32_t* slot_start;            // [nnz_sup_w+Tw*F]  at base_sup[tf] + tf + slot: first position of the slot in
                                    //                   the sorted list (absolute); sentinel at +n_slots
    int2* sup_sorted;               // [nnz_sup_w]       {row of the sample, slot} of every support lookup in sorted order
    int32_t* sup_slot;              // [nnz_sup_w]       by lookup
    int32_t* qry_slot;              // [nnz_qry_w]       by lookup, -1 when not in support
    int2* qry_sorted;               // [nnz_qry_w]       {row of the sample, slot or -1} of every query lookup, sorted
    int32_t* qseg_lo;               // [nnz_sup_w]       at base_sup[tf] + slot : range in the sorted query list
    int32_t* qseg_hi;
    // row of every sample (whole set) in the activation buffers, and the wave's first row
    const int32_t* sup_rows; int32_t sup_row_base;
    const int32_t* qry_rows; int32_t qry_row_base;
    u32* status;
};
void launch_tf_sort(hipStream_t st, const TfSortArgs& a, int max_tf, int max_set_rows);
int tf_sort_max_cap();

// How the value that travels with a lookup's row key names the lookup's bag in the gradient buffer.
// rshift == 0: value = (row of the sample) * F + field.  Otherwise bit fields: row << rshift | field << pshift |
// position of the lookup in its bag -- the form the per-(task, field) join needs (it finds every lookup's number again).
struct ValEnc {
    int rshift, pshift;
    u32 fmask;      // (1 << bits of a field number) - 1
};
void launch_build_keys(hipStream_t st, int F, const int64_t* field_base, const int64_t* bag_offsets,
                       const int32_t* indices, int64_t n_bags, int64_t lookup0, const int32_t* row_map, u32 row0, ValEnc enc,
                       u32* keys, u32* vals);
// Task of a bit-field value's sample: gradient-buffer rows below n_sup_rows are the wave's support rows, the others its
// query rows; row_task_* give the task (within the wave) of every padded row of a set.
struct TaskOf {
    const int32_t *row_task_s, *row_task_q;
    u32 n_sup_rows, n_rows;   // support rows; support + query rows
    int rshift;
    int uniform_shift;        // >= 0: every task has 1 << uniform_shift padded rows in each set (the tables are not read)
};
// (keys, vals) in (field, row) order -> (out_keys, out_vals) in (task, field, row) order, stable; the input is kept.
// (mid_keys, mid_vals) are needed when task_sort_passes(n_tasks) is 2.
void launch_task_sort(hipStream_t st, const u32* keys, const u32* vals, u32* mid_keys, u32* mid_vals, u32* out_keys,
                      u32* out_vals, int64_t n, int n_tasks, const TaskOf& tk, u32* hist /* radix_hist_words(n) */);
int task_sort_passes(int n_tasks);
// The outputs of launch_tf_sort, read off the (task, field, row)-ordered list instead of sorted per (task, field).
struct TfJoinArgs {
    int F, Tw;
    const u32 *keys, *vals;                        // the ordered list (bit-field values)
    const u32 *cnt_s, *base_s, *cnt_q, *base_q;    // per (task, field): lookups of each set and their exclusive scans
    int rshift, pshift;
    u32 n_sup_rows;
    u32* n_slots; u32* slot_rows; int32_t* slot_start;
    int2 *sup_sorted, *qry_sorted;
    int32_t *qseg_lo, *qseg_hi;
    int32_t *sup_slot, *qry_slot;                  // both null: the slot of every lookup is not written
    const int64_t *bag_s, *bag_q;                  // bag offsets of the two sets (whole sets)
    int64_t sample0_s, sample0_q, lookup0_s, lookup0_q;   // the wave's first sample / lookup in each set
    int64_t n_lookups_s, n_lookups_q;                     // the wave's lookups in each set
    const int32_t *row_off_s, *row_off_q, *real_off_s, *real_off_q;   // [Tw + 1] first padded row / first sample of each task
};
void launch_tf_join(hipStream_t st, const TfJoinArgs& a);
// Independent ranges of one list that a radix pass sorts side by side (device arrays of n_seg + 1 words): range i holds
// the keys at positions [key_base_pos[i], key_base_pos[i + 1]) in tiles [tile_base[i], tile_base[i + 1]), and its
// digits are taken from key - key_sub[i].  n_seg == 0: the whole list is one range.
struct SegTab {
    int n_seg;
    const u32 *tile_base, *key_base_pos, *key_sub;
};
#define RS_TILE_KEYS 2048   // keys per tile of a radix pass
// Stable LSD radix sort of (key, val) pairs on the low `bits` bits (of key - key_sub with ranges: every range by
// itself).  Returns the number of passes: after an odd number the result is in (keys_tmp, vals_tmp), else in (keys, vals).
int launch_radix_sort(hipStream_t st, u32* keys, u32* vals, u32* keys_tmp, u32* vals_tmp, int64_t n,
                      int bits, u32* hist /* radix_hist_words(n, ranges) */, const SegTab* seg = nullptr);
size_t radix_hist_words(int64_t n, int extra_tiles);
// The keys and bit-field values of a wave's lookups written field after field (a field's support lookups, then its
// query lookups, each in input order) from the per-(task, field) counts; `tables` (field_table_words(F) words) receives
// the fields' ranges, which field_seg_tab hands to the radix passes.
struct FieldKeysArgs {
    int F, t0, Tw;
    SetView sup, qry;
    const int64_t* field_base;
    const u32 *cnt_s, *cnt_q;        // [Tw * F]
    u32 *fm_off_s, *fm_off_q;        // [Tw * F] scratch: a (task, field)'s place inside its field's range, per set
    const int32_t *prow_s, *prow_q;  // padded row of every sample (whole sets)
    u32 row0_s, row0_q;              // added to it: the row in the gradient buffer
    ValEnc enc;                      // bit-field form (rshift != 0)
    u32 *keys, *vals;
    const u32 *key_pos, *tot;        // set by the launcher
};
void launch_build_keys_by_field(hipStream_t st, FieldKeysArgs a, u32* tables);
SegTab field_seg_tab(int F, u32* tables);
size_t field_table_words(int F);
void launch_segments(hipStream_t st, const u32* sorted_keys, int64_t n, u32* flags_scan, u32* scan_tmp,
                     int64_t* emb_rows, u32* seg_start, int64_t* seg_counts /* may be null */,
                     int64_t capacity, int64_t* n_rows_out, u32* status);

// ------------------------------------------------------------------ embedding kernels
void launch_gather_pool(hipStream_t st, int F, int D, int n_dense, const int64_t* field_base,
                        const int64_t* bag_offsets, const int32_t* indices, const float* dense,
                        const float* emb, int64_t sample0, int64_t n_samples, const int32_t* row_map,
                        int32_t row_base, float* x /* may be null */, int ldx, bf16_t* x_bf /* may be null */);
// Two-hop row arithmetic per (task, field): G[slot] = sum of Z over the slot's lookups (hop 1), then
// y_out[bag] = y_in[bag] + c * sum over the bag's lookups of G[slot] (hop 2), for up to two sets of bags.
struct TwoHopOut {
    int enabled;
    const int64_t* bag_offsets;     // the set's CSR (whole set)
    int64_t sample0, lookup0;       // the wave's first sample / lookup in the set
    const int32_t* real_offsets;    // [Tw+1] first sample of each task, relative to sample0
    const int32_t* slot_of_lookup;  // [lookups of the wave] slot of each lookup, -1 when its row is not in the support set
    const int32_t* row_map;         // row of each sample of the wave in the activation buffers
    int32_t row_base;
    const float* y_in;              // null: start from zero
    float* y_out;                   // may alias y_in; may be null
    bf16_t* y_bf;                   // may be null
    int64_t ld;
    float c;
};
struct TwoHopArgs {
    int F, D, dc, range, bag0;      // dc (columns per slice), range and bag0 are set by the launcher
    const u32 *tf_base, *n_slots;   // per (task, field): base of its slot / lookup lists, number of slots
    const int32_t *in_seg_lo, *in_seg_hi;  // lookups of slot u: positions [lo, hi) of in_sorted_row, at base + tf*stride + u
    int in_seg_tf_stride;
    const int2* in_sorted;          // {row of Z, slot or -1} of every lookup in slot order
    const int32_t* in_row_offsets;  // [Tw+1] first row (of Z) of each task
    int max_in_rows;                // largest number of rows of Z any task has
    const float* Z;                 // [rows, ldz], the (field f) block at column f*D
    int64_t ldz;
    TwoHopOut out[2];
    const u32* task_path;           // [Tw] tasks flagged 1 are left to the pair-count kernels (null: none is)
};
void launch_two_hop(hipStream_t st, TwoHopArgs a, int n_tasks, int max_bags);

// The same row arithmetic as a dense product: per (task, field) the pair-count matrix
// M[i][j] = number of (lookup of out-bag i, lookup of in-bag j) pairs on one row of the task's support set,
// stored as bytes, [pad64(n_out)][pad64(n_in)] per field, fields of a task back to back.
#define PAIR_LDS_BYTES (159 * 1024)   // LDS of the counting kernel: a tile of byte cells, two dense count blocks, the lists
#define PAIR_MAX_CAP 16384       // lookups of one (task, field) and set that the counting kernel stages
#define PAIR_MAX_BAG 127         // longest bag for which a (bag, row) count is a non-negative 8-bit integer
struct PairCountArgs {
    int F;
    const int32_t *real_off_s, *real_off_q;   // [Tw+1] first sample of each task (relative to the wave)
    const int32_t *row_off_s, *row_off_q;     // [Tw+1] first row of each task in the activation buffers
    const u32 *base_s, *base_q, *cnt_q, *n_slots;   // per (task, field)
    const int32_t *slot_start, *qseg_lo, *qseg_hi;
    const int2 *sup_sorted, *qry_sorted;
    const int64_t *off_ss, *off_qs, *off_sq;  // [Tw] byte offset of the task's first matrix of each kind
    uint8_t* mat;
    int want_ss, want_sq;
    int lds_bytes, n_max, max_tile_rows;      // set by the launcher
    int cls, small_n;                         // set by the launcher: 0 all, 1 only small (task, field)s, 2 only the others
    u32* task_path;                           // [Tw] only tasks flagged 1 are counted; cleared when a count exceeds 254
    u32* status;
};
void launch_pair_count(hipStream_t st, PairCountArgs a, int Tw, int max_tf, int max_rows, int min_rows, int max_tile_rows);
struct PairHopOut {
    int enabled;
    const int64_t* mat_off;                   // [Tw]
    const int32_t *real_off, *row_off;        // the out set
    const float* y_in;                        // null: start from zero
    float* y_out;                             // may alias y_in; may be null
    bf16_t* y_bf;                             // may be null
    int64_t ld;
    float c;
};
struct PairHopArgs {
    int F, D, row_blocks, n_out, n_work;      // row_blocks, n_out (enabled out sets) and n_work (workgroups) are set by the launcher
    const uint8_t* mat;
    const int32_t *in_real_off, *in_row_off;  // the in set
    const float* Z;                           // [rows, ldz], the (field f) block at column f*D
    int64_t ldz;
    PairHopOut out[2];
    const u32* task_path;                     // [Tw] only tasks flagged 1 are touched
};
void launch_pair_hop(hipStream_t st, PairHopArgs a, int Tw, int max_out_rows);
void launch_copy_tail(hipStream_t st, int FD, const float* x_base, int64_t n_rows, float* x_out, int ldx, bf16_t* x_bf);

// keys: the sorted row keys; scan: exclusive scan of their segment-head flags and n_rows: the number of segments
// (both as launch_segments left them; neither is read when the output is table-shaped)
void launch_seg_reduce(hipStream_t st, int D, int F, ValEnc enc, const u32* keys, const u32* scan, const int64_t* n_rows,
                       int64_t capacity, int64_t n, const u32* sorted_vals, const float* gx,
                       float* emb_grad, float* partial /* seg_reduce_partial_floats(n, D) */,
                       float* table /* null, or [all rows, D]: every segment is ADDED to its row instead of listed */);
size_t seg_reduce_partial_floats(int64_t n, int D);
void launch_scatter_add(hipStream_t st, int D, float* table, const int64_t* rows, const float* grad,
                        int64_t n_rows, float scale);

// ------------------------------------------------------------------ MLP kernels
enum { EPI_NONE = 0, EPI_BIAS_RELU = 1, EPI_BIAS_MASK = 2, EPI_MASK = 3, EPI_AXPBY = 4 };

struct GemmArgs {
    // up to two products accumulated: C = A1*B1 (+ A2*B2)
    const float* A[2];
    const float* B[2];
    int64_t sAm[2], sAk[2], gA[2];   // element (m,k) of group g: A + g*gA + r0(g)*rA + m*sAm + k*sAk
    int64_t sBk[2], sBn[2], gB[2];
    int64_t rA[2], rB[2];            // multiplier of the group's first row r0(g)
    int n_pairs;
    float* C;
    int64_t ldc, gC, rC;             // element (m,n): C + g*gC + r0(g)*rC + m*ldc + n
    int M, N, K;                     // fixed extents; -1 means "rows of the group" (variable)
    const int32_t* row_offsets;      // [G+1] device: first row of each group
    int G;
    // tiles over variable M: per m-tile the group and its first row inside the group
    const int32_t* tile_group;       // [n_mtiles] (null when M is fixed)
    const int32_t* tile_m0;
    int n_mtiles;
    int epi;
    const float* bias; int64_t gBias;           // bias + g*gBias + n
    const float* mask; int64_t ld_mask;         // mask + (r0+m)*ld_mask + n
    const float* Cin; int64_t gCin;             // Cin + g*gCin + m*ldc + n   (EPI_AXPBY)
    float c0, c1;
};
void launch_gemm_f32(hipStream_t st, const GemmArgs& a);

// bf16 operands, both stored contraction-contiguous: C[M,N] = sum_p A_p[M,K] * Bt_p[N,K]^T
#define GEMM_MAX_PAIRS 4   // products accumulated into one output (the pipelined kernel takes at most two)
struct GemmBArgs {
    const bf16_t* A[GEMM_MAX_PAIRS];
    const bf16_t* B[GEMM_MAX_PAIRS];
    int64_t lda[GEMM_MAX_PAIRS], gA[GEMM_MAX_PAIRS], rA[GEMM_MAX_PAIRS];   // element (m,k) of group g: A + g*gA + r0(g)*rA + m*lda + k
    int64_t ldb[GEMM_MAX_PAIRS], gB[GEMM_MAX_PAIRS], rB[GEMM_MAX_PAIRS];   // element (n,k) of group g: B + g*gB + r0(g)*rB + n*ldb + k
    int n_pairs;
    int M, N, K;                    // -1: rows of the group
    const int32_t* row_offsets;     // [G+1]
    int G;
    const int32_t* tile_group;      // per m-tile (null: fixed M, tiles enumerated per group)
    const int32_t* tile_m0;
    int n_mtiles;
    int epi;
    const float* bias; int64_t gBias;
    const bf16_t* mask; int64_t ld_mask;   // mask + (r0+m)*ld_mask + n
    const float* Cin; int64_t gCin, ldcin; // Cin + g*gCin + m*ldcin + n (EPI_AXPBY)
    float c0, c1;
    float* Cf; int64_t ldcf, gCf, rCf;     // fp32 output        (either may be null)
    bf16_t* Cb; int64_t ldcb, gCb, rCb;    // bf16 output
    float* Cacc; int64_t ldcacc, rCacc; float cacc;  // Cacc[(r0 + m)*ldcacc + n] += cacc * value (not with EPI_AXPBY + Cin)
    int cacc_init;                                   // 1: Cacc is not read, = cacc * value (first term of a sum)
};
void launch_gemm_bf16(hipStream_t st, const GemmBArgs& a, int bm, int bn = 128);   // bn = 256 (with bm = 256): the pipelined 256 x 256 kernel
// same product with both operands stored contraction-slowest: A_p element (k, m) at A + g*gA + r0*rA + k*lda + m,
// B_p element (k, n) at B + g*gB + r0*rB + k*ldb + n
void launch_gemm_bf16_kmajor(hipStream_t st, const GemmBArgs& a, int tile = 128);   // tile: 128, or 256 (N % 256 == 0)
// A contraction-contiguous as in launch_gemm_bf16, B stored contraction-slowest (element (k, n) at ... + k*ldb + n)
void launch_gemm_bf16_bkmajor(hipStream_t st, const GemmBArgs& a, int bm, int bn = 128);
void launch_convert_weights(hipStream_t st, const float* src, int64_t g_src, int G, int rows, int cols, bf16_t* w,
                            bf16_t* wT, int64_t g_dst);

// out[g*g_out + n] = c0*in[g*g_in + n] + c1 * sum_{s in group g} (X1[s,n]*w1[s] + X2[s,n]*w2[s])
void launch_task_colsum(hipStream_t st, int G, const int32_t* row_offsets, int N, const float* X1,
                        const float* w1, const float* X2, const float* w2, int64_t ldx, float* out,
                        int64_t g_out, const float* in, int64_t g_in, float c0, float c1);
void launch_task_colsum_bf(hipStream_t st, int G, const int32_t* row_offsets, int N, const bf16_t* X1,
                           const float* w1, const bf16_t* X2, const float* w2, int64_t ldx, float* out,
                           int64_t g_out, const float* in, int64_t g_in, float c0, float c1);
// z[s] = a[s,:].w_g + b_g (+ ta[s,:].w_g + a[s,:].tw_g + tb_g when tangent)
struct LastFwdArgs {
    int64_t n; int N; int64_t ld;       // rows (padded), width of the last hidden layer, its leading dimension
    int bf16;                           // activations a / ta are bf16 (else fp32)
    const int32_t* row_task;            // [n] task of every row
    const int32_t* row_offsets;         // [G+1] first (padded) row of each task
    const int32_t* real_offsets;        // [G+1] first sample of each task (labels are indexed by sample)
    const void* a; const void* ta;      // ta null: plain forward
    const float* w; int64_t gW; const float* b;      // w + g*gW [N], b + g*gW scalar
    const float* tw; int64_t gTW; const float* tb;
    const float* labels; const float* z_in;          // tangent: z of the primal pass
    float* z_out; float* delta_out; float* loss_out; // plain: z, (sigma-y)/N_g, bce/N_g
                                                     // tangent: delta_out = sigma'(z) * tz / N_g
};
void launch_last_fwd(hipStream_t st, const LastFwdArgs& a);
void launch_last_bwd(hipStream_t st, int bf16, int64_t n, int N, int64_t ld_a, int64_t ld_d, const int32_t* row_task,
                     const float* dl, const float* w, int64_t gW, const float* dl2, const float* w2, int64_t gW2,
                     const void* act, void* d, float* d_f32);
void launch_reduce_tasks(hipStream_t st, const float* v, int64_t ld, int G, int64_t n, float* out, int accumulate,
                         float scale = 1.f);
void launch_fill_sample_task(hipStream_t st, const int32_t* row_offsets, int G, int32_t* sample_task);
void launch_pack_weights(hipStream_t st, const float* W, int din, int dout, int ld_in, int ld_out, float* dst);
void launch_unpack_weights(hipStream_t st, const float* src, int din, int dout, int ld_out, float* W);
void launch_axpy(hipStream_t st, int64_t n, float a, const float* x, float* y);  // y += a*x
void launch_axpy_clear(hipStream_t st, int64_t n, float a, float* x, float* y);  // y += a*x, x = 0 (n % 4 == 0, 16-byte aligned)
void launch_sum_to_scalar(hipStream_t st, const float* x, int n, float* out, int accumulate);
void launch_fill_u32(hipStream_t st, u32* p, int64_t n, u32 v);
void launch_fill_f32(hipStream_t st, float* p, int64_t n, float v);

// ------------------------------------------------------------------ on-box ceilings (measurement only)
void launch_stream_copy(hipStream_t st, const void* src, void* dst, int64_t bytes);
void launch_stream_read(hipStream_t st, const void* src, int64_t bytes, u32* sink);
double launch_mfma_loop(hipStream_t st, int iters, float* sink);   // returns the flops of the launch
double launch_mfma_loop_random(hipStream_t st, int iters, float* sink);
