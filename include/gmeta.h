/*
 * gmeta.h -- C ABI of the MI355X-native per-task MAML step over a DLRM-style model.
 *
 * What is computed (G-Meta, Algorithm 1, with "worker i" read as "task t"; MAML as
 * the paper adopts it in Section 2):
 *   prefetch of support and query embedding rows in one pass        (Alg. 1, prefetch step; Sec. 2.1.1)
 *   inner forward L^Sup, local back-propagation on the looked-up
 *   rows and on theta with step alpha, repeated inner_steps times    (Alg. 1, inner steps)
 *   overlap update of the query rows that the support set adapted    (Alg. 1, overlap step; Sec. 2.1.2)
 *   outer forward L^Query with the adapted parameters                (Alg. 1, outer forward)
 *   gradients of L^Query w.r.t. the META parameters, summed over
 *   tasks: dense part (theta) and sparse part (xi)                   (Alg. 1, global back-propagation
 *                                                                     steps; Sec. 2.1.3 sum rule)
 * The beta update: gm_meta_train_step (the step and the update in one call), or gm_scatter_add (sparse half alone).
 *
 * Model: x_s = concat_f( sum_{r in bag(s,f)} xi_f[r] ) || dense_s ; MLP d_0 -> ... -> d_L = 1 with
 * ReLU on hidden layers; loss = mean over a set's samples of the binary cross-entropy with logits.
 * Tasks are summed.  order = 1 drops the Hessian-vector term, order = 2 keeps it.
 *
 * Pointer convention: every pointer below is marked HOST or DEVICE.  DEVICE memory is allocated
 * and owned by the caller; the library never frees or reallocates it and never writes to inputs.
 * All calls of one context are issued on the HIP stream given at gm_create and every entry point
 * returns after that stream has drained (results are valid on return).
 * Return value: GM_OK (0) or a negative gm_status; gm_last_error() gives a message.  On error the
 * outputs are unspecified, but no out-of-bounds access is made: indices, offsets and capacities are
 * checked on the device before they are used.
 */
#ifndef GMETA_H
#define GMETA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GM_OK = 0,
    GM_ERR_ARG = -1,        /* null pointer, negative size, unsupported shape, bad order          */
    GM_ERR_INDEX = -2,      /* an index is outside its table, or offsets are not monotone          */
    GM_ERR_CAPACITY = -3,   /* emb_rows_capacity too small, or a (task, field) exceeds the limits  */
    GM_ERR_WORKSPACE = -4,  /* the context's workspace cannot hold even one task                   */
    GM_ERR_HIP = -5         /* a HIP runtime call failed                                           */
} gm_status;

typedef struct gm_ctx gm_ctx; /* opaque; owns only its workspace */

/* Model shape.  HOST struct, HOST arrays (copied by gm_create). */
typedef struct {
    int32_t n_fields;              /* F sparse fields                                       */
    const int64_t* rows_per_field; /* HOST [F] rows of each field's table                   */
    int32_t emb_dim;               /* D, a power of two in 4..256                           */
    int32_t n_dense;               /* dense features per sample                             */
    int32_t n_layers;              /* L                                                     */
    const int32_t* layer_dims;     /* HOST [L+1] d_0..d_L; d_0 = F*D + n_dense, d_L = 1     */
    int32_t mlp_dtype;             /* 0: fp32 GEMMs; 1: bf16 operands, fp32 accumulation    */
} gm_model_desc;

/* One set (support or query) of all tasks, CSR over (sample, field) bags. */
typedef struct {
    int64_t n_samples;           /* over all tasks                                               */
    int64_t nnz;                 /* total lookups = bag_offsets[n_samples*F]                     */
    const int64_t* task_offsets; /* HOST   [T+1] sample range of each task, task_offsets[0] = 0  */
    const int64_t* bag_offsets;  /* DEVICE [n_samples*F+1], sample-major, field-minor            */
    const int32_t* indices;      /* DEVICE [nnz] row within its field's table                    */
    const float* dense;          /* DEVICE [n_samples, n_dense] row-major                        */
    const float* labels;         /* DEVICE [n_samples] in {0,1}                                  */
} gm_set;

/* Meta-parameters (never written). */
typedef struct {
    const float* emb;       /* DEVICE [sum rows_per_field, D] row-major, tables field after field */
    const float* const* W;  /* HOST array [L] of DEVICE pointers, W_l is [d_{l-1}, d_l] row-major */
    const float* const* b;  /* HOST array [L] of DEVICE pointers, b_l is [d_l]                    */
} gm_params;

/* Outputs of gm_meta_step. */
typedef struct {
    float* const* dW;          /* HOST array [L] of DEVICE pointers, same shapes as W            */
    float* const* db;          /* HOST array [L] of DEVICE pointers, same shapes as b            */
    int64_t* emb_rows;         /* DEVICE [capacity] ascending distinct global rows (field_base[f]
                                  + index) looked up by any support or query sample             */
    float* emb_grad;           /* DEVICE [capacity, D] gradient of the listed rows               */
    int64_t* n_emb_rows;       /* DEVICE scalar: number of rows listed                           */
    int64_t emb_rows_capacity; /* rows that emb_rows / emb_grad can hold                         */
    float* task_loss;          /* DEVICE [T] per-task L^Query, or NULL                           */
    float* emb_grad_table;     /* NULL, or DEVICE [sum rows_per_field, D] (the shape of params->emb):
                                  the sparse meta-gradient is ADDED to it row by row (the summation
                                  over tasks of Alg. 1's global back-propagation on xi, landing in a
                                  caller-owned accumulator) and no list is produced: emb_rows,
                                  emb_grad and emb_rows_capacity are ignored and *n_emb_rows = 0.
                                  Every wave of tasks orders and reduces its own lookups, so the
                                  call may hold more than 2^31 lookups per set; a row's sum is taken
                                  in a fixed order for a given workspace size.  Must not alias
                                  params->emb.                                                    */
} gm_grads;

/* Creates a context on `device` that enqueues on `hip_stream` (a hipStream_t, or NULL for the
 * default stream) and owns a workspace of `workspace_bytes` (see gm_workspace_bytes). */
int gm_create(gm_ctx** ctx, const gm_model_desc* model, int device, void* hip_stream,
              size_t workspace_bytes);
void gm_destroy(gm_ctx* ctx);
const char* gm_last_error(const gm_ctx* ctx);

/* Workspace that lets a batch of this size, with tasks of equal size, run in ONE wave of tasks.  A
 * smaller workspace is legal (and very uneven tasks may need more): gm_meta_step then processes the
 * tasks in several waves (Alg. 1 treats tasks independently). */
size_t gm_workspace_bytes(const gm_model_desc* model, int32_t n_tasks, int64_t n_support,
                          int64_t n_query, int64_t nnz_support, int64_t nnz_query,
                          int32_t inner_steps, int32_t order);

/* The whole step (Alg. 1 from the prefetch step to the two global back-propagation steps, without
 * the beta update).  loss: DEVICE scalar = sum_t L^Query_t.  order in {1,2}; inner_steps >= 0.
 * Size limits of a well-formed call (each reported as GM_ERR_CAPACITY with its own message, never as GM_ERR_INDEX):
 *   a bag holds at most 65,535 lookups and a task at most 65,536 samples per set;
 *   with the row-list output each set holds fewer than 2^31 lookups (any number with emb_grad_table);
 *   when the inner loop adapts embedding rows (inner_steps > 0, "adapt_rows" = 1, at least one field): a (task,
 *   field) holds at most 16,384 lookups per set, and a task at most 2,048 samples per set (rounded up to a
 *   multiple of 8 with bf16 operands);
 *   all tables together hold fewer than 2^32 rows, and one call fewer than 2^31 (sample, field) bags per set. */
int gm_meta_step(gm_ctx* ctx, int32_t n_tasks, const gm_set* support, const gm_set* query,
                 const gm_params* params, float inner_lr, int32_t inner_steps, int32_t order,
                 float* loss, gm_grads* out);

/* gm_meta_step for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): same arguments, same results, but every intermediate buffer lives in a static
 * device array of GM_STATIC_SCRATCH_MIB MiB that is part of the library's code object (each GPU the library runs on
 * holds its copy until the process ends) instead of the context's workspace, and the call allocates and frees
 * nothing on the device.  The caller still passes inputs and outputs; ctx must have been created before (gm_create
 * is where the array is located on the device).  Tasks run in waves as in gm_meta_step when the scratch does not
 * hold them all at once; a call whose batch-level buffers plus one task do not fit returns GM_ERR_WORKSPACE and says
 * so.  All calls on one GPU -- of any context -- share that GPU's array: calls that overlap in time on one GPU race,
 * and nothing in it survives from one call to the next (every call initialises what it reads).  Kernel timing
 * (gm_profile) is suspended for the call. */
#define GM_STATIC_SCRATCH_MIB 64
int gm_meta_step_static(gm_ctx* ctx, int32_t n_tasks, const gm_set* support, const gm_set* query,
                        const gm_params* params, float inner_lr, int32_t inner_steps, int32_t order,
                        float* loss, gm_grads* out);

/* One whole iteration of Alg. 1 on one shard: gm_meta_step, then the two global back-propagation steps
 * applied with the outer step size beta (plain SGD on the summed meta-gradient), IN PLACE:
 *   W_l -= outer_lr * dW_l,  b_l -= outer_lr * db_l,  emb[row, :] -= outer_lr * grad[row, :] for every row
 *   that a support or query sample looks up.
 * params: as for gm_meta_step, but the DEVICE arrays it points to are written (emb, every W_l, every b_l).
 * loss: DEVICE scalar, the step's sum_t L^Query_t (before the update).  task_loss: DEVICE [T] or NULL.
 * The meta-gradient lists live in the context's workspace (rows * (4 D + 8) bytes on top of what the step
 * needs, rows = min(lookups, table rows); GM_ERR_WORKSPACE if that does not fit).  The row-list form of the
 * sparse gradient is used, so each set must hold fewer than 2^31 lookups.  Errors as gm_meta_step; on an
 * error nothing has been updated. */
int gm_meta_train_step(gm_ctx* ctx, int32_t n_tasks, const gm_set* support, const gm_set* query,
                       const gm_params* params, float inner_lr, int32_t inner_steps, int32_t order,
                       float outer_lr, float* loss, float* task_loss);

/* gm_meta_train_step for batches of any size (the row-list form holds fewer than 2^31 lookups per set): the sparse
 * meta-gradient is accumulated, wave of tasks by wave of tasks, in emb_grad_table -- DEVICE [all table rows, D]
 * fp32, 16-byte aligned, ALL ZERO on entry -- and then applied to the tables in one streaming pass
 * (emb -= outer_lr * table) that also clears the buffer: it is all zero again on return, ready for the next
 * iteration.  Everything else as gm_meta_train_step (Alg. 1: the step, then both global back-propagation steps
 * applied with step size beta); the workspace only has to hold the dense meta-gradient beside the step. */
int gm_meta_train_step_table(gm_ctx* ctx, int32_t n_tasks, const gm_set* support, const gm_set* query,
                             const gm_params* params, float inner_lr, int32_t inner_steps, int32_t order,
                             float outer_lr, float* loss, float* task_loss, float* emb_grad_table);

/* n_iters iterations of Alg. 1 on one shard in one call: iteration i is gm_meta_train_step on (support[i], query[i]),
 * and the parameters after the call are bit for bit those of n_iters such calls in a row.  What the call adds is the
 * overlap of Alg. 1's outer loop as a sustained training loop: everything of batch i+1 that depends on its indices
 * only (validation, per-(task, field) row dictionaries and overlap join of Sec. 2.1.2, pair-count matrices, the order
 * of all lookups by row for the sparse gradient) is prepared on the context's second stream while batch i computes,
 * and the step itself then runs without a host synchronisation.
 * n_tasks: HOST [n_iters]; support, query: HOST arrays of n_iters gm_set (each as for gm_meta_step, row-list form:
 * fewer than 2^31 lookups per batch); params: updated in place; losses: DEVICE [n_iters], the loss of every step
 * before its update; n_done: HOST, iterations applied when the call returns (all of them on GM_OK; on an error the
 * failing iteration and the ones after it have not been applied), or NULL.
 * The overlap needs every batch to run as one wave of tasks and the workspace to hold, beside the dense buffers of
 * one batch, the index structures of two batches and the meta-gradient lists; otherwise the iterations simply run one
 * after the other (same results).  The "overlap_sort" / "overlap_pairs" settings are ignored during the call. */
int gm_meta_train(gm_ctx* ctx, int32_t n_iters, const int32_t* n_tasks, const gm_set* support, const gm_set* query,
                  const gm_params* params, float inner_lr, int32_t inner_steps, int32_t order, float outer_lr,
                  float* losses, int32_t* n_done);

/* Output buffers of gm_group_batch for one set.  Capacities are those of the whole stream (a set can at most
 * hold every record): task_offsets n_records + 1, bag_offsets n_records * F + 1, indices nnz, dense
 * n_records * n_dense, labels n_records.  n_samples and nnz are written by the call; afterwards the struct's
 * arrays are exactly a gm_set. */
typedef struct {
    int64_t n_samples;     /* out */
    int64_t nnz;           /* out */
    int64_t* task_offsets; /* HOST   */
    int64_t* bag_offsets;  /* DEVICE */
    int32_t* indices;      /* DEVICE */
    float* dense;          /* DEVICE */
    float* labels;         /* DEVICE */
} gm_set_buffers;

/* The step before the hot path (Sec. 2.2.2, Meta I/O pipeline; Alg. 1 "Split T_i"): assembles one-task
 * batches from a flat stream of records and splits each into its support and query set.  Records with equal
 * (task, batch_id) form one batch (the paper's GroupBatchOp); batches come out in ascending (task, batch_id)
 * order, records keep their stream order inside a batch, and the first ceil(n * support_num / support_den)
 * records of a batch of n are its support set (the paper fixes none of the three; see the oracle).
 * task, batch_id: HOST [n_records].  bag_offsets: DEVICE [n_records * F + 1] (sample-major, field-minor),
 * indices: DEVICE [nnz], dense: DEVICE [n_records, n_dense], labels: DEVICE [n_records].
 * *n_tasks: number of batches.  The stream must hold fewer than 2^31 records and 2^32 lookups.
 * GM_ERR_INDEX if bag_offsets is not monotone from 0 to nnz.  Uses the context's workspace
 * (about 12 bytes per bag). */
int gm_group_batch(gm_ctx* ctx, int64_t n_records, int64_t nnz, const int64_t* task, const int64_t* batch_id,
                   const int64_t* bag_offsets, const int32_t* indices, const float* dense, const float* labels,
                   int32_t support_num, int32_t support_den, gm_set_buffers* support, gm_set_buffers* query,
                   int32_t* n_tasks);

/* table[rows[i], :] += scale * grad[i, :]  (Alg. 1, global back-propagation on xi, on one shard,
 * with scale = -beta).  rows must be distinct (as gm_meta_step emits them).  All DEVICE. */
int gm_scatter_add(gm_ctx* ctx, float* table, const int64_t* rows, const float* grad,
                   int64_t n_rows, float scale);

/* The prefetch step alone: pooled model input of every sample of `set`,
 * x[s, :] = [ sum-pooled rows of field 0 | ... | field F-1 | dense_s ], DEVICE [n_samples, d_0]. */
int gm_gather_pool(gm_ctx* ctx, int32_t n_tasks, const gm_set* set, const float* emb, float* x);

/* The integer side of the step alone (the overlap join of Sec. 2.1.2 and the row routing of the
 * sparse gradient), for exact comparison.  All outputs DEVICE, sized by the caller:
 *   slot_counts [T*F]       distinct rows of the task's SUPPORT lookups in the field
 *   slot_rows   [nnz_sup]   those rows (global ids) ascending per (task, field), packed in
 *                           (task, field) order; first sum(slot_counts) entries are valid
 *   sup_slot    [nnz_sup]   rank of each support lookup's row in its (task, field) list
 *   qry_slot    [nnz_qry]   that rank for query lookups whose row is in the list, else -1
 *   emb_rows    [capacity], seg_counts [capacity], n_emb_rows: ascending distinct global rows over
 *                           all lookups, and how many lookups hit each */
int gm_index_prep(gm_ctx* ctx, int32_t n_tasks, const gm_set* support, const gm_set* query,
                  int64_t* slot_counts, int64_t* slot_rows, int32_t* sup_slot, int32_t* qry_slot,
                  int64_t* emb_rows, int64_t* seg_counts, int64_t* n_emb_rows,
                  int64_t emb_rows_capacity);

/* Settings of a context.  All but "adapt_rows" are implementation choices that change results by rounding
 * order only (for measurement and tests).
 *   "row_path": how the task-local row arithmetic (inner-loop row update, overlap update of Sec. 2.1.2 and
 *               their tangents) is carried out: 0 = chosen per wave of tasks (default); 1 = always the
 *               sparse two-hop kernel; 2 = always per-(task, field) pair-count matrices on the matrix
 *               cores (gm_meta_step then returns GM_ERR_CAPACITY when a wave exceeds that path's limits:
 *               bags of at most 127 lookups, pair counts of at most 254, 16384 lookups per task, field and set).
 *   "index_path": how the per-(task, field) row dictionaries, lookup lists and the overlap join of Sec. 2.1.2 are
 *               built: 0 = chosen per wave of tasks (default); 1 = every (task, field) sorted by itself; 2 = read
 *               off the row order of the wave's lookups (the order the sparse meta-gradient of Alg. 1 needs anyway,
 *               followed by one stable pass by task; GM_ERR_CAPACITY when that order is not the wave's own -- a
 *               row-list output over several waves -- or a gradient-buffer row, a field number and a position in a
 *               bag do not fit 32 bits together).  Identical integer structures, identical results.
 *   "sort_fields": with the row order of "index_path": 1 (default) = the wave's row keys are laid out field after field
 *               (the per-(task, field) counts give every lookup its place) and every field's range is sorted by
 *               its row bits alone, in fewer radix passes; 0 = one sort on (field, row).  The same order either way.
 *   "adapt_rows": 1 (default) = the inner loop adapts the dense parameters and the looked-up embedding rows
 *               (Alg. 1); 0 = it adapts the dense parameters only and reads the embeddings as they are (the
 *               dense-only family of optimisation-based meta learners that Sec. 3.1 runs on the same
 *               framework); the meta-gradient w.r.t. the embeddings then is the query loss's own plus, for
 *               order 2, the path through the adapted dense parameters.  THIS ONE CHANGES WHAT IS COMPUTED.
 *   "overlap_sort": 1 = the ordering of the lookups by row (it depends on the indices only) runs on a second
 *               stream of the context beside the dense phase and is joined before the segment reduction;
 *               0 (default) = everything on the context's stream.  Identical results.
 *   "overlap_pairs": 1 = the pair-count matrices (they depend on the indices only) are counted on the second
 *               stream beside the prefetch and the first forward / backward pass and joined before the first
 *               row hop; 0 (default) = on the context's stream.  Identical results; ignored while
 *               "overlap_sort" is 1.
 *   "gemm_tile_n": column tile of the forward / backward grouped products when tasks get 256-row tiles:
 *               0 = chosen by shape (256, the software-pipelined 256 x 256 tiles, when the contraction is at least
 *               1024 long and the width a multiple of 256; else 128), 128, or 256.  Identical results.
 *   "wgrad_wide": 1 (default) = weight-gradient products take the pipelined 256 x 256 tiles when a group (a task, or
 *               a run of consecutive tasks for the products that are only ever summed over tasks) has at least 512
 *               rows, the layer is at least 1024 wide on the input side and a multiple of 256 on the output side, and
 *               the tiles fill the device at least twice; 0 = always 128 x 128 tiles.  Identical results over the
 *               same groups.
 *   "theta_from_meta": bf16 operands, second order, 2 to 4 inner steps: 1 (default) = the weight matrices of inner step k
 *               are written as theta - alpha * (the gradients of steps 0..k), one product per step accumulated on the
 *               matrix cores, straight from the meta parameters (every step's activations and deltas are kept for the
 *               second-order chain anyway): no per-task fp32 copy of a weight matrix is written or read; 0 = every
 *               step updates a per-task fp32 master (theta_{k+1} = theta_k - alpha * gradient_k).  The same values up
 *               to fp32 rounding before the bf16 operand copy is taken.
 *   "coarse_groups": number of runs of consecutive tasks for those products: 0 (default) = 16, or, when the first
 *               layer's product takes the wide tiles, the count in [12, 16] whose tiles fill the device's last round
 *               best; 1..32 = that many.  Another grouping adds the same per-task terms in another order
 *               (fp32 rounding).
 *   "max_wave_tasks": most tasks processed at a time (0 = as many as the workspace holds).  Tasks are independent
 *               (Alg. 1): a call runs them in waves of nearly equal size, the fewest that fit the workspace.
 *   "pair_tile_rows": most out-rows of a pair-count matrix that the counting kernel holds in LDS at a time
 *               (0 = as many as fit); identical results.
 * Unknown keys or values give GM_ERR_ARG. */
int gm_configure(gm_ctx* ctx, const char* key, int64_t value);

/* Kernel timing for measurement harnesses (not part of the method): while enabled, every kernel family
 * launched by later calls is bracketed by HIP events on the context's stream.  gm_profile_report returns
 * HOST text owned by the context, one line per family: "name launches total_ms algorithmic_bytes
 * algorithmic_flops".  Enabling clears the accumulated figures. */
int gm_profile(gm_ctx* ctx, int enable);
const char* gm_profile_report(gm_ctx* ctx);

/* On-box ceilings for measurement harnesses (not part of the method): a streaming copy (bytes read + written per
 * second), a streaming read, and a register-resident v_mfma_f32_32x32x16_bf16 loop with constant operands and with
 * operands that change from one instruction to the next (pseudo-random values of the magnitude of activations and
 * weights: the rate the matrix cores sustain on real data), each run by a kernel of the library's own on the
 * context's workspace (at least 130 MiB; up to 2 GiB per buffer are used) and timed with HIP events: the best of
 * several repetitions.  Outputs are HOST: GB/s, GB/s, TFLOP/s, TFLOP/s, and (if not NULL) the bytes of one
 * buffer -- every stream_copy_kernel dispatch of the call reads that many bytes and writes as many, which gives
 * profiler byte counters a transfer of known size to be scaled by. */
int gm_ceilings(gm_ctx* ctx, double* copy_gbs, double* read_gbs, double* mfma_tflops, double* mfma_random_tflops,
                int64_t* buffer_bytes);

#ifdef __cplusplus
}
#endif
#endif /* GMETA_H */
