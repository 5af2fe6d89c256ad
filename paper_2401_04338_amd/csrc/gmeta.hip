// Host side of the library: the C ABI of include/gmeta.h and the orchestration of one MAML step
// (G-Meta Alg. 1 with "worker" read as "task") as a fixed sequence of kernel launches on one stream.
//
// Data layout in HBM (per wave of tasks; a wave is as many tasks as the workspace holds):
//   activations  [rows, ld]   rows = samples of the wave, each task's rows padded to a multiple of
//                             `row_pad` (1 for fp32, 8 for bf16); ld = width rounded up to 32
//   theta        [Tw, n_theta] fp32, per task once adapted; layer l at offW[l] ([ld_{l-1}, ld_l],
//                             zero padded) and offb[l]
//   bf16 mode    every GEMM operand also lives as bf16, once, in the orientation it is produced in
//                (activations and deltas [rows, ld], weights [ld_{l-1}, ld_l]); the GEMMs read an operand
//                whose contraction index is the slow one through LDS
//   row arithmetic: no row table in HBM; per (task, field) either byte matrices of pair counts or sorted
//                {row, slot} lists (see pairhop_kernels.hip / twohop_kernels.hip)
#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "../../include/gmeta.h"
#include "gm_internal.h"

struct Arena {
    char* base = nullptr;
    size_t cap = 0, off = 0;
    bool overflow = false;
    template <typename T>
    T* get(size_t n) {
        const size_t bytes = (n * sizeof(T) + 255) / 256 * 256;
        if (off + bytes > cap) {
            overflow = true;
            off += bytes;
            return nullptr;
        }
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += bytes;
        return p;
    }
};

struct ProfEntry {
    int64_t launches = 0;
    double ms = 0, bytes = 0, flops = 0;
};
struct ProfPending {
    std::string name;
    hipEvent_t e0, e1;
    double bytes, flops;
};

struct gm_ctx {
    int F = 0, D = 0, n_dense = 0, L = 0, mlp_dtype = 0;
    std::vector<int64_t> rows, field_base;
    std::vector<int> dims, ld;
    std::vector<int64_t> offW, offb;    // fp32 theta layout
    std::vector<int64_t> offWb;         // bf16 theta layout: W_l as stored ([d_in, d_out]), l = 1..L-1
    int64_t n_theta = 0, n_theta_b = 0;
    int FD = 0, row_pad = 1;
    int device = 0;
    hipStream_t stream = nullptr;
    char* ws = nullptr;
    size_t ws_bytes = 0;
    size_t persistent = 0;
    int64_t* d_field_base = nullptr;
    u32* d_status = nullptr;
    u32* d_status_side = nullptr;   // status words of the work on the side stream
    // The ordering of the lookups by row depends on the indices only: it runs on a stream of its own beside the dense
    // computation (same priority) and is joined before the segment reduction.
    hipStream_t side = nullptr;
    hipEvent_t ev_side = nullptr, ev_main = nullptr, ev_go = nullptr;
    // The pair-count matrices depend on the indices only and are first read by the first row hop: counting them on the
    // side stream lets the prefetch and the first forward / backward pass (bound by memory traffic) run beside a kernel
    // that is bound by latency and instruction issue.
    hipEvent_t ev_pairs_go = nullptr, ev_pairs = nullptr;
    int overlap_pairs = 0;
    int overlap_sort = 0;   // measured: 1-1.5 % (both streams contend for the same memory system), so off unless asked for
    std::string err;
    int pair_tile_rows = 0;
    int adapt_rows = 1;   // 0: the inner loop adapts the dense parameters only (embedding rows are read, not updated)
    int gemm_tile_n = 0;
    int wgrad_wide = 1;      // weight gradients over runs of tasks in 256 x 256 tiles where the shape allows
    int theta_from_meta = 1; // bf16, second order, several inner steps: a step's weights from theta and all steps' gradients
    int coarse_groups = 0;   // runs of tasks for the products only summed over tasks (0: chosen by shape)
    int n_cus = 256;
    int row_path = 0;   // task-local row arithmetic: 0 = choose per wave, 1 = sparse two-hop kernel, 2 = pair-count matrices
    int sort_fields = 1; // with index_path's row order: 1 = the keys are laid out field after field and every field's range sorted by row alone (fewer radix passes), 0 = one sort on (field, row)
    int index_path = 0; // per-(task, field) dictionaries: 0 = choose per wave, 1 = sorted per (task, field) in LDS, 2 = read off the wave's (task, field, row) order
    int max_wave_tasks = 0;   // 0: as many tasks per wave as the workspace holds
    char* static_scratch = nullptr;   // this device's copy of the static scratch array (gm_meta_step_static)
    // optional kernel timing
    bool prof_on = false;
    std::vector<ProfPending> prof_pending;
    std::vector<hipEvent_t> prof_free;
    std::map<std::string, ProfEntry> prof;
    std::string prof_text;
};

// Scratch of gm_meta_step_static: one array per GPU, part of the loaded code object (held until the process ends).
// Host code never passes the array's name to a kernel: the device address is looked up once per device at gm_create
// (hipGetSymbolAddress) and only that pointer is used.
#define GM_STATIC_SCRATCH_BYTES ((size_t)GM_STATIC_SCRATCH_MIB << 20)
static __device__ __align__(256) unsigned char scratch[GM_STATIC_SCRATCH_BYTES];
enum { GM_MAX_DEVICES = 64 };
static char* g_scratch_ptr[GM_MAX_DEVICES];   // device address of `scratch` on each GPU (null: not looked up yet)

static int fail(gm_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIPCHK(c, call)                                                                            \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(c, GM_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

// Brackets the launches issued during its lifetime with two events on the context's stream.
struct Prof {
    gm_ctx* c;
    ProfPending p;
    bool on;
    hipStream_t st;
    Prof(gm_ctx* c_, const char* name, double bytes, double flops, hipStream_t st_ = nullptr, bool use_st = false)
        : c(c_), on(c_->prof_on), st(use_st ? st_ : c_->stream) {
        if (!on) return;
        p.name = name;
        p.bytes = bytes;
        p.flops = flops;
        for (hipEvent_t* e : {&p.e0, &p.e1}) {
            if (!c->prof_free.empty()) {
                *e = c->prof_free.back();
                c->prof_free.pop_back();
            } else if (hipEventCreate(e) != hipSuccess) {
                on = false;
                return;
            }
        }
        (void)hipEventRecord(p.e0, st);
    }
    ~Prof() {
        if (!on) return;
        (void)hipEventRecord(p.e1, st);
        c->prof_pending.push_back(p);
    }
};

static void prof_drain(gm_ctx* c) {  // after the stream has been synchronised
    for (ProfPending& p : c->prof_pending) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.e0, p.e1) == hipSuccess) {
            ProfEntry& e = c->prof[p.name];
            e.launches += 1;
            e.ms += ms;
            e.bytes += p.bytes;
            e.flops += p.flops;
        }
        c->prof_free.push_back(p.e0);
        c->prof_free.push_back(p.e1);
    }
    c->prof_pending.clear();
}

static void zero_bf16(hipStream_t st, bf16_t* p, int64_t n) { launch_fill_u32(st, reinterpret_cast<u32*>(p), (n + 1) / 2, 0u); }

static int round_up(int x, int m) { return (x + m - 1) / m * m; }
static int64_t round_up64(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

static int model_layout(gm_ctx* c, const gm_model_desc* m) {
    if (!m || m->n_fields < 0 || m->n_layers < 1 || !m->layer_dims || (m->n_fields > 0 && !m->rows_per_field))
        return fail(c, GM_ERR_ARG, "bad model description");
    const int D = m->emb_dim;
    if (D < 4 || D > 256 || (D & (D - 1))) return fail(c, GM_ERR_ARG, "emb_dim must be a power of two in 4..256");
    if (m->mlp_dtype != 0 && m->mlp_dtype != 1) return fail(c, GM_ERR_ARG, "mlp_dtype must be 0 or 1");
    c->F = m->n_fields;
    c->D = D;
    c->n_dense = m->n_dense;
    c->L = m->n_layers;
    c->mlp_dtype = m->mlp_dtype;
    c->row_pad = m->mlp_dtype ? 8 : 1;
    c->FD = c->F * D;
    c->rows.assign(m->rows_per_field, m->rows_per_field + c->F);
    c->field_base.assign(c->F + 1, 0);
    for (int f = 0; f < c->F; ++f) {
        if (c->rows[f] <= 0) return fail(c, GM_ERR_ARG, "rows_per_field must be positive");
        c->field_base[f + 1] = c->field_base[f] + c->rows[f];
    }
    if (c->field_base[c->F] >= (int64_t)1 << 32) return fail(c, GM_ERR_ARG, "more than 2^32 rows in total");
    c->dims.assign(m->layer_dims, m->layer_dims + c->L + 1);
    if (c->n_dense < 0 || c->dims[0] != c->FD + c->n_dense || c->dims[c->L] != 1)
        return fail(c, GM_ERR_ARG, "layer_dims must start at F*D+n_dense and end at 1");
    c->ld.resize(c->L + 1);
    for (int l = 0; l <= c->L; ++l) {
        if (c->dims[l] <= 0) return fail(c, GM_ERR_ARG, "layer_dims must be positive");
        c->ld[l] = l == c->L ? 1 : round_up(c->dims[l], 32);
    }
    c->offW.assign(c->L + 1, 0);
    c->offb.assign(c->L + 1, 0);
    c->offWb.assign(c->L + 1, 0);
    int64_t o = 0, ob = 0;
    for (int l = 1; l <= c->L; ++l) {
        c->offW[l] = o;
        o += round_up64((int64_t)c->ld[l - 1] * c->ld[l], 32);
        c->offb[l] = o;
        o += round_up(c->ld[l], 32);
        if (l < c->L) {
            c->offWb[l] = ob;
            ob += (int64_t)c->ld[l - 1] * c->ld[l];
        }
    }
    c->n_theta = o;
    c->n_theta_b = std::max<int64_t>(ob, 32);
    return GM_OK;
}

// ------------------------------------------------------------------------------------------------
// handles
// ------------------------------------------------------------------------------------------------
struct Act {  // one activation-shaped buffer [rows, ld] in the type(s) the GEMMs read
    float* f = nullptr;    // fp32 mode
    bf16_t* b = nullptr;   // bf16 mode: [rows, ld]
    int ld = 0;
};
struct Theta {  // parameters as the GEMMs read them; stride 0 = shared by all tasks
    float* f = nullptr;
    int64_t sf = 0;
    bf16_t* b = nullptr;
    int64_t sb = 0;
};

struct StepState {  // what one inner step leaves behind for the second-order pass
    Act X;
    std::vector<Act> A, Dl;  // [1..L-1]
    float *dL = nullptr, *zL = nullptr;
    Theta th;                // parameters the step was taken at (GEMM operands)
    const float* wL = nullptr;  // last-layer weights of the step, fp32
    int64_t wL_stride = 0;
    float* wL_copy = nullptr;   // bf16 mode: copy of the last-layer weights (the master is updated in place)
};

// buffers of one sort + segment reduction of (row key, gradient-buffer slot) pairs
struct SortBufs {
    u32 *keys = nullptr, *vals = nullptr, *keys_tmp = nullptr, *vals_tmp = nullptr, *hist = nullptr, *scan_tmp = nullptr,
        *seg_start = nullptr;
    float* seg_partial = nullptr;
};

enum { COARSE_GROUPS = 32 };   // most runs of tasks (gm_configure "coarse_groups" says how many are used)

struct WaveBufs {
    int32_t *row_off_s, *row_off_q, *real_off_s, *real_off_q;
    int32_t *sample_task_s, *sample_task_q, *row_task_s, *row_task_q;
    int32_t *tile_g_s, *tile_m_s, *tile_g_q, *tile_m_q;
    u32 *cnt_s, *base_s, *cnt_q, *base_q, *n_slots, *scan_tmp;
    u32* slot_rows;
    int32_t *slot_start, *sup_slot, *qry_slot, *qseg_lo, *qseg_hi;
    int2 *sup_sorted, *qry_sorted;
    u32 *fm_off_s = nullptr, *fm_off_q = nullptr, *field_tab = nullptr;   // keys laid out field after field: places and ranges
    u32 *tmid_keys = nullptr, *tmid_vals = nullptr;   // more than 512 tasks: the first of the two passes that order the lookups by task
    bool slots_written = true;   // sup_slot / qry_slot hold the slot of every lookup (only the sparse row kernel reads them)
    float *Xs0, *Xq0, *TXf, *dX, *loss_q;
    Theta v;  // direction / query gradient w.r.t. theta'
    // the last weight-gradient products of a call are only ever summed over the tasks: they are taken over COARSE_GROUPS
    // runs of consecutive tasks instead (row offsets of the runs, one sum per run)
    int32_t *coarse_off_s, *coarse_off_q;
    Theta vsum;
    Act Xs_scratch;
    std::vector<StepState> steps;
    std::vector<Theta> thetas;
    Act Xq;
    std::vector<Act> Aq, Dq;
    float *dLq, *zq;
    Act TX;
    std::vector<Act> TA, TD;
    float* tdL;
    // pair-count matrices of the wave (null when the sparse kernel does the row arithmetic)
    uint8_t* pair_mat;
    int64_t *pair_off_ss, *pair_off_qs, *pair_off_sq;
    u32* task_path;   // [Tw] 1: pair-count path, 0: sparse kernel (the counting kernel clears it on overflow)
    // table-shaped sparse output only: the wave's own gradient buffer (support rows, then query rows) and sort
    float* GX = nullptr;
    int64_t* n_rows = nullptr;
    SortBufs so;
};

struct WaveDims {
    int Tw;
    int64_t Ss, Sq, Ps, Pq, nnz_s, nnz_q;  // real samples, padded rows, lookups
    int mt_s, mt_q;
    bool pair = false;                     // some task of the wave takes the pair-count path (matrices are allocated)
    bool any_sparse = false;               // some task of the wave takes the sparse kernel
    bool pair_ss = false, pair_sq = false; // which kinds besides query x support
    int64_t pair_bytes = 0;
    bool table = false;                    // the sparse gradient is reduced wave by wave into a table-shaped output
};

static Act alloc_act(const gm_ctx* c, Arena& ar, int64_t rows, int ld) {
    Act a;
    a.ld = ld;
    if (c->mlp_dtype == 0) {
        a.f = ar.get<float>(rows * ld);
    } else {
        a.b = ar.get<bf16_t>(rows * ld + 8);
    }
    return a;
}
static Theta alloc_theta(const gm_ctx* c, Arena& ar, int Tw, bool need_f) {
    Theta t;
    if (need_f) {
        t.f = ar.get<float>((int64_t)Tw * c->n_theta);
        t.sf = c->n_theta;
    }
    if (c->mlp_dtype) {
        t.b = ar.get<bf16_t>((int64_t)Tw * c->n_theta_b);
        t.sb = c->n_theta_b;
    }
    return t;
}

static void alloc_sort(const gm_ctx* c, Arena& ar, SortBufs& so, int64_t nnz, int64_t max_segs, size_t extra_hist_words,
                       bool need_gx) {
    so.keys = ar.get<u32>(nnz + 1);
    so.vals = ar.get<u32>(nnz + 1);
    so.keys_tmp = ar.get<u32>(nnz + 1);
    so.vals_tmp = ar.get<u32>(nnz + 1);
    so.hist = ar.get<u32>(radix_hist_words(nnz, c->F) + extra_hist_words);
    so.scan_tmp = ar.get<u32>(scan_tmp_words(nnz));
    so.seg_start = ar.get<u32>(std::min(nnz, max_segs) + 2);
    so.seg_partial = need_gx ? ar.get<float>(seg_reduce_partial_floats(nnz, c->D)) : nullptr;
}

// What depends on the indices only (row dictionaries, overlap join, pair-count matrices, and with the table-shaped
// output the wave's own sort buffers): a batch's can be prepared while another batch computes.
static void alloc_wave_index(const gm_ctx* c, Arena& ar, WaveBufs& w, const WaveDims& d) {
    const int F = c->F;
    const int64_t TF = (int64_t)d.Tw * F;
    w.row_off_s = ar.get<int32_t>(d.Tw + 1);
    w.row_off_q = ar.get<int32_t>(d.Tw + 1);
    w.real_off_s = ar.get<int32_t>(d.Tw + 1);
    w.real_off_q = ar.get<int32_t>(d.Tw + 1);
    w.sample_task_s = ar.get<int32_t>(d.Ss + 1);
    w.sample_task_q = ar.get<int32_t>(d.Sq + 1);
    w.row_task_s = ar.get<int32_t>(d.Ps + 1);
    w.row_task_q = ar.get<int32_t>(d.Pq + 1);
    w.tile_g_s = ar.get<int32_t>(d.mt_s + 1);
    w.tile_m_s = ar.get<int32_t>(d.mt_s + 1);
    w.tile_g_q = ar.get<int32_t>(d.mt_q + 1);
    w.tile_m_q = ar.get<int32_t>(d.mt_q + 1);
    w.cnt_s = ar.get<u32>(TF + 1);
    w.base_s = ar.get<u32>(TF + 1);
    w.cnt_q = ar.get<u32>(TF + 1);
    w.base_q = ar.get<u32>(TF + 1);
    w.n_slots = ar.get<u32>(TF + 1);
    w.scan_tmp = ar.get<u32>(scan_tmp_words(TF + 1));
    w.slot_rows = ar.get<u32>(d.nnz_s + 1);
    w.slot_start = ar.get<int32_t>(d.nnz_s + TF + 1);
    w.sup_sorted = ar.get<int2>(d.nnz_s + 1);
    w.sup_slot = ar.get<int32_t>(d.nnz_s + 1);
    w.qry_slot = ar.get<int32_t>(d.nnz_q + 1);
    w.qry_sorted = ar.get<int2>(d.nnz_q + 1);
    w.qseg_lo = ar.get<int32_t>(d.nnz_s + 1);
    w.qseg_hi = ar.get<int32_t>(d.nnz_s + 1);
    w.fm_off_s = ar.get<u32>(TF + 1);
    w.fm_off_q = ar.get<u32>(TF + 1);
    w.field_tab = ar.get<u32>(field_table_words(F));
    w.tmid_keys = w.tmid_vals = nullptr;
    if (F > 0 && c->adapt_rows && c->index_path != 1 && task_sort_passes(d.Tw) > 1) {
        w.tmid_keys = ar.get<u32>(d.nnz_s + d.nnz_q + 1);
        w.tmid_vals = ar.get<u32>(d.nnz_s + d.nnz_q + 1);
    }
    w.coarse_off_s = ar.get<int32_t>(COARSE_GROUPS + 1);
    w.coarse_off_q = ar.get<int32_t>(COARSE_GROUPS + 1);
    w.pair_mat = nullptr;
    w.pair_off_ss = w.pair_off_qs = w.pair_off_sq = nullptr;
    w.task_path = ar.get<u32>(d.Tw + 1);
    if (d.pair) {
        w.pair_off_ss = ar.get<int64_t>(d.Tw + 1);
        w.pair_off_qs = ar.get<int64_t>(d.Tw + 1);
        w.pair_off_sq = ar.get<int64_t>(d.Tw + 1);
        w.pair_mat = ar.get<uint8_t>(d.pair_bytes + 64);
    }
}

// activations, per-task parameters and gradient buffers of a wave
static void alloc_wave_dense(const gm_ctx* c, Arena& ar, WaveBufs& w, const WaveDims& d, int K, int order) {
    const int L = c->L;
    const bool bf = c->mlp_dtype != 0;
    const int ld0 = c->ld[0];
    w.Xs0 = ar.get<float>(d.Ps * ld0);
    w.Xq0 = ar.get<float>(d.Pq * ld0);
    const bool second = order == 2 && K > 0;
    w.TXf = (second && bf) ? ar.get<float>(d.Ps * ld0) : nullptr;
    w.dX = ar.get<float>(std::max(d.Ps, d.Pq) * (int64_t)std::max(c->FD, 1) + 4);
    w.loss_q = ar.get<float>(d.Pq + 1);
    w.v = alloc_theta(c, ar, d.Tw, true);
    w.vsum = Theta{ar.get<float>((int64_t)std::max(16, c->coarse_groups) * c->n_theta), c->n_theta, nullptr, 0};
    if (!second) w.v.b = nullptr;  // the direction is a GEMM operand only in the second-order pass
    w.Xs_scratch = Act();
    if (K > 1 && !second) {
        w.Xs_scratch = alloc_act(c, ar, d.Ps, ld0);
    }
    const int kept = second ? K : (K > 0 ? 1 : 0);
    w.steps.assign(kept, StepState());
    for (int k = 0; k < kept; ++k) {
        StepState& s = w.steps[k];
        // fp32: step 0 reads Xs0 itself; later steps (second order) keep their own input
        if (bf) s.X = alloc_act(c, ar, d.Ps, ld0);
        else if (k > 0) s.X = alloc_act(c, ar, d.Ps, ld0);
        s.X.ld = ld0;
        s.A.assign(L, Act());
        s.Dl.assign(L, Act());
        for (int l = 1; l < L; ++l) {
            s.A[l] = alloc_act(c, ar, d.Ps, c->ld[l]);
            s.Dl[l] = alloc_act(c, ar, d.Ps, c->ld[l]);
        }
        s.dL = ar.get<float>(d.Ps + 1);
        s.zL = ar.get<float>(d.Ps + 1);
        s.wL_copy = (bf && second && k > 0) ? ar.get<float>((int64_t)d.Tw * c->ld[L - 1]) : nullptr;
    }
    // theta^(k+1), k = 0..K-1.  fp32: one buffer per kept step (the second-order pass needs them all), or one
    // updated in place.  bf16: ONE fp32 master updated in place, and bf16 operand copies per kept step.
    const int n_bufs = second ? K : (K > 0 ? 1 : 0);
    w.thetas.assign(n_bufs, Theta());
    for (int k = 0; k < n_bufs; ++k) {
        if (bf) {
            w.thetas[k] = alloc_theta(c, ar, d.Tw, k == 0);
            if (k > 0) { w.thetas[k].f = w.thetas[0].f; w.thetas[k].sf = w.thetas[0].sf; }
        } else {
            w.thetas[k] = alloc_theta(c, ar, d.Tw, true);
        }
    }
    w.Xq = alloc_act(c, ar, d.Pq, ld0);
    w.Aq.assign(L, Act());
    w.Dq.assign(L, Act());
    for (int l = 1; l < L; ++l) {
        w.Aq[l] = alloc_act(c, ar, d.Pq, c->ld[l]);
        w.Dq[l] = alloc_act(c, ar, d.Pq, c->ld[l]);
    }
    w.dLq = ar.get<float>(d.Pq + 1);
    w.zq = ar.get<float>(d.Pq + 1);
    w.TX = Act();
    w.TA.assign(L, Act());
    w.TD.assign(L, Act());
    w.tdL = nullptr;
    if (second) {
        w.TX = alloc_act(c, ar, d.Ps, ld0);
        for (int l = 1; l < L; ++l) {
            w.TA[l] = alloc_act(c, ar, d.Ps, c->ld[l]);
            w.TD[l] = alloc_act(c, ar, d.Ps, c->ld[l]);
        }
        w.tdL = ar.get<float>(d.Ps + 1);
    }
    if (d.table) {
        w.GX = ar.get<float>((d.Ps + d.Pq) * (int64_t)std::max(c->FD, 1) + 4);
        w.n_rows = ar.get<int64_t>(2);
        alloc_sort(c, ar, w.so, d.nnz_s + d.nnz_q, c->field_base[c->F], 0, true);
    }
}

static void alloc_wave(const gm_ctx* c, Arena& ar, WaveBufs& w, const WaveDims& d, int K, int order) {
    alloc_wave_index(c, ar, w, d);
    alloc_wave_dense(c, ar, w, d, K, order);
}

struct BatchBufs {
    int64_t *toff_s, *toff_q;
    int32_t *prow_s, *prow_q, *prow_off_s, *prow_off_q;
    float *GX, *g_theta, *task_loss;
    Theta theta0;
    SortBufs so;
};

// per batch, from the indices only: device copies of the task offsets, the row of every sample in the activation
// buffers, and the buffers of the batch-wide sort
static void alloc_batch_index(const gm_ctx* c, Arena& ar, BatchBufs& b, int T, int64_t Ss, int64_t Sq, int64_t nnz,
                              int64_t capacity, bool need_gx) {
    b.toff_s = ar.get<int64_t>(T + 1);
    b.toff_q = ar.get<int64_t>(T + 1);
    b.prow_off_s = ar.get<int32_t>(T + 1);
    b.prow_off_q = ar.get<int32_t>(T + 1);
    b.prow_s = ar.get<int32_t>(Ss + 1);
    b.prow_q = ar.get<int32_t>(Sq + 1);
    // the histogram area doubles as the scratch of the per-task lookup offsets (2 (T+1) 64-bit words) before any sort
    alloc_sort(c, ar, b.so, nnz, capacity, 2 * (size_t)(T + 1) * 2, need_gx);
}
static void alloc_batch_dense(const gm_ctx* c, Arena& ar, BatchBufs& b, int T, int64_t Ps, int64_t Pq, bool need_gx) {
    b.GX = need_gx ? ar.get<float>((Ps + Pq) * (int64_t)std::max(c->FD, 1) + 4) : nullptr;
    b.theta0 = Theta();
    b.theta0.f = ar.get<float>(c->n_theta);
    if (c->mlp_dtype) b.theta0.b = ar.get<bf16_t>(c->n_theta_b);
    b.g_theta = ar.get<float>(c->n_theta);
    b.task_loss = ar.get<float>(T + 1);
}
static void alloc_batch(const gm_ctx* c, Arena& ar, BatchBufs& b, int T, int64_t Ss, int64_t Sq, int64_t Ps, int64_t Pq,
                        int64_t nnz, int64_t capacity, bool need_gx) {
    alloc_batch_index(c, ar, b, T, Ss, Sq, nnz, capacity, need_gx);
    alloc_batch_dense(c, ar, b, T, Ps, Pq, need_gx);
}

// ------------------------------------------------------------------------------------------------
// ABI: create / destroy / sizes / timing
// ------------------------------------------------------------------------------------------------
extern "C" int gm_create(gm_ctx** out, const gm_model_desc* model, int device, void* hip_stream,
                         size_t workspace_bytes) {
    if (!out) return GM_ERR_ARG;
    gm_ctx* c = new gm_ctx();
    *out = c;  // kept on failure too, so that the message can be read; gm_destroy frees it
    int rc = model_layout(c, model);
    if (rc != GM_OK) return rc;
    c->device = device;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    HIPCHK(c, hipSetDevice(device));
    {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && n > 0) c->n_cus = n;
    }
    if (device < 0 || device >= GM_MAX_DEVICES) return fail(c, GM_ERR_ARG, "device must be in [0, %d)", (int)GM_MAX_DEVICES);
    if (!g_scratch_ptr[device]) {   // once per device, with that device current: every GPU holds its own copy
        void* p = nullptr;
        HIPCHK(c, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        g_scratch_ptr[device] = static_cast<char*>(p);
    }
    c->static_scratch = g_scratch_ptr[device];
    c->ws_bytes = std::max<size_t>(workspace_bytes, 1 << 20);
    HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->ws), c->ws_bytes));
    Arena ar;
    ar.base = c->ws;
    ar.cap = c->ws_bytes;
    c->d_field_base = ar.get<int64_t>(c->F + 1);
    c->d_status = ar.get<u32>(ST_WORDS);
    c->d_status_side = ar.get<u32>(ST_WORDS);
    HIPCHK(c, hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
    HIPCHK(c, hipEventCreateWithFlags(&c->ev_side, hipEventDisableTiming));
    HIPCHK(c, hipEventCreateWithFlags(&c->ev_main, hipEventDisableTiming));
    HIPCHK(c, hipEventCreateWithFlags(&c->ev_go, hipEventDisableTiming));
    HIPCHK(c, hipEventCreateWithFlags(&c->ev_pairs_go, hipEventDisableTiming));
    HIPCHK(c, hipEventCreateWithFlags(&c->ev_pairs, hipEventDisableTiming));
    c->persistent = ar.off;
    HIPCHK(c, hipMemcpy(c->d_field_base, c->field_base.data(), (c->F + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    return GM_OK;
}

extern "C" void gm_destroy(gm_ctx* c) {
    if (!c) return;
    if (c->ws) {
        (void)hipSetDevice(c->device);
        for (ProfPending& p : c->prof_pending) {
            (void)hipEventDestroy(p.e0);
            (void)hipEventDestroy(p.e1);
        }
        for (hipEvent_t e : c->prof_free) (void)hipEventDestroy(e);
        if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
        if (c->ev_side) (void)hipEventDestroy(c->ev_side);
        if (c->ev_main) (void)hipEventDestroy(c->ev_main);
        if (c->ev_go) (void)hipEventDestroy(c->ev_go);
        if (c->ev_pairs_go) (void)hipEventDestroy(c->ev_pairs_go);
        if (c->ev_pairs) (void)hipEventDestroy(c->ev_pairs);
        (void)hipFree(c->ws);
    }
    delete c;
}

extern "C" const char* gm_last_error(const gm_ctx* c) { return c ? c->err.c_str() : "null context"; }

extern "C" int gm_configure(gm_ctx* c, const char* key, int64_t value) {
    if (!c) return GM_ERR_ARG;
    if (!key) return fail(c, GM_ERR_ARG, "null key");
    if (!strcmp(key, "pair_tile_rows")) {   // most out-rows of a pair-count matrix counted at a time (0: as many as fit)
        if (value < 0 || value > 1024) return fail(c, GM_ERR_ARG, "pair_tile_rows must be in [0, 1024]");
        c->pair_tile_rows = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "gemm_tile_n")) {   // column tile of the forward / backward products with 256-row tiles (0: chosen by shape)
        if (value != 0 && value != 128 && value != 256) return fail(c, GM_ERR_ARG, "gemm_tile_n must be 0, 128 or 256");
        c->gemm_tile_n = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "wgrad_wide")) {
        if (value != 0 && value != 1) return fail(c, GM_ERR_ARG, "wgrad_wide must be 0 or 1");
        c->wgrad_wide = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "theta_from_meta")) {
        if (value != 0 && value != 1) return fail(c, GM_ERR_ARG, "theta_from_meta must be 0 or 1");
        c->theta_from_meta = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "coarse_groups")) {
        if (value < 0 || value > COARSE_GROUPS) return fail(c, GM_ERR_ARG, "coarse_groups must be in [0, 32]");
        c->coarse_groups = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "adapt_rows")) {
        if (value != 0 && value != 1) return fail(c, GM_ERR_ARG, "adapt_rows must be 0 or 1");
        c->adapt_rows = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "overlap_pairs")) {   // (ignored while overlap_sort is on: one side stream, one set of status words)
        if (value != 0 && value != 1) return fail(c, GM_ERR_ARG, "overlap_pairs must be 0 or 1");
        c->overlap_pairs = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "overlap_sort")) {
        if (value != 0 && value != 1) return fail(c, GM_ERR_ARG, "overlap_sort must be 0 or 1");
        c->overlap_sort = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "max_wave_tasks")) {
        if (value < 0 || value > 32768) return fail(c, GM_ERR_ARG, "max_wave_tasks must be in [0, 32768]");
        c->max_wave_tasks = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "row_path")) {
        if (value < 0 || value > 2) return fail(c, GM_ERR_ARG, "row_path must be 0, 1 or 2");
        c->row_path = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "sort_fields")) {
        if (value != 0 && value != 1) return fail(c, GM_ERR_ARG, "sort_fields must be 0 or 1");
        c->sort_fields = (int)value;
        return GM_OK;
    }
    if (!strcmp(key, "index_path")) {
        if (value < 0 || value > 2) return fail(c, GM_ERR_ARG, "index_path must be 0, 1 or 2");
        c->index_path = (int)value;
        return GM_OK;
    }
    return fail(c, GM_ERR_ARG, "unknown key '%s'", key);
}

extern "C" int gm_profile(gm_ctx* c, int enable) {
    if (!c) return GM_ERR_ARG;
    c->prof_on = enable != 0;
    if (enable) c->prof.clear();
    return GM_OK;
}

extern "C" const char* gm_profile_report(gm_ctx* c) {
    if (!c) return "";
    c->prof_text.clear();
    char line[256];
    for (auto& kv : c->prof) {
        snprintf(line, sizeof line, "%s %lld %.6f %.6e %.6e\n", kv.first.c_str(), (long long)kv.second.launches,
                 kv.second.ms, kv.second.bytes, kv.second.flops);
        c->prof_text += line;
    }
    return c->prof_text.c_str();
}

// Streaming and matrix-core ceilings of this GPU, measured with kernels of the library's own on the context's
// workspace (whose contents are scratch between calls anyway).
extern "C" int gm_ceilings(gm_ctx* c, double* copy_gbs, double* read_gbs, double* mfma_tflops, double* mfma_random_tflops,
                           int64_t* buffer_bytes) {
    if (!c) return GM_ERR_ARG;
    if (!copy_gbs || !read_gbs || !mfma_tflops || !mfma_random_tflops) return fail(c, GM_ERR_ARG, "null outputs");
    HIPCHK(c, hipSetDevice(c->device));
    hipStream_t st = c->stream;
    const size_t avail = (c->ws_bytes - c->persistent) / 2 / 4096 * 4096;
    const int64_t bytes = (int64_t)std::min<size_t>(avail, (size_t)2 << 30);
    if (bytes < (64 << 20)) return fail(c, GM_ERR_WORKSPACE, "gm_ceilings needs a workspace of at least 130 MiB");
    char* a = c->ws + (c->persistent + 4095) / 4096 * 4096;
    char* b = a + bytes;
    if (buffer_bytes) *buffer_bytes = bytes;
    hipEvent_t e0, e1;
    HIPCHK(c, hipEventCreate(&e0));
    HIPCHK(c, hipEventCreate(&e1));
    auto timed = [&](auto&& launch, int reps, float* best) -> int {
        *best = 1e30f;
        for (int r = 0; r < reps + 1; ++r) {   // the first repetition warms up
            HIPCHK(c, hipEventRecord(e0, st));
            launch();
            HIPCHK(c, hipEventRecord(e1, st));
            HIPCHK(c, hipEventSynchronize(e1));
            float ms = 0.f;
            HIPCHK(c, hipEventElapsedTime(&ms, e0, e1));
            if (r > 0) *best = std::min(*best, ms);
        }
        return GM_OK;
    };
    launch_fill_u32(st, reinterpret_cast<u32*>(a), bytes / 4, 0x3f800000u);
    float ms = 0.f;
    int rc = timed([&] { launch_stream_copy(st, a, b, bytes); }, 5, &ms);
    if (rc == GM_OK) {
        *copy_gbs = 2.0 * bytes / (ms * 1e-3) / 1e9;
        rc = timed([&] { launch_stream_read(st, a, bytes, reinterpret_cast<u32*>(b)); }, 5, &ms);
    }
    if (rc == GM_OK) {
        *read_gbs = (double)bytes / (ms * 1e-3) / 1e9;
        double flops = 0.0;
        rc = timed([&] { flops = launch_mfma_loop(st, 20000, reinterpret_cast<float*>(b)); }, 3, &ms);
        if (rc == GM_OK) {
            *mfma_tflops = flops / (ms * 1e-3) / 1e12;
            rc = timed([&] { flops = launch_mfma_loop_random(st, 40000, reinterpret_cast<float*>(b)); }, 3, &ms);
            if (rc == GM_OK) *mfma_random_tflops = flops / (ms * 1e-3) / 1e12;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != GM_OK) return rc;
    HIPCHK(c, hipStreamSynchronize(st));
    HIPCHK(c, hipGetLastError());
    return GM_OK;
}

static int64_t padded_upper(const gm_ctx* c, int64_t n, int T) { return n + (int64_t)T * (c->row_pad - 1); }

extern "C" size_t gm_workspace_bytes(const gm_model_desc* model, int32_t n_tasks, int64_t n_support, int64_t n_query,
                                     int64_t nnz_support, int64_t nnz_query, int32_t inner_steps, int32_t order) {
    gm_ctx c;
    if (model_layout(&c, model) != GM_OK || n_tasks < 0) return 0;
    Arena ar;
    ar.cap = ~(size_t)0 >> 1;
    ar.get<int64_t>(c.F + 1);
    ar.get<u32>(ST_WORDS);
    BatchBufs b;
    const int64_t total_rows = c.field_base[c.F];
    const int64_t Ps = padded_upper(&c, n_support, n_tasks), Pq = padded_upper(&c, n_query, n_tasks);
    alloc_batch(&c, ar, b, n_tasks, n_support, n_query, Ps, Pq, nnz_support + nnz_query,
                std::min(total_rows, nnz_support + nnz_query), true);
    WaveBufs w;
    WaveDims d;
    d.Tw = n_tasks;
    d.Ss = n_support; d.Sq = n_query; d.Ps = Ps; d.Pq = Pq;
    d.nnz_s = nnz_support; d.nnz_q = nnz_query;
    d.mt_s = (int)(Ps / 64 + n_tasks + 1);  // upper bound on m-tiles
    d.mt_q = (int)(Pq / 64 + n_tasks + 1);
    // pair-count matrices, for tasks of equal size (a batch of uneven tasks may need more and then runs in waves)
    if (n_tasks > 0 && inner_steps > 0 && c.F > 0 && c.D % 32 == 0) {
        const int64_t ns = (n_support + n_tasks - 1) / n_tasks, nq = (n_query + n_tasks - 1) / n_tasks;
        if (std::max(ns, nq) > 0 && std::max(ns, nq) <= 512) {
            const int64_t ps = (ns + 63) & ~(int64_t)63, pq = (nq + 63) & ~(int64_t)63;
            d.pair = true;
            d.pair_ss = inner_steps >= 2;
            d.pair_sq = order == 2;
            d.pair_bytes = (int64_t)n_tasks * c.F * ((d.pair_ss ? ps * ps : 0) + pq * ps * (d.pair_sq ? 2 : 1));
        }
    }
    alloc_wave(&c, ar, w, d, inner_steps, order);
    return ar.off + (1 << 20);
}

// ------------------------------------------------------------------------------------------------
// argument checks shared by the entry points
// ------------------------------------------------------------------------------------------------
static int check_set(gm_ctx* c, const gm_set* s, int T, const char* name, bool any_nnz = false) {
    if (!s || !s->task_offsets) return fail(c, GM_ERR_ARG, "%s: null set or task_offsets", name);
    if (s->n_samples < 0 || s->nnz < 0) return fail(c, GM_ERR_ARG, "%s: negative size", name);
    if (s->task_offsets[0] != 0 || s->task_offsets[T] != s->n_samples)
        return fail(c, GM_ERR_ARG, "%s: task_offsets must start at 0 and end at n_samples", name);
    for (int t = 0; t < T; ++t)
        if (s->task_offsets[t + 1] < s->task_offsets[t]) return fail(c, GM_ERR_ARG, "%s: task_offsets not monotone", name);
    if (s->n_samples > 0 && (!s->bag_offsets || !s->labels || (c->n_dense > 0 && !s->dense)))
        return fail(c, GM_ERR_ARG, "%s: null array", name);
    if (s->nnz > 0 && !s->indices) return fail(c, GM_ERR_ARG, "%s: null indices", name);
    if (s->n_samples == 0 && s->nnz != 0) return fail(c, GM_ERR_ARG, "%s: nnz without samples", name);
    // any_nnz: the call orders lookups wave by wave, so only a wave's lookups must number below 2^31
    if ((s->n_samples + (int64_t)T * 8) * (int64_t)std::max(c->F, 1) >= ((int64_t)1 << 31) ||
        (!any_nnz && s->nnz >= ((int64_t)1 << 31)))
        return fail(c, GM_ERR_ARG, "%s: more than 2^31 bags or lookups in one call", name);
    return GM_OK;
}

static SetView make_view(const gm_set* s, const int64_t* d_toff, int64_t sample0, int64_t lookup0) {
    SetView v;
    v.bag_offsets = s->bag_offsets;
    v.indices = s->indices;
    v.task_offsets = d_toff;
    v.sample0 = sample0;
    v.lookup0 = lookup0;
    v.n_samples = s->n_samples;
    return v;
}

static int read_status(gm_ctx* c, u32* host) {
    HIPCHK(c, hipMemcpyAsync(host, c->d_status, ST_WORDS * sizeof(u32), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return GM_OK;
}

// ------------------------------------------------------------------------------------------------
// dense operators on handles (fp32: vector-FMA GEMM; bf16: MFMA GEMM)
// ------------------------------------------------------------------------------------------------
struct Grp {  // grouping of one set's rows by task inside the wave
    const int32_t *row_off, *real_off, *row_task;
    const int32_t *tile_g, *tile_m;
    int n_mtiles, G, bm;
    int64_t rows;  // padded rows of the set in the wave
};


// column tile of a forward / backward product.  256 selects the pipelined 256 x 256 kernel (256-row tiles, a multiple of
// 256 columns): it wins where the contraction is long enough to pay for its unhidden prologue and epilogue (one
// workgroup per compute unit), measured from about 2,048 on; results are identical either way.
static int gemm_bn(const gm_ctx* c, int bm, int N, int K) {
    if (bm != 256 || N < 256 || N % 256 != 0) return 128;
    if (c->gemm_tile_n) return c->gemm_tile_n;
    return K >= 1024 ? 256 : 128;
}

// out[rows, ld_l] = epi( sum_p in_p[rows, ld_{l-1}] * W_p,l + bias )
static void dense_nn(gm_ctx* c, const Grp& g, int l, int np, const Act* in0, const Theta* th0, const Act* in1,
                     const Theta* th1, const float* bias, int64_t bias_stride, const Act* mask, int epi, Act& out) {
    const int K = c->ld[l - 1], N = c->ld[l];
    // algorithmic bytes: operands once (per-task weights once per task), every output once
    const double esz = c->mlp_dtype ? 2.0 : 4.0;
    double by = (double)g.rows * N * esz + (mask ? (double)g.rows * N * esz : 0.0);
    for (int i = 0; i < np; ++i) {
        const Theta* t = i ? th1 : th0;
        by += (double)g.rows * K * esz + (double)((c->mlp_dtype ? t->sb : t->sf) ? g.G : 1) * K * N * esz;
    }
    Prof p(c, "gemm_fwd", by, 2.0 * g.rows * N * K * np);
    const Act* ins[2] = {in0, in1};
    const Theta* ths[2] = {th0, th1};
    if (c->mlp_dtype == 0) {
        GemmArgs a;
        memset(&a, 0, sizeof a);
        a.row_offsets = g.row_off; a.G = g.G; a.n_pairs = np;
        for (int i = 0; i < np; ++i) {
            a.A[i] = ins[i]->f; a.sAm[i] = K; a.sAk[i] = 1; a.rA[i] = K;
            a.B[i] = ths[i]->f + c->offW[l]; a.sBk[i] = N; a.sBn[i] = 1; a.gB[i] = ths[i]->sf;
        }
        a.C = out.f; a.ldc = N; a.rC = N; a.M = -1; a.N = N; a.K = K;
        a.tile_group = g.tile_g; a.tile_m0 = g.tile_m; a.n_mtiles = g.n_mtiles;
        a.epi = epi; a.bias = bias; a.gBias = bias_stride;
        if (mask) { a.mask = mask->f; a.ld_mask = mask->ld; }
        launch_gemm_f32(c->stream, a);
    } else {
        GemmBArgs a;
        memset(&a, 0, sizeof a);
        a.row_offsets = g.row_off; a.G = g.G; a.n_pairs = np;
        for (int i = 0; i < np; ++i) {   // W as stored, [d_in, d_out]: the contraction index is its slow one
            a.A[i] = ins[i]->b; a.lda[i] = K; a.rA[i] = K;
            a.B[i] = ths[i]->b + c->offWb[l]; a.ldb[i] = N; a.gB[i] = ths[i]->sb;
        }
        a.Cb = out.b; a.ldcb = N; a.rCb = N; a.M = -1; a.N = N; a.K = K;
        a.tile_group = g.tile_g; a.tile_m0 = g.tile_m; a.n_mtiles = g.n_mtiles;
        a.epi = epi; a.bias = bias; a.gBias = bias_stride;
        if (mask) { a.mask = mask->b; a.ld_mask = mask->ld; }
        launch_gemm_bf16_bkmajor(c->stream, a, g.bm, gemm_bn(c, g.bm, N, K * np));
    }
}

// out[rows, ld_{l-1}] = mask .* sum_p d_p[rows, ld_l] * W_p,l^T ; for l == 1: dX[rows, FD] fp32, no mask
// dX (layer 1 only): the fp32 gradient w.r.t. the pooled input.  bf16 mode can also accumulate it, scaled, into
// gx_acc (gx_acc += gx_scale * dX, or = with gx_init) in the same pass; with write_dx = false only that is stored.
static void dense_nt(gm_ctx* c, const Grp& g, int l, int np, const Act* d0, const Theta* th0, const Act* d1,
                     const Theta* th1, const Act* mask, Act* out, float* dX, float* gx_acc = nullptr, float gx_scale = 0.f,
                     bool write_dx = true, bool gx_init = false) {
    const int K = c->ld[l], N = dX ? c->FD : c->ld[l - 1];
    if (N <= 0) return;
    const double esz = c->mlp_dtype ? 2.0 : 4.0;
    double by = dX ? (double)g.rows * N * 4.0 * ((write_dx ? 1 : 0) + (gx_acc ? (gx_init ? 1 : 2) : 0)) : (double)g.rows * N * esz;
    if (mask) by += (double)g.rows * N * esz;
    for (int i = 0; i < np; ++i) {
        const Theta* t = i ? th1 : th0;
        by += (double)g.rows * K * esz + (double)((c->mlp_dtype ? t->sb : t->sf) ? g.G : 1) * K * N * esz;
    }
    Prof p(c, "gemm_bwd", by, 2.0 * g.rows * N * K * np);
    const Act* ds[2] = {d0, d1};
    const Theta* ths[2] = {th0, th1};
    if (c->mlp_dtype == 0) {
        GemmArgs a;
        memset(&a, 0, sizeof a);
        a.row_offsets = g.row_off; a.G = g.G; a.n_pairs = np;
        for (int i = 0; i < np; ++i) {
            a.A[i] = ds[i]->f; a.sAm[i] = K; a.sAk[i] = 1; a.rA[i] = K;
            a.B[i] = ths[i]->f + c->offW[l]; a.sBk[i] = 1; a.sBn[i] = K; a.gB[i] = ths[i]->sf;
        }
        a.M = -1; a.N = N; a.K = K;
        a.tile_group = g.tile_g; a.tile_m0 = g.tile_m; a.n_mtiles = g.n_mtiles;
        if (dX) { a.C = dX; a.ldc = N; a.rC = N; a.epi = EPI_NONE; }
        else { a.C = out->f; a.ldc = N; a.rC = N; a.epi = EPI_MASK; a.mask = mask->f; a.ld_mask = mask->ld; }
        launch_gemm_f32(c->stream, a);
    } else {
        GemmBArgs a;
        memset(&a, 0, sizeof a);
        a.row_offsets = g.row_off; a.G = g.G; a.n_pairs = np;
        for (int i = 0; i < np; ++i) {
            a.A[i] = ds[i]->b; a.lda[i] = K; a.rA[i] = K;
            a.B[i] = ths[i]->b + c->offWb[l]; a.ldb[i] = K; a.gB[i] = ths[i]->sb;
        }
        a.M = -1; a.N = N; a.K = K;
        a.tile_group = g.tile_g; a.tile_m0 = g.tile_m; a.n_mtiles = g.n_mtiles;
        if (dX) {
            if (write_dx) { a.Cf = dX; a.ldcf = N; a.rCf = N; }
            a.epi = EPI_NONE;
            if (gx_acc) { a.Cacc = gx_acc; a.ldcacc = N; a.rCacc = N; a.cacc = gx_scale; a.cacc_init = gx_init ? 1 : 0; }
        } else {
            a.Cb = out->b; a.ldcb = N; a.rCb = N; a.epi = EPI_MASK; a.mask = mask->b; a.ld_mask = mask->ld;
        }
        launch_gemm_bf16(c->stream, a, g.bm, gemm_bn(c, g.bm, N, K * np));
    }
}

// Weight gradient [M, N] of G groups over `rows` rows in all: the pipelined 256 x 256 tiles pay once the contraction of a
// group is at least 512 rows long (clearly so from thousands of rows on) and the tiles fill the device several times over.
static bool wgrad_wide_ok(const gm_ctx* c, int M, int N, int64_t rows, int G) {
    return c->wgrad_wide && c->mlp_dtype && M >= 1024 && N % 256 == 0 && G > 0 && rows / G >= 512 &&
           (int64_t)((M + 255) / 256) * (N / 256) * G >= 2 * (int64_t)c->n_cus;
}

// Runs of consecutive tasks that the products only summed over tasks are taken over.  16, unless the first layer's
// product then runs in 256 x 256 tiles, one workgroup per compute unit: the count in [12, 16] whose tiles fill the
// last round over the compute units best (the larger count on a tie).
static int coarse_group_count(const gm_ctx* c, int Tw, int64_t rows) {
    if (c->coarse_groups) return std::min(Tw, c->coarse_groups);
    int n = std::min(Tw, 16);
    if (n < 16 || c->L < 1) return n;
    const int M = c->ld[0], N = c->ld[1];
    if (!wgrad_wide_ok(c, M, N, rows, 16) || rows / 16 < 2048) return n;
    const int64_t per = (int64_t)((M + 255) / 256) * (N / 256);
    double best = -1.0;
    for (int k = 12; k <= 16; ++k) {
        const int64_t tiles = per * k, rounds = (tiles + c->n_cus - 1) / c->n_cus;
        const double fill = (double)tiles / (double)(rounds * c->n_cus);
        if (fill >= best) { best = fill; n = k; }
    }
    return n;
}

// out_g[ld_{l-1}, ld_l] = c0*in_g + c1 * sum_p a_p[rows_g, ld_{l-1}]^T d_p[rows_g, ld_l]  (and its bf16 copies)
static void dense_tn_n(gm_ctx* c, const Grp& g, int l, int np, const Act* const* as, const Act* const* ds, Theta& out,
                       const float* in, int64_t in_stride, float c0, float c1, bool write_f32 = true) {
    const int M = c->ld[l - 1], N = c->ld[l];
    {
        const double esz = c->mlp_dtype ? 2.0 : 4.0;
        const double out_b = c->mlp_dtype ? ((write_f32 || !out.b) ? 4.0 : 0.0) + (out.b ? 2.0 : 0.0) : 4.0;
        const double by = (double)np * g.rows * (M + N) * esz + (double)g.G * M * N * (out_b + ((in && in_stride) ? 4.0 : 0.0));
        Prof p(c, "gemm_wgrad", by, 2.0 * g.rows * N * M * np);
        if (c->mlp_dtype == 0) {
            GemmArgs a;
            memset(&a, 0, sizeof a);
            a.row_offsets = g.row_off; a.G = g.G; a.n_pairs = np;
            for (int i = 0; i < np; ++i) {
                a.A[i] = as[i]->f; a.sAm[i] = 1; a.sAk[i] = M; a.rA[i] = M;
                a.B[i] = ds[i]->f; a.sBk[i] = N; a.sBn[i] = 1; a.rB[i] = N;
            }
            a.C = out.f + c->offW[l]; a.ldc = N; a.gC = out.sf; a.M = M; a.N = N; a.K = -1;
            a.epi = EPI_AXPBY; a.Cin = in ? in + c->offW[l] : nullptr; a.gCin = in_stride; a.c0 = c0; a.c1 = c1;
            launch_gemm_f32(c->stream, a);
        } else {
            GemmBArgs a;
            memset(&a, 0, sizeof a);
            a.row_offsets = g.row_off; a.G = g.G; a.n_pairs = np;
            for (int i = 0; i < np; ++i) {   // activations and deltas as they are stored: [rows, width]
                a.A[i] = as[i]->b; a.lda[i] = M; a.rA[i] = M;
                a.B[i] = ds[i]->b; a.ldb[i] = N; a.rB[i] = N;
            }
            if (write_f32 || !out.b) { a.Cf = out.f + c->offW[l]; a.ldcf = N; a.gCf = out.sf; }
            a.M = M; a.N = N; a.K = -1;
            if (out.b) {  // the bf16 operand copy of W
                a.Cb = out.b + c->offWb[l]; a.ldcb = N; a.gCb = out.sb;
            }
            a.epi = EPI_AXPBY; a.Cin = in ? in + c->offW[l] : nullptr; a.gCin = in_stride; a.ldcin = N; a.c0 = c0; a.c1 = c1;
            launch_gemm_bf16_kmajor(c->stream, a, wgrad_wide_ok(c, M, N, g.rows, g.G) ? 256 : 128);
        }
    }
}

static void dense_tn(gm_ctx* c, const Grp& g, int l, int np, const Act* a0, const Act* d0, const Act* a1, const Act* d1,
                     Theta& out, const float* in, int64_t in_stride, float c0, float c1, bool write_f32 = true) {
    const Act* as[2] = {a0, a1};
    const Act* ds[2] = {d0, d1};
    dense_tn_n(c, g, l, np, as, ds, out, in, in_stride, c0, c1, write_f32);
}

static void colsum(gm_ctx* c, const Grp& g, int N, const Act* X1, const float* w1, const Act* X2, const float* w2,
                   float* out, int64_t g_out, const float* in, int64_t g_in, float c0, float c1) {
    // algorithmic bytes: every operand row once (and its per-row weights), one output row per task (read back when updated)
    Prof p(c, "task_colsum", (double)g.rows * N * (c->mlp_dtype ? 2.0 : 4.0) * (X2 ? 2 : 1) + 4.0 * g.rows * ((w1 ? 1 : 0) + (w2 ? 1 : 0)) +
                                 4.0 * g.G * N * (in ? 2 : 1), 0);
    if (c->mlp_dtype == 0)
        launch_task_colsum(c->stream, g.G, g.row_off, N, X1->f, w1, X2 ? X2->f : nullptr, w2, X1->ld, out, g_out, in, g_in,
                           c0, c1);
    else
        launch_task_colsum_bf(c->stream, g.G, g.row_off, N, X1->b, w1, X2 ? X2->b : nullptr, w2, X1->ld, out, g_out, in,
                              g_in, c0, c1);
}
static void colsum_f32(gm_ctx* c, const Grp& g, int N, const float* X1, int64_t ldx, float* out, int64_t g_out,
                       const float* in, int64_t g_in, float c0, float c1) {
    Prof p(c, "task_colsum", 4.0 * g.rows * N + 4.0 * g.G * N * (in ? 2 : 1), 0);
    launch_task_colsum(c->stream, g.G, g.row_off, N, X1, nullptr, nullptr, nullptr, ldx, out, g_out, in, g_in, c0, c1);
}

static const void* act_ptr(const gm_ctx* c, const Act& a) { return c->mlp_dtype ? (const void*)a.b : (const void*)a.f; }
static void* act_ptr(const gm_ctx* c, Act& a) { return c->mlp_dtype ? (void*)a.b : (void*)a.f; }

struct Pass {  // activations of one forward/backward pass over one set
    Act* X;
    std::vector<Act>*A, *Dl;
    float *dL, *zL;
};

// forward with parameters th (GEMM operands) / thf (fp32: biases and the last layer), loss and delta_L; then
// backward to the deltas of every layer and, when dX is given, to the pooled-input gradient [rows, FD].
static void forward_backward(gm_ctx* c, const Grp& g, const float* labels, const Pass& p, const Theta& th,
                             const float* thf, int64_t thf_stride, float* loss_out, float* dX) {
    hipStream_t st = c->stream;
    const int L = c->L;
    const Act* prev = p.X;
    for (int l = 1; l < L; ++l) {
        dense_nn(c, g, l, 1, prev, &th, nullptr, nullptr, thf + c->offb[l], thf_stride, nullptr, EPI_BIAS_RELU, (*p.A)[l]);
        prev = &(*p.A)[l];
    }
    const float* wL = thf + c->offW[L];
    {
        // algorithmic bytes: the last hidden activations read twice (logit; mask of the backward pass), the delta of the
        // last hidden layer written, 20 bytes of per-row scalars (label, logit, delta, loss, task)
        const double esz_l = c->mlp_dtype ? 2.0 : 4.0;
        Prof pr(c, "last_layer", (double)g.rows * c->ld[L - 1] * esz_l * (L > 1 ? 3 : 1) + 20.0 * g.rows + (L == 1 && dX ? 4.0 * g.rows * c->FD : 0.0), 0);
        LastFwdArgs f;
        memset(&f, 0, sizeof f);
        f.n = g.rows; f.N = c->ld[L - 1]; f.ld = c->ld[L - 1]; f.bf16 = c->mlp_dtype;
        f.row_task = g.row_task; f.row_offsets = g.row_off; f.real_offsets = g.real_off;
        f.a = act_ptr(c, *prev); f.w = wL; f.gW = thf_stride; f.b = thf + c->offb[L];
        f.labels = labels; f.z_out = p.zL; f.delta_out = p.dL; f.loss_out = loss_out;
        launch_last_fwd(st, f);
        if (L == 1) {
            if (dX) launch_last_bwd(st, 0, g.rows, c->FD, c->ld[0], c->FD, g.row_task, p.dL, wL, thf_stride, nullptr, nullptr,
                                    0, nullptr, nullptr, dX);
            return;
        }
        launch_last_bwd(st, c->mlp_dtype, g.rows, c->ld[L - 1], c->ld[L - 1], c->ld[L - 1], g.row_task, p.dL, wL,
                        thf_stride, nullptr, nullptr, 0, act_ptr(c, (*p.A)[L - 1]), act_ptr(c, (*p.Dl)[L - 1]), nullptr);
    }
    for (int l = L - 1; l >= 1; --l) {
        if (l == 1) {
            if (dX) dense_nt(c, g, l, 1, &(*p.Dl)[l], &th, nullptr, nullptr, nullptr, nullptr, dX);
        } else {
            dense_nt(c, g, l, 1, &(*p.Dl)[l], &th, nullptr, nullptr, &(*p.A)[l - 1], &(*p.Dl)[l - 1], nullptr);
        }
    }
}

// out = c0*in + c1 * (gradient of the pass w.r.t. theta), per task; out.b (if any) gets the bf16 operand copies.
// coarse / coarse_out: the hidden layers' weight matrices are summed over runs of tasks instead (c1 times the gradient,
// nothing added), for a caller that only wants their sum over the tasks; biases and the last layer stay per task.
// hist / in0 (bf16 operands, an inner step of a second-order call): the passes of all inner steps so far, this one
// last, and the meta parameters.  The step's weight matrices are then written as theta - alpha * (sum of the steps'
// gradients), one product per step accumulated in the matrix cores, from the shared fp32 theta: no per-task fp32
// master of a weight matrix is written or read (it was most of what a step of small tasks moved); biases and the
// last layer keep their per-task fp32 chain (in, in_stride).
static void theta_grad(gm_ctx* c, const Grp& g, const Pass& p, Theta& out, const float* in, int64_t in_stride, float c0,
                       float c1, float* wL_copy, bool write_f32 = true, const Grp* coarse = nullptr,
                       Theta* coarse_out = nullptr, const std::vector<Pass>* hist = nullptr, const float* in0 = nullptr) {
    const int L = c->L;
    const int64_t nt = out.sf;
    for (int l = 1; l < L; ++l) {
        const Act* prev = l == 1 ? p.X : &(*p.A)[l - 1];
        if (coarse) dense_tn(c, *coarse, l, 1, prev, &(*p.Dl)[l], nullptr, nullptr, *coarse_out, nullptr, 0, 0.f, c1);
        else if (hist) {
            const Act* as[GEMM_MAX_PAIRS];
            const Act* ds[GEMM_MAX_PAIRS];
            const int np = (int)hist->size();
            for (int j = 0; j < np; ++j) {
                as[j] = l == 1 ? (*hist)[j].X : &(*(*hist)[j].A)[l - 1];
                ds[j] = &(*(*hist)[j].Dl)[l];
            }
            dense_tn_n(c, g, l, np, as, ds, out, in0, 0, c0, c1, false);
        } else dense_tn(c, g, l, 1, prev, &(*p.Dl)[l], nullptr, nullptr, out, in, in_stride, c0, c1, write_f32);
        colsum(c, g, c->ld[l], &(*p.Dl)[l], nullptr, nullptr, nullptr, out.f + c->offb[l], nt, in ? in + c->offb[l] : nullptr,
               in_stride, c0, c1);
    }
    const Act* prev = L == 1 ? p.X : &(*p.A)[L - 1];
    colsum(c, g, c->ld[L - 1], prev, p.dL, nullptr, nullptr, out.f + c->offW[L], nt, in ? in + c->offW[L] : nullptr,
           in_stride, c0, c1);
    colsum_f32(c, g, 1, p.dL, 1, out.f + c->offb[L], nt, in ? in + c->offb[L] : nullptr, in_stride, c0, c1);
    if (wL_copy)
        (void)hipMemcpy2DAsync(wL_copy, c->ld[L - 1] * sizeof(float), out.f + c->offW[L], nt * sizeof(float),
                               c->ld[L - 1] * sizeof(float), g.G, hipMemcpyDeviceToDevice, c->stream);
}

// v <- v - alpha * (H v)_theta ;  w.dX [rows, FD] <- (H v)'s pooled-input part
// (tangent pass through the forward and the backward pass of step s, direction (v, TX))
// gx_acc (bf16 mode): the support rows of the sparse-gradient buffer, which take -alpha * (tangent of dX) in the
// layer-1 product itself; need_dx: the tangent of dX is also wanted in w.dX (for the row arithmetic of the next step)
// coarse (the chain's last step): the weight matrices' part of H v is not folded into every task's v but summed over
// runs of tasks into w.vsum (unscaled); the caller adds -alpha times their sum to the reduced v
static void hvp_step(gm_ctx* c, const Grp& g, const StepState& s, WaveBufs& w, float alpha, bool refresh_v_copies,
                     float* gx_acc, bool need_dx, bool gx_init, bool tx, const Grp* coarse = nullptr) {
    hipStream_t st = c->stream;
    const int L = c->L;
    Theta& v = w.v;
    const int64_t nt = v.sf;
    const Act* tprev = &w.TX;
    const Act* prev = &s.X;
    for (int l = 1; l < L; ++l) {
        // (tx false: no direction on the inputs -- rows not adapted -- so layer 1 has one product only)
        if (l == 1 && !tx) dense_nn(c, g, l, 1, prev, &v, nullptr, nullptr, v.f + c->offb[l], nt, &s.A[l], EPI_BIAS_MASK, w.TA[l]);
        else dense_nn(c, g, l, 2, tprev, &s.th, prev, &v, v.f + c->offb[l], nt, &s.A[l], EPI_BIAS_MASK, w.TA[l]);
        tprev = &w.TA[l];
        prev = &s.A[l];
    }
    const float* vwL = v.f + c->offW[L];
    {
        // (tangent pass: activations and their tangents read, the mask read, the tangent delta written)
        const double esz_l = c->mlp_dtype ? 2.0 : 4.0;
        Prof pr(c, "last_layer", (double)g.rows * c->ld[L - 1] * esz_l * (L > 1 ? 4 : 2) + 24.0 * g.rows + (L == 1 ? 4.0 * g.rows * c->FD : 0.0), 0);
        LastFwdArgs f;
        memset(&f, 0, sizeof f);
        f.n = g.rows; f.N = c->ld[L - 1]; f.ld = c->ld[L - 1]; f.bf16 = c->mlp_dtype;
        f.row_task = g.row_task; f.row_offsets = g.row_off; f.real_offsets = g.real_off;
        f.a = act_ptr(c, *prev); f.ta = act_ptr(c, *tprev); f.w = s.wL; f.gW = s.wL_stride; f.b = nullptr;
        f.tw = vwL; f.gTW = nt; f.tb = v.f + c->offb[L];
        f.z_in = s.zL; f.delta_out = w.tdL;
        launch_last_fwd(st, f);
        // tangent of the backward pass, top layer first; each layer's direction is consumed before it is updated
        if (L == 1)
            launch_last_bwd(st, 0, g.rows, c->FD, c->ld[0], c->FD, g.row_task, w.tdL, s.wL, s.wL_stride, s.dL, vwL, nt,
                            nullptr, nullptr, w.dX);
        else
            launch_last_bwd(st, c->mlp_dtype, g.rows, c->ld[L - 1], c->ld[L - 1], c->ld[L - 1], g.row_task, w.tdL, s.wL,
                            s.wL_stride, s.dL, vwL, nt, act_ptr(c, s.A[L - 1]), act_ptr(c, w.TD[L - 1]), nullptr);
    }
    colsum(c, g, c->ld[L - 1], tprev, s.dL, prev, w.tdL, v.f + c->offW[L], nt, v.f + c->offW[L], nt, 1.f, -alpha);
    colsum_f32(c, g, 1, w.tdL, 1, v.f + c->offb[L], nt, v.f + c->offb[L], nt, 1.f, -alpha);
    Theta vout = v;
    if (!refresh_v_copies) vout.b = nullptr;
    for (int l = L - 1; l >= 1; --l) {
        if (l == 1) dense_nt(c, g, l, 2, &w.TD[l], &s.th, &s.Dl[l], &v, nullptr, nullptr, w.dX, gx_acc, -alpha, need_dx || !gx_acc, gx_init);
        else dense_nt(c, g, l, 2, &w.TD[l], &s.th, &s.Dl[l], &v, &s.A[l - 1], &w.TD[l - 1], nullptr);
        const Act* ta_prev = l == 1 ? &w.TX : &w.TA[l - 1];
        const Act* a_prev = l == 1 ? &s.X : &s.A[l - 1];
        if (coarse) {
            if (l == 1 && !tx) dense_tn(c, *coarse, l, 1, a_prev, &w.TD[l], nullptr, nullptr, w.vsum, nullptr, 0, 0.f, 1.f);
            else dense_tn(c, *coarse, l, 2, ta_prev, &s.Dl[l], a_prev, &w.TD[l], w.vsum, nullptr, 0, 0.f, 1.f);
        } else if (l == 1 && !tx) dense_tn(c, g, l, 1, a_prev, &w.TD[l], nullptr, nullptr, vout, v.f, nt, 1.f, -alpha);
        else dense_tn(c, g, l, 2, ta_prev, &s.Dl[l], a_prev, &w.TD[l], vout, v.f, nt, 1.f, -alpha);
        colsum(c, g, c->ld[l], &w.TD[l], nullptr, nullptr, nullptr, v.f + c->offb[l], nt, v.f + c->offb[l], nt, 1.f, -alpha);
    }
}

// ------------------------------------------------------------------------------------------------
// the step
// ------------------------------------------------------------------------------------------------
struct WavePlan {
    int t0, t1;
    int64_t s0, s1, q0, q1;      // sample ranges
    int64_t ps0, ps1, pq0, pq1;  // padded row ranges
    int64_t ls0, ls1, lq0, lq1;  // lookup ranges
};

__global__ void gather_task_lookup_offsets(const int64_t* toff, const int64_t* bag_offsets, int F, int T, int64_t* out) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t <= T) out[t] = bag_offsets[toff[t] * F];
}

// prow[s] = padded row of sample s (whole set): prow_off[t] + (s - toff[t])
__global__ void fill_prow_kernel(const int64_t* toff, const int32_t* prow_off, int32_t* prow) {
    const int t = blockIdx.x;
    const int64_t lo = toff[t], hi = toff[t + 1];
    for (int64_t s = lo + threadIdx.x; s < hi; s += blockDim.x) prow[s] = prow_off[t] + (int32_t)(s - lo);
}

static void build_tiles(const std::vector<int64_t>& poff, int t0, int t1, int bm, std::vector<int32_t>& row_off,
                        std::vector<int32_t>& tg, std::vector<int32_t>& tm) {
    row_off.clear(); tg.clear(); tm.clear();
    const int64_t base = poff[t0];
    for (int t = t0; t < t1; ++t) {
        row_off.push_back((int32_t)(poff[t] - base));
        const int n = (int)(poff[t + 1] - poff[t]);
        for (int m = 0; m < n; m += bm) {
            tg.push_back(t - t0);
            tm.push_back(m);
        }
    }
    row_off.push_back((int32_t)(poff[t1] - base));
}

static int upload_i32(gm_ctx* c, int32_t* dst, const std::vector<int32_t>& v) {
    if (v.empty()) return GM_OK;
    HIPCHK(c, hipMemcpyAsync(dst, v.data(), v.size() * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    return GM_OK;
}

struct Batch {  // host-side description of one call
    int T;
    const gm_set *sup, *qry;
    std::vector<int64_t> poff_s, poff_q;  // padded row offsets per task, whole batch
    std::vector<int64_t> ls, lq;          // lookup offsets per task (filled when several waves are needed)
    bool table = false;                   // table-shaped sparse output: every wave sorts and reduces its own lookups
    BatchBufs b;
};

// The lookups of samples [s0, s1) of the support set and [q0, q1) of the query set, ordered by global row and cut into
// one segment per distinct row.  Gradient-buffer rows are row0_* + the batch-wide padded row of the sample (mod 2^32).
struct SortRange {
    int64_t s0, s1, q0, q1;      // samples
    int64_t ls0, ls1, lq0, lq1;  // their lookups
    u32 row0_s, row0_q;
};

static const ValEnc kPlainVals{0, 0, 0u};

enum { ORDER_SORT = 1, ORDER_SEGMENTS = 2, ORDER_ALL = 3 };

// parts: the sort (keys built, ordered by row: left in so.keys / so.vals), the segments (one per distinct row, from
// the sorted keys), or both
static int global_order(gm_ctx* c, Batch& B, SortBufs& so, const SortRange& r, int64_t* emb_rows, int64_t* seg_counts,
                        int64_t capacity, int64_t* n_rows, bool on_side = false, ValEnc enc = kPlainVals, int parts = ORDER_ALL) {
    hipStream_t st = on_side ? c->side : c->stream;
    u32* status = on_side ? c->d_status_side : c->d_status;
    const int F = c->F;
    const gm_set *sup = B.sup, *qry = B.qry;
    BatchBufs& b = B.b;
    const int64_t n_s = r.ls1 - r.ls0, nnz = n_s + (r.lq1 - r.lq0);
    Prof p(c, "global_sort", 0, 0, st, true);
    if (parts & ORDER_SORT) {
        if (F > 0) {
            launch_build_keys(st, F, c->d_field_base, sup->bag_offsets + r.s0 * F, sup->indices, (r.s1 - r.s0) * F, r.ls0,
                              b.prow_s + r.s0, r.row0_s, enc, so.keys, so.vals);
            launch_build_keys(st, F, c->d_field_base, qry->bag_offsets + r.q0 * F, qry->indices, (r.q1 - r.q0) * F, r.lq0,
                              b.prow_q + r.q0, r.row0_q, enc, so.keys + n_s, so.vals + n_s);
        }
        int bits = 1;
        while (((int64_t)1 << bits) < c->field_base[c->F]) ++bits;
        const int passes = launch_radix_sort(st, so.keys, so.vals, so.keys_tmp, so.vals_tmp, nnz, bits, so.hist);
        // algorithmic bytes: keys built from the lookups (4 B index read, 8 B of key and value written, 8 B of offsets per bag),
        // 20 B per key and radix pass (the key read for the digit counts; key and value read and written by the scatter)
        p.p.bytes += (double)nnz * (12.0 + 20.0 * passes) + 8.0 * F * ((r.s1 - r.s0) + (r.q1 - r.q0));
        if (passes & 1) {
            std::swap(so.keys, so.keys_tmp);   // an odd number of passes leaves the result in the second pair of buffers
            std::swap(so.vals, so.vals_tmp);
        }
    }
    // the table-shaped output adds every segment to the row its key names: no segment numbers, no row list
    if ((parts & ORDER_SEGMENTS) && n_rows) {
        p.p.bytes += 4.0 * (double)nnz;   // the sorted keys read once more
        launch_segments(st, so.keys, nnz, so.keys_tmp, so.scan_tmp, emb_rows, so.seg_start, seg_counts, capacity, n_rows,
                        status);
    }
    return GM_OK;
}

// Asks run_index_wave to take the wave's per-(task, field) dictionaries from the (field, row) order of its lookups --
// the order the sparse meta-gradient needs anyway -- instead of sorting every (task, field) by itself: the wave's
// lookups are ordered by row first (left in `so` for the segment reduction), one more stable pass orders them by task,
// and the dictionaries, the lookup lists and the overlap join are read off that list.  Applies when the sort's range is
// exactly the wave and a gradient-buffer row, a field number and a position in a bag fit 32 bits together.
struct JoinReq {
    SortBufs* so = nullptr;
    SortRange range{};
    int64_t* emb_rows = nullptr;     // row-list output: the segments are cut right after the sort (n_rows null: table-shaped output)
    int64_t* seg_counts = nullptr;
    int64_t capacity = 0;
    int64_t* n_rows = nullptr;
    int64_t n_sup_rows = 0, n_qry_rows = 0;   // padded rows of the wave's two sets (gradient-buffer rows: support first)
    bool slots = false;              // the slot of every lookup is wanted whatever the row path
    bool pair_only = false;          // every task of the wave is planned for the pair-count matrices (which do not read those slots)
    bool used = false;               // out: the wave's lookups are ordered, `enc` says how their values read
    ValEnc enc = kPlainVals;
};

static int64_t uniform_rows(const gm_ctx* c) {   // rows of every table when they are all of one size, else -1
    for (int f = 1; f < c->F; ++f)
        if (c->rows[f] != c->rows[0]) return -1;
    return c->F > 0 ? c->rows[0] : -1;
}

static int bits_for(int64_t n) {   // bits that hold every value below n
    int b = 0;
    while (((int64_t)1 << b) < n) ++b;
    return b;
}

// The per-(task, field) dictionaries, lookup lists and overlap join of a wave, every (task, field) sorted by itself in LDS
// (w.cnt_* / w.base_* are in place).
static void sort_task_fields(gm_ctx* c, const Batch& B, const WavePlan& wp, WaveBufs& w, int max_tf) {
    const int F = c->F, Tw = wp.t1 - wp.t0;
    TfSortArgs a;
    a.F = F; a.t0 = wp.t0; a.Tw = Tw;
    a.sup = make_view(B.sup, B.b.toff_s, wp.s0, wp.ls0); a.qry = make_view(B.qry, B.b.toff_q, wp.q0, wp.lq0);
    a.field_base = c->d_field_base;
    a.cnt_sup = w.cnt_s; a.base_sup = w.base_s; a.cnt_qry = w.cnt_q; a.base_qry = w.base_q;
    a.n_slots = w.n_slots; a.slot_rows = w.slot_rows; a.slot_start = w.slot_start;
    a.sup_sorted = w.sup_sorted; a.sup_slot = w.sup_slot; a.qry_slot = w.qry_slot;
    a.qry_sorted = w.qry_sorted; a.qseg_lo = w.qseg_lo; a.qseg_hi = w.qseg_hi; a.status = c->d_status;
    a.sup_rows = B.b.prow_s; a.sup_row_base = (int32_t)wp.ps0;
    a.qry_rows = B.b.prow_q; a.qry_row_base = (int32_t)wp.pq0;
    Prof p(c, "tf_sort", 12.0 * ((wp.ls1 - wp.ls0) + (wp.lq1 - wp.lq0)), 0);
    int64_t max_set_rows = 0;
    for (int t = wp.t0; t < wp.t1; ++t)
        max_set_rows = std::max(max_set_rows, std::max(B.sup->task_offsets[t + 1] - B.sup->task_offsets[t],
                                                       B.qry->task_offsets[t + 1] - B.qry->task_offsets[t]));
    launch_tf_sort(c->stream, a, max_tf, (int)std::min<int64_t>(max_set_rows, 1 << 30));
    w.slots_written = true;
}

static int run_index_wave(gm_ctx* c, Batch& B, const WavePlan& wp, WaveBufs& w, int* cap_out = nullptr,
                          int* max_bag_out = nullptr, int* max_tf_out = nullptr, JoinReq* jr = nullptr) {
    hipStream_t st = c->stream;
    const int F = c->F, Tw = wp.t1 - wp.t0;
    if (jr) jr->used = false;
    if (F == 0 || Tw == 0) return GM_OK;
    const int64_t TF = (int64_t)Tw * F;
    SetView vs = make_view(B.sup, B.b.toff_s, wp.s0, wp.ls0), vq = make_view(B.qry, B.b.toff_q, wp.q0, wp.lq0);
    launch_fill_u32(st, c->d_status, ST_WORDS, 0);
    {
        Prof p(c, "tf_count", 8.0 * ((wp.s1 - wp.s0) + (wp.q1 - wp.q0)) * F + 4.0 * ((wp.ls1 - wp.ls0) + (wp.lq1 - wp.lq0)), 0);
        launch_tf_count(st, F, wp.t0, Tw, vs, vq, c->d_field_base, B.sup->nnz, B.qry->nnz, uniform_rows(c), w.cnt_s, w.cnt_q, c->d_status);
    }
    u32 hs[ST_WORDS];
    int rc = read_status(c, hs);
    if (rc != GM_OK) return rc;
    if (hs[ST_BAD_INDEX]) return fail(c, GM_ERR_INDEX, "index outside its table, or bag_offsets not monotone / beyond nnz");
    if (hs[ST_TOO_LARGE])
        return fail(c, GM_ERR_CAPACITY, "a bag has more than 65535 lookups, or a task more than 65536 samples in one set");
    int cap = 1024;
    while (cap < (int)hs[ST_MAX_TF]) cap <<= 1;
    if (cap_out) *cap_out = cap;
    if (max_bag_out) *max_bag_out = (int)hs[ST_MAX_BAG];
    if (max_tf_out) *max_tf_out = (int)hs[ST_MAX_TF];
    if (!c->adapt_rows) return GM_OK;   // validated; no row arithmetic, so no per-(task, field) dictionaries
    if (cap > tf_sort_max_cap())
        return fail(c, GM_ERR_CAPACITY, "a (task, field) has %u lookups in one set; the limit is %d", hs[ST_MAX_TF],
                    tf_sort_max_cap());
    launch_scan_u32(st, w.cnt_s, w.base_s, TF, w.scan_tmp, nullptr);
    launch_scan_u32(st, w.cnt_q, w.base_q, TF, w.scan_tmp, nullptr);
    const double tf_bytes = 12.0 * ((wp.ls1 - wp.ls0) + (wp.lq1 - wp.lq0));
    // ---- the dictionaries read off the row order of the wave's lookups
    bool join = jr && jr->so && c->index_path != 1;
    ValEnc enc = kPlainVals;
    if (join) {
        const int pbits = bits_for((int64_t)hs[ST_MAX_BAG]), fbits = bits_for(F);
        const int rbits = bits_for(jr->n_sup_rows + jr->n_qry_rows);
        if (rbits + fbits + pbits > 32 || (task_sort_passes(Tw) > 1 && !w.tmid_keys)) join = false;
        else enc = ValEnc{fbits + pbits > 0 ? fbits + pbits : 1, pbits, (1u << fbits) - 1u};
        if (join && enc.rshift + rbits > 32) join = false;   // (no field and no position bits: the shift of 1 marks the form)
    }
    if (jr && c->index_path == 2 && !join)
        return fail(c, GM_ERR_CAPACITY, "index_path 2: the wave's lookups cannot be ordered as one list of 32-bit bit-field values");
    if (join) {
        SortBufs& so = *jr->so;
        if (c->sort_fields) {
            // the keys field after field (the per-(task, field) counts give every lookup its place), then every field's
            // range sorted by its row bits alone
            const int64_t nw = (wp.ls1 - wp.ls0) + (wp.lq1 - wp.lq0);
            Prof p(c, "global_sort", 0, 0, st, true);
            FieldKeysArgs fa;
            memset(&fa, 0, sizeof fa);
            fa.F = F; fa.t0 = wp.t0; fa.Tw = Tw; fa.sup = vs; fa.qry = vq; fa.field_base = c->d_field_base;
            fa.cnt_s = w.cnt_s; fa.cnt_q = w.cnt_q; fa.fm_off_s = w.fm_off_s; fa.fm_off_q = w.fm_off_q;
            fa.prow_s = B.b.prow_s; fa.prow_q = B.b.prow_q; fa.row0_s = jr->range.row0_s; fa.row0_q = jr->range.row0_q;
            fa.enc = enc; fa.keys = so.keys; fa.vals = so.vals;
            launch_build_keys_by_field(st, fa, w.field_tab);
            int64_t max_rows = 1;
            for (int f = 0; f < F; ++f) max_rows = std::max(max_rows, c->field_base[f + 1] - c->field_base[f]);
            const SegTab seg = field_seg_tab(F, w.field_tab);
            const int passes = launch_radix_sort(st, so.keys, so.vals, so.keys_tmp, so.vals_tmp, nw, std::max(1, bits_for(max_rows)), so.hist, &seg);
            p.p.bytes += (double)nw * (12.0 + 20.0 * passes) + 8.0 * F * ((wp.s1 - wp.s0) + (wp.q1 - wp.q0));
            if (passes & 1) {
                std::swap(so.keys, so.keys_tmp);
                std::swap(so.vals, so.vals_tmp);
            }
        } else {
            global_order(c, B, so, jr->range, nullptr, nullptr, jr->capacity, nullptr, false, enc, ORDER_SORT);
        }
        {
            Prof p(c, "tf_sort", tf_bytes, 0);
            const int64_t nw = (wp.ls1 - wp.ls0) + (wp.lq1 - wp.lq0);
            int uniform_shift = -1;   // all tasks of the wave of one power-of-two size (padded rows, both sets alike)?
            {
                const int64_t r0 = B.poff_s[wp.t0 + 1] - B.poff_s[wp.t0];
                bool same = r0 > 0 && (r0 & (r0 - 1)) == 0;
                for (int t = wp.t0; t < wp.t1 && same; ++t)
                    same = B.poff_s[t + 1] - B.poff_s[t] == r0 && B.poff_q[t + 1] - B.poff_q[t] == r0;
                if (same) uniform_shift = bits_for(r0);
            }
            TaskOf tk{w.row_task_s, w.row_task_q, (u32)jr->n_sup_rows, (u32)(jr->n_sup_rows + jr->n_qry_rows), enc.rshift, uniform_shift};
            launch_task_sort(st, so.keys, so.vals, w.tmid_keys, w.tmid_vals, so.keys_tmp, so.vals_tmp, nw, Tw, tk, so.hist);
            TfJoinArgs a;
            memset(&a, 0, sizeof a);
            a.F = F; a.Tw = Tw; a.keys = so.keys_tmp; a.vals = so.vals_tmp;
            a.cnt_s = w.cnt_s; a.base_s = w.base_s; a.cnt_q = w.cnt_q; a.base_q = w.base_q;
            a.rshift = enc.rshift; a.pshift = enc.pshift; a.n_sup_rows = (u32)jr->n_sup_rows;
            a.n_slots = w.n_slots; a.slot_rows = w.slot_rows; a.slot_start = w.slot_start;
            a.sup_sorted = w.sup_sorted; a.qry_sorted = w.qry_sorted; a.qseg_lo = w.qseg_lo; a.qseg_hi = w.qseg_hi;
            // the slot of every lookup (scattered 4-byte writes) only where the sparse row kernel may read it
            const bool write_slots = jr->slots || !jr->pair_only || cap > PAIR_MAX_CAP || (int)hs[ST_MAX_BAG] > PAIR_MAX_BAG;
            a.sup_slot = write_slots ? w.sup_slot : nullptr;
            a.qry_slot = write_slots ? w.qry_slot : nullptr;
            w.slots_written = write_slots;
            a.bag_s = B.sup->bag_offsets; a.bag_q = B.qry->bag_offsets;
            a.sample0_s = wp.s0; a.sample0_q = wp.q0; a.lookup0_s = wp.ls0; a.lookup0_q = wp.lq0;
            a.n_lookups_s = wp.ls1 - wp.ls0; a.n_lookups_q = wp.lq1 - wp.lq0;
            a.row_off_s = w.row_off_s; a.row_off_q = w.row_off_q; a.real_off_s = w.real_off_s; a.real_off_q = w.real_off_q;
            launch_tf_join(st, a);
        }
        // (the list in task order is done with: the second pair of buffers is free for the segment scan)
        if (jr->n_rows)
            global_order(c, B, so, jr->range, jr->emb_rows, jr->seg_counts, jr->capacity, jr->n_rows, false, enc, ORDER_SEGMENTS);
        jr->used = true;
        jr->enc = enc;
        return GM_OK;
    }
    w.slots_written = true;
    sort_task_fields(c, B, wp, w, (int)hs[ST_MAX_TF]);
    return GM_OK;
}

static SortRange whole_batch_range(const Batch& B) {
    return SortRange{0, B.sup->n_samples, 0, B.qry->n_samples, 0, B.sup->nnz, 0, B.qry->nnz, 0u, (u32)B.poff_s[B.T]};
}

static inline int64_t pad64(int64_t n) { return (n + 63) & ~(int64_t)63; }

// Whether a task's row arithmetic should go through pair-count matrices: the product costs
// n_out * n_in * D per (task, field) against lookups * D for the sparse kernel, on units that are far
// faster, so it pays while the task is moderately small.
static bool task_pair_ok(const gm_ctx* c, const Batch& B, int t, int K) {
    if (c->row_path == 1 || K <= 0 || c->F == 0 || c->D % 32 != 0 || !c->adapt_rows) return false;
    const int64_t mx = std::max(B.sup->task_offsets[t + 1] - B.sup->task_offsets[t], B.qry->task_offsets[t + 1] - B.qry->task_offsets[t]);
    return mx > 0 && mx <= (c->row_path == 2 ? 1024 : 512);
}

// Byte offsets of every task's pair-count matrices (kind by kind, fields back to back; nothing for a task
// that takes the sparse kernel); returns the total.
static int64_t pair_layout(const gm_ctx* c, const Batch& B, const WavePlan& p, int K, bool ss, bool sq,
                           std::vector<int64_t>* off_ss, std::vector<int64_t>* off_qs, std::vector<int64_t>* off_sq,
                           std::vector<u32>* path) {
    int64_t acc = 0;
    for (int t = p.t0; t < p.t1; ++t) {
        const bool ok = task_pair_ok(c, B, t, K);
        const int64_t ns = ok ? pad64(B.sup->task_offsets[t + 1] - B.sup->task_offsets[t]) : 0;
        const int64_t nq = ok ? pad64(B.qry->task_offsets[t + 1] - B.qry->task_offsets[t]) : 0;
        if (path) path->push_back(ok ? 1u : 0u);
        if (off_ss) off_ss->push_back(acc);
        if (ss) acc += c->F * ns * ns;
        if (off_qs) off_qs->push_back(acc);
        acc += c->F * nq * ns;
        if (off_sq) off_sq->push_back(acc);
        if (sq) acc += c->F * ns * nq;
    }
    return acc;
}

static WaveDims wave_dims(const gm_ctx* c, const Batch& B, const WavePlan& p, int bm, int K, int order) {
    WaveDims d;
    d.table = B.table;
    for (int t = p.t0; t < p.t1; ++t) {
        if (task_pair_ok(c, B, t, K)) d.pair = true;
        else d.any_sparse = true;
    }
    if (d.pair) {
        d.pair_ss = K >= 2;
        d.pair_sq = order == 2;
        d.pair_bytes = pair_layout(c, B, p, K, d.pair_ss, d.pair_sq, nullptr, nullptr, nullptr, nullptr);
    }
    d.Tw = p.t1 - p.t0;
    d.Ss = p.s1 - p.s0; d.Sq = p.q1 - p.q0; d.Ps = p.ps1 - p.ps0; d.Pq = p.pq1 - p.pq0;
    d.nnz_s = p.ls1 - p.ls0; d.nnz_q = p.lq1 - p.lq0;
    int64_t ms = 0, mq = 0;
    for (int t = p.t0; t < p.t1; ++t) {
        ms += (B.poff_s[t + 1] - B.poff_s[t] + bm - 1) / bm;
        mq += (B.poff_q[t + 1] - B.poff_q[t] + bm - 1) / bm;
    }
    d.mt_s = (int)ms; d.mt_q = (int)mq;
    return d;
}

static int pick_bm(const gm_ctx* c, const Batch& B) {
    if (B.T == 0) return 64;
    const int64_t avg = (B.poff_s[B.T] + B.poff_q[B.T]) / (2 * (int64_t)B.T);
    if (!c->mlp_dtype) return 64;
    return avg >= 192 ? 256 : (avg >= 96 ? 128 : 64);
}

// splits the tasks into waves that fit `avail` bytes of workspace
static int plan_waves(gm_ctx* c, Batch& B, size_t avail, int K, int order, int bm, std::vector<WavePlan>& plans) {
    const int F = c->F, T = B.T;
    const gm_set *sup = B.sup, *qry = B.qry;
    B.ls.assign(T + 1, 0);
    B.lq.assign(T + 1, 0);
    bool have_offsets = false;
    auto fetch = [&]() -> int {
        if (have_offsets || F == 0) return GM_OK;
        int64_t* d = reinterpret_cast<int64_t*>(B.b.so.hist);  // scratch: the histogram area is free until the global sort
        hipLaunchKernelGGL(gather_task_lookup_offsets, dim3((T + 256) / 256), dim3(256), 0, c->stream, B.b.toff_s,
                           sup->bag_offsets, F, T, d);
        hipLaunchKernelGGL(gather_task_lookup_offsets, dim3((T + 256) / 256), dim3(256), 0, c->stream, B.b.toff_q,
                           qry->bag_offsets, F, T, d + T + 1);
        HIPCHK(c, hipMemcpyAsync(B.ls.data(), d, (T + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipMemcpyAsync(B.lq.data(), d + T + 1, (T + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        for (int t = 0; t <= T; ++t)
            if (B.ls[t] < 0 || B.ls[t] > sup->nnz || B.lq[t] < 0 || B.lq[t] > qry->nnz ||
                (t && (B.ls[t] < B.ls[t - 1] || B.lq[t] < B.lq[t - 1])))
                return fail(c, GM_ERR_INDEX, "bag_offsets not monotone / beyond nnz at a task boundary");
        have_offsets = true;
        return GM_OK;
    };
    // Waves of (nearly) equal numbers of tasks: the fewest waves whose every wave fits.  A wave's tasks are one grid
    // dimension of several kernels, hence the cap.
    int max_per = std::min(std::max(T, 1), 32768);
    if (c->max_wave_tasks > 0) max_per = std::min(max_per, c->max_wave_tasks);
    int n_waves = (std::max(T, 1) + max_per - 1) / max_per;
    while (true) {
        const int per = (std::max(T, 1) + n_waves - 1) / n_waves;
        plans.clear();
        bool fits = true;
        if (per < T) {
            int rc = fetch();
            if (rc != GM_OK) return rc;
        } else {
            B.ls[T] = sup->nnz;
            B.lq[T] = qry->nnz;
        }
        for (int t0 = 0; t0 < T || (T == 0 && plans.empty()); t0 += per) {
            WavePlan p;
            p.t0 = t0;
            p.t1 = std::min(T, t0 + per);
            p.s0 = sup->task_offsets[p.t0]; p.s1 = sup->task_offsets[p.t1];
            p.q0 = qry->task_offsets[p.t0]; p.q1 = qry->task_offsets[p.t1];
            p.ps0 = B.poff_s[p.t0]; p.ps1 = B.poff_s[p.t1]; p.pq0 = B.poff_q[p.t0]; p.pq1 = B.poff_q[p.t1];
            p.ls0 = B.ls[p.t0]; p.ls1 = B.ls[p.t1]; p.lq0 = B.lq[p.t0]; p.lq1 = B.lq[p.t1];
            plans.push_back(p);
            // a wave's lookups are numbered in 32 bits
            if ((p.ls1 - p.ls0) + (p.lq1 - p.lq0) >= ((int64_t)1 << 31)) { fits = false; break; }
            Arena ar;
            ar.cap = avail;
            WaveBufs w;
            alloc_wave(c, ar, w, wave_dims(c, B, p, bm, K, order), K, order);
            if (ar.overflow) { fits = false; break; }
            if (T == 0) break;
        }
        if (fits) return GM_OK;
        if (per == 1) return fail(c, GM_ERR_WORKSPACE, "workspace of %zu bytes cannot hold one task", c->ws_bytes);
        n_waves = std::min(std::max(T, 1), std::max(n_waves + 1, n_waves + n_waves / 16));
    }
}

// batch-level set-up shared by gm_meta_step and gm_index_prep
// ar: where the index-side buffers go; dense_ar: where the batch's dense buffers go (null: the caller places them)
static int begin_batch(gm_ctx* c, Batch& B, Arena& ar, int64_t capacity, bool need_gx, Arena* dense_ar) {
    const int T = B.T, pad = c->row_pad;
    B.poff_s.assign(T + 1, 0);
    B.poff_q.assign(T + 1, 0);
    for (int t = 0; t < T; ++t) {
        B.poff_s[t + 1] = B.poff_s[t] + round_up64(B.sup->task_offsets[t + 1] - B.sup->task_offsets[t], pad);
        B.poff_q[t + 1] = B.poff_q[t] + round_up64(B.qry->task_offsets[t + 1] - B.qry->task_offsets[t], pad);
    }
    if ((B.poff_s[T] + B.poff_q[T]) * (int64_t)std::max(c->F, 1) >= ((int64_t)1 << 32))
        return fail(c, GM_ERR_ARG, "more than 2^32 (row, field) pairs in one call");
    // (no batch-wide sort when every wave reduces its own lookups into a table)
    alloc_batch_index(c, ar, B.b, T, B.sup->n_samples, B.qry->n_samples, B.table ? 0 : B.sup->nnz + B.qry->nnz, capacity, need_gx);
    if (dense_ar) alloc_batch_dense(c, *dense_ar, B.b, T, B.poff_s[T], B.poff_q[T], need_gx);
    if (ar.overflow || (dense_ar && dense_ar->overflow))
        return fail(c, GM_ERR_WORKSPACE, "workspace too small for the batch-level buffers (%zu needed)", ar.off);
    hipStream_t st = c->stream;
    HIPCHK(c, hipMemcpyAsync(B.b.toff_s, B.sup->task_offsets, (T + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(B.b.toff_q, B.qry->task_offsets, (T + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    std::vector<int32_t> ps(B.poff_s.begin(), B.poff_s.end()), pq(B.poff_q.begin(), B.poff_q.end());
    int rc;
    if ((rc = upload_i32(c, B.b.prow_off_s, ps)) || (rc = upload_i32(c, B.b.prow_off_q, pq))) return rc;
    if (T > 0) {
        hipLaunchKernelGGL(fill_prow_kernel, dim3(T), dim3(256), 0, st, B.b.toff_s, B.b.prow_off_s, B.b.prow_s);
        hipLaunchKernelGGL(fill_prow_kernel, dim3(T), dim3(256), 0, st, B.b.toff_q, B.b.prow_off_q, B.b.prow_q);
    }
    HIPCHK(c, hipStreamSynchronize(st));  // the host vectors above go out of scope
    return GM_OK;
}

static int setup_wave(gm_ctx* c, const Batch& B, const WavePlan& wp, int bm, int K, WaveBufs& w, const WaveDims& d, Grp& gs,
                      Grp& gq) {
    hipStream_t st = c->stream;
    std::vector<int32_t> ro_s, tg_s, tm_s, ro_q, tg_q, tm_q, re_s, re_q;
    build_tiles(B.poff_s, wp.t0, wp.t1, bm, ro_s, tg_s, tm_s);
    build_tiles(B.poff_q, wp.t0, wp.t1, bm, ro_q, tg_q, tm_q);
    for (int t = wp.t0; t <= wp.t1; ++t) {
        re_s.push_back((int32_t)(B.sup->task_offsets[t] - wp.s0));
        re_q.push_back((int32_t)(B.qry->task_offsets[t] - wp.q0));
    }
    // runs of consecutive tasks for the products that are only summed over the tasks
    std::vector<int32_t> co_s, co_q;
    const int n_coarse = coarse_group_count(c, d.Tw, std::min(d.Ps, d.Pq));
    for (int i = 0; i <= n_coarse; ++i) {
        const int t = (int)((int64_t)i * d.Tw / n_coarse);
        co_s.push_back(ro_s[t]);
        co_q.push_back(ro_q[t]);
    }
    int rc;
    if ((rc = upload_i32(c, w.coarse_off_s, co_s)) || (rc = upload_i32(c, w.coarse_off_q, co_q))) return rc;
    if ((rc = upload_i32(c, w.row_off_s, ro_s)) || (rc = upload_i32(c, w.row_off_q, ro_q)) ||
        (rc = upload_i32(c, w.real_off_s, re_s)) || (rc = upload_i32(c, w.real_off_q, re_q)) ||
        (rc = upload_i32(c, w.tile_g_s, tg_s)) || (rc = upload_i32(c, w.tile_m_s, tm_s)) ||
        (rc = upload_i32(c, w.tile_g_q, tg_q)) || (rc = upload_i32(c, w.tile_m_q, tm_q)))
        return rc;
    std::vector<int64_t> po_ss, po_qs, po_sq;
    std::vector<u32> path;
    pair_layout(c, B, wp, K, d.pair_ss, d.pair_sq, &po_ss, &po_qs, &po_sq, &path);
    if (!path.empty())
        HIPCHK(c, hipMemcpyAsync(w.task_path, path.data(), path.size() * sizeof(u32), hipMemcpyHostToDevice, st));
    if (d.pair) {
        HIPCHK(c, hipMemcpyAsync(w.pair_off_ss, po_ss.data(), po_ss.size() * sizeof(int64_t), hipMemcpyHostToDevice, st));
        HIPCHK(c, hipMemcpyAsync(w.pair_off_qs, po_qs.data(), po_qs.size() * sizeof(int64_t), hipMemcpyHostToDevice, st));
        HIPCHK(c, hipMemcpyAsync(w.pair_off_sq, po_sq.data(), po_sq.size() * sizeof(int64_t), hipMemcpyHostToDevice, st));
    }
    launch_fill_sample_task(st, w.real_off_s, d.Tw, w.sample_task_s);
    launch_fill_sample_task(st, w.real_off_q, d.Tw, w.sample_task_q);
    launch_fill_sample_task(st, w.row_off_s, d.Tw, w.row_task_s);
    launch_fill_sample_task(st, w.row_off_q, d.Tw, w.row_task_q);
    HIPCHK(c, hipStreamSynchronize(st));  // host vectors go out of scope
    gs = Grp{w.row_off_s, w.real_off_s, w.row_task_s, w.tile_g_s, w.tile_m_s, d.mt_s, d.Tw, bm, d.Ps};
    gq = Grp{w.row_off_q, w.real_off_q, w.row_task_q, w.tile_g_q, w.tile_m_q, d.mt_q, d.Tw, bm, d.Pq};
    return GM_OK;
}

// Pair-count matrices for the tasks that qualify, when the wave's bags and (task, field)s are within the counting
// kernel's limits; a task with a count that does not fit a byte is handed to the sparse kernel (its flag is cleared on
// the device).  allow_side: the counting may run on the second stream (gm_configure "overlap_pairs"); the caller then
// joins it before the first row hop.
static int count_pairs(gm_ctx* c, const Batch& B, const WavePlan& wp, WaveBufs& w, const WaveDims& d, int K, int tf_cap,
                       int max_bag, int max_tf, bool allow_side, bool& pair, bool& any_sparse, bool& pairs_on_side) {
    hipStream_t st = c->stream;
    const int F = c->F, Tw = wp.t1 - wp.t0;
    const gm_set *sup = B.sup, *qry = B.qry;
    pair = d.pair && tf_cap <= PAIR_MAX_CAP && max_bag <= PAIR_MAX_BAG;
    any_sparse = d.any_sparse || (d.pair && !pair);
    pairs_on_side = false;
    if (d.pair && !pair) launch_fill_u32(st, w.task_path, Tw, 0u);
    if (!pair) return GM_OK;
    PairCountArgs pa;
    memset(&pa, 0, sizeof pa);
    pa.F = F;
    pa.real_off_s = w.real_off_s; pa.real_off_q = w.real_off_q; pa.row_off_s = w.row_off_s; pa.row_off_q = w.row_off_q;
    pa.base_s = w.base_s; pa.base_q = w.base_q; pa.cnt_q = w.cnt_q; pa.n_slots = w.n_slots;
    pa.slot_start = w.slot_start; pa.qseg_lo = w.qseg_lo; pa.qseg_hi = w.qseg_hi;
    pa.sup_sorted = w.sup_sorted; pa.qry_sorted = w.qry_sorted;
    pa.off_ss = w.pair_off_ss; pa.off_qs = w.pair_off_qs; pa.off_sq = w.pair_off_sq;
    pa.mat = w.pair_mat; pa.want_ss = d.pair_ss; pa.want_sq = d.pair_sq; pa.status = c->d_status;
    pa.task_path = w.task_path;
    pairs_on_side = allow_side && c->overlap_pairs && !c->overlap_sort;
    hipStream_t pst = pairs_on_side ? c->side : st;
    if (pairs_on_side) {   // everything the kernel reads is in place once the main stream gets here
        HIPCHK(c, hipEventRecord(c->ev_pairs_go, st));
        HIPCHK(c, hipStreamWaitEvent(c->side, c->ev_pairs_go, 0));
        launch_fill_u32(c->side, c->d_status_side, ST_WORDS, 0);
        pa.status = c->d_status_side;
    }
    {
        Prof p(c, "pair_count", 8.0 * (d.nnz_s + d.nnz_q) + (double)d.pair_bytes, 0, pst, true);
        int max_rows = 0, min_rows = 1 << 30;
        for (int t = wp.t0; t < wp.t1; ++t)
            if (task_pair_ok(c, B, t, K)) {
                const int r = (int)std::max(sup->task_offsets[t + 1] - sup->task_offsets[t],
                                            qry->task_offsets[t + 1] - qry->task_offsets[t]);
                max_rows = std::max(max_rows, r);
                min_rows = std::min(min_rows, r);
            }
        launch_pair_count(pst, pa, Tw, max_tf, max_rows, min_rows, c->pair_tile_rows);
    }
    if (pairs_on_side) {
        HIPCHK(c, hipEventRecord(c->ev_pairs, c->side));
    } else {
        u32 hs[ST_WORDS];
        int rc = read_status(c, hs);
        if (rc != GM_OK) return rc;
        if (hs[ST_PAIR_OVF]) any_sparse = true;   // some task's flag was cleared on the device
        // the sparse kernel reads the slot of every lookup: written now if the wave was planned without it
        if (any_sparse && !w.slots_written) sort_task_fields(c, B, wp, w, max_tf);
    }
    return GM_OK;
}

// Everything of a one-wave batch with the row-list output that depends on its indices only, prepared ahead of the step
// (by gm_meta_train, on the second stream, while the previous batch computes): validated offsets and indices, padded
// row numbers, tile lists, per-(task, field) dictionaries and overlap join, pair-count matrices, the batch-wide order
// of the lookups by row and its segments.  The buffers live in an arena of their own.
struct Prepared {
    Batch B;
    WavePlan wp;
    WaveDims d;
    WaveBufs w;        // index part only
    Grp gs, gq;
    int bm = 64;
    int tf_cap = 0, max_bag = 0, max_tf = 0;
    bool pair = false, any_sparse = false;
    ValEnc enc = kPlainVals;   // how the values of the ordered lookups name their bags
};

// The step.  pre: null, or the batch's index side prepared beforehand (one wave, row-list output); no_sync: return with
// the work enqueued and the stream not drained (the caller synchronises and reads nothing from the host side but the
// stream's error state; only with pre).
static int meta_step_impl(gm_ctx* c, int32_t T, const gm_set* sup, const gm_set* qry, const gm_params* params, float alpha,
                          int32_t K, int32_t order, float* loss, gm_grads* out, Prepared* pre, bool no_sync) {
    if (!c) return GM_ERR_ARG;
    if (T < 0 || K < 0 || (order != 1 && order != 2)) return fail(c, GM_ERR_ARG, "bad n_tasks / inner_steps / order");
    if (!out) return fail(c, GM_ERR_ARG, "null outputs");
    float* const table = c->F > 0 ? out->emb_grad_table : nullptr;
    int rc = check_set(c, sup, T, "support", table != nullptr);
    if (rc != GM_OK) return rc;
    rc = check_set(c, qry, T, "query", table != nullptr);
    if (rc != GM_OK) return rc;
    if (!params || !params->W || !params->b || (c->F > 0 && !params->emb)) return fail(c, GM_ERR_ARG, "null params");
    if (!loss || !out->dW || !out->db || !out->n_emb_rows) return fail(c, GM_ERR_ARG, "null outputs");
    for (int l = 0; l < c->L; ++l)
        if (!params->W[l] || !params->b[l] || !out->dW[l] || !out->db[l]) return fail(c, GM_ERR_ARG, "null layer pointer");
    if (!table && (out->emb_rows_capacity < 0 || (out->emb_rows_capacity > 0 && (!out->emb_rows || !out->emb_grad))))
        return fail(c, GM_ERR_ARG, "bad sparse output buffers");
    HIPCHK(c, hipSetDevice(c->device));
    hipStream_t st = c->stream;
    const int F = c->F, D = c->D, L = c->L, FD = c->FD, ld0 = c->ld[0];
    const bool bf = c->mlp_dtype != 0;
    const int64_t nt = c->n_theta;
    const int64_t nnz = sup->nnz + qry->nnz;
    const int64_t capacity = table ? 0 : out->emb_rows_capacity;

    if (pre && table) return fail(c, GM_ERR_ARG, "internal: a prepared batch uses the row-list output");
    Arena ar;
    ar.base = c->ws; ar.cap = c->ws_bytes; ar.off = c->persistent;
    Batch local_batch;
    Batch& B = pre ? pre->B : local_batch;
    std::vector<WavePlan> plans;
    int bm;
    if (pre) {   // the index side exists already; the dense buffers of the batch go to this call's arena
        alloc_batch_dense(c, ar, B.b, T, B.poff_s[T], B.poff_q[T], true);
        if (ar.overflow) return fail(c, GM_ERR_WORKSPACE, "workspace too small for the batch-level buffers (%zu needed)", ar.off);
        bm = pre->bm;
        plans.push_back(pre->wp);
    } else {
        B.T = T; B.sup = sup; B.qry = qry;
        B.table = table != nullptr;
        rc = begin_batch(c, B, ar, capacity, !B.table, &ar);
        if (rc != GM_OK) return rc;
        bm = pick_bm(c, B);
        rc = plan_waves(c, B, c->ws_bytes - ar.off, K, order, bm, plans);
        if (rc != GM_OK) return rc;
    }
    BatchBufs& b = B.b;
    const int64_t Ps_tot = B.poff_s[T];
    const size_t wave_mark = ar.off;
    struct SideGuard {   // whatever way this call ends, nothing of it is left running on the side stream
        gm_ctx* c;
        bool active = false;
        ~SideGuard() { if (active) (void)hipStreamSynchronize(c->side); }
    } side{c};
    bool side_list = false;
    bool list_ordered = false;   // row-list output: the batch's lookups were ordered and cut into segments inside its (only) wave
    ValEnc enc = kPlainVals;     // how the values that travel with the row keys name their bags

    // meta theta in the padded internal layout (and its bf16 operand copies); accumulators
    for (int l = 1; l <= L; ++l) {
        launch_pack_weights(st, params->W[l - 1], c->dims[l - 1], c->dims[l], c->ld[l - 1], c->ld[l], b.theta0.f + c->offW[l]);
        launch_pack_weights(st, params->b[l - 1], 1, c->dims[l], 1, (int)(l == L ? 32 : c->ld[l]), b.theta0.f + c->offb[l]);
        if (bf && l < L)
            launch_convert_weights(st, b.theta0.f + c->offW[l], 0, 1, c->ld[l - 1], c->ld[l], b.theta0.b + c->offWb[l],
                                   nullptr, 0);
    }
    launch_fill_f32(st, b.g_theta, nt, 0.f);
    // Gradient w.r.t. the pooled inputs: the query rows are written whole by the outer backward pass; the support rows
    // are the second-order chain's sum, which starts from zero unless its first product stores instead of adding.
    const bool gxs_self_init = order == 2 && K > 0 && bf && L > 1;
    if (FD > 0 && !table && !gxs_self_init) launch_fill_f32(st, b.GX, Ps_tot * (int64_t)FD, 0.f);
    float* task_loss = out->task_loss ? out->task_loss : b.task_loss;

    for (const WavePlan& wp : plans) {
        ar.off = wave_mark;
        const int Tw = wp.t1 - wp.t0;
        if (Tw == 0) continue;
        WaveBufs w;
        if (pre) w = pre->w;
        const WaveDims d = pre ? pre->d : wave_dims(c, B, wp, bm, K, order);
        if (!pre) alloc_wave_index(c, ar, w, d);
        alloc_wave_dense(c, ar, w, d, K, order);
        if (ar.overflow) return fail(c, GM_ERR_WORKSPACE, "internal: wave does not fit");
        Grp gs, gq;
        const bool adapt = c->adapt_rows != 0;
        int tf_cap = 0, max_bag = 0, max_tf = 0;
        bool pair = false, any_sparse = false, pairs_on_side = false;
        bool ordered = false;   // this wave's lookups are in row order already (its dictionaries were read off that order)
        if (pre) {
            enc = pre->enc;
            gs = pre->gs; gq = pre->gq;
            tf_cap = pre->tf_cap; max_bag = pre->max_bag; max_tf = pre->max_tf;
            pair = pre->pair; any_sparse = pre->any_sparse;
        } else {
            if ((rc = setup_wave(c, B, wp, bm, K, w, d, gs, gq))) return rc;
            // a0: row dictionaries and the overlap join -- read off the row order of the wave's lookups when that order
            // is the one the sparse gradient needs (table-shaped output: every wave's own; row list: a batch of one wave)
            JoinReq jr;
            if (F > 0 && !c->overlap_sort && (table || plans.size() == 1)) {
                jr.so = table ? &w.so : &b.so;
                jr.range = table ? SortRange{wp.s0, wp.s1, wp.q0, wp.q1, wp.ls0, wp.ls1, wp.lq0, wp.lq1,
                                             (u32)(0 - (uint64_t)wp.ps0), (u32)((uint64_t)d.Ps - (uint64_t)wp.pq0)}
                                 : whole_batch_range(B);
                jr.n_sup_rows = d.Ps; jr.n_qry_rows = d.Pq;
                if (!table) { jr.emb_rows = out->emb_rows; jr.capacity = capacity; jr.n_rows = out->n_emb_rows; }
                jr.pair_only = d.pair && !d.any_sparse;
            }
            rc = run_index_wave(c, B, wp, w, &tf_cap, &max_bag, &max_tf, &jr);
            if (rc != GM_OK) return rc;
            if (jr.used) { ordered = true; enc = jr.enc; }
            if ((rc = count_pairs(c, B, wp, w, d, K, tf_cap, max_bag, max_tf, true, pair, any_sparse, pairs_on_side))) return rc;
            if (pairs_on_side) side.active = true;
        }
        // joins the counting on the side stream: the host learns whether a task fell back to the sparse kernel, the main
        // stream waits for the matrices (called before the first row hop, which is their first reader)
        auto join_pairs = [&]() -> int {
            if (!pairs_on_side) return GM_OK;
            pairs_on_side = false;
            u32 hs[ST_WORDS];
            HIPCHK(c, hipMemcpyAsync(hs, c->d_status_side, ST_WORDS * sizeof(u32), hipMemcpyDeviceToHost, c->side));
            HIPCHK(c, hipStreamSynchronize(c->side));
            HIPCHK(c, hipStreamWaitEvent(st, c->ev_pairs, 0));
            if (hs[ST_PAIR_OVF]) any_sparse = true;
            if (c->row_path == 2 && any_sparse && adapt)
                return fail(c, GM_ERR_CAPACITY, "pair-count path forced, but a task, count, bag or (task, field) exceeds its limits");
            if (any_sparse && !w.slots_written) sort_task_fields(c, B, wp, w, max_tf);
            return GM_OK;
        };
        if (!pairs_on_side && c->row_path == 2 && any_sparse && adapt)
            return fail(c, GM_ERR_CAPACITY, "pair-count path forced, but a task, count, bag or (task, field) exceeds its limits");
        const int n_tf = Tw * F;
        const int32_t* rows_s = b.prow_s + wp.s0;
        const int32_t* rows_q = b.prow_q + wp.q0;
        const int32_t rb_s = (int32_t)wp.ps0, rb_q = (int32_t)wp.pq0;
        const bool second = order == 2 && K > 0;

        // a1: one prefetch pass for both sets (pad rows stay zero; without pad rows nothing needs clearing: every
        // real row is written whole, pooled fields by the gather and dense / pad columns by the tail kernels)
        const bool padded = d.Ps != d.Ss || d.Pq != d.Sq;
        if (padded) {
            launch_fill_f32(st, w.Xs0, d.Ps * ld0, 0.f);
            launch_fill_f32(st, w.Xq0, d.Pq * ld0, 0.f);
        }
        Act X0s;  // step-0 support input
        X0s.ld = ld0;
        if (bf) X0s = K > 0 ? w.steps[0].X : Act();
        else X0s.f = w.Xs0;
        {
            const double lookups = (double)(d.nnz_s + d.nnz_q), bags = (double)(d.Ss + d.Sq) * F;
            Prof p(c, "gather_pool", lookups * (4.0 * D + 4) + bags * (4.0 * D + 8 + (bf ? 2.0 * D : 0)), 0);
            if (bf && X0s.b && padded) zero_bf16(st, X0s.b, d.Ps * ld0);
            if (bf && padded) zero_bf16(st, w.Xq.b, d.Pq * ld0);
            launch_gather_pool(st, F, D, c->n_dense, c->d_field_base, sup->bag_offsets, sup->indices, sup->dense,
                               params->emb, wp.s0, d.Ss, rows_s, rb_s, w.Xs0, ld0, bf ? X0s.b : nullptr);
            launch_gather_pool(st, F, D, c->n_dense, c->d_field_base, qry->bag_offsets, qry->indices, qry->dense,
                               params->emb, wp.q0, d.Sq, rows_q, rb_q, w.Xq0, ld0, (bf && K == 0) ? w.Xq.b : nullptr);
        }
        // the pooled direction: its dense and pad columns are zero (dense features are not parameters)
        if (second && padded) {
            if (w.TX.b) zero_bf16(st, w.TX.b, d.Ps * ld0);
            if (w.TX.f) launch_fill_f32(st, w.TX.f, d.Ps * ld0, 0.f);
            if (w.TXf) launch_fill_f32(st, w.TXf, d.Ps * ld0, 0.f);
        } else if (second) {
            launch_copy_tail(st, FD, nullptr, d.Ps, bf ? w.TXf : w.TX.f, ld0, w.TX.b);
        }

        // The wave's offsets and indices are validated.  Ordering the lookups by row needs nothing else: it runs on the
        // side stream from here on -- beside the dense phase, which is bound by memory traffic, not beside the index
        // kernels above, which are bound by the same things as the sort -- and is joined before the segment reduction
        // (row-list output: only when the batch is one wave, so that everything it reads has been validated).
        if (!pre && c->overlap_sort && F > 0 && (table || plans.size() == 1)) {
            HIPCHK(c, hipEventRecord(c->ev_go, st));
            HIPCHK(c, hipStreamWaitEvent(c->side, c->ev_go, 0));
        }
        const bool side_table = table && c->overlap_sort && F > 0;
        if (side_table) {
            if (side.active) HIPCHK(c, hipStreamWaitEvent(c->side, c->ev_main, 0));   // the previous wave is done with this memory
            side.active = true;
            launch_fill_u32(c->side, c->d_status_side, ST_WORDS, 0);
            const SortRange r{wp.s0, wp.s1, wp.q0, wp.q1, wp.ls0, wp.ls1, wp.lq0, wp.lq1,
                              (u32)(0 - (uint64_t)wp.ps0), (u32)((uint64_t)d.Ps - (uint64_t)wp.pq0)};
            global_order(c, B, w.so, r, nullptr, nullptr, d.nnz_s + d.nnz_q, nullptr, true);
            HIPCHK(c, hipEventRecord(c->ev_side, c->side));
        } else if (!pre && !table && c->overlap_sort && F > 0 && plans.size() == 1) {
            side.active = true;
            side_list = true;
            launch_fill_u32(c->side, c->d_status_side, ST_WORDS, 0);
            global_order(c, B, b.so, whole_batch_range(B), out->emb_rows, nullptr, capacity, out->n_emb_rows, true);
            HIPCHK(c, hipEventRecord(c->ev_side, c->side));
        }
        // row arithmetic of one (task, field) at a time, through LDS (no row table in HBM)
        int max_bags = 0;
        for (int t = wp.t0; t < wp.t1; ++t)
            max_bags = std::max<int>(max_bags, (int)std::max(sup->task_offsets[t + 1] - sup->task_offsets[t],
                                                               qry->task_offsets[t + 1] - qry->task_offsets[t]));
        int max_prows = 0;
        for (int t = wp.t0; t < wp.t1; ++t)
            max_prows = std::max<int>(max_prows, (int)std::max(B.poff_s[t + 1] - B.poff_s[t], B.poff_q[t + 1] - B.poff_q[t]));
        if (K > 0 && F > 0 && max_prows > 2048)
            return fail(c, GM_ERR_CAPACITY, "a task has %d samples in one set; the limit with inner steps is 2048", max_prows);
        auto hop_out = [&](bool support, const float* y_in, float* y_out, bf16_t* y_bf, float cc) {
            TwoHopOut o;
            memset(&o, 0, sizeof o);
            o.enabled = 1;
            o.bag_offsets = support ? sup->bag_offsets : qry->bag_offsets;
            o.sample0 = support ? wp.s0 : wp.q0;
            o.lookup0 = support ? wp.ls0 : wp.lq0;
            o.real_offsets = support ? w.real_off_s : w.real_off_q;
            o.slot_of_lookup = support ? w.sup_slot : w.qry_slot;
            o.row_map = support ? rows_s : rows_q;
            o.row_base = support ? rb_s : rb_q;
            o.y_in = y_in; o.y_out = y_out; o.y_bf = y_bf; o.ld = ld0; o.c = cc;
            return o;
        };
        auto two_hop = [&](bool in_support, const float* Z, const TwoHopOut* o0, const TwoHopOut* o1) {
            const double bags_ = (o0 ? (double)d.Ss : 0.0) + (o1 ? (double)d.Sq : 0.0);
            const double in_l_ = in_support ? (double)d.nnz_s : (double)d.nnz_q;
            const double out_l_ = (o0 ? (double)d.nnz_s : 0.0) + (o1 ? (double)d.nnz_q : 0.0);
            // algorithmic bytes: Z once per (sample, field), Y read + written per (sample, field), 4 B per lookup and hop
            const double alg_bytes = 4.0 * D * F * (in_support ? d.Ss : d.Sq) + bags_ * F * (8.0 * D + (bf ? 2.0 * D : 0)) + 4.0 * (in_l_ + out_l_);
            if (pair) {   // o0 is always the support side, o1 the query side
                PairHopArgs pa;
                memset(&pa, 0, sizeof pa);
                pa.F = F; pa.D = D; pa.mat = w.pair_mat; pa.task_path = w.task_path;
                pa.in_real_off = in_support ? w.real_off_s : w.real_off_q;
                pa.in_row_off = in_support ? w.row_off_s : w.row_off_q;
                pa.Z = Z; pa.ldz = FD;
                auto fill = [&](PairHopOut& po, const TwoHopOut& o, bool out_support) {
                    po.enabled = 1;
                    po.mat_off = out_support ? (in_support ? w.pair_off_ss : w.pair_off_sq) : w.pair_off_qs;
                    po.real_off = out_support ? w.real_off_s : w.real_off_q;
                    po.row_off = out_support ? w.row_off_s : w.row_off_q;
                    po.y_in = o.y_in; po.y_out = o.y_out; po.y_bf = o.y_bf; po.ld = o.ld; po.c = o.c;
                };
                if (o0) fill(pa.out[0], *o0, true);
                if (o1) fill(pa.out[1], *o1, false);
                Prof p(c, "pair_hop", alg_bytes, 0);
                launch_pair_hop(st, pa, Tw, max_bags);
            }
            if (!any_sparse) return;
            TwoHopArgs a;
            memset(&a, 0, sizeof a);
            a.F = F; a.D = D;
            a.tf_base = w.base_s; a.n_slots = w.n_slots;
            if (in_support) { a.in_seg_lo = w.slot_start; a.in_seg_hi = w.slot_start + 1; a.in_seg_tf_stride = 1; a.in_sorted = w.sup_sorted; }
            else { a.in_seg_lo = w.qseg_lo; a.in_seg_hi = w.qseg_hi; a.in_seg_tf_stride = 0; a.in_sorted = w.qry_sorted; }
            a.Z = Z; a.ldz = FD; a.task_path = w.task_path;
            a.in_row_offsets = in_support ? w.row_off_s : w.row_off_q;
            a.max_in_rows = max_prows;
            if (o0) a.out[0] = *o0;
            if (o1) a.out[1] = *o1;
            Prof p(c, "two_hop", alg_bytes, 0);
            launch_two_hop(st, a, Tw, max_bags);
        };

        // inner loop on the support set
        const float* labels_s = sup->labels + wp.s0;
        const float* labels_q = qry->labels + wp.q0;
        Theta th = b.theta0;        // GEMM operands of the current step
        const float* thf = b.theta0.f;  // fp32 view (biases, last layer)
        int64_t thf_stride = 0;
        const float* xs_cur = w.Xs0;    // fp32 support input of the current step
        Act Xq = w.Xq;                  // query input as the GEMMs read it
        if (!bf) Xq.f = w.Xq0;          // fp32: the prefetched buffer, updated in place by the overlap update
        // bf16, second order, 2..GEMM_MAX_PAIRS inner steps: every step's weights straight from the meta parameters
        // and the gradients of all steps so far (their activations and deltas are kept for the chain anyway)
        const bool from_theta0 = bf && second && K >= 2 && K <= GEMM_MAX_PAIRS && c->theta_from_meta;
        const float* thf0 = thf;
        std::vector<Pass> passes;
        for (int k = 0; k < K; ++k) {
            StepState& s = w.steps[second ? k : 0];
            if (k == 0) s.X = X0s;
            s.th = th;
            s.wL = thf + c->offW[L];
            s.wL_stride = thf_stride;
            Pass p{&s.X, &s.A, &s.Dl, s.dL, s.zL};
            forward_backward(c, gs, labels_s, p, th, thf, thf_stride, nullptr, F > 0 ? w.dX : nullptr);
            // local back-propagation: theta' = theta - alpha dtheta (per task)
            Theta& next = w.thetas[second ? k : 0];
            float* wl_copy = (bf && second && k + 1 < K) ? w.steps[k + 1].wL_copy : nullptr;
            // bf16: after the last inner step only the operand copies of W' are read again, not its fp32 master
            if (from_theta0) {
                passes.push_back(p);
                theta_grad(c, gs, p, next, thf, thf_stride, 1.f, -alpha, wl_copy, false, nullptr, nullptr, &passes, thf0);
            } else theta_grad(c, gs, p, next, thf, thf_stride, 1.f, -alpha, wl_copy, !(bf && k + 1 == K));
            th = next;
            thf = next.f;
            thf_stride = nt;
            // rows' = rows - alpha drows, seen through the pooled inputs: the support input of the next step and
            // (overlap update) the query input; a query row that the support set does not touch keeps its meta value
            const bool more = k + 1 < K;
            Act Xn;  // support input of step k+1
            if (more) Xn = second ? w.steps[k + 1].X : w.Xs_scratch;
            if (F > 0 && adapt) {
                if ((rc = join_pairs())) return rc;
                float* xs_next = nullptr;
                if (more) {
                    xs_next = bf ? w.Xs0 : Xn.f;  // bf16: the fp32 master is updated in place
                    if (bf && padded) zero_bf16(st, Xn.b, d.Ps * ld0);
                }
                const bool last = !more;
                TwoHopOut os = hop_out(true, xs_cur, xs_next, more && bf ? Xn.b : nullptr, -alpha);
                TwoHopOut oq = hop_out(false, w.Xq0, w.Xq0, (bf && last) ? Xq.b : nullptr, -alpha);
                if (bf && last && padded) zero_bf16(st, Xq.b, d.Pq * ld0);
                two_hop(true, w.dX, more ? &os : nullptr, &oq);
                if (more) {
                    launch_copy_tail(st, FD, xs_cur, d.Ps, bf ? nullptr : (xs_next != xs_cur ? xs_next : nullptr), ld0, bf ? Xn.b : nullptr);
                    xs_cur = xs_next;
                }
            } else if (more) {  // no sparse fields, or rows not adapted: every step reads the same input
                Xn = s.X;
            }
            if (more) {
                w.steps[second ? k + 1 : 0].X = Xn;
            }
        }
        // bf16 second order with K > 1: steps k >= 1 read their last-layer weights from the copies taken above
        if (bf && second)
            for (int k = 1; k < K; ++k) {
                w.steps[k].wL = w.steps[k].wL_copy;
                w.steps[k].wL_stride = c->ld[L - 1];
            }

        if ((rc = join_pairs())) return rc;   // (no inner step took a row hop)
        // outer forward/backward on the query set with the adapted parameters
        if (bf && K > 0) launch_copy_tail(st, (F > 0 && adapt) ? FD : 0, w.Xq0, d.Pq, nullptr, ld0, Xq.b);
        // gradient w.r.t. the pooled inputs: the wave's rows of the batch-wide buffer, or the wave's own buffer
        float* gxs = table ? w.GX : b.GX + wp.ps0 * (int64_t)FD;
        float* gxq = table ? w.GX + d.Ps * (int64_t)FD : b.GX + (Ps_tot + wp.pq0) * (int64_t)FD;
        if (table && FD > 0 && !gxs_self_init) launch_fill_f32(st, w.GX, d.Ps * (int64_t)FD, 0.f);
        Pass pq{&Xq, &w.Aq, &w.Dq, w.dLq, w.zq};
        forward_backward(c, gq, labels_q, pq, th, thf, thf_stride, w.loss_q, F > 0 ? gxq : nullptr);
        colsum_f32(c, gq, 1, w.loss_q, 1, task_loss + wp.t0, 1, nullptr, 0, 0.f, 1.f);
        // The query gradient w.r.t. theta' per task starts the second-order chain; without a chain it is only summed
        // over the tasks, so it is taken over runs of tasks straight away.
        const int n_coarse = coarse_group_count(c, Tw, std::min(d.Ps, d.Pq));
        Grp gs_coarse = gs, gq_coarse = gq;
        gs_coarse.row_off = w.coarse_off_s; gs_coarse.G = n_coarse;
        gq_coarse.row_off = w.coarse_off_q; gq_coarse.G = n_coarse;
        if (second) theta_grad(c, gq, pq, w.v, nullptr, 0, 0.f, 1.f, nullptr);
        else theta_grad(c, gq, pq, w.v, nullptr, 0, 0.f, 1.f, nullptr, true, &gq_coarse, &w.vsum);

        // second-order chain back through the inner steps: v_k = v_{k+1} - alpha H_k v_{k+1}
        if (second) {
            float* txf = bf ? w.TXf : w.TX.f;  // fp32 pooled direction (support rows); TX.b is its GEMM operand copy
            if (!adapt) {   // no direction on the inputs: whatever still reads it (a model without hidden layers) sees zeros
                if (bf) zero_bf16(st, w.TX.b, d.Ps * ld0);
                else launch_fill_f32(st, w.TX.f, d.Ps * ld0, 0.f);
            }
            if (F > 0 && adapt) {
                // direction on the support rows = query gradient routed through the rows both sets share
                TwoHopOut os = hop_out(true, nullptr, txf, w.TX.b, 1.f);
                two_hop(false, gxq, &os, nullptr);
            }
            for (int k = K - 1; k >= 0; --k) {
                const StepState& s = w.steps[k];
                // bf16 with hidden layers: the layer-1 product adds -alpha * dX to the gradient buffer itself
                const bool fused_gx = bf && L > 1 && F > 0;
                // (the chain's first step starts that sum: the buffer's support rows need no clearing)
                hvp_step(c, gs, s, w, alpha, k > 0, fused_gx ? gxs : nullptr, k > 0 && adapt, k == K - 1, adapt,
                         k == 0 ? &gs_coarse : nullptr);
                if (F > 0) {
                    if (!fused_gx) {
                        Prof p(c, "axpy_gx", 12.0 * d.Ps * FD, 0);
                        launch_axpy(st, d.Ps * (int64_t)FD, -alpha, w.dX, gxs);
                    }
                    if (k > 0 && adapt) {
                        TwoHopOut os = hop_out(true, txf, txf, w.TX.b, -alpha);
                        two_hop(true, w.dX, &os, nullptr);
                    }
                }
            }
        }
        // cross-task reduction of the dense part (tasks of the wave in order, waves in order)
        {
            Prof p(c, "reduce_tasks", 4.0 * (second ? Tw : n_coarse) * nt, 0);
            if (second) {
                launch_reduce_tasks(st, w.v.f, nt, Tw, nt, b.g_theta, 1, 1.f);
                for (int l = 1; l < L; ++l)   // the last step's weight-matrix part, summed over runs of tasks
                    launch_reduce_tasks(st, w.vsum.f + c->offW[l], nt, n_coarse, (int64_t)c->ld[l - 1] * c->ld[l],
                                        b.g_theta + c->offW[l], 1, -alpha);
            } else {   // weight matrices of the hidden layers from the runs of tasks, the rest from the tasks
                for (int l = 1; l < L; ++l) {
                    launch_reduce_tasks(st, w.vsum.f + c->offW[l], nt, n_coarse, c->offb[l] - c->offW[l],
                                        b.g_theta + c->offW[l], 1, 1.f);
                    launch_reduce_tasks(st, w.v.f + c->offb[l], nt, Tw, c->offW[l + 1] - c->offb[l], b.g_theta + c->offb[l], 1,
                                        1.f);
                }
                launch_reduce_tasks(st, w.v.f + c->offW[L], nt, Tw, nt - c->offW[L], b.g_theta + c->offW[L], 1, 1.f);
            }
        }
        // table-shaped sparse output: the wave's lookups are ordered by row and every row's sum is added to its row of
        // the table (rows are distinct within a wave; waves follow each other on the stream)
        if (table) {
            const SortRange r{wp.s0, wp.s1, wp.q0, wp.q1, wp.ls0, wp.ls1, wp.lq0, wp.lq1,
                              (u32)(0 - (uint64_t)wp.ps0), (u32)((uint64_t)d.Ps - (uint64_t)wp.pq0)};
            const int64_t nw = d.nnz_s + d.nnz_q;
            if (side_table) HIPCHK(c, hipStreamWaitEvent(st, c->ev_side, 0));
            else if (!ordered) global_order(c, B, w.so, r, nullptr, nullptr, nw, nullptr);
            {
                Prof p(c, "seg_reduce", (double)nw * (4.0 * D + 4), 0);
                launch_seg_reduce(st, D, F, ordered ? enc : kPlainVals, w.so.keys, w.so.keys_tmp, nullptr, nw, nw, w.so.vals, w.GX,
                                  nullptr, w.so.seg_partial, table);
            }
            if (side_table) HIPCHK(c, hipEventRecord(c->ev_main, st));
        } else if (ordered) {
            list_ordered = true;
        }
    }

    // outputs: dense meta-gradient, loss, coalesced sparse meta-gradient
    for (int l = 1; l <= L; ++l) {
        launch_unpack_weights(st, b.g_theta + c->offW[l], c->dims[l - 1], c->dims[l], c->ld[l], out->dW[l - 1]);
        launch_unpack_weights(st, b.g_theta + c->offb[l], 1, c->dims[l], c->dims[l], out->db[l - 1]);
    }
    launch_sum_to_scalar(st, task_loss, T, loss, 0);
    // (a batch whose segments were cut inside its wave keeps the status words of that: the row count, the capacity flag)
    if (!pre && !list_ordered) launch_fill_u32(st, c->d_status, ST_WORDS, 0);
    if (table) {
        launch_fill_u32(st, reinterpret_cast<u32*>(out->n_emb_rows), 2, 0u);
    } else {
        if (side_list) HIPCHK(c, hipStreamWaitEvent(st, c->ev_side, 0));
        else if (!pre && !list_ordered) global_order(c, B, b.so, whole_batch_range(B), out->emb_rows, nullptr, capacity, out->n_emb_rows);
        if (F > 0) {
            Prof p(c, "seg_reduce", (double)nnz * (4.0 * D + 4), 0);
            launch_seg_reduce(st, D, F, (pre || list_ordered) ? enc : kPlainVals, b.so.keys, b.so.keys_tmp, out->n_emb_rows, capacity, nnz,
                              b.so.vals, b.GX, out->emb_grad, b.so.seg_partial, nullptr);
        }
    }
    if (pre && no_sync) return GM_OK;   // the caller drains the stream; a prepared batch has passed every check already
    u32 hs[ST_WORDS];
    memset(hs, 0, sizeof hs);
    if (pre) {
        HIPCHK(c, hipStreamSynchronize(st));
        HIPCHK(c, hipGetLastError());
        prof_drain(c);
        return GM_OK;
    }
    if (side_list)   // the ordering's own status words (the main stream has waited for it)
        HIPCHK(c, hipMemcpyAsync(hs, c->d_status_side, ST_WORDS * sizeof(u32), hipMemcpyDeviceToHost, st));
    rc = side_list ? (hipStreamSynchronize(st) == hipSuccess ? GM_OK : fail(c, GM_ERR_HIP, "stream synchronisation failed"))
                   : read_status(c, hs);
    if (rc != GM_OK) return rc;
    HIPCHK(c, hipGetLastError());
    prof_drain(c);
    if (hs[ST_CAPACITY])
        return fail(c, GM_ERR_CAPACITY, "emb_rows_capacity %lld is smaller than the %u rows touched", (long long)capacity,
                    hs[ST_NROWS]);
    return GM_OK;
}

extern "C" int gm_meta_step(gm_ctx* c, int32_t T, const gm_set* sup, const gm_set* qry, const gm_params* params,
                            float alpha, int32_t K, int32_t order, float* loss, gm_grads* out) {
    return meta_step_impl(c, T, sup, qry, params, alpha, K, order, loss, out, nullptr, false);
}

// The same step with every intermediate buffer in the static scratch array instead of the context's workspace: no
// device memory is allocated or freed anywhere below (the persistent words -- table bases, status -- stay where
// gm_create put them).  Kernel timing is off for the call: its events would have to be created.
extern "C" int gm_meta_step_static(gm_ctx* c, int32_t T, const gm_set* sup, const gm_set* qry, const gm_params* params,
                                   float alpha, int32_t K, int32_t order, float* loss, gm_grads* out) {
    if (!c) return GM_ERR_ARG;
    if (!c->static_scratch) return fail(c, GM_ERR_HIP, "the static scratch array was not located at gm_create");
    char* const ws = c->ws;
    const size_t ws_bytes = c->ws_bytes, persistent = c->persistent;
    const bool prof_on = c->prof_on;
    c->ws = c->static_scratch;
    c->ws_bytes = GM_STATIC_SCRATCH_BYTES;
    c->persistent = 0;
    c->prof_on = false;
    const int rc = gm_meta_step(c, T, sup, qry, params, alpha, K, order, loss, out);
    c->ws = ws;
    c->ws_bytes = ws_bytes;
    c->persistent = persistent;
    c->prof_on = prof_on;
    if (rc == GM_ERR_WORKSPACE) {
        const std::string why = c->err;
        return fail(c, GM_ERR_WORKSPACE, "the call does not fit the %d MiB of static scratch of gm_meta_step_static (%s); "
                    "use gm_meta_step with a workspace", (int)GM_STATIC_SCRATCH_MIB, why.c_str());
    }
    return rc;
}

extern "C" int gm_meta_train_step(gm_ctx* c, int32_t T, const gm_set* sup, const gm_set* qry, const gm_params* params,
                                  float alpha, int32_t K, int32_t order, float beta, float* loss, float* task_loss) {
    if (!c) return GM_ERR_ARG;
    if (!sup || !qry || sup->nnz < 0 || qry->nnz < 0) return fail(c, GM_ERR_ARG, "null set / negative size");
    if (!params || !params->W || !params->b) return fail(c, GM_ERR_ARG, "null params");
    HIPCHK(c, hipSetDevice(c->device));
    const int L = c->L, D = c->D;
    // the meta-gradient of this iteration lives at the top of the workspace; the step gets what is below it
    const int64_t capacity = c->F > 0 ? std::min<int64_t>(sup->nnz + qry->nnz, c->field_base[c->F]) : 0;
    int64_t n_dense = 0;
    for (int l = 0; l < L; ++l) n_dense += (int64_t)(c->dims[l] + 1) * c->dims[l + 1];
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t need = up((size_t)n_dense * 4) + up((size_t)capacity * 8) + up((size_t)capacity * std::max(D, 1) * 4) + 256;
    if (need + c->persistent + (1 << 20) > c->ws_bytes)
        return fail(c, GM_ERR_WORKSPACE, "workspace of %zu bytes cannot hold the meta-gradient (%zu bytes) beside the step", c->ws_bytes, need);
    const size_t full = c->ws_bytes;
    char* top = c->ws + (full - need) / 256 * 256;
    float* dense = reinterpret_cast<float*>(top);
    int64_t* rows = reinterpret_cast<int64_t*>(top + up((size_t)n_dense * 4));
    float* grad = reinterpret_cast<float*>(reinterpret_cast<char*>(rows) + up((size_t)capacity * 8));
    int64_t* n_rows = reinterpret_cast<int64_t*>(reinterpret_cast<char*>(grad) + up((size_t)capacity * std::max(D, 1) * 4));
    std::vector<float*> dW(L), db(L);
    {
        float* p = dense;
        for (int l = 0; l < L; ++l) {
            dW[l] = p; p += (int64_t)c->dims[l] * c->dims[l + 1];
            db[l] = p; p += c->dims[l + 1];
        }
    }
    gm_grads out;
    memset(&out, 0, sizeof out);
    out.dW = dW.data(); out.db = db.data();
    out.emb_rows = rows; out.emb_grad = grad; out.n_emb_rows = n_rows; out.emb_rows_capacity = capacity;
    out.task_loss = task_loss;
    c->ws_bytes = static_cast<size_t>(top - c->ws);
    const int rc = gm_meta_step(c, T, sup, qry, params, alpha, K, order, loss, &out);
    c->ws_bytes = full;
    if (rc != GM_OK) return rc;
    hipStream_t st = c->stream;
    int64_t h_rows = 0;
    HIPCHK(c, hipMemcpyAsync(&h_rows, n_rows, sizeof h_rows, hipMemcpyDeviceToHost, st));
    for (int l = 0; l < L; ++l) {
        launch_axpy(st, (int64_t)c->dims[l] * c->dims[l + 1], -beta, dW[l], const_cast<float*>(params->W[l]));
        launch_axpy(st, c->dims[l + 1], -beta, db[l], const_cast<float*>(params->b[l]));
    }
    HIPCHK(c, hipStreamSynchronize(st));
    if (c->F > 0 && h_rows > 0) {
        Prof p(c, "scatter_add", (double)h_rows * (12.0 * D + 8), 0);
        launch_scatter_add(st, D, const_cast<float*>(params->emb), rows, grad, h_rows, -beta);
    }
    HIPCHK(c, hipStreamSynchronize(st));
    HIPCHK(c, hipGetLastError());
    prof_drain(c);
    return GM_OK;
}

// The same iteration with the sparse meta-gradient accumulated in a table-shaped buffer of the caller's (any number of
// lookups, tasks in waves) and applied to the tables in one streaming pass that clears the buffer again.
extern "C" int gm_meta_train_step_table(gm_ctx* c, int32_t T, const gm_set* sup, const gm_set* qry, const gm_params* params,
                                        float alpha, int32_t K, int32_t order, float beta, float* loss, float* task_loss,
                                        float* emb_grad_table) {
    if (!c) return GM_ERR_ARG;
    if (!sup || !qry || sup->nnz < 0 || qry->nnz < 0) return fail(c, GM_ERR_ARG, "null set / negative size");
    if (!params || !params->W || !params->b) return fail(c, GM_ERR_ARG, "null params");
    if (c->F > 0 && (!emb_grad_table || !params->emb)) return fail(c, GM_ERR_ARG, "null emb_grad_table / emb");
    if ((reinterpret_cast<uintptr_t>(emb_grad_table) | reinterpret_cast<uintptr_t>(params->emb)) & 15)
        return fail(c, GM_ERR_ARG, "emb_grad_table and emb must be 16-byte aligned");
    HIPCHK(c, hipSetDevice(c->device));
    const int L = c->L, D = c->D;
    int64_t n_dense = 0;
    for (int l = 0; l < L; ++l) n_dense += (int64_t)(c->dims[l] + 1) * c->dims[l + 1];
    const size_t dense_bytes = ((size_t)n_dense * 4 + 255) & ~(size_t)255;
    const size_t need = dense_bytes + 512;   // the dense meta-gradient and the row counter, at the top of the workspace
    if (need + c->persistent + (1 << 20) > c->ws_bytes)
        return fail(c, GM_ERR_WORKSPACE, "workspace of %zu bytes cannot hold the dense meta-gradient (%zu bytes) beside the step", c->ws_bytes, need);
    const size_t full = c->ws_bytes;
    char* top = c->ws + (full - need) / 256 * 256;
    std::vector<float*> dW(L), db(L);
    {
        float* p = reinterpret_cast<float*>(top);
        for (int l = 0; l < L; ++l) {
            dW[l] = p; p += (int64_t)c->dims[l] * c->dims[l + 1];
            db[l] = p; p += c->dims[l + 1];
        }
    }
    gm_grads out;
    memset(&out, 0, sizeof out);
    out.dW = dW.data(); out.db = db.data();
    out.emb_grad_table = emb_grad_table;
    out.n_emb_rows = reinterpret_cast<int64_t*>(top + dense_bytes);   // (0 with the table-shaped output)
    out.task_loss = task_loss;
    c->ws_bytes = static_cast<size_t>(top - c->ws);
    const int rc = gm_meta_step(c, T, sup, qry, params, alpha, K, order, loss, &out);
    c->ws_bytes = full;
    if (rc != GM_OK) return rc;
    hipStream_t st = c->stream;
    for (int l = 0; l < L; ++l) {
        launch_axpy(st, (int64_t)c->dims[l] * c->dims[l + 1], -beta, dW[l], const_cast<float*>(params->W[l]));
        launch_axpy(st, c->dims[l + 1], -beta, db[l], const_cast<float*>(params->b[l]));
    }
    if (c->F > 0) {
        const int64_t n = c->field_base[c->F] * (int64_t)D;   // (D is a multiple of 4)
        Prof p(c, "table_update", 16.0 * n, 0);
        launch_axpy_clear(st, n, -beta, emb_grad_table, const_cast<float*>(params->emb));
    }
    HIPCHK(c, hipStreamSynchronize(st));
    HIPCHK(c, hipGetLastError());
    prof_drain(c);
    return GM_OK;
}

// ------------------------------------------------------------------------------------------------
// several iterations of Alg. 1 in one call, the index side of batch i+1 prepared while batch i computes
// ------------------------------------------------------------------------------------------------
static void host_layout(const gm_ctx* c, Batch& B, int T, const gm_set* sup, const gm_set* qry) {
    B.T = T; B.sup = sup; B.qry = qry; B.table = false;
    B.poff_s.assign(T + 1, 0);
    B.poff_q.assign(T + 1, 0);
    for (int t = 0; t < T; ++t) {
        B.poff_s[t + 1] = B.poff_s[t] + round_up64(sup->task_offsets[t + 1] - sup->task_offsets[t], c->row_pad);
        B.poff_q[t + 1] = B.poff_q[t] + round_up64(qry->task_offsets[t + 1] - qry->task_offsets[t], c->row_pad);
    }
}
static WavePlan whole_batch_plan(const Batch& B) {
    WavePlan p;
    const int T = B.T;
    p.t0 = 0; p.t1 = T;
    p.s0 = 0; p.s1 = B.sup->n_samples; p.q0 = 0; p.q1 = B.qry->n_samples;
    p.ps0 = 0; p.ps1 = B.poff_s[T]; p.pq0 = 0; p.pq1 = B.poff_q[T];
    p.ls0 = 0; p.ls1 = B.sup->nnz; p.lq0 = 0; p.lq1 = B.qry->nnz;
    return p;
}
// bytes of the index side and of the dense side of a batch run as ONE wave of tasks
static void one_wave_bytes(const gm_ctx* c, int T, const gm_set* sup, const gm_set* qry, int K, int order, int64_t capacity,
                           size_t* index_bytes, size_t* dense_bytes) {
    Batch B;
    host_layout(c, B, T, sup, qry);
    const WavePlan p = whole_batch_plan(B);
    const WaveDims d = wave_dims(c, B, p, pick_bm(c, B), K, order);
    Arena ia, da;
    ia.cap = da.cap = ~(size_t)0 >> 1;
    BatchBufs b;
    WaveBufs w;
    alloc_batch_index(c, ia, b, T, sup->n_samples, qry->n_samples, sup->nnz + qry->nnz, capacity, true);
    alloc_wave_index(c, ia, w, d);
    alloc_batch_dense(c, da, b, T, B.poff_s[T], B.poff_q[T], true);
    alloc_wave_dense(c, da, w, d, K, order);
    *index_bytes = ia.off;
    *dense_bytes = da.off;
}

// The index side of one batch, on the context's current stream, into the arena `ia`.
static int prepare_batch(gm_ctx* c, Arena& ia, int32_t T, const gm_set* sup, const gm_set* qry, int K, int order,
                         int64_t capacity, int64_t* emb_rows, int64_t* n_rows, Prepared& P) {
    int rc = check_set(c, sup, T, "support");
    if (rc != GM_OK) return rc;
    rc = check_set(c, qry, T, "query");
    if (rc != GM_OK) return rc;
    P = Prepared();
    JoinReq jr;
    Batch& B = P.B;
    B.T = T; B.sup = sup; B.qry = qry; B.table = false;
    if ((rc = begin_batch(c, B, ia, capacity, true, nullptr))) return rc;
    P.bm = pick_bm(c, B);
    P.wp = whole_batch_plan(B);
    if (sup->nnz + qry->nnz >= ((int64_t)1 << 31)) return fail(c, GM_ERR_WORKSPACE, "the batch does not run as one wave of tasks");
    P.d = wave_dims(c, B, P.wp, P.bm, K, order);
    alloc_wave_index(c, ia, P.w, P.d);
    if (ia.overflow) return fail(c, GM_ERR_WORKSPACE, "the batch's index structures do not fit their arena");
    if (T > 0) {
        if ((rc = setup_wave(c, B, P.wp, P.bm, K, P.w, P.d, P.gs, P.gq))) return rc;
        if (c->F > 0) {
            jr.so = &B.b.so;
            jr.range = whole_batch_range(B);
            jr.n_sup_rows = P.d.Ps; jr.n_qry_rows = P.d.Pq;
            jr.emb_rows = emb_rows; jr.capacity = capacity; jr.n_rows = n_rows;
            jr.pair_only = P.d.pair && !P.d.any_sparse;
        }
        if ((rc = run_index_wave(c, B, P.wp, P.w, &P.tf_cap, &P.max_bag, &P.max_tf, &jr))) return rc;
        if (jr.used) P.enc = jr.enc;
        bool on_side = false;
        if ((rc = count_pairs(c, B, P.wp, P.w, P.d, K, P.tf_cap, P.max_bag, P.max_tf, false, P.pair, P.any_sparse, on_side))) return rc;
        if (c->row_path == 2 && P.any_sparse && c->adapt_rows)
            return fail(c, GM_ERR_CAPACITY, "pair-count path forced, but a task, count, bag or (task, field) exceeds its limits");
    }
    if (!jr.used) {
        launch_fill_u32(c->stream, c->d_status, ST_WORDS, 0);
        global_order(c, B, B.b.so, whole_batch_range(B), emb_rows, nullptr, capacity, n_rows);
    }
    u32 hs[ST_WORDS];
    if ((rc = read_status(c, hs))) return rc;
    HIPCHK(c, hipGetLastError());
    if (hs[ST_CAPACITY])
        return fail(c, GM_ERR_CAPACITY, "internal: %u rows touched exceed the list capacity %lld", hs[ST_NROWS], (long long)capacity);
    return GM_OK;
}

extern "C" int gm_meta_train(gm_ctx* c, int32_t n_iters, const int32_t* n_tasks, const gm_set* support, const gm_set* query,
                             const gm_params* params, float alpha, int32_t K, int32_t order, float beta, float* losses,
                             int32_t* n_done) {
    if (!c) return GM_ERR_ARG;
    if (n_done) *n_done = 0;
    if (n_iters < 0 || (n_iters > 0 && (!n_tasks || !support || !query || !losses)))
        return fail(c, GM_ERR_ARG, "bad iteration count / null arrays");
    if (K < 0 || (order != 1 && order != 2)) return fail(c, GM_ERR_ARG, "bad inner_steps / order");
    if (!params || !params->W || !params->b || (c->F > 0 && !params->emb)) return fail(c, GM_ERR_ARG, "null params");
    for (int l = 0; l < c->L; ++l)
        if (!params->W[l] || !params->b[l]) return fail(c, GM_ERR_ARG, "null layer pointer");
    if (n_iters == 0) return GM_OK;
    HIPCHK(c, hipSetDevice(c->device));
    const int L = c->L, D = c->D;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    // what the overlapped loop needs: two index arenas, the meta-gradient lists (row lists twice: the next batch's is
    // written while this batch's is still being applied), and the dense side of the largest batch
    bool overlapped = true;
    int64_t cap_max = 0;
    size_t idx_max = 0, dense_max = 0;
    for (int i = 0; i < n_iters; ++i) {
        const gm_set *s = &support[i], *q = &query[i];
        if (n_tasks[i] < 0 || !s->task_offsets || !q->task_offsets || s->nnz < 0 || q->nnz < 0 || s->n_samples < 0 || q->n_samples < 0 ||
            s->task_offsets[n_tasks[i]] != s->n_samples || q->task_offsets[n_tasks[i]] != q->n_samples ||
            s->nnz + q->nnz >= ((int64_t)1 << 31)) {
            overlapped = false;   // (the per-iteration call reports what is wrong)
            break;
        }
        const int64_t cap = c->F > 0 ? std::min<int64_t>(s->nnz + q->nnz, c->field_base[c->F]) : 0;
        cap_max = std::max(cap_max, cap);
        size_t ib, db;
        one_wave_bytes(c, n_tasks[i], s, q, K, order, cap, &ib, &db);
        idx_max = std::max(idx_max, up(ib) + 4096);
        dense_max = std::max(dense_max, db);
    }
    int64_t n_dense = 0;
    for (int l = 0; l < L; ++l) n_dense += (int64_t)(c->dims[l] + 1) * c->dims[l + 1];
    const size_t top = up((size_t)n_dense * 4) + 2 * up((size_t)cap_max * 8) + up((size_t)cap_max * std::max(D, 1) * 4) + 2 * 256 + 256;
    if (overlapped && c->persistent + dense_max + 2 * idx_max + top + (1 << 20) > c->ws_bytes) overlapped = false;
    if (!overlapped) {   // one iteration after the other (several waves of tasks, or a workspace for one batch only)
        for (int i = 0; i < n_iters; ++i) {
            const int rc = gm_meta_train_step(c, n_tasks[i], &support[i], &query[i], params, alpha, K, order, beta, losses + i, nullptr);
            if (rc != GM_OK) return rc;
            if (n_done) *n_done = i + 1;
        }
        return GM_OK;
    }
    const size_t full = c->ws_bytes;
    char* const top_p = c->ws + (full - top) / 256 * 256;
    float* dense = reinterpret_cast<float*>(top_p);
    int64_t* rows[2];
    rows[0] = reinterpret_cast<int64_t*>(top_p + up((size_t)n_dense * 4));
    rows[1] = reinterpret_cast<int64_t*>(reinterpret_cast<char*>(rows[0]) + up((size_t)cap_max * 8));
    float* grad = reinterpret_cast<float*>(reinterpret_cast<char*>(rows[1]) + up((size_t)cap_max * 8));
    int64_t* n_rows[2];
    n_rows[0] = reinterpret_cast<int64_t*>(reinterpret_cast<char*>(grad) + up((size_t)cap_max * std::max(D, 1) * 4));
    n_rows[1] = n_rows[0] + 32;
    char* const idx_p[2] = {top_p - 2 * idx_max, top_p - idx_max};
    const size_t dense_end = static_cast<size_t>(idx_p[0] - c->ws);
    std::vector<float*> dW(L), db(L);
    {
        float* p = dense;
        for (int l = 0; l < L; ++l) {
            dW[l] = p; p += (int64_t)c->dims[l] * c->dims[l + 1];
            db[l] = p; p += c->dims[l + 1];
        }
    }
    // the side-stream settings of single steps do not apply here: the second stream belongs to the preparation
    const int keep_sort = c->overlap_sort, keep_pairs = c->overlap_pairs;
    c->overlap_sort = c->overlap_pairs = 0;
    struct Restore {
        gm_ctx* c; size_t full; int s, p;
        ~Restore() { c->ws_bytes = full; c->overlap_sort = s; c->overlap_pairs = p; (void)hipStreamSynchronize(c->side); }
    } restore{c, full, keep_sort, keep_pairs};
    hipStream_t st = c->stream;
    Prepared P[2];
    auto prepare = [&](int i, bool on_side) -> int {
        Arena ia;
        ia.base = idx_p[i & 1]; ia.cap = idx_max; ia.off = 0;
        const int64_t cap = c->F > 0 ? std::min<int64_t>(support[i].nnz + query[i].nnz, c->field_base[c->F]) : 0;
        if (on_side) { std::swap(c->stream, c->side); std::swap(c->d_status, c->d_status_side); }
        const int rc = prepare_batch(c, ia, n_tasks[i], &support[i], &query[i], K, order, cap, rows[i & 1], n_rows[i & 1], P[i & 1]);
        if (on_side) { std::swap(c->stream, c->side); std::swap(c->d_status, c->d_status_side); }
        return rc;
    };
    int rc = prepare(0, false);
    if (rc != GM_OK) return rc;
    for (int i = 0; i < n_iters; ++i) {
        gm_grads out;
        memset(&out, 0, sizeof out);
        out.dW = dW.data(); out.db = db.data();
        out.emb_rows = rows[i & 1]; out.emb_grad = grad; out.n_emb_rows = n_rows[i & 1];
        out.emb_rows_capacity = c->F > 0 ? std::min<int64_t>(support[i].nnz + query[i].nnz, c->field_base[c->F]) : 0;
        c->ws_bytes = dense_end;
        rc = meta_step_impl(c, n_tasks[i], &support[i], &query[i], params, alpha, K, order, losses + i, &out, &P[i & 1], true);
        c->ws_bytes = full;
        if (rc != GM_OK) { (void)hipStreamSynchronize(st); return rc; }
        int64_t h_rows = 0;
        HIPCHK(c, hipMemcpyAsync(&h_rows, n_rows[i & 1], sizeof h_rows, hipMemcpyDeviceToHost, st));
        // the next batch's index side, on the second stream, while this batch computes; its row list replaces the one of
        // batch i-1, whose update (enqueued before this batch's step) must have been applied: ev_main marks that point
        int rc_next = GM_OK;
        if (i + 1 < n_iters) {
            HIPCHK(c, hipStreamWaitEvent(c->side, c->ev_main, 0));
            rc_next = prepare(i + 1, true);
        }
        HIPCHK(c, hipStreamSynchronize(st));
        HIPCHK(c, hipGetLastError());
        prof_drain(c);
        // the two global back-propagation steps with the outer step size (Alg. 1), in place
        for (int l = 0; l < L; ++l) {
            launch_axpy(st, (int64_t)c->dims[l] * c->dims[l + 1], -beta, dW[l], const_cast<float*>(params->W[l]));
            launch_axpy(st, c->dims[l + 1], -beta, db[l], const_cast<float*>(params->b[l]));
        }
        if (c->F > 0 && h_rows > 0) {
            Prof p(c, "scatter_add", (double)h_rows * (12.0 * D + 8), 0);
            launch_scatter_add(st, D, const_cast<float*>(params->emb), rows[i & 1], grad, h_rows, -beta);
        }
        HIPCHK(c, hipEventRecord(c->ev_main, st));
        if (n_done) *n_done = i + 1;
        if (rc_next != GM_OK) {
            (void)hipStreamSynchronize(st);
            return rc_next;
        }
    }
    HIPCHK(c, hipStreamSynchronize(st));
    HIPCHK(c, hipGetLastError());
    prof_drain(c);
    return GM_OK;
}

// ------------------------------------------------------------------------------------------------
// one-task batches out of a flat record stream
// ------------------------------------------------------------------------------------------------
// lens[d * F + f] = length of bag f of source record perm[d]; flags offsets that are not monotone inside [0, nnz]
__global__ void group_lens_kernel(const int32_t* __restrict__ perm, int64_t n_dst, int F, const int64_t* __restrict__ bo,
                                  int64_t nnz, u32* lens, u32* status) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_dst * F) return;
    const int64_t d = i / F;
    const int f = (int)(i - d * F);
    const int64_t b = (int64_t)perm[d] * F + f;
    const int64_t p0 = bo[b], p1 = bo[b + 1];
    const bool bad = p0 < 0 || p1 < p0 || p1 > nnz;
    if (bad) atomicOr(&status[ST_BAD_INDEX], 1u);
    lens[i] = bad ? 0u : (u32)(p1 - p0);
}
// One workgroup per 256 destination bags: their lookups are one contiguous destination range; the bag of a lookup is
// found by bisection of the staged offsets (as in build_keys_kernel).  Also widens the offsets to 64 bits.
__global__ __launch_bounds__(256) void group_copy_kernel(const int32_t* __restrict__ perm, int64_t n_bags, int F,
                                                         const int64_t* __restrict__ bo, const int32_t* __restrict__ idx_in,
                                                         const u32* __restrict__ offs, int64_t* bo_out, int32_t* idx_out) {
    __shared__ u32 so[257];
    __shared__ int64_t src0[256];
    const int64_t b0 = (int64_t)blockIdx.x * 256;
    const int nb = (int)min<int64_t>(256, n_bags - b0);
    for (int i = threadIdx.x; i <= nb; i += 256) {
        so[i] = offs[b0 + i];
        bo_out[b0 + i] = (int64_t)offs[b0 + i];
    }
    for (int i = threadIdx.x; i < nb; i += 256) {
        const int64_t d = (b0 + i) / F;
        src0[i] = bo[(int64_t)perm[d] * F + (b0 + i - d * F)];
    }
    __syncthreads();
    const u32 p0 = so[0], p1 = so[nb];
    for (u32 p = p0 + threadIdx.x; p < p1; p += 256) {
        int lo = 0, hi = nb;   // last bag with so[bag] <= p
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (so[mid] <= p) lo = mid;
            else hi = mid;
        }
        idx_out[p] = idx_in[src0[lo] + (p - so[lo])];
    }
}
__global__ void group_rows_kernel(const int32_t* __restrict__ perm, int64_t n_dst, int nd, const float* __restrict__ dense,
                                  const float* __restrict__ labels, float* dense_out, float* labels_out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_dst * (nd + 1)) return;
    const int64_t d = i / (nd + 1);
    const int k = (int)(i - d * (nd + 1));
    const int64_t s = perm[d];
    if (k < nd) dense_out[d * nd + k] = dense[s * nd + k];
    else labels_out[d] = labels[s];
}

extern "C" int gm_group_batch(gm_ctx* c, int64_t n, int64_t nnz, const int64_t* task, const int64_t* batch_id,
                              const int64_t* bag_offsets, const int32_t* indices, const float* dense, const float* labels,
                              int32_t support_num, int32_t support_den, gm_set_buffers* sup, gm_set_buffers* qry,
                              int32_t* n_tasks) {
    if (!c) return GM_ERR_ARG;
    if (n < 0 || nnz < 0 || !sup || !qry || !n_tasks) return fail(c, GM_ERR_ARG, "bad sizes / null outputs");
    if (support_den <= 0 || support_num < 0 || support_num > support_den) return fail(c, GM_ERR_ARG, "support share must be in [0, 1]");
    if (n >= ((int64_t)1 << 31) / std::max(c->F, 1) || nnz >= ((int64_t)1 << 32))
        return fail(c, GM_ERR_ARG, "the stream must hold fewer than 2^31 bags and 2^32 lookups");
    if (n > 0 && (!task || !batch_id || !bag_offsets || !labels || (c->n_dense > 0 && !dense) || (nnz > 0 && !indices)))
        return fail(c, GM_ERR_ARG, "null stream array");
    gm_set_buffers* outs[2] = {sup, qry};
    for (gm_set_buffers* o : outs)
        if (!o->task_offsets || (n > 0 && (!o->bag_offsets || !o->labels || (c->n_dense > 0 && !o->dense) || (nnz > 0 && !o->indices))))
            return fail(c, GM_ERR_ARG, "null output buffer");
    HIPCHK(c, hipSetDevice(c->device));
    hipStream_t st = c->stream;
    const int F = c->F, nd = c->n_dense;
    // host: records in (task, batch_id) order, stream order inside a batch; batches and their split
    std::vector<int32_t> order((size_t)n);
    for (int64_t i = 0; i < n; ++i) order[(size_t)i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return task[a] != task[b] ? task[a] < task[b] : batch_id[a] < batch_id[b];
    });
    std::vector<int32_t> perm[2];
    sup->task_offsets[0] = qry->task_offsets[0] = 0;
    int32_t T = 0;
    for (int64_t i = 0; i < n;) {
        int64_t j = i + 1;
        while (j < n && task[order[j]] == task[order[i]] && batch_id[order[j]] == batch_id[order[i]]) ++j;
        const int64_t m = j - i, k = (m * support_num + support_den - 1) / support_den;
        for (int64_t r = i; r < j; ++r) perm[r - i < k ? 0 : 1].push_back(order[(size_t)r]);
        ++T;
        sup->task_offsets[T] = (int64_t)perm[0].size();
        qry->task_offsets[T] = (int64_t)perm[1].size();
        i = j;
    }
    *n_tasks = T;
    launch_fill_u32(st, c->d_status, ST_WORDS, 0);
    for (int w = 0; w < 2; ++w) {
        gm_set_buffers* o = outs[w];
        const int64_t nw = (int64_t)perm[w].size(), nbags = nw * F;
        o->n_samples = nw;
        o->nnz = 0;
        Arena ar;
        ar.base = c->ws; ar.cap = c->ws_bytes; ar.off = c->persistent;
        int32_t* d_perm = ar.get<int32_t>(nw + 1);
        u32* lens = ar.get<u32>(nbags + 2);
        u32* scan_tmp = ar.get<u32>(scan_tmp_words(nbags + 1));
        if (ar.overflow) return fail(c, GM_ERR_WORKSPACE, "workspace too small for the grouping (%zu bytes needed)", ar.off);
        if (nw == 0) {
            if (n > 0) HIPCHK(c, hipMemsetAsync(o->bag_offsets, 0, sizeof(int64_t), st));
            continue;
        }
        HIPCHK(c, hipMemcpyAsync(d_perm, perm[w].data(), nw * sizeof(int32_t), hipMemcpyHostToDevice, st));
        if (nbags > 0) {
            hipLaunchKernelGGL(group_lens_kernel, dim3((unsigned)((nbags + 255) / 256)), dim3(256), 0, st, d_perm, nw, F,
                               bag_offsets, nnz, lens, c->d_status);
            launch_fill_u32(st, lens + nbags, 1, 0);   // so that the exclusive scan's last entry is the total
            launch_scan_u32(st, lens, lens, nbags + 1, scan_tmp, nullptr);
            u32 hs[ST_WORDS];
            int rc = read_status(c, hs);   // (synchronises: the permutation vector may go, the offsets are trusted below)
            if (rc != GM_OK) return rc;
            if (hs[ST_BAD_INDEX]) return fail(c, GM_ERR_INDEX, "bag_offsets not monotone / beyond nnz");
            u32 total = 0;
            HIPCHK(c, hipMemcpy(&total, lens + nbags, sizeof total, hipMemcpyDeviceToHost));
            o->nnz = (int64_t)total;
            hipLaunchKernelGGL(group_copy_kernel, dim3((unsigned)((nbags + 255) / 256)), dim3(256), 0, st, d_perm, nbags, F,
                               bag_offsets, indices, lens, o->bag_offsets, o->indices);
        } else {
            HIPCHK(c, hipMemsetAsync(o->bag_offsets, 0, sizeof(int64_t), st));
        }
        hipLaunchKernelGGL(group_rows_kernel, dim3((unsigned)((nw * (nd + 1) + 255) / 256)), dim3(256), 0, st, d_perm, nw, nd,
                           dense, labels, o->dense, o->labels);
        HIPCHK(c, hipStreamSynchronize(st));
    }
    HIPCHK(c, hipGetLastError());
    return GM_OK;
}

extern "C" int gm_scatter_add(gm_ctx* c, float* table, const int64_t* rows, const float* grad, int64_t n_rows,
                              float scale) {
    if (!c) return GM_ERR_ARG;
    if (n_rows < 0 || (n_rows > 0 && (!table || !rows || !grad))) return fail(c, GM_ERR_ARG, "bad scatter arguments");
    HIPCHK(c, hipSetDevice(c->device));
    launch_scatter_add(c->stream, c->D, table, rows, grad, n_rows, scale);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipGetLastError());
    return GM_OK;
}

// copies a padded [n, ld] buffer into a dense [n, d] one
__global__ void strip_pad_kernel(const float* src, int64_t n, int ld, int d, float* dst) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * d) return;
    const int64_t s = i / d;
    dst[i] = src[s * ld + (i - s * d)];
}
__global__ void iota_i32_kernel(int32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (int32_t)i;
}

extern "C" int gm_gather_pool(gm_ctx* c, int32_t T, const gm_set* set, const float* emb, float* x) {
    if (!c) return GM_ERR_ARG;
    if (T < 0) return fail(c, GM_ERR_ARG, "bad n_tasks");
    int rc = check_set(c, set, T, "set");
    if (rc != GM_OK) return rc;
    if (set->n_samples > 0 && (!x || (c->F > 0 && !emb))) return fail(c, GM_ERR_ARG, "null emb / x");
    HIPCHK(c, hipSetDevice(c->device));
    hipStream_t st = c->stream;
    Arena ar;
    ar.base = c->ws; ar.cap = c->ws_bytes; ar.off = c->persistent;
    int64_t* toff = ar.get<int64_t>(T + 1);
    u32* cnt = ar.get<u32>(2 * ((int64_t)T * c->F + 1));
    if (ar.overflow) return fail(c, GM_ERR_WORKSPACE, "workspace too small");
    HIPCHK(c, hipMemcpyAsync(toff, set->task_offsets, (T + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    // validate before the gather trusts offsets and indices
    launch_fill_u32(st, c->d_status, ST_WORDS, 0);
    SetView v = make_view(set, toff, 0, 0);
    if (c->F > 0 && T > 0)
        launch_tf_count(st, c->F, 0, T, v, v, c->d_field_base, set->nnz, set->nnz, uniform_rows(c), cnt, cnt + (int64_t)T * c->F + 1, c->d_status);
    u32 hs[ST_WORDS];
    rc = read_status(c, hs);
    if (rc != GM_OK) return rc;
    if (hs[ST_BAD_INDEX]) return fail(c, GM_ERR_INDEX, "index outside its table, or bag_offsets not monotone / beyond nnz");
    if (hs[ST_TOO_LARGE])
        return fail(c, GM_ERR_CAPACITY, "a bag has more than 65535 lookups, or a task more than 65536 samples in one set");
    // process in chunks of samples that fit the workspace
    const size_t mark = ar.off;
    const int ld0 = c->ld[0], d0 = c->dims[0];
    const size_t avail = c->ws_bytes - mark;
    int64_t chunk = (int64_t)(avail / ((size_t)(ld0 + 1) * sizeof(float))) - 128;
    if (chunk < 1) return fail(c, GM_ERR_WORKSPACE, "workspace too small");
    chunk = std::min<int64_t>(chunk, (int64_t)1 << 30);
    for (int64_t s0 = 0; s0 < set->n_samples; s0 += chunk) {
        const int64_t n = std::min(chunk, set->n_samples - s0);
        ar.off = mark;
        float* xp = ar.get<float>(n * ld0);
        int32_t* ident = ar.get<int32_t>(n);
        hipLaunchKernelGGL(iota_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, ident, n);
        Prof p(c, "gather_pool", 0, 0);
        launch_gather_pool(st, c->F, c->D, c->n_dense, c->d_field_base, set->bag_offsets, set->indices, set->dense, emb, s0,
                           n, ident, 0, xp, ld0, nullptr);
        hipLaunchKernelGGL(strip_pad_kernel, dim3((unsigned)((n * d0 + 255) / 256)), dim3(256), 0, st, xp, n, ld0, d0,
                           x + s0 * d0);
    }
    HIPCHK(c, hipStreamSynchronize(st));
    HIPCHK(c, hipGetLastError());
    prof_drain(c);
    return GM_OK;
}

__global__ void widen_u32_kernel(const u32* src, int64_t n, int64_t* dst) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = (int64_t)src[i];
}
// packs the gapped per-(task, field) row lists: dst[packed_base[tf] + u] = slot_rows[base[tf] + u]
__global__ void pack_slot_rows_kernel(const u32* slot_rows, const u32* base, const u32* n_slots, const u32* packed_base,
                                      int64_t out0, int64_t* dst) {
    const int tf = blockIdx.x;
    for (u32 u = threadIdx.x; u < n_slots[tf]; u += blockDim.x)
        dst[out0 + packed_base[tf] + u] = (int64_t)slot_rows[base[tf] + u];
}

extern "C" int gm_index_prep(gm_ctx* c, int32_t T, const gm_set* sup, const gm_set* qry, int64_t* slot_counts,
                             int64_t* slot_rows, int32_t* sup_slot, int32_t* qry_slot, int64_t* emb_rows,
                             int64_t* seg_counts, int64_t* n_emb_rows, int64_t capacity) {
    if (!c) return GM_ERR_ARG;
    if (T < 0) return fail(c, GM_ERR_ARG, "bad n_tasks");
    int rc = check_set(c, sup, T, "support");
    if (rc != GM_OK) return rc;
    rc = check_set(c, qry, T, "query");
    if (rc != GM_OK) return rc;
    if (!n_emb_rows || capacity < 0) return fail(c, GM_ERR_ARG, "bad outputs");
    HIPCHK(c, hipSetDevice(c->device));
    hipStream_t st = c->stream;
    const int F = c->F;
    Arena ar;
    ar.base = c->ws; ar.cap = c->ws_bytes; ar.off = c->persistent;
    Batch B;
    B.T = T; B.sup = sup; B.qry = qry;
    rc = begin_batch(c, B, ar, capacity, false, &ar);
    if (rc != GM_OK) return rc;
    std::vector<WavePlan> plans;
    rc = plan_waves(c, B, c->ws_bytes - ar.off, 1, 2, 64, plans);
    if (rc != GM_OK) return rc;
    const size_t mark = ar.off;
    int64_t packed0 = 0;
    bool ordered = false;
    for (const WavePlan& wp : plans) {
        ar.off = mark;
        const int Tw = wp.t1 - wp.t0;
        if (Tw == 0 || F == 0) continue;
        WaveBufs w;
        const WaveDims d = wave_dims(c, B, wp, 64, 0, 1);
        alloc_wave(c, ar, w, d, 1, 2);
        if (ar.overflow) return fail(c, GM_ERR_WORKSPACE, "internal: wave does not fit");
        Grp gs, gq;
        if ((rc = setup_wave(c, B, wp, 64, 0, w, d, gs, gq))) return rc;
        JoinReq jr;
        if (plans.size() == 1) {   // the batch-wide order is this wave's: both come out of one sort
            jr.so = &B.b.so;
            jr.range = whole_batch_range(B);
            jr.n_sup_rows = d.Ps; jr.n_qry_rows = d.Pq;
            jr.emb_rows = emb_rows; jr.seg_counts = seg_counts; jr.capacity = capacity; jr.n_rows = n_emb_rows;
            jr.slots = true;
        }
        rc = run_index_wave(c, B, wp, w, nullptr, nullptr, nullptr, &jr);
        if (rc != GM_OK) return rc;
        ordered = jr.used;
        const int64_t TF = (int64_t)Tw * F;
        hipLaunchKernelGGL(widen_u32_kernel, dim3((unsigned)((TF + 255) / 256)), dim3(256), 0, st, w.n_slots, TF,
                           slot_counts + (int64_t)wp.t0 * F);
        u32* total = w.cnt_q + TF;  // spare word
        launch_scan_u32(st, w.n_slots, w.cnt_s, TF, w.scan_tmp, total);  // cnt_s reused as the packed base
        hipLaunchKernelGGL(pack_slot_rows_kernel, dim3((unsigned)TF), dim3(64), 0, st, w.slot_rows, w.base_s, w.n_slots,
                           w.cnt_s, packed0, slot_rows);
        u32 h_total = 0;
        HIPCHK(c, hipMemcpyAsync(&h_total, total, sizeof(u32), hipMemcpyDeviceToHost, st));
        HIPCHK(c, hipMemcpyAsync(sup_slot + wp.ls0, w.sup_slot, d.nnz_s * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        HIPCHK(c, hipMemcpyAsync(qry_slot + wp.lq0, w.qry_slot, d.nnz_q * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        HIPCHK(c, hipStreamSynchronize(st));
        packed0 += h_total;
    }
    if (!ordered) {
        launch_fill_u32(st, c->d_status, ST_WORDS, 0);
        global_order(c, B, B.b.so, whole_batch_range(B), emb_rows, seg_counts, capacity, n_emb_rows);
    }
    u32 hs[ST_WORDS];
    rc = read_status(c, hs);
    if (rc != GM_OK) return rc;
    HIPCHK(c, hipGetLastError());
    prof_drain(c);
    if (hs[ST_CAPACITY])
        return fail(c, GM_ERR_CAPACITY, "emb_rows_capacity %lld is smaller than the %u rows touched", (long long)capacity,
                    hs[ST_NROWS]);
    return GM_OK;
}
