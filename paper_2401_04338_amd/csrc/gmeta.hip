// Host side of the library: the C ABI of include/gmeta.h and the orchestration of one MAML step
// (G-Meta Alg. 1 with "worker" read as "task") as a fixed sequence of kernel launches on one stream.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/gmeta.h"
#include "gm_internal.h"

#define GEMM_BM 64

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

struct gm_ctx {
    int F = 0, D = 0, n_dense = 0, L = 0, mlp_dtype = 0;
    std::vector<int64_t> rows, field_base;
    std::vector<int> dims, ld;
    std::vector<int64_t> offW, offb;
    int64_t n_theta = 0;
    int FD = 0;
    int device = 0;
    hipStream_t stream = nullptr;
    char* ws = nullptr;
    size_t ws_bytes = 0;
    size_t persistent = 0;
    int64_t* d_field_base = nullptr;
    u32* d_status = nullptr;
    std::string err;
};

static int fail(gm_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIPCHK(c, call)                                                                              \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess) return fail(c, GM_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_));   \
    } while (0)

static int round_up(int x, int m) { return (x + m - 1) / m * m; }

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
    c->FD = c->F * D;
    c->rows.assign(m->rows_per_field, m->rows_per_field + c->F);
    c->field_base.assign(c->F + 1, 0);
    for (int f = 0; f < c->F; ++f) {
        if (c->rows[f] <= 0) return fail(c, GM_ERR_ARG, "rows_per_field must be positive");
        c->field_base[f + 1] = c->field_base[f] + c->rows[f];
    }
    if (c->field_base[c->F] >= (int64_t)1 << 32) return fail(c, GM_ERR_ARG, "more than 2^32 rows in total");
    c->dims.assign(m->layer_dims, m->layer_dims + c->L + 1);
    if (c->dims[0] != c->FD + c->n_dense || c->dims[c->L] != 1 || c->n_dense < 0)
        return fail(c, GM_ERR_ARG, "layer_dims must start at F*D+n_dense and end at 1");
    c->ld.resize(c->L + 1);
    for (int l = 0; l <= c->L; ++l) {
        if (c->dims[l] <= 0) return fail(c, GM_ERR_ARG, "layer_dims must be positive");
        c->ld[l] = l == c->L ? 1 : round_up(c->dims[l], 32);
    }
    c->offW.resize(c->L + 1);
    c->offb.resize(c->L + 1);
    int64_t o = 0;
    for (int l = 1; l <= c->L; ++l) {
        c->offW[l] = o;
        o += (int64_t)c->ld[l - 1] * c->ld[l];
        o = (o + 31) / 32 * 32;
        c->offb[l] = o;
        o += round_up(c->ld[l], 32);
    }
    c->n_theta = o;
    return GM_OK;
}

// ------------------------------------------------------------------------------------------------
// buffers
// ------------------------------------------------------------------------------------------------
struct StepState {  // what one inner step leaves behind for the second-order pass
    float* X = nullptr;                 // a_0 of the step [Ss, ld0]
    std::vector<float*> A, Dl;          // [1..L-1]
    float *dL = nullptr, *zL = nullptr; // [Ss]
    float* theta = nullptr;             // parameters the step was taken at
    int64_t theta_stride = 0;
};

struct WaveBufs {
    int32_t *row_off_s, *row_off_q, *sample_task_s, *sample_task_q;
    int32_t *tile_g_s, *tile_m_s, *tile_g_q, *tile_m_q;
    u32 *cnt_s, *base_s, *cnt_q, *base_q, *n_slots, *scan_tmp;
    u32* slot_rows;
    int32_t *slot_start, *sup_sorted_sample, *sup_slot, *qry_slot, *qry_sorted_sample, *qseg_lo, *qseg_hi;
    float *Xs0, *Xq0, *Xs_scratch, *Delta, *vXi, *dX, *v_theta, *loss_q;
    std::vector<StepState> steps;
    std::vector<float*> thetas;  // theta^(1..K)
    // query pass
    float* Xq;
    std::vector<float*> Aq, Dq;
    float *dLq, *zq;
    // tangent temporaries
    float* TX;
    std::vector<float*> TA, TD;
    float* tdL;
};

struct WaveDims {
    int Tw;
    int64_t Ss, Sq, nnz_s, nnz_q;
    int mt_s, mt_q;
};

static void alloc_wave(const gm_ctx* c, Arena& ar, WaveBufs& w, const WaveDims& d, int K, int order) {
    const int L = c->L, F = c->F, D = c->D;
    const int64_t TF = (int64_t)d.Tw * F;
    w.row_off_s = ar.get<int32_t>(d.Tw + 1);
    w.row_off_q = ar.get<int32_t>(d.Tw + 1);
    w.sample_task_s = ar.get<int32_t>(d.Ss);
    w.sample_task_q = ar.get<int32_t>(d.Sq);
    w.tile_g_s = ar.get<int32_t>(d.mt_s);
    w.tile_m_s = ar.get<int32_t>(d.mt_s);
    w.tile_g_q = ar.get<int32_t>(d.mt_q);
    w.tile_m_q = ar.get<int32_t>(d.mt_q);
    w.cnt_s = ar.get<u32>(TF + 1);
    w.base_s = ar.get<u32>(TF + 1);
    w.cnt_q = ar.get<u32>(TF + 1);
    w.base_q = ar.get<u32>(TF + 1);
    w.n_slots = ar.get<u32>(TF + 1);
    w.scan_tmp = ar.get<u32>(scan_tmp_words(TF + 1));
    w.slot_rows = ar.get<u32>(d.nnz_s + 1);
    w.slot_start = ar.get<int32_t>(d.nnz_s + TF + 1);
    w.sup_sorted_sample = ar.get<int32_t>(d.nnz_s + 1);
    w.sup_slot = ar.get<int32_t>(d.nnz_s + 1);
    w.qry_slot = ar.get<int32_t>(d.nnz_q + 1);
    w.qry_sorted_sample = ar.get<int32_t>(d.nnz_q + 1);
    w.qseg_lo = ar.get<int32_t>(d.nnz_s + 1);
    w.qseg_hi = ar.get<int32_t>(d.nnz_s + 1);
    const int ld0 = c->ld[0];
    w.Xs0 = ar.get<float>(d.Ss * ld0);
    w.Xq0 = ar.get<float>(d.Sq * ld0);
    w.Delta = K > 0 ? ar.get<float>((d.nnz_s + 1) * D) : nullptr;
    const bool second = order == 2 && K > 0;
    w.Xs_scratch = (K > 1 && !second) ? ar.get<float>(d.Ss * ld0) : nullptr;
    w.vXi = second ? ar.get<float>((d.nnz_s + 1) * D) : nullptr;
    w.dX = ar.get<float>(std::max(d.Ss, d.Sq) * (int64_t)std::max(c->FD, 1));
    w.v_theta = ar.get<float>((int64_t)d.Tw * c->n_theta);
    w.loss_q = ar.get<float>(d.Sq + 1);
    const int kept = second ? K : (K > 0 ? 1 : 0);
    w.steps.assign(kept, StepState());
    for (int k = 0; k < kept; ++k) {
        StepState& s = w.steps[k];
        s.X = (k == 0) ? w.Xs0 : ar.get<float>(d.Ss * ld0);
        s.A.assign(L, nullptr);
        s.Dl.assign(L, nullptr);
        for (int l = 1; l < L; ++l) {
            s.A[l] = ar.get<float>(d.Ss * c->ld[l]);
            s.Dl[l] = ar.get<float>(d.Ss * c->ld[l]);
        }
        s.dL = ar.get<float>(d.Ss + 1);
        s.zL = ar.get<float>(d.Ss + 1);
    }
    const int n_theta_bufs = second ? K : (K > 0 ? 1 : 0);
    w.thetas.assign(n_theta_bufs, nullptr);
    for (int k = 0; k < n_theta_bufs; ++k) w.thetas[k] = ar.get<float>((int64_t)d.Tw * c->n_theta);
    w.Xq = K > 0 ? ar.get<float>(d.Sq * ld0) : w.Xq0;
    w.Aq.assign(L, nullptr);
    w.Dq.assign(L, nullptr);
    for (int l = 1; l < L; ++l) {
        w.Aq[l] = ar.get<float>(d.Sq * c->ld[l]);
        w.Dq[l] = ar.get<float>(d.Sq * c->ld[l]);
    }
    w.dLq = ar.get<float>(d.Sq + 1);
    w.zq = ar.get<float>(d.Sq + 1);
    w.TX = nullptr;
    w.TA.assign(L, nullptr);
    w.TD.assign(L, nullptr);
    w.tdL = nullptr;
    if (second) {
        w.TX = ar.get<float>(d.Ss * ld0);
        for (int l = 1; l < L; ++l) {
            w.TA[l] = ar.get<float>(d.Ss * c->ld[l]);
            w.TD[l] = ar.get<float>(d.Ss * c->ld[l]);
        }
        w.tdL = ar.get<float>(d.Ss + 1);
    }
}

struct BatchBufs {
    int64_t *toff_s, *toff_q;
    float *GX, *theta0, *g_theta, *task_loss;
    u32 *keys, *vals, *keys_tmp, *vals_tmp, *hist, *scan_tmp, *seg_start;
};

static void alloc_batch(const gm_ctx* c, Arena& ar, BatchBufs& b, int T, int64_t Ss, int64_t Sq, int64_t nnz,
                        int64_t capacity, bool need_gx) {
    b.toff_s = ar.get<int64_t>(T + 1);
    b.toff_q = ar.get<int64_t>(T + 1);
    b.GX = need_gx ? ar.get<float>((Ss + Sq) * (int64_t)std::max(c->FD, 1) + 4) : nullptr;
    b.theta0 = ar.get<float>(c->n_theta);
    b.g_theta = ar.get<float>(c->n_theta);
    b.task_loss = ar.get<float>(T + 1);
    b.keys = ar.get<u32>(nnz + 1);
    b.vals = ar.get<u32>(nnz + 1);
    b.keys_tmp = ar.get<u32>(nnz + 1);
    b.vals_tmp = ar.get<u32>(nnz + 1);
    b.hist = ar.get<u32>(radix_hist_words(nnz));
    b.scan_tmp = ar.get<u32>(scan_tmp_words(nnz));
    b.seg_start = ar.get<u32>(std::min(nnz, capacity) + 2);
}

static int count_mtiles(const int64_t* toff, int t0, int t1) {
    int64_t n = 0;
    for (int t = t0; t < t1; ++t) n += (toff[t + 1] - toff[t] + GEMM_BM - 1) / GEMM_BM;
    return (int)n;
}

// ------------------------------------------------------------------------------------------------
// ABI: create / destroy / sizes
// ------------------------------------------------------------------------------------------------
extern "C" int gm_create(gm_ctx** out, const gm_model_desc* model, int device, void* hip_stream,
                         size_t workspace_bytes) {
    if (!out) return GM_ERR_ARG;
    *out = nullptr;
    gm_ctx* c = new gm_ctx();
    int rc = model_layout(c, model);
    if (rc != GM_OK) {
        // keep the context so that the message can be read
        *out = c;
        return rc;
    }
    *out = c;
    c->device = device;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    HIPCHK(c, hipSetDevice(device));
    c->ws_bytes = std::max<size_t>(workspace_bytes, 1 << 20);
    HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&c->ws), c->ws_bytes));
    Arena ar;
    ar.base = c->ws;
    ar.cap = c->ws_bytes;
    c->d_field_base = ar.get<int64_t>(c->F + 1);
    c->d_status = ar.get<u32>(ST_WORDS);
    c->persistent = ar.off;
    HIPCHK(c, hipMemcpy(c->d_field_base, c->field_base.data(), (c->F + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    return GM_OK;
}

extern "C" void gm_destroy(gm_ctx* c) {
    if (!c) return;
    if (c->ws) {
        hipSetDevice(c->device);
        hipFree(c->ws);
    }
    delete c;
}

extern "C" const char* gm_last_error(const gm_ctx* c) { return c ? c->err.c_str() : "null context"; }

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
    alloc_batch(&c, ar, b, n_tasks, n_support, n_query, nnz_support + nnz_query,
                std::min(total_rows, nnz_support + nnz_query), true);
    WaveBufs w;
    WaveDims d;
    d.Tw = n_tasks;
    d.Ss = n_support;
    d.Sq = n_query;
    d.nnz_s = nnz_support;
    d.nnz_q = nnz_query;
    d.mt_s = (int)(n_support / GEMM_BM + n_tasks + 1);  // upper bound on m-tiles
    d.mt_q = (int)(n_query / GEMM_BM + n_tasks + 1);
    alloc_wave(&c, ar, w, d, inner_steps, order);
    return ar.off + (1 << 20);
}

// ------------------------------------------------------------------------------------------------
// argument checks shared by the entry points
// ------------------------------------------------------------------------------------------------
static int check_set(gm_ctx* c, const gm_set* s, int T, const char* name) {
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
    if (s->n_samples * (int64_t)std::max(c->F, 1) >= ((int64_t)1 << 31) || s->nnz >= ((int64_t)1 << 31))
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
// GEMM argument builders
// ------------------------------------------------------------------------------------------------
struct Grp {  // the grouping of one set's samples by task inside the wave
    const int32_t* row_off;
    const int32_t *tile_g, *tile_m;
    int n_mtiles, G;
};

static GemmArgs gemm_base(const Grp& g) {
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.row_offsets = g.row_off;
    a.G = g.G;
    a.n_pairs = 1;
    return a;
}

// C[rows, N] = sum_p A_p[rows, K] * W_p[K, N]   (W row-major [K, ldw])
static void set_pair_nn(GemmArgs& a, int p, const float* A, int lda, const float* W, int ldw, int64_t w_stride) {
    a.A[p] = A; a.sAm[p] = lda; a.sAk[p] = 1; a.gA[p] = 0; a.rA[p] = lda;
    a.B[p] = W; a.sBk[p] = ldw; a.sBn[p] = 1; a.gB[p] = w_stride; a.rB[p] = 0;
}
// C[rows, N] = sum_p A_p[rows, K] * W_p^T   (W row-major [N, ldw], K = ldw's extent)
static void set_pair_nt(GemmArgs& a, int p, const float* A, int lda, const float* W, int ldw, int64_t w_stride) {
    a.A[p] = A; a.sAm[p] = lda; a.sAk[p] = 1; a.gA[p] = 0; a.rA[p] = lda;
    a.B[p] = W; a.sBk[p] = 1; a.sBn[p] = ldw; a.gB[p] = w_stride; a.rB[p] = 0;
}
// C_g[M, N] = sum_p A_p[rows_g, M]^T * B_p[rows_g, N]
static void set_pair_tn(GemmArgs& a, int p, const float* A, int lda, const float* B, int ldb) {
    a.A[p] = A; a.sAm[p] = 1; a.sAk[p] = lda; a.gA[p] = 0; a.rA[p] = lda;
    a.B[p] = B; a.sBk[p] = ldb; a.sBn[p] = 1; a.gB[p] = 0; a.rB[p] = ldb;
}
static void rows_out(GemmArgs& a, const Grp& g, float* C, int ldc, int N, int K) {
    a.C = C; a.ldc = ldc; a.gC = 0; a.rC = ldc;
    a.M = -1; a.N = N; a.K = K;
    a.tile_group = g.tile_g; a.tile_m0 = g.tile_m; a.n_mtiles = g.n_mtiles;
}
static void theta_out(GemmArgs& a, float* C, int64_t stride, int M, int N, const float* Cin, int64_t cin_stride,
                      float c0, float c1) {
    a.C = C; a.ldc = N; a.gC = stride; a.rC = 0;
    a.M = M; a.N = N; a.K = -1;
    a.tile_group = nullptr;
    a.epi = EPI_AXPBY; a.Cin = Cin; a.gCin = cin_stride; a.c0 = c0; a.c1 = c1;
}

struct Pass {  // activations of one forward/backward pass over one set
    float* X; int64_t n;
    std::vector<float*>*A, *Dl;
    float *dL, *zL;
};

// forward with parameters theta (stride 0: shared by all tasks), loss and delta_L; then backward to the
// deltas of every layer and, when dX is given, to the pooled-input gradient [n, FD].
static void forward_backward(gm_ctx* c, const Grp& g, const int32_t* sample_task, const float* labels,
                             const Pass& p, const float* theta, int64_t ts, float* loss_out, float* dX) {
    hipStream_t st = c->stream;
    const int L = c->L;
    const float* prev = p.X;
    for (int l = 1; l < L; ++l) {
        GemmArgs a = gemm_base(g);
        set_pair_nn(a, 0, prev, c->ld[l - 1], theta + c->offW[l], c->ld[l], ts);
        rows_out(a, g, (*p.A)[l], c->ld[l], c->ld[l], c->ld[l - 1]);
        a.epi = EPI_BIAS_RELU; a.bias = theta + c->offb[l]; a.gBias = ts;
        launch_gemm_f32(st, a);
        prev = (*p.A)[l];
    }
    LastFwdArgs f;
    memset(&f, 0, sizeof f);
    f.n = p.n; f.N = c->ld[L - 1]; f.ld = c->ld[L - 1];
    f.sample_task = sample_task; f.row_offsets = g.row_off;
    f.a = prev; f.w = theta + c->offW[L]; f.gW = ts; f.b = theta + c->offb[L];
    f.labels = labels; f.z_out = p.zL; f.delta_out = p.dL; f.loss_out = loss_out;
    launch_last_fwd(st, f);
    // backward
    if (L == 1) {
        if (dX) launch_last_bwd(st, p.n, c->FD, c->ld[0], c->FD, sample_task, p.dL, theta + c->offW[L], ts, nullptr,
                                nullptr, 0, nullptr, dX);
        return;
    }
    launch_last_bwd(st, p.n, c->ld[L - 1], c->ld[L - 1], c->ld[L - 1], sample_task, p.dL, theta + c->offW[L], ts,
                    nullptr, nullptr, 0, (*p.A)[L - 1], (*p.Dl)[L - 1]);
    for (int l = L - 1; l >= 1; --l) {
        if (l == 1 && !dX) break;
        GemmArgs a = gemm_base(g);
        set_pair_nt(a, 0, (*p.Dl)[l], c->ld[l], theta + c->offW[l], c->ld[l], ts);
        if (l == 1) {
            rows_out(a, g, dX, c->FD, c->FD, c->ld[l]);
            a.epi = EPI_NONE;
        } else {
            rows_out(a, g, (*p.Dl)[l - 1], c->ld[l - 1], c->ld[l - 1], c->ld[l]);
            a.epi = EPI_MASK; a.mask = (*p.A)[l - 1]; a.ld_mask = c->ld[l - 1];
        }
        launch_gemm_f32(st, a);
    }
}

// out = c0*in + c1 * (gradient of the pass w.r.t. theta), per task
static void theta_grad(gm_ctx* c, const Grp& g, const Pass& p, float* out, const float* in, int64_t in_stride, float c0,
                       float c1) {
    hipStream_t st = c->stream;
    const int L = c->L;
    const int64_t nt = c->n_theta;
    for (int l = 1; l < L; ++l) {
        const float* prev = l == 1 ? p.X : (*p.A)[l - 1];
        GemmArgs a = gemm_base(g);
        set_pair_tn(a, 0, prev, c->ld[l - 1], (*p.Dl)[l], c->ld[l]);
        theta_out(a, out + c->offW[l], nt, c->ld[l - 1], c->ld[l], in ? in + c->offW[l] : nullptr, in_stride, c0, c1);
        launch_gemm_f32(st, a);
        launch_task_colsum(st, g.G, g.row_off, c->ld[l], (*p.Dl)[l], nullptr, nullptr, nullptr, c->ld[l],
                           out + c->offb[l], nt, in ? in + c->offb[l] : nullptr, in_stride, c0, c1);
    }
    const float* prev = L == 1 ? p.X : (*p.A)[L - 1];
    launch_task_colsum(st, g.G, g.row_off, c->ld[L - 1], prev, p.dL, nullptr, nullptr, c->ld[L - 1], out + c->offW[L],
                       nt, in ? in + c->offW[L] : nullptr, in_stride, c0, c1);
    launch_task_colsum(st, g.G, g.row_off, 1, p.dL, nullptr, nullptr, nullptr, 1, out + c->offb[L], nt,
                       in ? in + c->offb[L] : nullptr, in_stride, c0, c1);
}

// v_theta <- v_theta - alpha * H_theta,. v ;  tdx [Ss, FD] <- (H v)'s pooled-input part
// (tangent pass through the forward and the backward pass of step `s`, direction (v_theta, TX))
static void hvp_step(gm_ctx* c, const Grp& g, const int32_t* sample_task, const StepState& s, int64_t n, WaveBufs& w,
                     float alpha) {
    hipStream_t st = c->stream;
    const int L = c->L;
    const int64_t nt = c->n_theta;
    float* v = w.v_theta;
    const float* tprev = w.TX;
    const float* prev = s.X;
    for (int l = 1; l < L; ++l) {
        GemmArgs a = gemm_base(g);
        a.n_pairs = 2;
        set_pair_nn(a, 0, tprev, c->ld[l - 1], s.theta + c->offW[l], c->ld[l], s.theta_stride);
        set_pair_nn(a, 1, prev, c->ld[l - 1], v + c->offW[l], c->ld[l], nt);
        rows_out(a, g, w.TA[l], c->ld[l], c->ld[l], c->ld[l - 1]);
        a.epi = EPI_BIAS_MASK; a.bias = v + c->offb[l]; a.gBias = nt; a.mask = s.A[l]; a.ld_mask = c->ld[l];
        launch_gemm_f32(st, a);
        tprev = w.TA[l];
        prev = s.A[l];
    }
    LastFwdArgs f;
    memset(&f, 0, sizeof f);
    f.n = n; f.N = c->ld[L - 1]; f.ld = c->ld[L - 1];
    f.sample_task = sample_task; f.row_offsets = g.row_off;
    f.a = prev; f.ta = tprev; f.w = s.theta + c->offW[L]; f.gW = s.theta_stride; f.b = s.theta + c->offb[L];
    f.tw = v + c->offW[L]; f.gTW = nt; f.tb = v + c->offb[L];
    f.z_in = s.zL; f.delta_out = w.tdL;
    launch_last_fwd(st, f);
    // tangent of the backward pass, top layer first; each layer's direction is consumed before it is updated
    if (L == 1) {
        launch_last_bwd(st, n, c->FD, c->ld[0], c->FD, sample_task, w.tdL, s.theta + c->offW[L], s.theta_stride, s.dL,
                        v + c->offW[L], nt, nullptr, w.dX);
    } else {
        launch_last_bwd(st, n, c->ld[L - 1], c->ld[L - 1], c->ld[L - 1], sample_task, w.tdL, s.theta + c->offW[L],
                        s.theta_stride, s.dL, v + c->offW[L], nt, s.A[L - 1], w.TD[L - 1]);
    }
    launch_task_colsum(st, g.G, g.row_off, c->ld[L - 1], tprev, s.dL, prev, w.tdL, c->ld[L - 1], v + c->offW[L], nt,
                       v + c->offW[L], nt, 1.f, -alpha);
    launch_task_colsum(st, g.G, g.row_off, 1, w.tdL, nullptr, nullptr, nullptr, 1, v + c->offb[L], nt, v + c->offb[L],
                       nt, 1.f, -alpha);
    for (int l = L - 1; l >= 1; --l) {
        GemmArgs a = gemm_base(g);
        a.n_pairs = 2;
        set_pair_nt(a, 0, w.TD[l], c->ld[l], s.theta + c->offW[l], c->ld[l], s.theta_stride);
        set_pair_nt(a, 1, s.Dl[l], c->ld[l], v + c->offW[l], c->ld[l], nt);
        if (l == 1) {
            rows_out(a, g, w.dX, c->FD, c->FD, c->ld[l]);
            a.epi = EPI_NONE;
        } else {
            rows_out(a, g, w.TD[l - 1], c->ld[l - 1], c->ld[l - 1], c->ld[l]);
            a.epi = EPI_MASK; a.mask = s.A[l - 1]; a.ld_mask = c->ld[l - 1];
        }
        if (c->FD > 0 || l > 1) launch_gemm_f32(st, a);
        const float* ta_prev = l == 1 ? w.TX : w.TA[l - 1];
        const float* a_prev = l == 1 ? s.X : s.A[l - 1];
        GemmArgs b = gemm_base(g);
        b.n_pairs = 2;
        set_pair_tn(b, 0, ta_prev, c->ld[l - 1], s.Dl[l], c->ld[l]);
        set_pair_tn(b, 1, a_prev, c->ld[l - 1], w.TD[l], c->ld[l]);
        theta_out(b, v + c->offW[l], nt, c->ld[l - 1], c->ld[l], v + c->offW[l], nt, 1.f, -alpha);
        launch_gemm_f32(st, b);
        launch_task_colsum(st, g.G, g.row_off, c->ld[l], w.TD[l], nullptr, nullptr, nullptr, c->ld[l], v + c->offb[l],
                           nt, v + c->offb[l], nt, 1.f, -alpha);
    }
}

// ------------------------------------------------------------------------------------------------
// the step
// ------------------------------------------------------------------------------------------------
struct WavePlan {
    int t0, t1;
    int64_t s0, s1, q0, q1;          // sample ranges
    int64_t ls0, ls1, lq0, lq1;      // lookup ranges
};

__global__ void gather_task_lookup_offsets(const int64_t* toff, const int64_t* bag_offsets, int F, int T, int64_t* out) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t <= T) out[t] = bag_offsets[toff[t] * F];
}

static void build_tiles(const int64_t* toff, int t0, int t1, std::vector<int32_t>& row_off, std::vector<int32_t>& tg,
                        std::vector<int32_t>& tm) {
    row_off.clear(); tg.clear(); tm.clear();
    const int64_t base = toff[t0];
    for (int t = t0; t < t1; ++t) {
        row_off.push_back((int32_t)(toff[t] - base));
        const int n = (int)(toff[t + 1] - toff[t]);
        for (int m = 0; m < n; m += GEMM_BM) {
            tg.push_back(t - t0);
            tm.push_back(m);
        }
    }
    row_off.push_back((int32_t)(toff[t1] - base));
}

static int upload_i32(gm_ctx* c, int32_t* dst, const std::vector<int32_t>& v) {
    if (v.empty()) return GM_OK;
    HIPCHK(c, hipMemcpyAsync(dst, v.data(), v.size() * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    return GM_OK;
}

static int run_index_wave(gm_ctx* c, const gm_set* sup, const gm_set* qry, const BatchBufs& b, const WavePlan& wp,
                          WaveBufs& w) {
    hipStream_t st = c->stream;
    const int F = c->F, Tw = wp.t1 - wp.t0;
    if (F == 0 || Tw == 0) return GM_OK;
    const int64_t TF = (int64_t)Tw * F;
    SetView vs = make_view(sup, b.toff_s, wp.s0, wp.ls0), vq = make_view(qry, b.toff_q, wp.q0, wp.lq0);
    launch_fill_u32(st, c->d_status, ST_WORDS, 0);
    launch_tf_count(st, F, wp.t0, Tw, vs, vq, c->d_field_base, sup->nnz, qry->nnz, w.cnt_s, w.cnt_q, c->d_status);
    u32 hs[ST_WORDS];
    int rc = read_status(c, hs);
    if (rc != GM_OK) return rc;
    if (hs[ST_BAD_INDEX]) return fail(c, GM_ERR_INDEX, "index outside its table, or bag_offsets not monotone / beyond nnz");
    int cap = 1024;
    while (cap < (int)hs[ST_MAX_TF]) cap <<= 1;
    if (cap > tf_sort_max_cap())
        return fail(c, GM_ERR_CAPACITY, "a (task, field) has %u lookups in one set; the limit is %d", hs[ST_MAX_TF],
                    tf_sort_max_cap());
    launch_scan_u32(st, w.cnt_s, w.base_s, TF, w.scan_tmp, nullptr);
    launch_scan_u32(st, w.cnt_q, w.base_q, TF, w.scan_tmp, nullptr);
    TfSortArgs a;
    a.F = F; a.t0 = wp.t0; a.Tw = Tw; a.sup = vs; a.qry = vq; a.field_base = c->d_field_base;
    a.cnt_sup = w.cnt_s; a.base_sup = w.base_s; a.cnt_qry = w.cnt_q; a.base_qry = w.base_q;
    a.n_slots = w.n_slots; a.slot_rows = w.slot_rows; a.slot_start = w.slot_start;
    a.sup_sorted_sample = w.sup_sorted_sample; a.sup_slot = w.sup_slot; a.qry_slot = w.qry_slot;
    a.qry_sorted_sample = w.qry_sorted_sample; a.qseg_lo = w.qseg_lo; a.qseg_hi = w.qseg_hi; a.status = c->d_status;
    launch_tf_sort(st, a, cap);
    return GM_OK;
}

static int global_order(gm_ctx* c, const gm_set* sup, const gm_set* qry, const BatchBufs& b, int64_t* emb_rows,
                        int64_t* seg_counts, int64_t capacity, int64_t* n_rows) {
    hipStream_t st = c->stream;
    const int F = c->F;
    const int64_t nnz = sup->nnz + qry->nnz;
    if (F > 0) {
        launch_build_keys(st, F, c->d_field_base, sup->bag_offsets, sup->indices, sup->n_samples * F, 0u, b.keys, b.vals,
                          c->d_status);
        launch_build_keys(st, F, c->d_field_base, qry->bag_offsets, qry->indices, qry->n_samples * F,
                          (u32)(sup->n_samples * F), b.keys + sup->nnz, b.vals + sup->nnz, c->d_status);
    }
    int bits = 1;
    while (((int64_t)1 << bits) < c->field_base[c->F]) ++bits;
    launch_radix_sort(st, b.keys, b.vals, b.keys_tmp, b.vals_tmp, nnz, bits, b.hist);
    launch_segments(st, b.keys, nnz, b.keys_tmp, b.scan_tmp, emb_rows, b.seg_start, seg_counts, capacity, n_rows,
                    c->d_status);
    return GM_OK;
}

// validates the lookups of the whole batch on the device (offsets monotone and inside nnz, indices inside
// their tables) before any kernel trusts them
static int plan_waves(gm_ctx* c, int T, const gm_set* sup, const gm_set* qry, const BatchBufs& b, size_t avail, int K,
                      int order, std::vector<WavePlan>& plans) {
    const int F = c->F;
    std::vector<int64_t> ls(T + 1, 0), lq(T + 1, 0);
    bool have_offsets = false;
    auto fetch = [&]() -> int {
        if (have_offsets || F == 0) return GM_OK;
        // lookup offset of every task boundary, read back once
        // the two small arrays reuse the radix-sort histogram scratch
        int64_t* d = reinterpret_cast<int64_t*>(b.hist);
        const size_t need = 2 * (size_t)(T + 1) * sizeof(int64_t);
        if (radix_hist_words(sup->nnz + qry->nnz) * sizeof(u32) < need) {
            // tiny batches: hist may be too small; fall back to per-element copies
            for (int t = 0; t <= T; ++t) {
                HIPCHK(c, hipMemcpy(&ls[t], sup->bag_offsets + sup->task_offsets[t] * F, sizeof(int64_t), hipMemcpyDeviceToHost));
                HIPCHK(c, hipMemcpy(&lq[t], qry->bag_offsets + qry->task_offsets[t] * F, sizeof(int64_t), hipMemcpyDeviceToHost));
            }
        } else {
            hipLaunchKernelGGL(gather_task_lookup_offsets, dim3((T + 256) / 256), dim3(256), 0, c->stream, b.toff_s,
                               sup->bag_offsets, F, T, d);
            hipLaunchKernelGGL(gather_task_lookup_offsets, dim3((T + 256) / 256), dim3(256), 0, c->stream, b.toff_q,
                               qry->bag_offsets, F, T, d + T + 1);
            HIPCHK(c, hipMemcpyAsync(ls.data(), d, (T + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, c->stream));
            HIPCHK(c, hipMemcpyAsync(lq.data(), d + T + 1, (T + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, c->stream));
            HIPCHK(c, hipStreamSynchronize(c->stream));
        }
        for (int t = 0; t <= T; ++t)
            if (ls[t] < 0 || ls[t] > sup->nnz || lq[t] < 0 || lq[t] > qry->nnz || (t && (ls[t] < ls[t - 1] || lq[t] < lq[t - 1])))
                return fail(c, GM_ERR_INDEX, "bag_offsets not monotone / beyond nnz at a task boundary");
        have_offsets = true;
        return GM_OK;
    };
    int per = std::max(T, 1);
    while (true) {
        plans.clear();
        bool fits = true;
        if (per < T) {
            int rc = fetch();
            if (rc != GM_OK) return rc;
        } else {
            ls[T] = sup->nnz;
            lq[T] = qry->nnz;
        }
        for (int t0 = 0; t0 < T || (T == 0 && plans.empty()); t0 += per) {
            WavePlan p;
            p.t0 = t0;
            p.t1 = std::min(T, t0 + per);
            p.s0 = sup->task_offsets[p.t0]; p.s1 = sup->task_offsets[p.t1];
            p.q0 = qry->task_offsets[p.t0]; p.q1 = qry->task_offsets[p.t1];
            p.ls0 = ls[p.t0]; p.ls1 = ls[p.t1]; p.lq0 = lq[p.t0]; p.lq1 = lq[p.t1];
            plans.push_back(p);
            Arena ar;
            ar.cap = avail;
            WaveBufs w;
            WaveDims d;
            d.Tw = p.t1 - p.t0; d.Ss = p.s1 - p.s0; d.Sq = p.q1 - p.q0; d.nnz_s = p.ls1 - p.ls0; d.nnz_q = p.lq1 - p.lq0;
            d.mt_s = count_mtiles(sup->task_offsets, p.t0, p.t1);
            d.mt_q = count_mtiles(qry->task_offsets, p.t0, p.t1);
            alloc_wave(c, ar, w, d, K, order);
            if (ar.overflow) { fits = false; break; }
            if (T == 0) break;
        }
        if (fits) return GM_OK;
        if (per == 1) return fail(c, GM_ERR_WORKSPACE, "workspace of %zu bytes cannot hold one task", c->ws_bytes);
        per = (per + 1) / 2;
    }
}

extern "C" int gm_meta_step(gm_ctx* c, int32_t T, const gm_set* sup, const gm_set* qry, const gm_params* params,
                            float alpha, int32_t K, int32_t order, float* loss, gm_grads* out) {
    if (!c) return GM_ERR_ARG;
    if (T < 0 || K < 0 || (order != 1 && order != 2)) return fail(c, GM_ERR_ARG, "bad n_tasks / inner_steps / order");
    if (c->mlp_dtype != 0) return fail(c, GM_ERR_ARG, "mlp_dtype 1 is not available in this build");
    int rc = check_set(c, sup, T, "support");
    if (rc != GM_OK) return rc;
    rc = check_set(c, qry, T, "query");
    if (rc != GM_OK) return rc;
    if (!params || !params->W || !params->b || (c->F > 0 && !params->emb)) return fail(c, GM_ERR_ARG, "null params");
    if (!loss || !out || !out->dW || !out->db || !out->n_emb_rows) return fail(c, GM_ERR_ARG, "null outputs");
    for (int l = 0; l < c->L; ++l)
        if (!params->W[l] || !params->b[l] || !out->dW[l] || !out->db[l]) return fail(c, GM_ERR_ARG, "null layer pointer");
    if (out->emb_rows_capacity < 0 || (out->emb_rows_capacity > 0 && (!out->emb_rows || !out->emb_grad)))
        return fail(c, GM_ERR_ARG, "bad sparse output buffers");
    HIPCHK(c, hipSetDevice(c->device));
    hipStream_t st = c->stream;
    const int F = c->F, D = c->D, L = c->L, FD = c->FD, ld0 = c->ld[0];
    const int64_t nt = c->n_theta;
    const int64_t Ss = sup->n_samples, Sq = qry->n_samples, nnz = sup->nnz + qry->nnz;
    const int64_t capacity = out->emb_rows_capacity;

    Arena ar;
    ar.base = c->ws; ar.cap = c->ws_bytes; ar.off = c->persistent;
    BatchBufs b;
    alloc_batch(c, ar, b, T, Ss, Sq, nnz, capacity, true);
    if (ar.overflow) return fail(c, GM_ERR_WORKSPACE, "workspace too small for the batch-level buffers (%zu needed)", ar.off);
    HIPCHK(c, hipMemcpyAsync(b.toff_s, sup->task_offsets, (T + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(b.toff_q, qry->task_offsets, (T + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    std::vector<WavePlan> plans;
    rc = plan_waves(c, T, sup, qry, b, c->ws_bytes - ar.off, K, order, plans);
    if (rc != GM_OK) return rc;
    const size_t wave_mark = ar.off;

    // meta theta in the padded internal layout; accumulators
    for (int l = 1; l <= L; ++l) {
        launch_pack_weights(st, params->W[l - 1], c->dims[l - 1], c->dims[l], c->ld[l - 1], c->ld[l], b.theta0 + c->offW[l]);
        launch_pack_weights(st, params->b[l - 1], 1, c->dims[l], 1, (int)(l == L ? 32 : c->ld[l]), b.theta0 + c->offb[l]);
    }
    launch_fill_f32(st, b.g_theta, nt, 0.f);
    if (b.GX) launch_fill_f32(st, b.GX, (Ss + Sq) * (int64_t)FD, 0.f);
    float* task_loss = out->task_loss ? out->task_loss : b.task_loss;

    for (const WavePlan& wp : plans) {
        ar.off = wave_mark;
        const int Tw = wp.t1 - wp.t0;
        if (Tw == 0) continue;
        WaveBufs w;
        WaveDims d;
        d.Tw = Tw; d.Ss = wp.s1 - wp.s0; d.Sq = wp.q1 - wp.q0; d.nnz_s = wp.ls1 - wp.ls0; d.nnz_q = wp.lq1 - wp.lq0;
        std::vector<int32_t> ro_s, tg_s, tm_s, ro_q, tg_q, tm_q;
        build_tiles(sup->task_offsets, wp.t0, wp.t1, ro_s, tg_s, tm_s);
        build_tiles(qry->task_offsets, wp.t0, wp.t1, ro_q, tg_q, tm_q);
        d.mt_s = (int)tg_s.size(); d.mt_q = (int)tg_q.size();
        alloc_wave(c, ar, w, d, K, order);
        if (ar.overflow) return fail(c, GM_ERR_WORKSPACE, "internal: wave does not fit");
        if ((rc = upload_i32(c, w.row_off_s, ro_s)) || (rc = upload_i32(c, w.row_off_q, ro_q)) ||
            (rc = upload_i32(c, w.tile_g_s, tg_s)) || (rc = upload_i32(c, w.tile_m_s, tm_s)) ||
            (rc = upload_i32(c, w.tile_g_q, tg_q)) || (rc = upload_i32(c, w.tile_m_q, tm_q)))
            return rc;
        launch_fill_sample_task(st, w.row_off_s, Tw, w.sample_task_s);
        launch_fill_sample_task(st, w.row_off_q, Tw, w.sample_task_q);
        Grp gs{w.row_off_s, w.tile_g_s, w.tile_m_s, d.mt_s, Tw}, gq{w.row_off_q, w.tile_g_q, w.tile_m_q, d.mt_q, Tw};

        // a0: row dictionaries and the overlap join
        rc = run_index_wave(c, sup, qry, b, wp, w);
        if (rc != GM_OK) return rc;
        const int n_tf = Tw * F;

        // a1: one prefetch pass for both sets
        launch_gather_pool(st, F, D, c->n_dense, c->d_field_base, sup->bag_offsets, sup->indices, sup->dense, params->emb,
                           wp.s0, d.Ss, w.Xs0, ld0, nullptr);
        launch_gather_pool(st, F, D, c->n_dense, c->d_field_base, qry->bag_offsets, qry->indices, qry->dense, params->emb,
                           wp.q0, d.Sq, w.Xq0, ld0, nullptr);
        if (K > 0 && F > 0) launch_fill_f32(st, w.Delta, (d.nnz_s + 1) * D, 0.f);

        // inner loop on the support set
        const float* labels_s = sup->labels + wp.s0;
        const float* labels_q = qry->labels + wp.q0;
        const bool second = order == 2 && K > 0;
        const float* theta = b.theta0;
        int64_t ts = 0;
        for (int k = 0; k < K; ++k) {
            StepState& s = w.steps[second ? k : 0];
            if (k > 0 && F > 0) {
                // support input of step k: meta rows plus the task's accumulated row deltas
                float* Xk = second ? s.X : w.Xs_scratch;
                launch_pool_slots(st, F, D, sup->bag_offsets, wp.s0, wp.ls0, d.Ss, w.sample_task_s, w.sup_slot, w.base_s,
                                  w.Delta, w.Xs0, Xk, ld0, nullptr);
                s.X = Xk;
            } else {
                s.X = w.Xs0;
            }
            s.theta = const_cast<float*>(theta);
            s.theta_stride = ts;
            Pass p{s.X, d.Ss, &s.A, &s.Dl, s.dL, s.zL};
            forward_backward(c, gs, w.sample_task_s, labels_s, p, theta, ts, nullptr, F > 0 ? w.dX : nullptr);
            // local back-propagation: theta' = theta - alpha dtheta (per task), rows' = rows - alpha drows
            float* theta_next = w.thetas[second ? k : 0];
            theta_grad(c, gs, p, theta_next, theta, ts, 1.f, -alpha);
            theta = theta_next;
            ts = nt;
            if (F > 0)
                launch_slot_segsum(st, F, D, n_tf, w.base_s, w.n_slots, w.slot_start, w.slot_start + 1, 1,
                                   w.sup_sorted_sample, w.dX, FD, w.Delta, 1.f, -alpha);
        }

        // overlap update + outer forward/backward on the query set
        if (K > 0 && F > 0)
            launch_pool_slots(st, F, D, qry->bag_offsets, wp.q0, wp.lq0, d.Sq, w.sample_task_q, w.qry_slot, w.base_s,
                              w.Delta, w.Xq0, w.Xq, ld0, nullptr);
        float* gxq = b.GX + (Ss + wp.q0) * (int64_t)FD;
        float* gxs = b.GX + wp.s0 * (int64_t)FD;
        Pass pq{K > 0 && F > 0 ? w.Xq : w.Xq0, d.Sq, &w.Aq, &w.Dq, w.dLq, w.zq};
        forward_backward(c, gq, w.sample_task_q, labels_q, pq, theta, ts, w.loss_q, F > 0 ? gxq : nullptr);
        launch_task_colsum(st, Tw, w.row_off_q, 1, w.loss_q, nullptr, nullptr, nullptr, 1, task_loss + wp.t0, 1, nullptr,
                           0, 0.f, 1.f);
        theta_grad(c, gq, pq, w.v_theta, nullptr, 0, 0.f, 1.f);

        // second-order chain back through the inner steps
        if (second) {
            if (F > 0)
                launch_slot_segsum(st, F, D, n_tf, w.base_s, w.n_slots, w.qseg_lo, w.qseg_hi, 0, w.qry_sorted_sample, gxq,
                                   FD, w.vXi, 0.f, 1.f);
            for (int k = K - 1; k >= 0; --k) {
                const StepState& s = w.steps[k];
                if (F > 0)
                    launch_pool_slots(st, F, D, sup->bag_offsets, wp.s0, wp.ls0, d.Ss, w.sample_task_s, w.sup_slot,
                                      w.base_s, w.vXi, nullptr, w.TX, ld0, nullptr);
                else
                    launch_fill_f32(st, w.TX, d.Ss * ld0, 0.f);
                hvp_step(c, gs, w.sample_task_s, s, d.Ss, w, alpha);
                if (F > 0) {
                    launch_axpy(st, d.Ss * (int64_t)FD, -alpha, w.dX, gxs);
                    if (k > 0)
                        launch_slot_segsum(st, F, D, n_tf, w.base_s, w.n_slots, w.slot_start, w.slot_start + 1, 1,
                                           w.sup_sorted_sample, w.dX, FD, w.vXi, 1.f, -alpha);
                }
            }
        }
        // cross-task reduction of the dense part (tasks of the wave in order, waves in order)
        launch_reduce_tasks(st, w.v_theta, nt, Tw, nt, b.g_theta, 1);
    }

    // outputs: dense meta-gradient, loss, coalesced sparse meta-gradient
    for (int l = 1; l <= L; ++l) {
        launch_unpack_weights(st, b.g_theta + c->offW[l], c->dims[l - 1], c->dims[l], c->ld[l], out->dW[l - 1]);
        launch_unpack_weights(st, b.g_theta + c->offb[l], 1, c->dims[l], c->dims[l], out->db[l - 1]);
    }
    launch_sum_to_scalar(st, task_loss, T, loss, 0);
    launch_fill_u32(st, c->d_status, ST_WORDS, 0);
    global_order(c, sup, qry, b, out->emb_rows, nullptr, capacity, out->n_emb_rows);
    if (F > 0)
        launch_seg_reduce(st, D, b.seg_start, out->n_emb_rows, capacity, std::min(nnz, capacity), b.vals, b.GX,
                          out->emb_grad);
    u32 hs[ST_WORDS];
    rc = read_status(c, hs);
    if (rc != GM_OK) return rc;
    HIPCHK(c, hipGetLastError());
    if (hs[ST_CAPACITY])
        return fail(c, GM_ERR_CAPACITY, "emb_rows_capacity %lld is smaller than the %u rows touched", (long long)capacity,
                    hs[ST_NROWS]);
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
        launch_tf_count(st, c->F, 0, T, v, v, c->d_field_base, set->nnz, set->nnz, cnt, cnt + (int64_t)T * c->F + 1, c->d_status);
    u32 hs[ST_WORDS];
    rc = read_status(c, hs);
    if (rc != GM_OK) return rc;
    if (hs[ST_BAD_INDEX]) return fail(c, GM_ERR_INDEX, "index outside its table, or bag_offsets not monotone / beyond nnz");
    // process in chunks of samples that fit the workspace
    const size_t mark = ar.off;
    const int ld0 = c->ld[0], d0 = c->dims[0];
    const size_t avail = c->ws_bytes - mark;
    int64_t chunk = (int64_t)(avail / ((size_t)ld0 * sizeof(float))) - 8;
    if (chunk < 1) return fail(c, GM_ERR_WORKSPACE, "workspace too small");
    for (int64_t s0 = 0; s0 < set->n_samples; s0 += chunk) {
        const int64_t n = std::min(chunk, set->n_samples - s0);
        ar.off = mark;
        float* xp = ar.get<float>(n * ld0);
        launch_gather_pool(st, c->F, c->D, c->n_dense, c->d_field_base, set->bag_offsets, set->indices, set->dense, emb, s0,
                           n, xp, ld0, nullptr);
        hipLaunchKernelGGL(strip_pad_kernel, dim3((unsigned)((n * d0 + 255) / 256)), dim3(256), 0, st, xp, n, ld0, d0,
                           x + s0 * d0);
    }
    HIPCHK(c, hipStreamSynchronize(st));
    HIPCHK(c, hipGetLastError());
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
    BatchBufs b;
    alloc_batch(c, ar, b, T, 0, 0, sup->nnz + qry->nnz, capacity, false);
    if (ar.overflow) return fail(c, GM_ERR_WORKSPACE, "workspace too small");
    HIPCHK(c, hipMemcpyAsync(b.toff_s, sup->task_offsets, (T + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIPCHK(c, hipMemcpyAsync(b.toff_q, qry->task_offsets, (T + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    std::vector<WavePlan> plans;
    rc = plan_waves(c, T, sup, qry, b, c->ws_bytes - ar.off, 1, 2, plans);
    if (rc != GM_OK) return rc;
    const size_t mark = ar.off;
    int64_t packed0 = 0;
    for (const WavePlan& wp : plans) {
        ar.off = mark;
        const int Tw = wp.t1 - wp.t0;
        if (Tw == 0 || F == 0) continue;
        WaveBufs w;
        WaveDims d;
        d.Tw = Tw; d.Ss = wp.s1 - wp.s0; d.Sq = wp.q1 - wp.q0; d.nnz_s = wp.ls1 - wp.ls0; d.nnz_q = wp.lq1 - wp.lq0;
        d.mt_s = count_mtiles(sup->task_offsets, wp.t0, wp.t1);
        d.mt_q = count_mtiles(qry->task_offsets, wp.t0, wp.t1);
        alloc_wave(c, ar, w, d, 1, 2);
        rc = run_index_wave(c, sup, qry, b, wp, w);
        if (rc != GM_OK) return rc;
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
    launch_fill_u32(st, c->d_status, ST_WORDS, 0);
    global_order(c, sup, qry, b, emb_rows, seg_counts, capacity, n_emb_rows);
    u32 hs[ST_WORDS];
    rc = read_status(c, hs);
    if (rc != GM_OK) return rc;
    HIPCHK(c, hipGetLastError());
    if (hs[ST_CAPACITY])
        return fail(c, GM_ERR_CAPACITY, "emb_rows_capacity %lld is smaller than the %u rows touched", (long long)capacity,
                    hs[ST_NROWS]);
    return GM_OK;
}
