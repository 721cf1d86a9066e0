// One isolated train step on one partition: forward, loss, backward, coverage statistics.
// Host-side orchestration of the kernels in spmm.hip / gemm.hip / elementwise.hip on one
// stream, with every intermediate carved out of the caller's workspace (no allocation, no
// host synchronisation).
//
// Per layer the neighbour aggregation runs at the narrower of the two widths (mean and the
// linear map commute): "aggregate first" when Fin <= Fout, "transform first" otherwise.
#include "common.h"

#include <vector>

namespace grp {

static inline int64_t ldp(int64_t f) { return round_up(f, 4); }

struct Bump {
    char* base;
    size_t cap, off = 0;
    bool measure;
    Bump(void* b, size_t c) : base((char*)b), cap(c), measure(b == nullptr) {}
    template <typename T> T* take(size_t count) {
        off = (off + 255) & ~(size_t)255;
        T* p = measure ? nullptr : (T*)(base + off);
        off += count * sizeof(T);
        return p;
    }
};

struct LayerBufs {
    float* Wp_s = nullptr;   // [Fin x ld(Fout)] aligned copy of W_self (GCN: W)
    float* Wp_n = nullptr;   // same for W_neigh
    float* Wt_s = nullptr;   // [Fout x ld(Fin)] transpose of W_self
    float* Wt_n = nullptr;
    float* M = nullptr;      // [n x ld(Fin)] aggregated input (aggregate-first SAGE layers)
    float* H_out = nullptr;  // [n x ld(Fout)] layer output (post-ReLU; logits for the last layer)
    int64_t off_ws = 0, off_wn = 0, off_b = 0;
    bool agg_first = false;
};

struct StepPlan {
    std::vector<LayerBufs> L;
    float *inv_in = nullptr, *gr = nullptr, *gs = nullptr, *grinv = nullptr;
    float *tmpA = nullptr, *tmpB = nullptr, *dZa = nullptr, *dZb = nullptr;
    void *tn_ws = nullptr, *colsum_ws = nullptr, *stats_ws = nullptr;
    float* partials = nullptr;   // partial rows of the split long rows (SpMM)
    size_t tn_ws_bytes = 0;
    size_t total = 0;
};

static bool valid_model(const grp_model_desc* m) {
    if (!m) return false;
    if (m->arch < GRP_ARCH_SAGE_MEAN || m->arch > GRP_ARCH_GCN_RESIDUAL) return false;
    if (m->n_layers < 1 || m->n_layers > GRP_MAX_LAYERS) return false;
    for (int l = 0; l <= m->n_layers; ++l)
        if (m->dims[l] <= 0 || m->dims[l] > 1024) return false;
    if (m->feat_dtype != GRP_DTYPE_FP32 && m->feat_dtype != GRP_DTYPE_BF16) return false;
    return true;
}

static int64_t param_count(const grp_model_desc* m) {
    const int per = m->arch == GRP_ARCH_SAGE_MEAN ? 2 : 1;
    int64_t p = 0;
    for (int l = 0; l < m->n_layers; ++l) p += (int64_t)per * m->dims[l] * m->dims[l + 1] + m->dims[l + 1];
    return p;
}

// Carves (or, with a null base, measures) the workspace.
static StepPlan make_plan(const grp_partition_t* part, const grp_model_desc* m, void* ws, size_t ws_bytes) {
    StepPlan p;
    const int64_t n = part->n;
    Bump b(ws, ws_bytes);
    const int k = m->n_layers;
    const bool sage = m->arch == GRP_ARCH_SAGE_MEAN;
    p.L.resize(k);
    int64_t off = 0, fmax = 0;
    size_t tn_bytes = 0, cs_bytes = 0;
    for (int l = 0; l < k; ++l) {
        LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        L.off_ws = off; off += (int64_t)fin * fout;
        if (sage) { L.off_wn = off; off += (int64_t)fin * fout; }
        L.off_b = off; off += fout;
        L.agg_first = sage && fin <= fout;
        L.Wp_s = b.take<float>((size_t)fin * ldp(fout));
        L.Wt_s = b.take<float>((size_t)fout * ldp(fin));
        if (sage) {
            L.Wp_n = b.take<float>((size_t)fin * ldp(fout));
            L.Wt_n = b.take<float>((size_t)fout * ldp(fin));
            if (L.agg_first) L.M = b.take<float>((size_t)n * ldp(fin));
        }
        L.H_out = b.take<float>((size_t)n * ldp(fout));
        if (ldp(fout) > fmax) fmax = ldp(fout);
        if (l > 0 && ldp(fin) > fmax) fmax = ldp(fin);
        const size_t t = gemm_tn_workspace_bytes(n, fin, fout);
        if (t > tn_bytes) tn_bytes = t;
        const size_t c = colsum_workspace_bytes(n, fout);
        if (c > cs_bytes) cs_bytes = c;
    }
    p.inv_in = b.take<float>((size_t)n);
    if (!sage) {
        p.gr = b.take<float>((size_t)n);
        p.gs = b.take<float>((size_t)n);
        p.grinv = b.take<float>((size_t)n);
    }
    p.tmpA = b.take<float>((size_t)n * fmax);
    p.tmpB = b.take<float>((size_t)n * fmax);
    p.dZa = b.take<float>((size_t)n * fmax);
    p.dZb = b.take<float>((size_t)n * fmax);
    p.tn_ws = b.take<char>(tn_bytes);
    p.tn_ws_bytes = tn_bytes;
    p.colsum_ws = b.take<char>(cs_bytes);
    p.stats_ws = b.take<char>(stats_workspace_bytes(n));
    {
        int64_t fsp = 0;
        for (int l = 0; l <= k; ++l)
            if (ldp(m->dims[l]) > fsp) fsp = ldp(m->dims[l]);
        const int64_t chunks = part->csr_long.n_chunks > part->csc_long.n_chunks ? part->csr_long.n_chunks : part->csc_long.n_chunks;
        p.partials = b.take<float>((size_t)chunks * fsp);
    }
    p.total = (b.off + 255) & ~(size_t)255;
    return p;
}

static grp_status check_step_args(const grp_partition_t* part, const grp_model_desc* model, const grp_step_opts* opts) {
    if (!part || !opts) return fail(GRP_EINVAL, "train_step: null partition or options");
    if (!valid_model(model)) return fail(GRP_EINVAL, "train_step: invalid model description");
    if (opts->estimator < GRP_EST_NONE || opts->estimator > GRP_EST_SHRINKAGE)
        return fail(GRP_EINVAL, "train_step: unknown estimator %d", opts->estimator);
    if (!opts->full_graph) return fail(GRP_EUNSUPPORTED, "train_step: mini-batch mode is not implemented in this build");
    if (model->arch == GRP_ARCH_GCN_RESIDUAL) return fail(GRP_EUNSUPPORTED, "train_step: residual GCN is not implemented in this build");
    return GRP_OK;
}

static grp_status sage_step(const grp_partition_t* g, const grp_model_desc* m, const grp_step_opts* o, const void* X,
                            const int32_t* labels, const uint8_t* mask, const float* theta, StepPlan& p, hipStream_t st,
                            float* grad, grp_step_stats* stats) {
    const int k = m->n_layers;
    const int64_t n = g->n;
    GRP_TRY(launch_degree_scales(g->d_local_in, g->d_local_out, n, 0, p.inv_in, nullptr, nullptr, nullptr, st));
    for (int l = 0; l < k; ++l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        GRP_TRY(launch_pad_copy(theta + L.off_ws, fin, fout, L.Wp_s, ldp(fout), st));
        GRP_TRY(launch_pad_copy(theta + L.off_wn, fin, fout, L.Wp_n, ldp(fout), st));
        if (l > 0) {
            GRP_TRY(launch_transpose(theta + L.off_ws, fin, fout, L.Wt_s, ldp(fin), fout, st));
            GRP_TRY(launch_transpose(theta + L.off_wn, fin, fout, L.Wt_n, ldp(fin), fout, st));
        }
    }
    GRP_TRY(launch_stats(n, nullptr, mask, g->d_local_in, g->d_global_in, nullptr, g->nnz, p.stats_ws, stats, st));

    // ---------------- forward
    const void* H = X;
    int64_t ldh = m->dims[0];
    int h_bf16 = m->feat_dtype == GRP_DTYPE_BF16;
    for (int l = 0; l < k; ++l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        const int relu = l < k - 1;
        if (L.agg_first) {
            SpmmArgs s;
            s.ptr = g->rowptr; s.idx = g->col; s.nnz = g->nnz; s.long_rows = &g->csr_long; s.partials = p.partials; s.n_rows = n; s.F = fin; s.X = H; s.ldx = ldh; s.x_bf16 = h_bf16;
            s.scale = GRP_SCALE_MEAN; s.Y = L.M; s.ldy = ldp(fin);
            GRP_TRY(launch_spmm(s, st));
            GemmNNArgs a;
            a.M = n; a.N = fout; a.K = fin; a.A = H; a.lda = ldh; a.a_bf16 = h_bf16; a.B = L.Wp_s; a.ldb = ldp(fout);
            a.K2 = fin; a.A2 = L.M; a.lda2 = ldp(fin); a.B2 = L.Wp_n; a.ldb2 = ldp(fout);
            a.bias = theta + L.off_b; a.relu = relu; a.C = L.H_out; a.ldc = ldp(fout); a.zero_pad_to = (int)ldp(fout);
            GRP_TRY(launch_gemm_nn(a, st));
        } else {
            GemmNNArgs a;
            a.M = n; a.N = fout; a.K = fin; a.A = H; a.lda = ldh; a.a_bf16 = h_bf16; a.B = L.Wp_n; a.ldb = ldp(fout);
            a.C = p.tmpA; a.ldc = ldp(fout); a.zero_pad_to = (int)ldp(fout);
            GRP_TRY(launch_gemm_nn(a, st));
            a.B = L.Wp_s; a.bias = theta + L.off_b; a.C = L.H_out;
            GRP_TRY(launch_gemm_nn(a, st));
            SpmmArgs s;
            s.ptr = g->rowptr; s.idx = g->col; s.nnz = g->nnz; s.long_rows = &g->csr_long; s.partials = p.partials; s.n_rows = n; s.F = fout; s.X = p.tmpA; s.ldx = ldp(fout);
            s.scale = GRP_SCALE_MEAN; s.addend = L.H_out; s.ld_add = ldp(fout); s.relu = relu; s.Y = L.H_out; s.ldy = ldp(fout);
            GRP_TRY(launch_spmm(s, st));
        }
        H = L.H_out; ldh = ldp(fout); h_bf16 = 0;
    }

    // ---------------- loss
    const int C = m->dims[k];
    float* dZ = p.dZa;
    float* dZ_other = p.dZb;
    GRP_TRY(launch_softmax_xent(n, C, p.L[k - 1].H_out, ldp(C), labels, nullptr, mask, o->estimator == GRP_EST_NODE_LEVEL,
                                g->d_local_in, g->d_global_in, nullptr, dZ, ldp(C), p.stats_ws, stats, st));

    // ---------------- backward
    for (int l = k - 1; l >= 0; --l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        const void* Hin = l == 0 ? X : (const void*)p.L[l - 1].H_out;
        const int64_t ldin = l == 0 ? m->dims[0] : ldp(fin);
        const int in_bf16 = l == 0 && m->feat_dtype == GRP_DTYPE_BF16;
        GRP_TRY(launch_colsum(dZ, n, fout, ldp(fout), grad + L.off_b, p.colsum_ws, st));
        GemmTNArgs t;
        t.M = n; t.K = fin; t.N = fout; t.A = Hin; t.lda = ldin; t.a_bf16 = in_bf16; t.B = dZ; t.ldb = ldp(fout);
        t.C = grad + L.off_ws; t.ldc = fout; t.workspace = p.tn_ws; t.workspace_bytes = p.tn_ws_bytes;
        GRP_TRY(launch_gemm_tn(t, st));
        if (L.agg_first) {
            t.A = L.M; t.lda = ldp(fin); t.a_bf16 = 0; t.C = grad + L.off_wn;
            GRP_TRY(launch_gemm_tn(t, st));
            if (l > 0) {
                GemmNNArgs a;      // dM' = (dZ Wn^T) / d_in
                a.M = n; a.N = fin; a.K = fout; a.A = dZ; a.lda = ldp(fout); a.B = L.Wt_n; a.ldb = ldp(fin);
                a.rowscale = p.inv_in; a.C = p.tmpA; a.ldc = ldp(fin); a.zero_pad_to = (int)ldp(fin);
                GRP_TRY(launch_gemm_nn(a, st));
                SpmmArgs s;        // P = A^T dM'
                s.ptr = g->colptr; s.idx = g->row; s.nnz = g->nnz; s.long_rows = &g->csc_long; s.partials = p.partials; s.n_rows = n; s.F = fin; s.X = p.tmpA; s.ldx = ldp(fin);
                s.Y = p.tmpB; s.ldy = ldp(fin);
                GRP_TRY(launch_spmm(s, st));
                GemmNNArgs c;      // dZ_prev = mask * (dZ Ws^T + P)
                c.M = n; c.N = fin; c.K = fout; c.A = dZ; c.lda = ldp(fout); c.B = L.Wt_s; c.ldb = ldp(fin);
                c.addend = p.tmpB; c.ld_add = ldp(fin); c.mask = p.L[l - 1].H_out; c.ld_mask = ldp(fin);
                c.C = dZ_other; c.ldc = ldp(fin); c.zero_pad_to = (int)ldp(fin);
                GRP_TRY(launch_gemm_nn(c, st));
            }
        } else {
            SpmmArgs s;            // dT = A^T (dZ / d_in)
            s.ptr = g->colptr; s.idx = g->row; s.nnz = g->nnz; s.long_rows = &g->csc_long; s.partials = p.partials; s.n_rows = n; s.F = fout; s.X = dZ; s.ldx = ldp(fout);
            s.colscale = p.inv_in; s.Y = p.tmpA; s.ldy = ldp(fout);
            GRP_TRY(launch_spmm(s, st));
            t.B = p.tmpA; t.C = grad + L.off_wn;
            GRP_TRY(launch_gemm_tn(t, st));
            if (l > 0) {
                GemmNNArgs c;      // dZ_prev = mask * (dZ Ws^T + dT Wn^T)
                c.M = n; c.N = fin; c.K = fout; c.A = dZ; c.lda = ldp(fout); c.B = L.Wt_s; c.ldb = ldp(fin);
                c.K2 = fout; c.A2 = p.tmpA; c.lda2 = ldp(fout); c.B2 = L.Wt_n; c.ldb2 = ldp(fin);
                c.mask = p.L[l - 1].H_out; c.ld_mask = ldp(fin);
                c.C = dZ_other; c.ldc = ldp(fin); c.zero_pad_to = (int)ldp(fin);
                GRP_TRY(launch_gemm_nn(c, st));
            }
        }
        float* sw = dZ; dZ = dZ_other; dZ_other = sw;
    }
    return GRP_OK;
}

static grp_status gcn_step(const grp_partition_t* g, const grp_model_desc* m, const grp_step_opts* o, const void* X,
                           const int32_t* labels, const uint8_t* mask, const float* theta, StepPlan& p, hipStream_t st,
                           float* grad, grp_step_stats* stats) {
    const int k = m->n_layers;
    const int64_t n = g->n;
    const int sl = m->gcn_self_loops ? 1 : 0;
    GRP_TRY(launch_degree_scales(g->d_local_in, g->d_local_out, n, sl, nullptr, p.gr, p.gs, p.grinv, st));
    for (int l = 0; l < k; ++l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        GRP_TRY(launch_pad_copy(theta + L.off_ws, fin, fout, L.Wp_s, ldp(fout), st));
        if (l > 0) GRP_TRY(launch_transpose(theta + L.off_ws, fin, fout, L.Wt_s, ldp(fin), fout, st));
    }
    GRP_TRY(launch_stats(n, nullptr, mask, g->d_local_in, g->d_global_in, nullptr, g->nnz, p.stats_ws, stats, st));

    // forward: T' = diag(s) (H W);  H' = ReLU(diag(r) (A T' + sl T') + b)
    const void* H = X;
    int64_t ldh = m->dims[0];
    int h_bf16 = m->feat_dtype == GRP_DTYPE_BF16;
    for (int l = 0; l < k; ++l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        GemmNNArgs a;
        a.M = n; a.N = fout; a.K = fin; a.A = H; a.lda = ldh; a.a_bf16 = h_bf16; a.B = L.Wp_s; a.ldb = ldp(fout);
        a.rowscale = p.gs; a.C = p.tmpA; a.ldc = ldp(fout); a.zero_pad_to = (int)ldp(fout);
        GRP_TRY(launch_gemm_nn(a, st));
        SpmmArgs s;
        s.ptr = g->rowptr; s.idx = g->col; s.nnz = g->nnz; s.long_rows = &g->csr_long; s.partials = p.partials; s.n_rows = n; s.F = fout; s.X = p.tmpA; s.ldx = ldp(fout);
        s.scale = GRP_SCALE_RSQRT; s.self_term = sl; s.bias = theta + L.off_b; s.relu = l < k - 1;
        s.Y = L.H_out; s.ldy = ldp(fout);
        GRP_TRY(launch_spmm(s, st));
        H = L.H_out; ldh = ldp(fout); h_bf16 = 0;
    }

    // loss: dZ' = diag(r) dZ
    const int C = m->dims[k];
    float* dZ = p.dZa;
    float* dZ_other = p.dZb;
    GRP_TRY(launch_softmax_xent(n, C, p.L[k - 1].H_out, ldp(C), labels, nullptr, mask, o->estimator == GRP_EST_NODE_LEVEL,
                                g->d_local_in, g->d_global_in, p.gr, dZ, ldp(C), p.stats_ws, stats, st));

    // backward: dT = diag(s) (A^T dZ' + sl dZ');  dW = H^T dT;  db = 1^T dZ;  dZ'_prev = diag(r) mask (dT W^T)
    for (int l = k - 1; l >= 0; --l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        const void* Hin = l == 0 ? X : (const void*)p.L[l - 1].H_out;
        const int64_t ldin = l == 0 ? m->dims[0] : ldp(fin);
        const int in_bf16 = l == 0 && m->feat_dtype == GRP_DTYPE_BF16;
        GRP_TRY(launch_colsum_scaled(dZ, n, fout, ldp(fout), p.grinv, grad + L.off_b, p.colsum_ws, st));
        SpmmArgs s;
        s.ptr = g->colptr; s.idx = g->row; s.nnz = g->nnz; s.long_rows = &g->csc_long; s.partials = p.partials; s.n_rows = n; s.F = fout; s.X = dZ; s.ldx = ldp(fout);
        s.scale = GRP_SCALE_RSQRT; s.self_term = sl; s.Y = p.tmpA; s.ldy = ldp(fout);
        GRP_TRY(launch_spmm(s, st));
        GemmTNArgs t;
        t.M = n; t.K = fin; t.N = fout; t.A = Hin; t.lda = ldin; t.a_bf16 = in_bf16; t.B = p.tmpA; t.ldb = ldp(fout);
        t.C = grad + L.off_ws; t.ldc = fout; t.workspace = p.tn_ws; t.workspace_bytes = p.tn_ws_bytes;
        GRP_TRY(launch_gemm_tn(t, st));
        if (l > 0) {
            GemmNNArgs c;
            c.M = n; c.N = fin; c.K = fout; c.A = p.tmpA; c.lda = ldp(fout); c.B = L.Wt_s; c.ldb = ldp(fin);
            c.rowscale = p.gr; c.mask = p.L[l - 1].H_out; c.ld_mask = ldp(fin);
            c.C = dZ_other; c.ldc = ldp(fin); c.zero_pad_to = (int)ldp(fin);
            GRP_TRY(launch_gemm_nn(c, st));
        }
        float* sw = dZ; dZ = dZ_other; dZ_other = sw;
    }
    return GRP_OK;
}

}  // namespace grp

extern "C" int64_t grp_param_count(const grp_model_desc* model) {
    if (!grp::valid_model(model)) return -1;
    return grp::param_count(model);
}

extern "C" grp_status grp_step_workspace_bytes(const grp_partition_t* part, const grp_model_desc* model,
                                               const grp_step_opts* opts, size_t* bytes) {
    using namespace grp;
    if (!bytes) return fail(GRP_EINVAL, "grp_step_workspace_bytes: null output");
    *bytes = 0;
    GRP_TRY(check_step_args(part, model, opts));
    *bytes = make_plan(part, model, nullptr, 0).total;
    return GRP_OK;
}

extern "C" grp_status grp_train_step(const grp_partition_t* part, const grp_model_desc* model, const grp_step_opts* opts,
                                     const void* features, const int32_t* labels, const uint8_t* train_mask,
                                     const float* weights, void* workspace, size_t workspace_bytes, void* stream,
                                     float* grad_out, grp_step_stats* stats_out) {
    using namespace grp;
    GRP_TRY(check_step_args(part, model, opts));
    if (!weights || !grad_out || !stats_out) return fail(GRP_EINVAL, "train_step: null weights / grad_out / stats_out");
    if (part->n > 0 && (!features || !labels)) return fail(GRP_EINVAL, "train_step: null features or labels");
    StepPlan need = make_plan(part, model, nullptr, 0);
    if (!workspace || workspace_bytes < need.total)
        return fail(GRP_EWORKSPACE, "train_step: workspace %zu bytes, need %zu", workspace_bytes, need.total);
    if ((uintptr_t)workspace % 256 != 0) return fail(GRP_EINVAL, "train_step: workspace must be 256-byte aligned");
    StepPlan p = make_plan(part, model, workspace, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    if (model->arch == GRP_ARCH_SAGE_MEAN)
        return sage_step(part, model, opts, features, labels, train_mask, weights, p, st, grad_out, stats_out);
    return gcn_step(part, model, opts, features, labels, train_mask, weights, p, st, grad_out, stats_out);
}
