// One isolated train step on one partition: (sampling,) forward, loss, backward, coverage
// statistics.  Host-side orchestration of the kernels in sampler.hip / spmm.hip / gemm.hip /
// elementwise.hip on one stream, with every intermediate carved out of the caller's
// workspace (no allocation; full-graph mode never synchronises the stream, mini-batch mode
// does once per layer above the input layer to learn the sampled block sizes).
//
// Every layer is a bipartite block (common.h): in full-graph mode all layers share the
// partition's CSR/CSC, in mini-batch mode each layer has its sampled block.  Per GraphSAGE
// layer the neighbour aggregation runs at the narrower of the two widths (mean and the
// linear map commute): "aggregate first" when Fin <= Fout, "transform first" otherwise.
#include "common.h"

#include <vector>

namespace grp {

static inline int64_t ldp(int64_t f) { return round_up(f, 4); }
static inline bool measure_only(const void* p) { return p == nullptr; }

struct LayerBufs {
    float* Wp_s = nullptr;   // [ld(Fin) x ld(Fout)] aligned, zero-padded copy of W_self (GCN: W)
    float* Wp_n = nullptr;   // same for W_neigh
    float* Wt_s = nullptr;   // [ld(Fout) x ld(Fin)] transpose of W_self
    float* Wt_n = nullptr;
    float* M = nullptr;      // [rows x ld(Fin)] aggregated input (aggregate-first SAGE layers)
    float* H_out = nullptr;  // [rows x ld(Fout)] layer output (post-activation; logits for the last layer)
    float* Act = nullptr;    // [rows x ld(Fout)] ReLU(z) of a residual layer (its derivative mask)
    int64_t off_ws = 0, off_wn = 0, off_b = 0;
    int64_t ldwp = 0, ldwt = 0;   // pitches of Wp_* / Wt_* (SAGE keeps [W_neigh | W_self] side by side)
    bool agg_first = false;
    bool skip = false;       // residual GCN: H_out = H_in + ReLU(z)
};

struct StepPlan {
    std::vector<LayerBufs> L;
    float *inv_in = nullptr, *gr = nullptr, *gs = nullptr, *grinv = nullptr;
    float* Xpad = nullptr;       // residual first layer: zero-padded copy of features whose rows are not 16-byte friendly
    float* gr_drop = nullptr;    // gr / (1 - dropout rate): the row scale of the backward pass through a dropped layer
    float *tmpA = nullptr, *tmpB = nullptr, *dZa = nullptr, *dZb = nullptr, *Ga = nullptr, *Gb = nullptr;
    void *tn_ws = nullptr, *colsum_ws = nullptr, *stats_ws = nullptr, *sampler_ws = nullptr;
    float* partials = nullptr;   // partial rows of the split long rows (SpMM)
    size_t tn_ws_bytes = 0, sampler_bytes = 0;
    size_t total = 0;
};

static bool valid_model(const grp_model_desc* m) {
    if (!m) return false;
    if (m->arch < GRP_ARCH_SAGE_MEAN || m->arch > GRP_ARCH_GAT) return false;
    if (m->n_layers < 1 || m->n_layers > GRP_MAX_LAYERS) return false;
    for (int l = 0; l <= m->n_layers; ++l)
        if (m->dims[l] <= 0 || m->dims[l] > 1024) return false;
    if (m->feat_dtype != GRP_DTYPE_FP32 && m->feat_dtype != GRP_DTYPE_BF16) return false;
    return true;
}

static int64_t param_count(const grp_model_desc* m) {
    if (m->arch == GRP_ARCH_GAT) {        // per layer W, a_src, a_dst, b
        int64_t p = 0;
        for (int l = 0; l < m->n_layers; ++l) p += (int64_t)m->dims[l] * m->dims[l + 1] + 3 * m->dims[l + 1];
        return p;
    }
    const int per = m->arch == GRP_ARCH_SAGE_MEAN ? 2 : 1;
    int64_t p = 0;
    for (int l = 0; l < m->n_layers; ++l) p += (int64_t)per * m->dims[l] * m->dims[l + 1] + m->dims[l + 1];
    return p;
}

// Carves (or, with a null base, measures) the workspace.  Row counts are exact in full-graph
// mode and upper bounds from the seeds and fanouts in mini-batch mode.
static StepPlan make_plan(const grp_partition_t* part, const grp_model_desc* m, const grp_step_opts* o, void* ws,
                          size_t ws_bytes) {
    StepPlan p;
    const int64_t n = part->n;
    Bump b(ws, ws_bytes);
    const int k = m->n_layers;
    const bool sage = m->arch == GRP_ARCH_SAGE_MEAN;
    const bool mb = !o->full_graph;
    SamplerBounds bd;
    // partial rows of the split long rows: one per task of the sliced schedule, else one per chunk
    auto slots = [](const LongRows& lr) { return lr.n_tasks > 0 ? lr.n_tasks : (int64_t)lr.n_chunks; };
    int64_t chunks_cap = slots(part->csr_long) > slots(part->csc_long) ? slots(part->csr_long) : slots(part->csc_long);
    if (mb) {
        sampler_bounds(n, o->n_seeds, o->fanouts, k, &bd);
        p.sampler_bytes = sampler_workspace_bytes(n, bd, k);
        p.sampler_ws = b.take<char>(p.sampler_bytes);
        chunks_cap = 0;
        for (int l = 1; l < k; ++l) {
            const int64_t c = bd.nnz[l] / SPMM_CHUNK + bd.nnz[l] / SPMM_LONG_ROW + 2;
            if (c > chunks_cap) chunks_cap = c;
        }
    }
    p.L.resize(k);
    int64_t off = 0, fmax = 0, max_rows = 1;
    size_t tn_bytes = 0, cs_bytes = 0;
    for (int l = 0; l < k; ++l) {
        LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        const int64_t rows = mb ? bd.dst[l] : n;
        const int64_t rows_in = mb ? (l == 0 ? bd.dst[0] : bd.src[l]) : n;
        if (rows > max_rows) max_rows = rows;
        if (rows_in > max_rows) max_rows = rows_in;
        L.off_ws = off; off += (int64_t)fin * fout;
        if (sage) { L.off_wn = off; off += (int64_t)fin * fout; }
        L.off_b = off; off += fout;
        L.agg_first = sage && (fin <= fout || (mb && l == 0));
        L.skip = m->arch == GRP_ARCH_GCN_RESIDUAL && fin == fout && l < k - 1;
        if (sage) {
            // W_neigh stacked on top of W_self (row offset rounded up to 4, pad rows zero), so that
            // one product can span both: [.. | ..] = X [Wn | Ws] reads the stack as one Bt.
            L.ldwp = ldp(fout);
            L.ldwt = ldp(fin);
            float* wp = b.take<float>((size_t)2 * ldp(fin) * L.ldwp);
            float* wt = b.take<float>((size_t)2 * ldp(fout) * L.ldwt);
            L.Wp_n = wp; L.Wp_s = measure_only(wp) ? nullptr : wp + ldp(fin) * L.ldwp;
            L.Wt_n = wt; L.Wt_s = measure_only(wt) ? nullptr : wt + ldp(fout) * L.ldwt;
            if (L.agg_first) L.M = b.take<float>((size_t)rows * ldp(fin));
        } else {
            L.ldwp = ldp(fout);
            L.ldwt = ldp(fin);
            L.Wp_s = b.take<float>((size_t)ldp(fin) * ldp(fout));
            L.Wt_s = b.take<float>((size_t)ldp(fout) * ldp(fin));
        }
        L.H_out = b.take<float>((size_t)rows * ldp(fout));
        if (L.skip) L.Act = b.take<float>((size_t)rows * ldp(fout));
        if (ldp(fout) > fmax) fmax = ldp(fout);
        if (l > 0 && ldp(fin) > fmax) fmax = ldp(fin);
        const size_t t = gemm_tn_workspace_bytes(rows_in > rows ? rows_in : rows, fin, fout);
        if (t > tn_bytes) tn_bytes = t;
        const size_t c = colsum_workspace_bytes(rows, fout);
        if (c > cs_bytes) cs_bytes = c;
    }
    if (!mb) p.inv_in = b.take<float>((size_t)n);
    if (!sage) {
        p.gr = b.take<float>((size_t)n);
        p.gs = b.take<float>((size_t)n);
        p.grinv = b.take<float>((size_t)n);
        if (o->dropout_rate > 0.f) p.gr_drop = b.take<float>((size_t)n);
        if (p.L[0].skip) p.Xpad = b.take<float>((size_t)n * ldp(m->dims[0]));
    }
    p.tmpA = b.take<float>((size_t)max_rows * 2 * fmax);   // holds two matrices side by side in the fused layers
    p.tmpB = b.take<float>((size_t)max_rows * fmax);
    p.dZa = b.take<float>((size_t)max_rows * fmax);
    p.dZb = b.take<float>((size_t)max_rows * fmax);
    if (m->arch == GRP_ARCH_GCN_RESIDUAL) {
        p.Ga = b.take<float>((size_t)max_rows * fmax);
        p.Gb = b.take<float>((size_t)max_rows * fmax);
    }
    p.tn_ws = b.take<char>(tn_bytes);
    p.tn_ws_bytes = tn_bytes;
    p.colsum_ws = b.take<char>(cs_bytes);
    p.stats_ws = b.take<char>(stats_workspace_bytes(n));
    {
        int64_t fsp = 0;                                   // the widest aggregation of the step
        for (int l = 0; l < k; ++l) {
            const int64_t w = sage ? (p.L[l].agg_first ? ldp(m->dims[l]) : ldp(m->dims[l + 1]))
                                   : (ldp(m->dims[l]) > ldp(m->dims[l + 1]) ? ldp(m->dims[l]) : ldp(m->dims[l + 1]));
            if (w > fsp) fsp = w;
        }
        p.partials = b.take<float>((size_t)chunks_cap * fsp);
    }
    p.total = b.total();
    return p;
}

static grp_status check_step_args(const grp_partition_t* part, const grp_model_desc* model, const grp_step_opts* opts) {
    if (!part || !opts) return fail(GRP_EINVAL, "train_step: null partition or options");
    if (!valid_model(model)) return fail(GRP_EINVAL, "train_step: invalid model description");
    if (opts->estimator < GRP_EST_NONE || opts->estimator > GRP_EST_SHRINKAGE)
        return fail(GRP_EINVAL, "train_step: unknown estimator %d", opts->estimator);
    if (model->arch == GRP_ARCH_GCN_RESIDUAL && model->feat_dtype == GRP_DTYPE_BF16 && model->n_layers > 1 &&
        model->dims[0] == model->dims[1])
        return fail(GRP_EUNSUPPORTED, "train_step: a residual first layer needs fp32 features");
    if (part->csr_w && (model->arch != GRP_ARCH_SAGE_MEAN || !opts->full_graph))
        return fail(GRP_EUNSUPPORTED, "train_step: a weighted partition trains GraphSAGE in full-graph mode only");
    if (!(opts->dropout_rate >= 0.f && opts->dropout_rate < 1.f))
        return fail(GRP_EINVAL, "train_step: dropout rate outside [0, 1)");
    if (!opts->full_graph) {
        if (model->arch != GRP_ARCH_SAGE_MEAN)
            return fail(GRP_EUNSUPPORTED, "train_step: mini-batch mode is implemented for GraphSAGE only");
        if (opts->n_seeds < 1 || !opts->seeds) return fail(GRP_EINVAL, "train_step: mini-batch mode needs seed nodes");
        for (int l = 0; l < model->n_layers; ++l)
            if (opts->fanouts[l] < 1 || opts->fanouts[l] > 64)
                return fail(GRP_EINVAL, "train_step: fanout %d outside [1, 64]", opts->fanouts[l]);
    }
    return GRP_OK;
}

static void fill_spmm(SpmmArgs& s, const Block& B, bool transposed, float* partials) {
    s.ptr = transposed ? B.ptrT : B.ptr;
    s.idx = transposed ? B.idxT : B.idx;
    s.nnz = B.nnz;
    s.n_rows = transposed ? B.n_in : B.n_dst;
    s.n_rows_dev = transposed ? B.n_in_dev : B.n_dst_dev;
    s.n_src = transposed ? B.n_dst : B.n_in;
    s.long_rows = transposed ? B.long_bwd : B.long_fwd;
    s.partials = partials;
    s.val = transposed ? B.valT : B.val;
}

// The mean aggregator of a block: 1 / row length, or on a weighted partition the explicit
// 1 / (local weight mass) beside the per-edge weights fill_spmm has set.
static void set_mean(SpmmArgs& s, const Block& B) {
    if (B.val) s.rowscale = B.inv_in;
    else s.scale = GRP_SCALE_MEAN;
}

// bwd_scale multiplies the weights of the products that carry a gradient back through a layer
// output: 1 / (1 - rate) with dropout (the kept elements were scaled by it), else 1.
static grp_status prep_weights(const grp_model_desc* m, const float* theta, StepPlan& p, float bwd_scale, hipStream_t st) {
    const bool sage = m->arch == GRP_ARCH_SAGE_MEAN;
    PackJobs jobs;
    for (int l = 0; l < m->n_layers; ++l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        // the products read their weights transposed: forward uses W^T (rows = outputs), the
        // backward pass to the layer below uses W itself (rows = inputs)
        pack_jobs_add(jobs, theta + L.off_ws, fin, fout, true, (int)ldp(fout), L.Wt_s, L.ldwt);
        if (sage) pack_jobs_add(jobs, theta + L.off_wn, fin, fout, true, (int)ldp(fout), L.Wt_n, L.ldwt);
        if (l > 0) {
            pack_jobs_add(jobs, theta + L.off_ws, fin, fout, false, (int)ldp(fin), L.Wp_s, L.ldwp, bwd_scale);
            if (sage) pack_jobs_add(jobs, theta + L.off_wn, fin, fout, false, (int)ldp(fin), L.Wp_n, L.ldwp, bwd_scale);
        }
    }
    return launch_pack_weights(jobs, st);
}

static grp_status sage_step(const grp_partition_t* g, const grp_model_desc* m, const grp_step_opts* o, const Block* blk,
                            const void* X, const int32_t* labels, const uint8_t* mask, const int32_t* loss_nodes,
                            const float* theta, StepPlan& p, hipStream_t st, float* grad, grp_step_stats* stats,
                            hipEvent_t transposed_ready = nullptr) {
    const int k = m->n_layers;
    const DropoutPlan drop = dropout_plan(o);
    GRP_TRY(prep_weights(m, theta, p, drop.scale, st));

    // ---------------- forward
    const void* H = X;
    int64_t ldh = m->dims[0];
    int h_bf16 = m->feat_dtype == GRP_DTYPE_BF16;
    for (int l = 0; l < k; ++l) {
        const LayerBufs& L = p.L[l];
        const Block& B = blk[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        const int relu = l < k - 1;
        if (B.n_dst == 0) { H = L.H_out; ldh = ldp(fout); h_bf16 = 0; continue; }
        if (L.agg_first) {
            SpmmArgs s;
            fill_spmm(s, B, false, p.partials);
            s.F = fin; s.X = H; s.ldx = ldh; s.x_bf16 = h_bf16; set_mean(s, B); s.Y = L.M; s.ldy = ldp(fin);
            GRP_TRY(launch_spmm(s, st));
            GemmNNArgs a;
            a.M = B.n_dst; a.M_dev = B.n_dst_dev; a.N = fout; a.K = fin; a.A = H; a.lda = ldh; a.a_bf16 = h_bf16;
            a.a_rows = B.self_rows; a.Bt = L.Wt_s; a.ldbt = L.ldwt;
            a.K2 = fin; a.A2 = L.M; a.lda2 = ldp(fin); a.Bt2 = L.Wt_n; a.ldbt2 = L.ldwt;
            a.bias = theta + L.off_b; a.relu = relu; a.C = L.H_out; a.ldc = ldp(fout); a.zero_pad_to = (int)ldp(fout);
            GRP_TRY(launch_gemm_nn(a, st));
        } else if (B.n_in == B.n_dst && !B.self_rows && !B.n_dst_dev) {
            // [T | Z0] = H [Wn | Ws] (+ b on the second half) in one pass over H, then
            // H' = ReLU(mean-aggregate(T) + Z0)
            const int64_t w2 = 2 * ldp(fout);
            GemmNNArgs a;
            a.M = B.n_dst; a.N = (int)(ldp(fout) + fout); a.K = fin; a.A = H; a.lda = ldh; a.a_bf16 = h_bf16;
            a.Bt = L.Wt_n; a.ldbt = L.ldwt; a.bias = theta + L.off_b; a.bias_col0 = (int)ldp(fout); a.bias_n = fout;
            a.C = p.tmpA; a.ldc = w2; a.zero_pad_to = (int)w2;
            GRP_TRY(launch_gemm_nn(a, st));
            SpmmArgs s;
            fill_spmm(s, B, false, p.partials);
            s.F = fout; s.X = p.tmpA; s.ldx = w2; set_mean(s, B);
            s.addend = p.tmpA + ldp(fout); s.ld_add = w2; s.relu = relu; s.Y = L.H_out; s.ldy = ldp(fout);
            GRP_TRY(launch_spmm(s, st));
        } else {
            GemmNNArgs a;      // T = H Wn over every input row, Z0 = H_self Ws + b
            a.M = B.n_in; a.M_dev = B.n_in_dev; a.N = fout; a.K = fin; a.A = H; a.lda = ldh; a.a_bf16 = h_bf16;
            a.Bt = L.Wt_n; a.ldbt = L.ldwt;
            a.C = p.tmpA; a.ldc = ldp(fout); a.zero_pad_to = (int)ldp(fout);
            GRP_TRY(launch_gemm_nn(a, st));
            a.M = B.n_dst; a.M_dev = B.n_dst_dev; a.a_rows = B.self_rows; a.Bt = L.Wt_s; a.bias = theta + L.off_b; a.C = L.H_out;
            GRP_TRY(launch_gemm_nn(a, st));
            SpmmArgs s;
            fill_spmm(s, B, false, p.partials);
            s.F = fout; s.X = p.tmpA; s.ldx = ldp(fout); set_mean(s, B);
            s.addend = L.H_out; s.ld_add = ldp(fout); s.relu = relu; s.Y = L.H_out; s.ldy = ldp(fout);
            GRP_TRY(launch_spmm(s, st));
        }
        if (relu) GRP_TRY(launch_dropout(drop, l, g->l2g, B.n_dst, fout, L.H_out, ldp(fout), nullptr, 0, nullptr, 0, st, B.dst_nodes,
                                          B.n_dst_dev));
        H = L.H_out; ldh = ldp(fout); h_bf16 = 0;
    }

    // ---------------- loss
    const int C = m->dims[k];
    const int64_t n_loss_rows = blk[k - 1].n_dst;
    float* dZ = p.dZa;
    float* dZ_other = p.dZb;
    GRP_TRY(launch_softmax_xent(n_loss_rows, C, p.L[k - 1].H_out, ldp(C), labels, loss_nodes, mask,
                                o->estimator == GRP_EST_NODE_LEVEL, g->d_local_in, g->d_global_in, nullptr, dZ, ldp(C),
                                p.stats_ws, stats, st, g->w_local_in, g->w_global_in));

    // ---------------- backward
    if (transposed_ready) GRP_HIP(hipStreamWaitEvent(st, transposed_ready, 0));   // the blocks' transposed structures
    for (int l = k - 1; l >= 0; --l) {
        const LayerBufs& L = p.L[l];
        const Block& B = blk[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        const void* Hin = l == 0 ? X : (const void*)p.L[l - 1].H_out;
        const int64_t ldin = l == 0 ? m->dims[0] : ldp(fin);
        const int in_bf16 = l == 0 && m->feat_dtype == GRP_DTYPE_BF16;
        GemmTNArgs t;      // dW_self = H_self^T dZ, and db = 1^T dZ from the same pass over dZ
        t.M = B.n_dst; t.M_dev = B.n_dst_dev; t.K = fin; t.N = fout; t.A = Hin; t.lda = ldin; t.a_bf16 = in_bf16; t.a_rows = B.self_rows;
        t.B = dZ; t.ldb = ldp(fout); t.C = grad + L.off_ws; t.ldc = fout; t.workspace = p.tn_ws; t.workspace_bytes = p.tn_ws_bytes;
        t.colsum_out = grad + L.off_b;
        // the same rows of the input feed both weight gradients of a transform-first layer
        const bool shared_rows = !L.agg_first && B.n_in == B.n_dst && !B.self_rows && !B.n_dst_dev;
        if (L.agg_first) {
            t.A2 = L.M; t.lda2 = ldp(fin); t.C2 = grad + L.off_wn;       // dW_neigh = M^T dZ in the same launch
            GRP_TRY(launch_gemm_tn(t, st));
        } else if (!shared_rows) {
            GRP_TRY(launch_gemm_tn(t, st));
        }
        if (L.agg_first) {
            if (l > 0 && B.n_in > 0) {
                // [dM' | dS] = dZ [Wn^T | Ws^T], dM' rows divided by |N_v|, in one pass over dZ;
                // then dZ_prev = mask * (A^T dM' + [dS ; 0]) in the aggregation's epilogue.
                const int64_t w2 = 2 * ldp(fin);
                if (B.n_dst > 0) {
                    GemmNNArgs a;
                    a.M = B.n_dst; a.M_dev = B.n_dst_dev; a.N = (int)(ldp(fin) + fin); a.K = fout; a.A = dZ; a.lda = ldp(fout);
                    a.Bt = L.Wp_n; a.ldbt = L.ldwp; a.rowscale = B.inv_in; a.rowscale_cols = (int)ldp(fin);
                    a.C = p.tmpA; a.ldc = w2; a.zero_pad_to = (int)w2;
                    GRP_TRY(launch_gemm_nn(a, st));
                }
                SpmmArgs s;
                fill_spmm(s, B, true, p.partials);
                s.F = fin; s.X = p.tmpA; s.ldx = w2; s.addend = p.tmpA + ldp(fin); s.ld_add = w2;
                s.addend_rows = B.n_dst; s.addend_rows_dev = B.n_dst_dev; s.mask = p.L[l - 1].H_out; s.ld_mask = ldp(fin);
                s.Y = dZ_other; s.ldy = ldp(fin);
                GRP_TRY(launch_spmm(s, st));
            }
        } else {
            SpmmArgs s;            // dT = A^T (dZ / |N_v|)  over the block's inputs
            fill_spmm(s, B, true, p.partials);
            s.F = fout; s.X = dZ; s.ldx = ldp(fout); s.colscale = B.inv_in; s.Y = p.tmpA; s.ldy = ldp(fout);
            // The per-edge gather of 1/|N_v| costs a cache line per edge once that array outgrows the L2:
            // where a row has more edges than an eighth of its width it is cheaper to scale dZ's rows once.
            if (B.nnz > (int64_t)B.n_dst * fout / 8) {
                GRP_TRY(launch_scale_rows(dZ, ldp(fout), B.inv_in, B.n_dst, fout, p.tmpB, ldp(fout), st, B.n_dst_dev));
                s.X = p.tmpB;
                s.colscale = nullptr;
            }
            GRP_TRY(launch_spmm(s, st));
            if (shared_rows) {     // [dW_self | dW_neigh] = H^T [dZ | dT] in one launch
                t.B2 = p.tmpA; t.ldb2 = ldp(fout); t.C2 = grad + L.off_wn;
            } else {
                t.colsum_out = nullptr;
                t.M = B.n_in; t.M_dev = B.n_in_dev; t.a_rows = nullptr; t.B = p.tmpA; t.C = grad + L.off_wn;
            }
            GRP_TRY(launch_gemm_tn(t, st));
            if (l > 0 && B.n_in > 0) {
                GemmNNArgs c;      // dZ_prev = mask * ([dZ Ws^T ; 0] + dT Wn^T)
                c.M = B.n_in; c.M_dev = B.n_in_dev; c.N = fin; c.K = fout; c.A = dZ; c.lda = ldp(fout);
                c.a_valid_rows = B.n_dst; c.a_valid_rows_dev = B.n_dst_dev;
                c.Bt = L.Wp_s; c.ldbt = L.ldwp;
                c.K2 = fout; c.A2 = p.tmpA; c.lda2 = ldp(fout); c.Bt2 = L.Wp_n; c.ldbt2 = L.ldwp;
                c.mask = p.L[l - 1].H_out; c.ld_mask = ldp(fin);
                c.C = dZ_other; c.ldc = ldp(fin); c.zero_pad_to = (int)ldp(fin);
                GRP_TRY(launch_gemm_nn(c, st));
            }
        }
        float* sw = dZ; dZ = dZ_other; dZ_other = sw;
    }
    return GRP_OK;
}

// GCN / residual GCN, full-graph mode.
//   forward:  T' = diag(s) (H W);  A = ReLU(diag(r) (Adj T' + sl T') + b);  H' = A (+ H on a residual layer)
//   backward: with G = dL/dH' and dZ' = diag(r) (A > 0) G:
//             db = 1^T diag(1/r) dZ';  dT = diag(s) (Adj^T dZ' + sl dZ');  dW = H^T dT;
//             G_in = dT W^T (+ G on a residual layer)
static grp_status gcn_step(const grp_partition_t* g, const grp_model_desc* m, const grp_step_opts* o, const void* X,
                           const int32_t* labels, const uint8_t* mask, const float* theta, StepPlan& p, hipStream_t st,
                           float* grad, grp_step_stats* stats) {
    const int k = m->n_layers;
    const int64_t n = g->n;
    const int sl = m->gcn_self_loops ? 1 : 0;
    GRP_TRY(launch_degree_scales(g->d_local_in, g->d_local_out, n, sl, nullptr, p.gr, p.gs, p.grinv, st));
    GRP_TRY(prep_weights(m, theta, p, 1.f, st));
    // With dropout the gradient that reaches a hidden activation is also multiplied by 1 / (1 - rate);
    // the residual path bypasses it, so the factor rides on the row scale of the masked output.
    const DropoutPlan drop = dropout_plan(o);
    if (drop.on) GRP_TRY(launch_scale_copy(p.gr, drop.scale, p.gr_drop, n, st));
    const float* gr_bwd = drop.on ? p.gr_drop : p.gr;
    Block B;
    B.n_dst = B.n_in = n; B.nnz = g->nnz; B.ptr = g->rowptr; B.idx = g->col; B.ptrT = g->colptr; B.idxT = g->row;
    B.long_fwd = &g->csr_long; B.long_bwd = &g->csc_long;

    const void* H = X;
    int64_t ldh = m->dims[0];
    int h_bf16 = m->feat_dtype == GRP_DTYPE_BF16;
    for (int l = 0; l < k && n > 0; ++l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        if (l == 0 && L.skip && (ldh % 4 != 0 || (uintptr_t)H % 16 != 0)) {
            // the skip is added from 16-byte vectors: give the layer an aligned copy of the features
            GRP_TRY(launch_pad_rows((const float*)X, ldh, n, fin, p.Xpad, ldp(fin), st));
            H = p.Xpad;
            ldh = ldp(fin);
        }
        GemmNNArgs a;
        a.M = n; a.N = fout; a.K = fin; a.A = H; a.lda = ldh; a.a_bf16 = h_bf16; a.Bt = L.Wt_s; a.ldbt = L.ldwt;
        a.rowscale = p.gs; a.C = p.tmpA; a.ldc = ldp(fout); a.zero_pad_to = (int)ldp(fout);
        GRP_TRY(launch_gemm_nn(a, st));
        SpmmArgs s;
        fill_spmm(s, B, false, p.partials);
        s.F = fout; s.X = p.tmpA; s.ldx = ldp(fout); s.scale = GRP_SCALE_RSQRT; s.self_term = sl;
        s.bias = theta + L.off_b; s.relu = l < k - 1; s.Y = L.H_out; s.ldy = ldp(fout);
        if (L.skip) { s.residual = (const float*)H; s.ld_res = ldh; s.Y2 = L.Act; s.ldy2 = ldp(fout); }
        GRP_TRY(launch_spmm(s, st));
        if (l < k - 1)
            GRP_TRY(launch_dropout(drop, l, g->l2g, n, fout, L.H_out, ldp(fout), L.skip ? L.Act : nullptr, ldp(fout),
                                   L.skip ? (const float*)H : nullptr, ldh, st));
        H = L.H_out; ldh = ldp(fout); h_bf16 = 0;
    }

    const int C = m->dims[k];
    float* dZ = p.dZa;          // dZ' of the current layer
    float* dZ_other = p.dZb;
    float* G = p.Ga;            // dL/dH' of the current layer (residual models only)
    float* G_other = p.Gb;
    GRP_TRY(launch_softmax_xent(n, C, p.L[k - 1].H_out, ldp(C), labels, nullptr, mask, o->estimator == GRP_EST_NODE_LEVEL,
                                g->d_local_in, g->d_global_in, p.gr, dZ, ldp(C), p.stats_ws, stats, st));

    for (int l = k - 1; l >= 0; --l) {
        const LayerBufs& L = p.L[l];
        const int fin = m->dims[l], fout = m->dims[l + 1];
        const void* Hin = l == 0 ? X : (const void*)p.L[l - 1].H_out;
        const int64_t ldin = l == 0 ? m->dims[0] : ldp(fin);
        const int in_bf16 = l == 0 && m->feat_dtype == GRP_DTYPE_BF16;
        GRP_TRY(launch_colsum_scaled(dZ, n, fout, ldp(fout), p.grinv, grad + L.off_b, p.colsum_ws, st));
        SpmmArgs s;
        fill_spmm(s, B, true, p.partials);
        s.F = fout; s.X = dZ; s.ldx = ldp(fout); s.scale = GRP_SCALE_RSQRT; s.self_term = sl; s.Y = p.tmpA; s.ldy = ldp(fout);
        GRP_TRY(launch_spmm(s, st));
        GemmTNArgs t;
        t.M = n; t.K = fin; t.N = fout; t.A = Hin; t.lda = ldin; t.a_bf16 = in_bf16; t.B = p.tmpA; t.ldb = ldp(fout);
        t.C = grad + L.off_ws; t.ldc = fout; t.workspace = p.tn_ws; t.workspace_bytes = p.tn_ws_bytes;
        GRP_TRY(launch_gemm_tn(t, st));
        if (l > 0 && n > 0) {
            const LayerBufs& Lp = p.L[l - 1];
            GemmNNArgs c;      // G_in = dT W^T (+ G);  dZ'_prev = diag(r) (A_prev > 0) G_in
            c.M = n; c.N = fin; c.K = fout; c.A = p.tmpA; c.lda = ldp(fout); c.Bt = L.Wp_s; c.ldbt = L.ldwp;
            if (L.skip) { c.addend = G; c.ld_add = ldp(fout); }
            if (Lp.skip) { c.C_raw = G_other; c.ld_raw = ldp(fin); }
            c.rowscale = gr_bwd; c.mask = Lp.skip ? Lp.Act : Lp.H_out; c.ld_mask = ldp(fin);
            c.C = dZ_other; c.ldc = ldp(fin); c.zero_pad_to = (int)ldp(fin);
            GRP_TRY(launch_gemm_nn(c, st));
            float* sg = G; G = G_other; G_other = sg;
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
    *bytes = model->arch == GRP_ARCH_GAT ? gat_step_workspace_bytes(part, model) : make_plan(part, model, opts, nullptr, 0).total;
    return GRP_OK;
}

extern "C" grp_status grp_step_activation(const grp_partition_t* part, const grp_model_desc* model, const grp_step_opts* opts,
                                          void* workspace, size_t workspace_bytes, int32_t layer, const float** act_out,
                                          int64_t* ld_out) {
    using namespace grp;
    if (!act_out || !ld_out) return fail(GRP_EINVAL, "grp_step_activation: null output");
    *act_out = nullptr;
    *ld_out = 0;
    GRP_TRY(check_step_args(part, model, opts));
    if (layer < 0 || layer >= model->n_layers) return fail(GRP_EINVAL, "grp_step_activation: layer %d", layer);
    if (!workspace || (uintptr_t)workspace % 256 != 0) return fail(GRP_EINVAL, "grp_step_activation: bad workspace");
    if (model->arch == GRP_ARCH_GAT) {
        if (workspace_bytes < gat_step_workspace_bytes(part, model))
            return fail(GRP_EWORKSPACE, "grp_step_activation: workspace too small");
        gat_step_activation(part, model, workspace, workspace_bytes, layer, act_out, ld_out);
        return GRP_OK;
    }
    const StepPlan p = make_plan(part, model, opts, workspace, workspace_bytes);
    if (workspace_bytes < p.total) return fail(GRP_EWORKSPACE, "grp_step_activation: workspace too small");
    const LayerBufs& L = p.L[layer];
    *act_out = L.skip ? L.Act : L.H_out;
    *ld_out = ldp(model->dims[layer + 1]);
    return GRP_OK;
}

extern "C" grp_status grp_step_block(const grp_partition_t* part, const grp_model_desc* model, const grp_step_opts* opts,
                                     void* workspace, size_t workspace_bytes, int32_t layer, grp_block_view_t* view) {
    using namespace grp;
    if (!view) return fail(GRP_EINVAL, "grp_step_block: null output");
    memset(view, 0, sizeof *view);
    GRP_TRY(check_step_args(part, model, opts));
    if (opts->full_graph || model->arch != GRP_ARCH_SAGE_MEAN) return fail(GRP_EINVAL, "grp_step_block: not a mini-batch step");
    if (layer < 0 || layer >= model->n_layers) return fail(GRP_EINVAL, "grp_step_block: layer %d", layer);
    if (!workspace || (uintptr_t)workspace % 256 != 0) return fail(GRP_EINVAL, "grp_step_block: bad workspace");
    const StepPlan p = make_plan(part, model, opts, workspace, workspace_bytes);
    if (workspace_bytes < p.total) return fail(GRP_EWORKSPACE, "grp_step_block: workspace too small");
    return sampler_block_view(part, opts, model->n_layers, p.sampler_ws, p.sampler_bytes, layer, view);
}

extern "C" grp_status grp_train_step(const grp_partition_t* part, const grp_model_desc* model, const grp_step_opts* opts,
                                     const void* features, const int32_t* labels, const uint8_t* train_mask,
                                     const float* weights, void* workspace, size_t workspace_bytes, void* stream,
                                     float* grad_out, grp_step_stats* stats_out) {
    using namespace grp;
    GRP_TRY(check_step_args(part, model, opts));
    if (!weights || !grad_out || !stats_out) return fail(GRP_EINVAL, "train_step: null weights / grad_out / stats_out");
    if (part->n > 0 && (!features || !labels)) return fail(GRP_EINVAL, "train_step: null features or labels");
    if (model->arch == GRP_ARCH_GAT) {
        const size_t need_gat = gat_step_workspace_bytes(part, model);
        if (!workspace || workspace_bytes < need_gat)
            return fail(GRP_EWORKSPACE, "train_step: workspace %zu bytes, need %zu", workspace_bytes, need_gat);
        if ((uintptr_t)workspace % 256 != 0) return fail(GRP_EINVAL, "train_step: workspace must be 256-byte aligned");
        return gat_step(part, model, opts, features, labels, train_mask, weights, workspace, workspace_bytes,
                        (hipStream_t)stream, grad_out, stats_out);
    }
    StepPlan need = make_plan(part, model, opts, nullptr, 0);
    if (!workspace || workspace_bytes < need.total)
        return fail(GRP_EWORKSPACE, "train_step: workspace %zu bytes, need %zu", workspace_bytes, need.total);
    if ((uintptr_t)workspace % 256 != 0) return fail(GRP_EINVAL, "train_step: workspace must be 256-byte aligned");
    StepPlan p = make_plan(part, model, opts, workspace, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    const int k = model->n_layers;
    const int64_t n = part->n;

    if (model->arch != GRP_ARCH_SAGE_MEAN) {
        GRP_TRY(launch_stats(n, nullptr, train_mask, part->d_local_in, part->d_global_in, nullptr, part->nnz, nullptr, 0,
                             p.stats_ws, stats_out, st));
        return gcn_step(part, model, opts, features, labels, train_mask, weights, p, st, grad_out, stats_out);
    }

    Block blocks[GRP_MAX_LAYERS];
    if (opts->full_graph) {
        if (part->csr_w) GRP_TRY(launch_inverse_mass(part->w_local_in, n, p.inv_in, st));
        else GRP_TRY(launch_degree_scales(part->d_local_in, part->d_local_out, n, 0, p.inv_in, nullptr, nullptr, nullptr, st));
        for (int l = 0; l < k; ++l) {
            Block& B = blocks[l];
            B.n_dst = B.n_in = n; B.nnz = part->nnz; B.ptr = part->rowptr; B.idx = part->col;
            B.ptrT = part->colptr; B.idxT = part->row; B.long_fwd = &part->csr_long; B.long_bwd = &part->csc_long;
            B.inv_in = p.inv_in; B.val = part->csr_w; B.valT = part->csc_w;
        }
        GRP_TRY(launch_stats(n, nullptr, train_mask, part->d_local_in, part->d_global_in, nullptr, part->nnz, nullptr, 0,
                             p.stats_ws, stats_out, st, part->w_local_in, part->w_global_in));
        return sage_step(part, model, opts, blocks, features, labels, train_mask, nullptr, weights, p, st, grad_out,
                         stats_out);
    }

    // mini-batch: isolated sampling, then the same layers over the sampled blocks
    LongRows long_bwd[GRP_MAX_LAYERS];
    const int64_t* nnz_parts[GRP_MAX_LAYERS];
    const int32_t* seed_counts = nullptr;
    const int64_t* bad_seeds = nullptr;
    hipEvent_t transposed_ready = nullptr;
    GRP_TRY(sample_blocks(part, opts, k, p.sampler_ws, p.sampler_bytes, blocks, long_bwd, nnz_parts, &seed_counts, &bad_seeds,
                          st, &transposed_ready));
    const int32_t* const seeds = blocks[k - 1].dst_nodes;     // the range-checked copy of the caller's list
    GRP_TRY(launch_stats(opts->n_seeds, seeds, nullptr, part->d_local_in, part->d_global_in, seed_counts, 0, nnz_parts, k,
                         p.stats_ws, stats_out, st, nullptr, nullptr, bad_seeds));
    return sage_step(part, model, opts, blocks, features, labels, nullptr, seeds, weights, p, st, grad_out, stats_out,
                     transposed_ready);
}
