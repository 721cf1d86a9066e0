// Internal helpers shared by the HIP translation units of libgrappa_hip.so.
#pragma once

#include <hip/hip_runtime.h>

#include <vector>
#include <hip/hip_bf16.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>

#include "../../include/grappa.h"

namespace grp {

// ---------------------------------------------------------------- errors
void set_error(const char* fmt, ...);
grp_status fail(grp_status code, const char* fmt, ...);

#define GRP_HIP(call)                                                                   \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess)                                                           \
            return grp::fail(GRP_EHIP, "%s failed: %s (%s:%d)", #call,                  \
                             hipGetErrorString(e_), __FILE__, __LINE__);                \
    } while (0)

#define GRP_TRY(call)                                                                   \
    do {                                                                                \
        grp_status s_ = (call);                                                         \
        if (s_ != GRP_OK) return s_;                                                    \
    } while (0)

// ---------------------------------------------------------------- profiling
// Brackets a kernel launch with two events when profiling is enabled.
// flops / bytes: the algorithmic work of the launch (what the operation must compute and
// move, not what the kernel happens to touch); summed per kernel name in the report.
void prof_begin(const char* name, hipStream_t st, double flops, double bytes);
void prof_end(hipStream_t st);
// Optional shape suffix for the next prof_begin on this thread (only with profile mode 2).
void prof_detail(const char* fmt, ...);

struct ProfScope {
    hipStream_t st;
    ProfScope(const char* name, hipStream_t s, double flops = 0.0, double bytes = 0.0) : st(s) {
        prof_begin(name, s, flops, bytes);
    }
    ~ProfScope() { prof_end(st); }
};

// Checks the launch itself (bad configuration etc.); kernels run asynchronously.
#define GRP_LAUNCH_CHECK()                                                              \
    do {                                                                                \
        hipError_t e_ = hipGetLastError();                                              \
        if (e_ != hipSuccess)                                                           \
            return grp::fail(GRP_EHIP, "kernel launch failed: %s (%s:%d)",              \
                             hipGetErrorString(e_), __FILE__, __LINE__);                \
    } while (0)

// ---------------------------------------------------------------- partition handle
}  // namespace grp

namespace grp {
// Rows longer than SPMM_LONG_ROW edges are cut into chunks of at most SPMM_CHUNK edges
// (device arrays, built once with the partition; see spmm.hip).
constexpr int SPMM_LONG_ROW = 128;
constexpr int SPMM_CHUNK = 512;
// Source-sliced schedule of the long rows of a large structure (slices.hip): a long row is cut where its
// sorted sources cross from one of SLICES equal ranges of node ids into the next, and each segment into tasks
// of at most SLICE_TASK_MAX edges; the tasks are processed slice by slice.
constexpr int SLICES = 64;
constexpr int SLICE_PIECE = 128;       // edges a wavefront takes in one pass (two indices per lane)
constexpr int SLICE_TASK_MAX = 1024;   // edges of a task: up to this many consecutive edges of one piece share a partial row
                                       // (128, i.e. a partial row per pass: 40 % more partial rows, step 142.3 against 139.0 ms; 4096: 139.7)
constexpr int SLICE_MIN_PIECE = 112; // a row is not cut at a slice boundary before its current piece has this many edges
                                     // (measured on the 2^32-edge share, ms per step: 64: 153.3 and 96: 145.5 with tasks of at most 128
                                     //  edges; with tasks of up to 1024: 80: 143.1, 96: 139.0, 112: 137.3, 128: 137.6, 144: 137.6; the
                                     //  10^8-edge share with 1 KB rows prefers shorter pieces: 96: 291, 112: 295, 128: 297 ms per step)
struct SliceTask {
    int64_t begin;                   // first edge of the task
    uint32_t id;                     // its number in row-major order: where its partial row goes
    uint32_t len;                    // 1 .. SLICE_TASK_MAX edges
};
struct LongRows {
    int32_t n_long = 0, n_chunks = 0;
    int32_t* long_row = nullptr;     // [n_long]    row index
    int32_t* long_first = nullptr;   // [n_long+1]  first chunk of each long row
    int64_t* chunk_begin = nullptr;  // [n_chunks]  edge range of the chunk
    int64_t* chunk_end = nullptr;    // [n_chunks]
    // the sliced schedule of the same rows (n_tasks = 0: not built; the aggregation then walks the chunks)
    int64_t n_tasks = 0;
    SliceTask* tasks = nullptr;      // [n_tasks] in processing order (slice-major, rows ascending inside a slice)
    int64_t* row_task = nullptr;     // [n_long+1] first task id of each long row
};
// Structures with fewer rows than this keep the chunk schedule (their gathered rows fit the caches anyway).
grp_status build_slice_tasks(const int64_t* ptr, const int32_t* idx, int64_t n, int64_t nnz, LongRows* lr, hipStream_t st);
}  // namespace grp

struct grp_partition_s {
    grp::LongRows csr_long, csc_long;
    int64_t n = 0, nnz = 0;
    int64_t* l2g = nullptr;
    int64_t* rowptr = nullptr;
    int32_t* col = nullptr;
    int64_t* colptr = nullptr;
    int32_t* row = nullptr;
    int32_t* d_local_in = nullptr;
    int32_t* d_local_out = nullptr;
    int64_t* d_global_in = nullptr;
    // weighted partitions only (null otherwise): edge weights in CSR / CSC order and the weight
    // masses of every node's local / global in-edges
    float* csr_w = nullptr;
    float* csc_w = nullptr;
    double* w_local_in = nullptr;
    double* w_global_in = nullptr;
    uint8_t* base_mask = nullptr;    // partitions built from chunks: 1 for the base chunk's nodes
    void* slab = nullptr;            // one allocation that holds the CSR / CSC arrays and the long-row schedules
    size_t slab_bytes = 0;
    bool borrowed_csr = false;       // rowptr / col belong to the caller (grp_partition_from_csr): never freed here
    int device = 0;
};

// The graph split once into chunks: edges grouped by (chunk(dst), chunk(src)) so that the
// partition base + swept reads only its four groups, and the global in-degree of every node.
struct grp_chunks_s {
    int32_t n_chunks = 0;
    uint64_t seed = 0;
    int64_t N = 0, E = 0;
    int64_t* src = nullptr;          // [E] global ids, grouped by bucket (order inside a bucket arbitrary)
    int64_t* dst = nullptr;
    int64_t* d_global_all = nullptr; // [N]
    int32_t* assign = nullptr;       // [N] caller-supplied chunk of every node (null: the random split by seed)
    std::vector<int64_t> bucket_ptr; // host, [n_chunks^2 + 1], bucket = chunk(dst) * n_chunks + chunk(src)
    int device = 0;
};

namespace grp {

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int64_t round_up(int64_t a, int64_t b) { return cdiv(a, b) * b; }

// ---------------------------------------------------------------- kernels (host launchers)
// Neighbour aggregation over a CSR-like structure (ptr/idx), one output row per group of
// lanes.  Y[i,:] = a_i (sum_e X[idx[e],:] + self*X[i,:]) (+ addend[i,:]) (+ bias) (ReLU).
struct SpmmArgs {
    const int64_t* ptr = nullptr;   // [n_rows+1]
    const int32_t* idx = nullptr;   // [nnz]
    int64_t nnz = 0;                // only used for the profiler's byte count
    int64_t n_src = 0;              // rows of X (0 = n_rows); profiler only
    int64_t n_rows = 0;
    int32_t F = 0;
    const void* X = nullptr;
    int64_t ldx = 0;
    int32_t x_bf16 = 0;
    int32_t scale = GRP_SCALE_NONE;
    int32_t self_term = 0;
    const float* colscale = nullptr;  // per gathered row multiplier [n_src] or null
    const float* addend = nullptr;  // [n_rows x F] or null (may alias Y)
    int64_t ld_add = 0;
    const float* bias = nullptr;    // [F] or null
    int32_t relu = 0;
    float* Y = nullptr;
    int64_t ldy = 0;
    const LongRows* long_rows = nullptr;  // null = no row is split
    float* partials = nullptr;            // [n_chunks x round_up(F,4)] scratch when rows are split
    int64_t addend_rows = 0;              // rows >= this have no addend (0: every row has one)
    const float* mask = nullptr;          // result kept where mask[i,c] > 0, else 0 (after the ReLU)
    int64_t ld_mask = 0;
    const float* residual = nullptr;      // added after the ReLU: Y = residual + act (residual layers)
    int64_t ld_res = 0;
    float* Y2 = nullptr;                  // also receives act (before the residual is added)
    int64_t ldy2 = 0;
    const float* val = nullptr;           // [nnz] per-edge multiplier of the gathered row, or null
    const float* rowscale = nullptr;      // [n_rows] a_i given explicitly (replaces `scale`), or null
    // Sizes known on the device only (blocks sampled without a host round trip).  When set, n_rows and
    // addend_rows above are upper bounds that size the launch (ptr must be valid, with empty rows, up to
    // n_rows) and the kernels stop at the values stored here.
    const int64_t* n_rows_dev = nullptr;
    const int64_t* addend_rows_dev = nullptr;
};
grp_status launch_spmm(const SpmmArgs& a, hipStream_t st);
size_t spmm_partials_bytes(const LongRows* lr, int32_t F);

// C[M x N] = epilogue(A[M x K] B[K x N] + A2[M x K2] B2[K2 x N])
// epilogue: (+ bias[N]) (+ addend[M x N]) (* rowscale[M]) (ReLU) (* (mask[M x N] > 0))
struct GemmNNArgs {
    int64_t M = 0;
    int32_t N = 0, K = 0;
    const void* A = nullptr;
    int64_t lda = 0;
    int32_t a_bf16 = 0;
    const float* B = nullptr;
    int64_t ldb = 0;
    int32_t K2 = 0;                 // 0 = no second product
    const float* A2 = nullptr;
    int64_t lda2 = 0;
    const float* B2 = nullptr;
    int64_t ldb2 = 0;
    const float* bias = nullptr;
    const float* addend = nullptr;
    int64_t ld_add = 0;
    const float* rowscale = nullptr;
    int32_t relu = 0;
    const float* mask = nullptr;
    int64_t ld_mask = 0;
    float* C = nullptr;
    int64_t ldc = 0;
    int32_t zero_pad_to = 0;        // also write zeros to columns [N, zero_pad_to)
    const int32_t* a_rows = nullptr; // row i of A is stored at row a_rows[i] (null: i)
    int64_t a_valid_rows = 0;       // rows >= this of the FIRST product's A read as zero (0: M)
    float* C_raw = nullptr;         // also receives acc + bias + addend (before scale / ReLU / mask)
    int64_t ld_raw = 0;
    int32_t rowscale_cols = 0;      // rowscale applies to columns < this only (0: all columns)
    int32_t bias_col0 = 0;          // bias[c - bias_col0] is added to columns c in [bias_col0, bias_col0 + bias_n)
    int32_t bias_n = 0;             // (0: N - bias_col0)
    const float* Bt = nullptr;      // when set: B given transposed, Bt[N x K] (pitch ldbt), fast path
    int64_t ldbt = 0;
    const float* Bt2 = nullptr;     // same for the second product
    int64_t ldbt2 = 0;
    // Row counts known on the device only: when set, M (and a_valid_rows) above are upper bounds that
    // size the launch, and the kernels read the real values here.
    const int64_t* M_dev = nullptr;
    const int64_t* a_valid_rows_dev = nullptr;
};
grp_status launch_gemm_nn(const GemmNNArgs& a, hipStream_t st);

// C[K x N] = A[M x K]^T B[M x N], fixed-order split over M.
size_t gemm_tn_workspace_bytes(int64_t M, int32_t K, int32_t N);
struct GemmTNArgs {
    int64_t M = 0;
    int32_t K = 0, N = 0;
    const void* A = nullptr;
    int64_t lda = 0;
    int32_t a_bf16 = 0;
    const float* B = nullptr;
    int64_t ldb = 0;
    float* C = nullptr;
    int64_t ldc = 0;
    void* workspace = nullptr;
    size_t workspace_bytes = 0;
    const int32_t* a_rows = nullptr; // row i of A is stored at row a_rows[i] (null: i)
    float* colsum_out = nullptr;     // optional [N]: column sums of B (each row times colsum_scale[m] if set)
    const float* colsum_scale = nullptr;
    // A second product from the same launch (at most one of the two):
    const float* A2 = nullptr;       // C2[K x N] = A2[M x K]^T B   (fp32, rows not gathered)
    int64_t lda2 = 0;
    const float* B2 = nullptr;       // C2[K x N] = A^T B2[M x N]
    int64_t ldb2 = 0;
    float* C2 = nullptr;             // pitch ldc
    const int64_t* M_dev = nullptr;  // when set: the real number of rows (on the device); M above is an upper bound
};
grp_status launch_gemm_tn(const GemmTNArgs& a, hipStream_t st);

// out[N] = column sums of A[M x N]; scratch holds the per-block partials.
size_t colsum_workspace_bytes(int64_t M, int32_t N);
grp_status launch_colsum(const float* A, int64_t M, int32_t N, int64_t lda, float* out,
                         void* scratch, hipStream_t st);
// Same with every row multiplied by rowmul[m] first (rowmul may be null).
grp_status launch_colsum_scaled(const float* A, int64_t M, int32_t N, int64_t lda, const float* rowmul,
                                float* out, void* scratch, hipStream_t st);
// inv_in = 1/max(d_in,1); r = 1/sqrt(max(d_in+sl,1)); s = 1/sqrt(max(d_out+sl,1)); rinv = 1/r.
grp_status launch_degree_scales(const int32_t* d_in, const int32_t* d_out, int64_t n, int sl,
                                float* inv_in, float* r, float* s, float* rinv, hipStream_t st);
// Weight re-packing jobs of one step (at most four per layer), run by a single launch.
struct PackJob {
    const float* in;
    float* out;
    int32_t rows, cols;      // shape of `in` (dense, pitch cols)
    int32_t transpose;       // 0: out = in;  1: out = in^T
    int64_t ld_out;
    float scale;             // every element is multiplied by this
};
struct PackJobs {
    int32_t n = 0;
    PackJob job[4 * GRP_MAX_LAYERS];
    int64_t begin[4 * GRP_MAX_LAYERS + 1] = {0};
};
// Appends a job: the output is written with its columns zero-padded to a multiple of 4 and its
// rows zero-padded to out_rows_pad.
void pack_jobs_add(PackJobs& jobs, const float* in, int32_t rows, int32_t cols, bool transpose, int32_t out_rows_pad,
                   float* out, int64_t ld_out, float scale = 1.f);

// Inverted dropout of a layer's output (rows = local nodes, F columns), in place:
//   keep(v, f) = (mix(key + (l2g[node(v)] * F + f + 1) * GAMMA) >> 40) >= thresh;  a' = keep ? a * scale : 0.
// Plain layer: H holds the activation.  Residual layer (act != null): act holds the activation and
// is overwritten with a'; H = a' + res.
struct DropoutPlan {
    bool on = false;
    uint32_t thresh = 0;
    float scale = 1.f;
    uint64_t seed = 0, batch_id = 0;
    const uint64_t* batch_id_dev = nullptr;   // when set: the batch id is read on the device instead
};
DropoutPlan dropout_plan(const grp_step_opts* o);
uint64_t dropout_layer_key(const DropoutPlan& d, int layer);
grp_status launch_dropout(const DropoutPlan& d, int layer, const int64_t* l2g, int64_t n, int32_t F, float* H, int64_t ldh,
                          float* act, int64_t ld_act, const float* res, int64_t ld_res, hipStream_t st,
                          const int32_t* node_of_row = nullptr /*row i is local node node_of_row[i] (null: i)*/,
                          const int64_t* n_dev = nullptr /*when set: the real row count (on the device), n an upper bound*/);
// Y[i, :F] = rowscale[i] * X[i, :F] (whole 16-byte column groups)
grp_status launch_scale_rows(const float* X, int64_t ldx, const float* rowscale, int64_t n, int32_t F, float* Y, int64_t ldy,
                             hipStream_t st, const int64_t* n_dev = nullptr /*as for launch_dropout*/);
// Y[i, :] = [X[i, :F] | 0 ...] up to the pitch ldy
grp_status launch_pad_rows(const float* X, int64_t ldx, int64_t n, int32_t F, float* Y, int64_t ldy, hipStream_t st);
// out[i] = in[i] * s
grp_status launch_scale_copy(const float* in, float s, float* out, int64_t n, hipStream_t st);
grp_status launch_pack_weights(const PackJobs& jobs, hipStream_t st);

// Graph attention model (full-graph mode): workspace size and the whole train step.
size_t gat_step_workspace_bytes(const grp_partition_t* part, const grp_model_desc* m);
// Where layer `layer`'s stored output lives inside a workspace laid out for this partition and model.
void gat_step_activation(const grp_partition_t* part, const grp_model_desc* m, void* ws, size_t ws_bytes, int layer,
                         const float** out, int64_t* ld);
grp_status gat_step(const grp_partition_t* g, const grp_model_desc* m, const grp_step_opts* o, const void* X,
                    const int32_t* labels, const uint8_t* mask, const float* theta, void* ws, size_t ws_bytes,
                    hipStream_t st, float* grad, grp_step_stats* stats);

// Coverage statistics over the loss nodes and the weighted softmax cross-entropy.
size_t stats_workspace_bytes(int64_t n);
// nnz_used = nnz_const + the sum of the n_parts device counters nnz_parts[i][0]; or, when the device counter
// *bad_seeds is set and positive, minus that count (the record of a step whose seed list was invalid).
grp_status launch_stats(int64_t n_loss, const int32_t* loss_nodes /*null = 0..n-1 by mask*/,
                        const uint8_t* mask, const int32_t* d_local, const int64_t* d_global,
                        const int32_t* sampled_count /*null = full graph*/, int64_t nnz_const,
                        const int64_t* const* nnz_parts /*HOST array of device pointers*/, int n_parts,
                        void* scratch, grp_step_stats* out, hipStream_t st,
                        const double* w_local = nullptr, const double* w_global = nullptr /*weight masses: full graph*/,
                        const int64_t* bad_seeds = nullptr);
grp_status launch_softmax_xent(int64_t n_rows, int32_t C, const float* Z, int64_t ldz,
                               const int32_t* labels, const int32_t* node_of_row /*null = row*/,
                               const uint8_t* mask, int32_t node_level,
                               const int32_t* d_local, const int64_t* d_global,
                               const float* rowscale /*null; multiplies dZ rows*/,
                               float* dZ, int64_t lddz, void* scratch,
                               grp_step_stats* stats /*reads S, writes loss*/, hipStream_t st,
                               const double* w_local = nullptr, const double* w_global = nullptr);
// inv[v] = mass[v] > 0 ? 1 / mass[v] : 0
grp_status launch_inverse_mass(const double* mass, int64_t n, float* inv, hipStream_t st);

grp_status launch_fill_zero(void* p, size_t bytes, hipStream_t st);

}  // namespace grp

// ---------------------------------------------------------------- device primitives (partition.hip)
namespace grp {
// rocPRIM wrappers with caller-provided temporary storage (sizes from the *_temp_bytes calls).
size_t sort_keys_temp_bytes(int64_t count);
grp_status sort_keys_u64(void* temp, size_t temp_bytes, const uint64_t* in, uint64_t* out, int64_t count,
                         unsigned end_bit, hipStream_t st);
size_t scan_temp_bytes(int64_t count);
grp_status exclusive_scan_i64(void* temp, size_t temp_bytes, const int64_t* in, int64_t* out, int64_t count,
                              hipStream_t st);
grp_status exclusive_scan_i32(void* temp, size_t temp_bytes, const int32_t* in, int32_t* out, int64_t count,
                              hipStream_t st);
// out[i] = number of set bits in words[0 .. i), i in [0, count): reads `count` words
grp_status exclusive_scan_popcount(void* temp, size_t temp_bytes, const uint32_t* words, int32_t* out, int64_t count,
                                   hipStream_t st);
// From sorted keys (row << 32 | col): idx[i] = low half, ptr[r] = first position with high half >= r.
grp_status launch_csr_from_sorted_keys(const uint64_t* keys, int64_t nnz, int64_t n, int64_t* ptr, int32_t* idx,
                                       hipStream_t st);
// The split schedule of the long rows of a device pointer array, written into caller-provided device
// arrays without a host pass: out->n_long / n_chunks are set to the capacities (the launches cover
// them) and the slots beyond the real counts are filled so that they do nothing (row -1, empty
// chunks).  Capacities must cover every possible schedule: cap_long >= nnz / SPMM_LONG_ROW,
// cap_chunks >= nnz / SPMM_CHUNK + cap_long.  scanned: [n + 1] int64 scratch.
grp_status build_long_rows_device(const int64_t* ptr_dev, int64_t n, LongRows* out, int64_t cap_long, int64_t cap_chunks,
                                  int64_t* scanned, void* scan_tmp, size_t scan_bytes, hipStream_t st);

// M(x): the SplitMix64 finaliser of x + 0x9E3779B97F4A7C15 (the sampler's and the seed order's hash step)
__host__ __device__ __forceinline__ uint64_t mixM(uint64_t x) {
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// A helper stream beside a caller's stream, for work of a step that is off its critical path: the caller's
// stream records fork[i], the helper waits for it, works, records `join`, and the caller's stream waits for
// `join` before it needs the result (a fork and join that a graph capture of the caller's stream follows).
// Null when none can be had (creation failed, or the first request for this stream came while it was being
// captured): the work then stays on the caller's stream.  Calls that use the same caller stream from
// several host threads at once would mix up the events; the steps of one stream come from one thread.
struct SideLane {
    hipStream_t stream = nullptr;
    hipEvent_t fork[GRP_MAX_LAYERS] = {};
    hipEvent_t join = nullptr;
};
SideLane* side_lane(hipStream_t main);

// ---------------------------------------------------------------- blocks and sampling (sampler.hip)
// One bipartite message-passing layer.  Rows of `ptr/idx` are the layer's outputs
// (destinations); `idx` indexes rows of the layer's input matrix.  The outputs are the first
// n_dst inputs unless `self_rows` says where output i's own input row is stored.
struct Block {
    int64_t n_dst = 0, n_in = 0, nnz = 0;
    const int64_t* ptr = nullptr;
    const int32_t* idx = nullptr;
    const int64_t* ptrT = nullptr;       // transposed structure over the n_in inputs (null if unused)
    const int32_t* idxT = nullptr;
    const LongRows* long_fwd = nullptr;
    const LongRows* long_bwd = nullptr;
    const int32_t* self_rows = nullptr;  // [n_dst] or null (row i)
    float* inv_in = nullptr;             // [n_dst] 1 / max(row length, 1); weighted: 1 / local weight mass (0 if none)
    const int32_t* dst_nodes = nullptr;  // mini-batch: partition-local id of every destination row (null: row i is node i)
    const float* val = nullptr;          // weighted partitions: edge weights in ptr/idx order
    const float* valT = nullptr;         //                      and in ptrT/idxT order
    // Sampled blocks: n_dst, n_in and nnz above are upper bounds (from the seeds and fanouts) that size the
    // launches, and the real sizes live on the device (ptr and ptrT are valid up to the bounds: the rows
    // past the real ones are empty).  Null for a block whose sizes the host knows (n_in_dev is also null for
    // the input-side block, whose inputs are the partition's n nodes).
    const int64_t* n_dst_dev = nullptr;
    const int64_t* n_in_dev = nullptr;
};

struct SamplerBounds {                   // upper bounds per layer, from seeds and fanouts alone
    int64_t dst[GRP_MAX_LAYERS], nnz[GRP_MAX_LAYERS], src[GRP_MAX_LAYERS];
};
void sampler_bounds(int64_t n, int64_t n_seeds, const int32_t* fanouts, int k, SamplerBounds* out);
size_t sampler_workspace_bytes(int64_t n, const SamplerBounds& b, int k);
// Isolated k-hop sampling inside the partition; fills blocks[0..k) (layer 0 = input side).
// Layer 0's idx holds partition-local node ids (rows of the feature matrix) and its self_rows
// the destinations' ids; deeper layers are relabelled to block-local indices.  seeds_out
// receives the device pointer of the seed list; nnz_parts_dev[k] the per-layer edge counts
// (device); *bad_seeds_dev the number of seeds outside [0, n) (device; such a seed is replaced by node 0).
// Nothing here waits for the device: every launch is sized by the bounds and reads the real sizes from
// device memory, so the whole step can be queued (or captured in a graph) at once.
grp_status sample_blocks(const grp_partition_t* part, const grp_step_opts* opts, int k, void* ws, size_t ws_bytes,
                         Block* blocks, LongRows* long_bwd_store, const int64_t** nnz_parts_dev,
                         const int32_t** seed_counts_dev, const int64_t** bad_seeds_dev, hipStream_t st,
                         hipEvent_t* transposed_ready);
// *transposed_ready: null, or the event the caller's stream has to wait for before it reads a block's
// transposed structure (ptrT, idxT, long_bwd): those are built on a helper stream beside the sampling of the
// next layers, since only the backward pass reads them.
grp_status sampler_block_view(const grp_partition_t* part, const grp_step_opts* o, int k, void* ws, size_t ws_bytes, int layer,
                              grp_block_view_t* out);
}  // namespace grp

namespace grp {
// Bump allocator over a caller-provided workspace (null base: only measures).
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
    size_t total() const { return (off + 255) & ~(size_t)255; }
};
}  // namespace grp
