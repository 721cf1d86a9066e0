// Bandwidth-bound kernels of the train step and the aggregation:
//   weight preparation (aligned copies and transposes of the layer matrices, degree scales),
//   column sums (bias gradients), coverage statistics over the loss nodes, weighted softmax
//   cross-entropy with its logit gradient, and the K-way weighted gradient aggregation.
// All reductions are two-stage with a fixed block count and a fixed tree, so results are
// bit-reproducible (no floating-point atomics).
#include "common.h"

#include <cmath>

namespace grp {

// ------------------------------------------------------------------ small utilities
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* __restrict__ p, size_t words) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < words; i += stride) p[i] = 0u;
}

grp_status launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
    if (bytes == 0) return GRP_OK;
    if (bytes % 4 != 0 || (uintptr_t)p % 4 != 0) return fail(GRP_EINVAL, "fill_zero: unaligned");
    const size_t words = bytes / 4;
    size_t blocks = (words + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    ProfScope ps("fill_zero", st);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t*)p, words);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// All weight re-packing jobs of a step in one launch: job j owns the flat element range
// [begin_j, begin_{j+1}) of the grid and is either a zero-padded copy or a zero-padded transpose.
__global__ __launch_bounds__(256) void pack_weights_kernel(PackJobs jobs) {
    const int64_t e0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e0 >= jobs.begin[jobs.n]) return;
    int j = 0;
    while (e0 >= jobs.begin[j + 1]) ++j;
    const PackJob& J = jobs.job[j];
    const int64_t e = e0 - jobs.begin[j];
    if (J.transpose) {        // out[cols x rows] = in[rows x cols]^T; pad columns and rows [cols, out_rows_pad) are zero
        const int width = (J.rows + 3) & ~3;
        const int r = (int)(e / width), c = (int)(e % width);
        J.out[(int64_t)r * J.ld_out + c] = (r < J.cols && c < J.rows) ? J.in[(int64_t)c * J.cols + r] * J.scale : 0.f;
    } else {                  // out[rows x cols] = in; pad columns and rows [rows, out_rows_pad) are zero
        const int width = (J.cols + 3) & ~3;
        const int r = (int)(e / width), c = (int)(e % width);
        J.out[(int64_t)r * J.ld_out + c] = (r < J.rows && c < J.cols) ? J.in[(int64_t)r * J.cols + c] * J.scale : 0.f;
    }
}

void pack_jobs_add(PackJobs& jobs, const float* in, int32_t rows, int32_t cols, bool transpose, int32_t out_rows_pad,
                   float* out, int64_t ld_out, float scale) {
    PackJob& J = jobs.job[jobs.n];
    J.in = in; J.out = out; J.rows = rows; J.cols = cols; J.transpose = transpose ? 1 : 0; J.ld_out = ld_out;
    J.scale = scale;
    const int32_t out_rows = transpose ? cols : rows;
    if (out_rows_pad < out_rows) out_rows_pad = out_rows;
    const int64_t width = round_up(transpose ? rows : cols, 4);
    jobs.begin[jobs.n + 1] = jobs.begin[jobs.n] + (int64_t)out_rows_pad * width;
    ++jobs.n;
}

grp_status launch_pack_weights(const PackJobs& jobs, hipStream_t st) {
    if (jobs.n == 0 || jobs.begin[jobs.n] == 0) return GRP_OK;
    ProfScope ps("pack_weights", st);
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)cdiv(jobs.begin[jobs.n], 256)), dim3(256), 0, st, jobs);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// ------------------------------------------------------------------ dropout
// Output function and increment of SplitMix64 (Steele, Lea, Flood 2014).
constexpr uint64_t SM64_GAMMA = 0x9E3779B97F4A7C15ull;
__host__ __device__ static inline uint64_t sm64_mix(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

DropoutPlan dropout_plan(const grp_step_opts* o) {
    DropoutPlan d;
    if (o->dropout_rate > 0.f && o->dropout_rate < 1.f) {
        d.on = true;
        d.thresh = (uint32_t)(o->dropout_rate * 16777216.0f);      // exact: a power-of-two scaling, then truncation
        d.scale = 1.0f / (1.0f - o->dropout_rate);
        d.seed = o->dropout_seed;
        d.batch_id = o->batch_id;
        d.batch_id_dev = o->batch_id_dev;
    }
    return d;
}

uint64_t dropout_layer_key(const DropoutPlan& d, int layer) {
    return sm64_mix(d.seed + (d.batch_id * (uint64_t)GRP_MAX_LAYERS + (uint64_t)layer + 1ull) * SM64_GAMMA);
}

// One thread per 4 columns of a row.  VEC: every pitch is a multiple of 4 and every base 16-byte
// aligned, so the 4 columns (pad columns included, which stay zero) move as one float4.
template <bool VEC>
__global__ __launch_bounds__(256) void dropout_kernel(const int64_t* __restrict__ l2g, int64_t n, int F, uint64_t key,
                                                      uint32_t thresh, float scale, float* __restrict__ H, int64_t ldh,
                                                      float* __restrict__ act, int64_t ld_act,
                                                      const float* __restrict__ res, int64_t ld_res,
                                                      const int32_t* __restrict__ node_of_row,
                                                      const int64_t* __restrict__ n_dev, uint64_t seed, int layer,
                                                      const uint64_t* __restrict__ batch_id_dev) {
    if (batch_id_dev)                 // the layer's key from a batch id that lives on the device
        key = sm64_mix(seed + (*batch_id_dev * (uint64_t)GRP_MAX_LAYERS + (uint64_t)layer + 1ull) * SM64_GAMMA);
    const int C4 = (F + 3) / 4;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n_dev) n = *n_dev;            // the launch was sized by an upper bound
    if (e >= n * C4) return;
    const int64_t v = e / C4;
    const int f0 = 4 * (int)(e % C4);
    const int64_t node = node_of_row ? (int64_t)node_of_row[v] : v;
    const uint64_t base = (uint64_t)l2g[node] * (uint64_t)F + (uint64_t)f0 + 1ull;
    float m[4];                       // keep ? scale : 0
#pragma unroll
    for (int q = 0; q < 4; ++q)
        m[q] = (f0 + q < F && (uint32_t)(sm64_mix(key + (base + (uint64_t)q) * SM64_GAMMA) >> 40) >= thresh) ? scale : 0.f;
    float* const src = act ? act + v * ld_act + f0 : H + v * ldh + f0;
    if (VEC) {
        float4 a = *reinterpret_cast<const float4*>(src);
        a.x *= m[0]; a.y *= m[1]; a.z *= m[2]; a.w *= m[3];
        if (act) {
            *reinterpret_cast<float4*>(src) = a;
            const float4 r = *reinterpret_cast<const float4*>(res + v * ld_res + f0);
            a.x += r.x; a.y += r.y; a.z += r.z; a.w += r.w;
        }
        *reinterpret_cast<float4*>(H + v * ldh + f0) = a;
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (f0 + q >= F) break;
            float a = src[q] * m[q];
            if (act) { src[q] = a; a += res[v * ld_res + f0 + q]; }
            H[v * ldh + f0 + q] = a;
        }
    }
}

grp_status launch_dropout(const DropoutPlan& d, int layer, const int64_t* l2g, int64_t n, int32_t F, float* H, int64_t ldh,
                          float* act, int64_t ld_act, const float* res, int64_t ld_res, hipStream_t st,
                          const int32_t* node_of_row, const int64_t* n_dev) {
    if (!d.on || n <= 0) return GRP_OK;
    if (!l2g || !H || (act && !res)) return fail(GRP_EINVAL, "dropout: null argument");
    ProfScope ps("dropout", st, 0.0, 8.0 * n * F * (act ? 2 : 1));
    const int64_t work = n * ((F + 3) / 4);
    const bool vec = ldh % 4 == 0 && ldh >= round_up(F, 4) && (uintptr_t)H % 16 == 0 &&
                     (!act || (ld_act % 4 == 0 && ld_act >= round_up(F, 4) && (uintptr_t)act % 16 == 0 && ld_res % 4 == 0 &&
                               ld_res >= round_up(F, 4) && (uintptr_t)res % 16 == 0));
    const uint64_t key = dropout_layer_key(d, layer);
    if (vec)
        hipLaunchKernelGGL(dropout_kernel<true>, dim3((unsigned)cdiv(work, 256)), dim3(256), 0, st, l2g, n, (int)F, key,
                           d.thresh, d.scale, H, ldh, act, ld_act, res, ld_res, node_of_row, n_dev, d.seed, layer, d.batch_id_dev);
    else
        hipLaunchKernelGGL(dropout_kernel<false>, dim3((unsigned)cdiv(work, 256)), dim3(256), 0, st, l2g, n, (int)F, key,
                           d.thresh, d.scale, H, ldh, act, ld_act, res, ld_res, node_of_row, n_dev, d.seed, layer, d.batch_id_dev);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

__global__ __launch_bounds__(256) void scale_copy_kernel(const float* __restrict__ in, float s, float* __restrict__ out,
                                                         int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = in[i] * s;
}

// Y[i, :] = rowscale[i] * X[i, :] over c4 float4 columns (pitches multiples of 4, 16-byte aligned bases).
__global__ __launch_bounds__(256) void scale_rows_kernel(const float* __restrict__ X, int64_t ldx,
                                                         const float* __restrict__ rowscale, int64_t n, int c4,
                                                         float* __restrict__ Y, int64_t ldy,
                                                         const int64_t* __restrict__ n_dev) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n_dev) n = *n_dev;            // the launch was sized by an upper bound
    if (e >= n * c4) return;
    const int64_t i = e / c4;
    const int c = 4 * (int)(e % c4);
    float4 v = *reinterpret_cast<const float4*>(X + i * ldx + c);
    const float a = rowscale[i];
    v.x *= a; v.y *= a; v.z *= a; v.w *= a;
    *reinterpret_cast<float4*>(Y + i * ldy + c) = v;
}

grp_status launch_scale_rows(const float* X, int64_t ldx, const float* rowscale, int64_t n, int32_t F, float* Y, int64_t ldy,
                             hipStream_t st, const int64_t* n_dev) {
    if (n <= 0) return GRP_OK;
    const int c4 = (F + 3) / 4;
    if (ldx % 4 || ldy % 4 || ldx < 4 * c4 || ldy < 4 * c4 || (uintptr_t)X % 16 || (uintptr_t)Y % 16)
        return fail(GRP_EINVAL, "scale_rows: operands must be 16-byte friendly");
    ProfScope ps("scale_rows", st, 0.0, 8.0 * n * F);
    hipLaunchKernelGGL(scale_rows_kernel, dim3((unsigned)cdiv(n * c4, 256)), dim3(256), 0, st, X, ldx, rowscale, n, c4, Y, ldy, n_dev);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// Y[i, :] = [X[i, :F] | 0 ...] up to the pitch ldy (a zero-padded, 16-byte friendly copy)
__global__ __launch_bounds__(256) void pad_rows_kernel(const float* __restrict__ X, int64_t ldx, int64_t n, int F,
                                                       float* __restrict__ Y, int64_t ldy) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n * ldy) return;
    const int64_t i = e / ldy;
    const int c = (int)(e % ldy);
    Y[e] = c < F ? X[i * ldx + c] : 0.f;
}

grp_status launch_pad_rows(const float* X, int64_t ldx, int64_t n, int32_t F, float* Y, int64_t ldy, hipStream_t st) {
    if (n <= 0) return GRP_OK;
    hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)cdiv(n * ldy, 256)), dim3(256), 0, st, X, ldx, n, (int)F, Y, ldy);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

grp_status launch_scale_copy(const float* in, float s, float* out, int64_t n, hipStream_t st) {
    if (n <= 0) return GRP_OK;
    hipLaunchKernelGGL(scale_copy_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, in, s, out, n);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// ------------------------------------------------------------------ block reductions
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

template <typename T>
__device__ __forceinline__ T block_sum(T v, T* sm /*[4]*/) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    return sm[0] + sm[1] + sm[2] + sm[3];
}

// ------------------------------------------------------------------ column sums
constexpr int COLSUM_ROWS = 256;     // rows per block

size_t colsum_workspace_bytes(int64_t M, int32_t N) { return (size_t)cdiv(M > 0 ? M : 1, COLSUM_ROWS) * N * sizeof(float); }

// part[b][c] = sum over the block's rows of A[m][c] * (rowmul ? rowmul[m] : 1)
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float* __restrict__ A, int64_t M, int N, int64_t lda,
                                                             const float* __restrict__ rowmul,
                                                             float* __restrict__ part) {
    const int64_t m0 = (int64_t)blockIdx.x * COLSUM_ROWS;
    const int64_t m1 = m0 + COLSUM_ROWS < M ? m0 + COLSUM_ROWS : M;
    for (int c = threadIdx.x; c < N; c += 256) {
        float s = 0.f;
        for (int64_t m = m0; m < m1; ++m) s += rowmul ? A[m * lda + c] * rowmul[m] : A[m * lda + c];
        part[(int64_t)blockIdx.x * N + c] = s;
    }
}

// out[c] = sum_b part[b][c]: 8 columns per workgroup, 32 lanes per column take the blocks
// b = j, j + 32, ... and are added in lane order.
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ part, int64_t blocks, int N,
                                                           float* __restrict__ out) {
    __shared__ float red[32][8];
    const int cl = threadIdx.x & 7, j = threadIdx.x >> 3;
    const int c = blockIdx.x * 8 + cl;
    float s = 0.f;
    if (c < N)
        for (int64_t b = j; b < blocks; b += 32) s += part[b * N + c];
    red[j][cl] = s;
    __syncthreads();
    if (j == 0 && c < N) {
        float t = 0.f;
#pragma unroll
        for (int q = 0; q < 32; ++q) t += red[q][cl];
        out[c] = t;
    }
}

// Same partial sums with 16-byte loads: thread t owns the float4 column t % C4 and the rows
// t / C4, t / C4 + R, ... of the block's slab (R = 256 / C4 row lanes); the row lanes are then
// added through LDS in lane order.  Needs N <= 1024, lda % 4 == 0 and a 16-byte aligned A.
__global__ __launch_bounds__(256) void colsum_partial_vec_kernel(const float* __restrict__ A, int64_t M, int N,
                                                                 int64_t lda, const float* __restrict__ rowmul,
                                                                 float* __restrict__ part) {
    __shared__ float red[256 * 4];
    const int C4 = (N + 3) / 4;
    const int R = 256 / C4;
    const int c4 = threadIdx.x % C4, r0 = threadIdx.x / C4;
    const int64_t m0 = (int64_t)blockIdx.x * COLSUM_ROWS;
    const int64_t m1 = m0 + COLSUM_ROWS < M ? m0 + COLSUM_ROWS : M;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r0 < R) {
        // four rows per trip, all requested before the first is added (in row order)
        int64_t m = m0 + r0;
        for (; m + 3 * R < m1; m += 4 * R) {
            float4 v[4];
            float w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v[q] = *reinterpret_cast<const float4*>(A + (m + q * R) * lda + 4 * c4);
                w[q] = rowmul ? rowmul[m + q * R] : 1.f;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                s.x = fmaf(v[q].x, w[q], s.x); s.y = fmaf(v[q].y, w[q], s.y);
                s.z = fmaf(v[q].z, w[q], s.z); s.w = fmaf(v[q].w, w[q], s.w);
            }
        }
        for (; m < m1; m += R) {
            const float4 v = *reinterpret_cast<const float4*>(A + m * lda + 4 * c4);
            const float w = rowmul ? rowmul[m] : 1.f;
            s.x = fmaf(v.x, w, s.x); s.y = fmaf(v.y, w, s.y); s.z = fmaf(v.z, w, s.z); s.w = fmaf(v.w, w, s.w);
        }
    }
    *reinterpret_cast<float4*>(&red[threadIdx.x * 4]) = s;
    __syncthreads();
    for (int c = threadIdx.x; c < N; c += 256) {
        float acc = 0.f;
        for (int r = 0; r < R; ++r) acc += red[(r * C4 + c / 4) * 4 + (c & 3)];
        part[(int64_t)blockIdx.x * N + c] = acc;
    }
}

grp_status launch_colsum_scaled(const float* A, int64_t M, int32_t N, int64_t lda, const float* rowmul, float* out,
                                void* scratch, hipStream_t st) {
    const int64_t blocks = cdiv(M > 0 ? M : 1, COLSUM_ROWS);
    ProfScope ps("colsum", st, 0.0, 4.0 * M * N);
    const bool vec = N <= 1024 && lda % 4 == 0 && lda >= round_up(N, 4) && (uintptr_t)A % 16 == 0;
    if (vec)
        hipLaunchKernelGGL(colsum_partial_vec_kernel, dim3((unsigned)blocks), dim3(256), 0, st, A, M, N, lda, rowmul,
                           (float*)scratch);
    else
        hipLaunchKernelGGL(colsum_partial_kernel, dim3((unsigned)blocks), dim3(256), 0, st, A, M, N, lda, rowmul,
                           (float*)scratch);
    GRP_LAUNCH_CHECK();
    hipLaunchKernelGGL(colsum_final_kernel, dim3((unsigned)cdiv(N, 8)), dim3(256), 0, st, (const float*)scratch,
                       blocks, N, out);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

grp_status launch_colsum(const float* A, int64_t M, int32_t N, int64_t lda, float* out, void* scratch, hipStream_t st) {
    return launch_colsum_scaled(A, M, N, lda, nullptr, out, scratch, st);
}

// ------------------------------------------------------------------ degree scales
// inv_in[v] = 1/max(d_in,1); r[v] = 1/sqrt(max(d_in+sl,1)); s[v] = 1/sqrt(max(d_out+sl,1));
// rinv[v] = sqrt(max(d_in+sl,1)).  Null outputs are skipped.
__global__ __launch_bounds__(256) void degree_scales_kernel(const int32_t* __restrict__ d_in,
                                                            const int32_t* __restrict__ d_out, int64_t n, int sl,
                                                            float* __restrict__ inv_in, float* __restrict__ r,
                                                            float* __restrict__ s, float* __restrict__ rinv) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n) return;
    const int di = d_in[v], dout = d_out[v];
    if (inv_in) inv_in[v] = 1.0f / (float)(di > 1 ? di : 1);
    const float a = (float)(di + sl > 1 ? di + sl : 1), b = (float)(dout + sl > 1 ? dout + sl : 1);
    if (r) r[v] = 1.0f / sqrtf(a);
    if (rinv) rinv[v] = sqrtf(a);
    if (s) s[v] = 1.0f / sqrtf(b);
}

grp_status launch_degree_scales(const int32_t* d_in, const int32_t* d_out, int64_t n, int sl, float* inv_in, float* r,
                                float* s, float* rinv, hipStream_t st) {
    if (n == 0) return GRP_OK;
    ProfScope ps("degree_scales", st);
    hipLaunchKernelGGL(degree_scales_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, d_in, d_out, n, sl, inv_in,
                       r, s, rinv);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// ------------------------------------------------------------------ coverage statistics
constexpr int STATS_BLOCKS = 2048;

struct StatsPartial {
    double ratio, r_dbl;
    int64_t s, r_int;
};

size_t stats_workspace_bytes(int64_t) { return (size_t)STATS_BLOCKS * sizeof(StatsPartial) + STATS_BLOCKS * sizeof(double); }

__device__ __forceinline__ double degree_ratio(int64_t dl, int64_t dg) { return dg > 0 ? (double)dl / (double)dg : 1.0; }

// What a node's coverage ratio is computed from: in-degrees, or (weighted partitions) the weight
// masses of its local and global in-edges.
struct CoverageIn {
    const int32_t* d_local;
    const int64_t* d_global;
    const double* w_local;
    const double* w_global;
};
__device__ __forceinline__ double coverage_ratio(const CoverageIn& c, int64_t v) {
    if (c.w_local) { const double wg = c.w_global[v]; return wg > 0.0 ? c.w_local[v] / wg : 1.0; }
    return degree_ratio(c.d_local[v], c.d_global[v]);
}

// Rows are loss candidates: node = nodes ? nodes[i] : i; kept if !mask || mask[node].
__global__ __launch_bounds__(256) void stats_partial_kernel(int64_t n_rows, const int32_t* __restrict__ nodes,
                                                            const uint8_t* __restrict__ mask, CoverageIn cv,
                                                            const int32_t* __restrict__ sampled,
                                                            StatsPartial* __restrict__ part) {
    __shared__ double smd[4];
    __shared__ int64_t smi[4];
    double ratio = 0.0, rd = 0.0;
    int64_t s = 0, ri = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_rows; i += (int64_t)gridDim.x * 256) {
        const int64_t v = nodes ? nodes[i] : i;
        if (mask && !mask[v]) continue;
        const int64_t dl = cv.d_local[v], dg = cv.d_global[v];
        s += 1;
        ratio += coverage_ratio(cv, v);
        if (cv.w_local) {         // full graph, weight masses: missing mass in units of the mean local edge weight
            const double wl = cv.w_local[v];
            rd += dl > 0 ? (cv.w_global[v] - wl) * (double)dl / wl : (double)dg;
        } else if (sampled) {
            if (dl > 0) rd += (double)(dg - dl) * (double)sampled[i] / (double)dl;
        } else {
            ri += dg - dl;
        }
    }
    ratio = block_sum<double>(ratio, smd);
    rd = block_sum<double>(rd, smd);
    s = block_sum<int64_t>(s, smi);
    ri = block_sum<int64_t>(ri, smi);
    if (threadIdx.x == 0) part[blockIdx.x] = StatsPartial{ratio, rd, s, ri};
}

struct NnzParts {
    const int64_t* p[GRP_MAX_LAYERS];
    int n;
    const int64_t* bad_seeds;      // null, or the number of seeds that were outside the partition
};

__global__ __launch_bounds__(256) void stats_final_kernel(const StatsPartial* __restrict__ part, int blocks,
                                                          int full_graph, int64_t nnz_const, NnzParts np,
                                                          grp_step_stats* __restrict__ out) {
    __shared__ double smd[4];
    __shared__ int64_t smi[4];
    double ratio = 0.0, rd = 0.0;
    int64_t s = 0, ri = 0;
    for (int b = threadIdx.x; b < blocks; b += 256) {
        ratio += part[b].ratio; rd += part[b].r_dbl; s += part[b].s; ri += part[b].r_int;
    }
    ratio = block_sum<double>(ratio, smd);
    rd = block_sum<double>(rd, smd);
    s = block_sum<int64_t>(s, smi);
    ri = block_sum<int64_t>(ri, smi);
    if (threadIdx.x == 0) {
        out->loss = 0.0;
        out->sum_ratio = ratio;
        out->R = full_graph ? (double)ri : rd;
        out->S = s;
        int64_t nnz_used = nnz_const;
        for (int i = 0; i < np.n; ++i) nnz_used += np.p[i][0];
        if (np.bad_seeds && *np.bad_seeds > 0) nnz_used = -*np.bad_seeds;
        out->nnz_used = nnz_used;
    }
}

grp_status launch_stats(int64_t n_rows, const int32_t* nodes, const uint8_t* mask, const int32_t* d_local,
                        const int64_t* d_global, const int32_t* sampled_count, int64_t nnz_const,
                        const int64_t* const* nnz_parts, int n_parts, void* scratch, grp_step_stats* out, hipStream_t st,
                        const double* w_local, const double* w_global, const int64_t* bad_seeds) {
    NnzParts np;
    np.n = n_parts;
    np.bad_seeds = bad_seeds;
    for (int i = 0; i < GRP_MAX_LAYERS; ++i) np.p[i] = i < n_parts ? nnz_parts[i] : nullptr;
    ProfScope ps("coverage_stats", st);
    StatsPartial* part = (StatsPartial*)scratch;
    if (w_local && sampled_count) return fail(GRP_EUNSUPPORTED, "coverage statistics: weight masses in mini-batch mode");
    const CoverageIn cv{d_local, d_global, w_local, w_global};
    hipLaunchKernelGGL(stats_partial_kernel, dim3(STATS_BLOCKS), dim3(256), 0, st, n_rows, nodes, mask, cv, sampled_count,
                       part);
    GRP_LAUNCH_CHECK();
    hipLaunchKernelGGL(stats_final_kernel, dim3(1), dim3(256), 0, st, (const StatsPartial*)part, STATS_BLOCKS,
                       (sampled_count || w_local) ? 0 : 1, nnz_const, np, out);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// ------------------------------------------------------------------ softmax cross-entropy
// 16 lanes per row; dZ[row,:] = w (softmax(z) - onehot(y)) / |S| for loss rows, 0 otherwise
// (pad columns up to the pitch's multiple of 4 are written as zeros too).
__global__ __launch_bounds__(256) void softmax_xent_kernel(int64_t n_rows, int C, const float* __restrict__ Z,
                                                           int64_t ldz, const int32_t* __restrict__ labels,
                                                           const int32_t* __restrict__ nodes,
                                                           const uint8_t* __restrict__ mask, int node_level,
                                                           CoverageIn cv,
                                                           const float* __restrict__ rowscale,
                                                           float* __restrict__ dZ, int64_t lddz, int c_store,
                                                           const grp_step_stats* __restrict__ stats,
                                                           double* __restrict__ loss_part) {
    __shared__ double smd[4];
    const int t = threadIdx.x & 15;
    const int64_t S = stats->S;
    const float inv_s = S > 0 ? 1.0f / (float)S : 0.f;
    double loss = 0.0;
    for (int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4); row < n_rows; row += (int64_t)gridDim.x * 16) {
        const int64_t v = nodes ? nodes[row] : row;
        const bool in_loss = !mask || mask[v];
        if (!in_loss) {
            for (int c = t; c < c_store; c += 16) dZ[row * lddz + c] = 0.f;
            continue;
        }
        const float* z = Z + row * ldz;
        float mx = -INFINITY;
        for (int c = t; c < C; c += 16) mx = fmaxf(mx, z[c]);
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 16));
        float sum = 0.f;
        for (int c = t; c < C; c += 16) sum += expf(z[c] - mx);
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 16);
        const int y = labels[v];
        float w = 1.f;
        if (node_level) w = (float)coverage_ratio(cv, v);
        const float k = w * inv_s * (rowscale ? rowscale[v] : 1.f), inv_sum = 1.0f / sum;
        for (int c = t; c < c_store; c += 16) {
            float g = 0.f;
            if (c < C) g = (expf(z[c] - mx) * inv_sum - (c == y ? 1.f : 0.f)) * k;
            dZ[row * lddz + c] = g;
        }
        if (t == 0) loss += (double)w * (double)(logf(sum) + mx - z[y]);
    }
    loss = block_sum<double>(loss, smd);
    if (threadIdx.x == 0) loss_part[blockIdx.x] = loss;
}

// Same for C <= 16*NV: a lane keeps its NV logits in registers (one pass over Z, one expf per
// element) and the logits of the group's next row are requested before the current row is
// reduced, so the load latency overlaps the shuffles and exponentials.
template <int NV>
__global__ __launch_bounds__(256) void softmax_xent_reg_kernel(int64_t n_rows, int C, const float* __restrict__ Z,
                                                               int64_t ldz, const int32_t* __restrict__ labels,
                                                               const int32_t* __restrict__ nodes,
                                                               const uint8_t* __restrict__ mask, int node_level,
                                                               CoverageIn cv,
                                                               const float* __restrict__ rowscale,
                                                               float* __restrict__ dZ, int64_t lddz, int c_store,
                                                               const grp_step_stats* __restrict__ stats,
                                                               double* __restrict__ loss_part) {
    __shared__ double smd[4];
    const int t = threadIdx.x & 15;
    const int64_t S = stats->S;
    const float inv_s = S > 0 ? 1.0f / (float)S : 0.f;
    const int64_t stride = (int64_t)gridDim.x * 16;
    double loss = 0.0;
    int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    float cur[NV], nxt[NV];
    auto load = [&](int64_t r, float (&v)[NV]) {
#pragma unroll
        for (int q = 0; q < NV; ++q) v[q] = (r < n_rows && t + 16 * q < C) ? Z[r * ldz + t + 16 * q] : -INFINITY;
    };
    load(row, cur);
    for (; row < n_rows; row += stride) {
        load(row + stride, nxt);
        const int64_t v = nodes ? nodes[row] : row;
        const bool in_loss = !mask || mask[v];
        if (in_loss) {
            float mx = cur[0];
#pragma unroll
            for (int q = 1; q < NV; ++q) mx = fmaxf(mx, cur[q]);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 16));
            float e[NV], sum = 0.f;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                e[q] = t + 16 * q < C ? expf(cur[q] - mx) : 0.f;
                sum += e[q];
            }
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 16);
            const int y = labels[v];
            float w = 1.f;
            if (node_level) w = (float)coverage_ratio(cv, v);
            const float k = w * inv_s * (rowscale ? rowscale[v] : 1.f), inv_sum = 1.0f / sum;
            float zy = 0.f;                           // the label's logit sits in lane y%16, slot y/16
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const int c = t + 16 * q;
                if (c == y) zy = cur[q];
                if (c < c_store) dZ[row * lddz + c] = c < C ? (e[q] * inv_sum - (c == y ? 1.f : 0.f)) * k : 0.f;
            }
            zy = __shfl(zy, y & 15, 16);
            if (t == 0) loss += (double)w * (double)(logf(sum) + mx - zy);
        } else {
#pragma unroll
            for (int q = 0; q < NV; ++q)
                if (t + 16 * q < c_store) dZ[row * lddz + t + 16 * q] = 0.f;
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) cur[q] = nxt[q];
    }
    loss = block_sum<double>(loss, smd);
    if (threadIdx.x == 0) loss_part[blockIdx.x] = loss;
}

__global__ __launch_bounds__(256) void loss_final_kernel(const double* __restrict__ part, int blocks,
                                                         grp_step_stats* __restrict__ stats) {
    __shared__ double smd[4];
    double s = 0.0;
    for (int b = threadIdx.x; b < blocks; b += 256) s += part[b];
    s = block_sum<double>(s, smd);
    if (threadIdx.x == 0) stats->loss = stats->S > 0 ? s / (double)stats->S : 0.0;
}

grp_status launch_softmax_xent(int64_t n_rows, int32_t C, const float* Z, int64_t ldz, const int32_t* labels,
                               const int32_t* node_of_row, const uint8_t* mask, int32_t node_level,
                               const int32_t* d_local, const int64_t* d_global, const float* rowscale, float* dZ,
                               int64_t lddz, void* scratch, grp_step_stats* stats, hipStream_t st,
                               const double* w_local, const double* w_global) {
    ProfScope ps("softmax_xent", st, 0.0, 8.0 * n_rows * C);
    const CoverageIn cv{d_local, d_global, w_local, w_global};
    double* loss_part = (double*)((char*)scratch + (size_t)STATS_BLOCKS * sizeof(StatsPartial));
    int c_store = (int)round_up(C, 4);
    if (c_store > lddz) c_store = (int)lddz;
#define GRP_SOFTMAX_ARGS                                                                                     \
    n_rows, C, Z, ldz, labels, node_of_row, mask, node_level, cv, rowscale, dZ, lddz, c_store,               \
        (const grp_step_stats*)stats, loss_part
    if (c_store <= 16)
        hipLaunchKernelGGL(softmax_xent_reg_kernel<1>, dim3(STATS_BLOCKS), dim3(256), 0, st, GRP_SOFTMAX_ARGS);
    else if (c_store <= 32)
        hipLaunchKernelGGL(softmax_xent_reg_kernel<2>, dim3(STATS_BLOCKS), dim3(256), 0, st, GRP_SOFTMAX_ARGS);
    else if (c_store <= 64)
        hipLaunchKernelGGL(softmax_xent_reg_kernel<4>, dim3(STATS_BLOCKS), dim3(256), 0, st, GRP_SOFTMAX_ARGS);
    else
        hipLaunchKernelGGL(softmax_xent_kernel, dim3(STATS_BLOCKS), dim3(256), 0, st, GRP_SOFTMAX_ARGS);
#undef GRP_SOFTMAX_ARGS
    GRP_LAUNCH_CHECK();
    hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(256), 0, st, (const double*)loss_part, STATS_BLOCKS, stats);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

__global__ __launch_bounds__(256) void inverse_mass_kernel(const double* __restrict__ mass, int64_t n,
                                                           float* __restrict__ inv) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < n) inv[v] = mass[v] > 0.0 ? (float)(1.0 / mass[v]) : 0.f;
}

grp_status launch_inverse_mass(const double* mass, int64_t n, float* inv, hipStream_t st) {
    if (n <= 0) return GRP_OK;
    hipLaunchKernelGGL(inverse_mass_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, mass, n, inv);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// ------------------------------------------------------------------ aggregation
// G[i] = (1/K) sum_p c_p g_p[i], p ascending, fp32 FMAs.  c_p is derived from the statistics
// record of partition p inside the kernel (no host round trip).
__device__ __forceinline__ float coverage_factor(const grp_step_stats& s, int variant) {
    if (variant == GRP_EST_BATCH_MIN_DIST) return s.S > 0 ? (float)(s.sum_ratio / (double)s.S) : 1.f;
    if (variant == GRP_EST_SHRINKAGE) return s.R > 0.0 ? (float)(1.0 / s.R) : 1.f;
    return 1.f;
}

constexpr int AGG_MAX_K_LDS = 1024;

// PTRS: partition p's gradient starts at ptrs[p] instead of grads + p * ld.
// The K loads of an element are issued B at a time before the multiply-adds that consume them (the adds stay
// in ascending p, so the bits do not depend on the batching).  Measured at K = 64, P = 2^26: B = 1, 2, 4 all give
// 5.19 TB/s, B = 8 and 16 give 4.7: the kernel sits at what a read-only stream reaches on this chip (a plain
// device copy moves 4.7 TB/s, a fill 6.8), and B = 4 is kept for small K * P where latency shows.
template <bool VEC, bool PTRS, int B>
__global__ __launch_bounds__(256) void aggregate_kernel(const float* __restrict__ grads, int64_t ld,
                                                        const float* const* __restrict__ ptrs,
                                                        const grp_step_stats* __restrict__ stats, int K, int64_t P,
                                                        int variant, float* __restrict__ out,
                                                        float* __restrict__ c_out) {
    __shared__ float cs[AGG_MAX_K_LDS];
    __shared__ const float* base[PTRS ? AGG_MAX_K_LDS : 1];
    for (int p = threadIdx.x; p < K; p += 256) {
        const float c = coverage_factor(stats[p], variant);
        cs[p] = c;
        if (PTRS) base[p] = ptrs[p];
        if (c_out && blockIdx.x == 0) c_out[p] = c;
    }
    __syncthreads();
    auto row = [&](int p) -> const float* { return PTRS ? base[p] : grads + (int64_t)p * ld; };
    const float inv_k = 1.0f / (float)K;
    const int64_t stride = (int64_t)gridDim.x * 256;
    if constexpr (VEC) {
        const int64_t P4 = P / 4;
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < P4; i += stride) {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
            int p = 0;
            for (; p + B <= K; p += B) {
                float4 g[B];
#pragma unroll
                for (int u = 0; u < B; ++u) g[u] = *reinterpret_cast<const float4*>(row(p + u) + 4 * i);
#pragma unroll
                for (int u = 0; u < B; ++u) {
                    const float c = cs[p + u];
                    a.x = fmaf(c, g[u].x, a.x); a.y = fmaf(c, g[u].y, a.y); a.z = fmaf(c, g[u].z, a.z); a.w = fmaf(c, g[u].w, a.w);
                }
            }
            for (; p < K; ++p) {
                const float4 g = *reinterpret_cast<const float4*>(row(p) + 4 * i);
                const float c = cs[p];
                a.x = fmaf(c, g.x, a.x); a.y = fmaf(c, g.y, a.y); a.z = fmaf(c, g.z, a.z); a.w = fmaf(c, g.w, a.w);
            }
            *reinterpret_cast<float4*>(out + 4 * i) = make_float4(a.x * inv_k, a.y * inv_k, a.z * inv_k, a.w * inv_k);
        }
        for (int64_t i = 4 * P4 + (int64_t)blockIdx.x * 256 + threadIdx.x; i < P; i += stride) {
            float a = 0.f;
            for (int p = 0; p < K; ++p) a = fmaf(cs[p], row(p)[i], a);
            out[i] = a * inv_k;
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < P; i += stride) {
            float a = 0.f;
            int p = 0;
            for (; p + B <= K; p += B) {
                float g[B];
#pragma unroll
                for (int u = 0; u < B; ++u) g[u] = row(p + u)[i];
#pragma unroll
                for (int u = 0; u < B; ++u) a = fmaf(cs[p + u], g[u], a);
            }
            for (; p < K; ++p) a = fmaf(cs[p], row(p)[i], a);
            out[i] = a * inv_k;
        }
    }
}

// ------------------------------------------------------------------ optimizer step
// One pass: Adam reads theta, g, m, v and writes theta, m, v (28 bytes per parameter); SGD
// reads theta, g and writes theta (12 bytes).
template <bool ADAM, bool VEC>
__global__ __launch_bounds__(256) void optimizer_kernel(int64_t P, float* __restrict__ theta,
                                                        const float* __restrict__ g, float* __restrict__ m,
                                                        float* __restrict__ v, float lr, float b1, float b2,
                                                        float eps, float inv_c1, float inv_c2) {
    auto upd = [&](float& th, float gi, float& mi, float& vi) {
        if (ADAM) {
            mi = b1 * mi + (1.f - b1) * gi;
            vi = b2 * vi + (1.f - b2) * gi * gi;
            th -= lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
        } else {
            th -= lr * gi;
        }
    };
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if constexpr (VEC) {
        const int64_t P4 = P / 4;
        for (int64_t i = i0; i < P4; i += stride) {
            float4 th = reinterpret_cast<float4*>(theta)[i];
            const float4 gi = reinterpret_cast<const float4*>(g)[i];
            float4 mi = make_float4(0.f, 0.f, 0.f, 0.f), vi = mi;
            if (ADAM) { mi = reinterpret_cast<float4*>(m)[i]; vi = reinterpret_cast<float4*>(v)[i]; }
            upd(th.x, gi.x, mi.x, vi.x); upd(th.y, gi.y, mi.y, vi.y);
            upd(th.z, gi.z, mi.z, vi.z); upd(th.w, gi.w, mi.w, vi.w);
            reinterpret_cast<float4*>(theta)[i] = th;
            if (ADAM) { reinterpret_cast<float4*>(m)[i] = mi; reinterpret_cast<float4*>(v)[i] = vi; }
        }
        for (int64_t i = 4 * P4 + i0; i < P; i += stride) {
            float mi = 0.f, vi = 0.f;
            if (ADAM) { mi = m[i]; vi = v[i]; }
            upd(theta[i], g[i], mi, vi);
            if (ADAM) { m[i] = mi; v[i] = vi; }
        }
    } else {
        for (int64_t i = i0; i < P; i += stride) {
            float mi = 0.f, vi = 0.f;
            if (ADAM) { mi = m[i]; vi = v[i]; }
            upd(theta[i], g[i], mi, vi);
            if (ADAM) { m[i] = mi; v[i] = vi; }
        }
    }
}

}  // namespace grp

namespace grp {
// out[r, :] = src[idx[r], :] for rows of `units` elements of type U; a row whose index is outside
// [0, n_src) or whose keep byte is 0 is zero-filled.
template <typename U>
__global__ __launch_bounds__(256) void gather_rows_kernel(const U* __restrict__ src, int64_t n_src, int64_t units,
                                                          const int64_t* __restrict__ idx, int64_t n,
                                                          const uint8_t* __restrict__ keep, U* __restrict__ out) {
    const int64_t total = n * units;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / units, c = i - r * units;
        const int64_t from = idx[r];
        U v{};
        if (from >= 0 && from < n_src && (!keep || keep[r])) v = src[from * units + c];
        out[i] = v;
    }
}
}  // namespace grp

extern "C" grp_status grp_gather_rows(const void* src, int64_t n_src, int64_t row_bytes, const int64_t* idx, int64_t n,
                                      const uint8_t* keep, void* out, void* stream) {
    using namespace grp;
    if (n < 0 || n_src < 0 || row_bytes < 1) return fail(GRP_EINVAL, "grp_gather_rows: n = %lld, n_src = %lld, row_bytes = %lld",
                                                         (long long)n, (long long)n_src, (long long)row_bytes);
    if (n == 0) return GRP_OK;
    if (!src || !idx || !out) return fail(GRP_EINVAL, "grp_gather_rows: null pointer");
    hipStream_t st = (hipStream_t)stream;
    const uintptr_t both = (uintptr_t)src | (uintptr_t)out;
    const double bytes = 2.0 * (double)n * (double)row_bytes + 8.0 * (double)n;
    ProfScope ps("gather_rows", st, 0.0, bytes);
    auto blocks = [](int64_t work) { int64_t b = (work + 255) / 256; return (unsigned)(b > 65536 ? 65536 : (b > 0 ? b : 1)); };
    if (row_bytes % 16 == 0 && both % 16 == 0) {
        const int64_t units = row_bytes / 16;
        hipLaunchKernelGGL(gather_rows_kernel<uint4>, dim3(blocks(n * units)), dim3(256), 0, st, (const uint4*)src, n_src, units,
                           idx, n, keep, (uint4*)out);
    } else if (row_bytes % 4 == 0 && both % 4 == 0) {
        const int64_t units = row_bytes / 4;
        hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, dim3(blocks(n * units)), dim3(256), 0, st, (const uint32_t*)src, n_src,
                           units, idx, n, keep, (uint32_t*)out);
    } else {
        hipLaunchKernelGGL(gather_rows_kernel<uint8_t>, dim3(blocks(n * row_bytes)), dim3(256), 0, st, (const uint8_t*)src, n_src,
                           row_bytes, idx, n, keep, (uint8_t*)out);
    }
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

extern "C" grp_status grp_optimizer_step(const grp_optimizer_desc* opt, int64_t P, int64_t step, float* theta,
                                         const float* update, float* m, float* v, void* stream) {
    using namespace grp;
    if (!opt || !theta || !update) return fail(GRP_EINVAL, "grp_optimizer_step: null argument");
    if (P < 0 || step < 1) return fail(GRP_EINVAL, "grp_optimizer_step: P = %lld, step = %lld", (long long)P, (long long)step);
    if (opt->kind != GRP_OPT_SGD && opt->kind != GRP_OPT_ADAM) return fail(GRP_EINVAL, "grp_optimizer_step: bad kind %d", opt->kind);
    if (!(opt->lr > 0.f)) return fail(GRP_EINVAL, "grp_optimizer_step: lr must be positive");
    const bool adam = opt->kind == GRP_OPT_ADAM;
    if (adam) {
        if (!m || !v) return fail(GRP_EINVAL, "grp_optimizer_step: Adam needs the moment arrays");
        if (!(opt->beta1 >= 0.f && opt->beta1 < 1.f && opt->beta2 >= 0.f && opt->beta2 < 1.f && opt->eps > 0.f))
            return fail(GRP_EINVAL, "grp_optimizer_step: Adam hyper-parameters out of range");
    }
    if (P == 0) return GRP_OK;
    hipStream_t st = (hipStream_t)stream;
    const bool vec = (uintptr_t)theta % 16 == 0 && (uintptr_t)update % 16 == 0 &&
                     (!adam || ((uintptr_t)m % 16 == 0 && (uintptr_t)v % 16 == 0));
    int64_t blocks = cdiv(vec ? cdiv(P, 4) : P, 256);
    if (blocks > 8192) blocks = 8192;
    // bias corrections 1 - beta^t in double on the host (t can be large)
    const float inv_c1 = adam ? (float)(1.0 / (1.0 - pow((double)opt->beta1, (double)step))) : 1.f;
    const float inv_c2 = adam ? (float)(1.0 / (1.0 - pow((double)opt->beta2, (double)step))) : 1.f;
    ProfScope ps("optimizer_step", st, 0.0, (adam ? 28.0 : 12.0) * P);
#define GRP_OPT_LAUNCH(A, V)                                                                                         \
    hipLaunchKernelGGL((optimizer_kernel<A, V>), dim3((unsigned)blocks), dim3(256), 0, st, P, theta, update, m, v, \
                       opt->lr, opt->beta1, opt->beta2, opt->eps, inv_c1, inv_c2)
    if (adam) { if (vec) GRP_OPT_LAUNCH(true, true); else GRP_OPT_LAUNCH(true, false); }
    else { if (vec) GRP_OPT_LAUNCH(false, true); else GRP_OPT_LAUNCH(false, false); }
#undef GRP_OPT_LAUNCH
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

static grp_status aggregate_impl(const float* grads, int64_t ld_grads, const float* const* ptrs, bool vec_ok,
                                 const grp_step_stats* stats, int32_t K, int64_t P, int32_t variant, void* stream, float* update,
                                 float* c_out, const char* who) {
    using namespace grp;
    if ((!grads && !ptrs) || !stats || !update) return fail(GRP_EINVAL, "%s: null argument", who);
    if (K < 1 || K > AGG_MAX_K_LDS) return fail(GRP_EINVAL, "%s: K = %d outside [1, %d]", who, K, AGG_MAX_K_LDS);
    if (P < 0 || (!ptrs && K > 1 && ld_grads < P)) return fail(GRP_EINVAL, "%s: bad P / pitch", who);
    if (variant < GRP_EST_NONE || variant > GRP_EST_SHRINKAGE) return fail(GRP_EINVAL, "%s: bad variant", who);
    hipStream_t st = (hipStream_t)stream;
    const bool vec = vec_ok && (uintptr_t)update % 16 == 0;
    int64_t blocks = cdiv((vec ? P / 4 : P) > 0 ? (vec ? P / 4 : P) : 1, 256);
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    ProfScope ps("aggregate", st, 2.0 * K * P, 4.0 * P * (K + 1.0));
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(256), 0, st, grads, ld_grads, ptrs, stats, K, P, variant, update, c_out);
    };
    if (ptrs) { if (vec) go(aggregate_kernel<true, true, 4>); else go(aggregate_kernel<false, true, 4>); }
    else { if (vec) go(aggregate_kernel<true, false, 4>); else go(aggregate_kernel<false, false, 4>); }
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

extern "C" grp_status grp_aggregate(const float* grads, int64_t ld_grads, const grp_step_stats* stats, int32_t K,
                                    int64_t P, int32_t variant, void* stream, float* update, float* c_out) {
    const bool vec = ld_grads % 4 == 0 && (uintptr_t)grads % 16 == 0;
    return aggregate_impl(grads, ld_grads, nullptr, vec, stats, K, P, variant, stream, update, c_out, "grp_aggregate");
}

extern "C" grp_status grp_aggregate_ptrs(const float* const* grads, int32_t aligned16, const grp_step_stats* stats, int32_t K,
                                         int64_t P, int32_t variant, void* stream, float* update, float* c_out) {
    return aggregate_impl(nullptr, 0, grads, aligned16 != 0, stats, K, P, variant, stream, update, c_out, "grp_aggregate_ptrs");
}
