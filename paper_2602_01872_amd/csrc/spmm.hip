// Row-parallel neighbour aggregation (SpMM) for gfx950.
//
// Y[i,:] = a_i (sum_{e in row i} w_e c_{idx[e]} X[idx[e],:] + self * X[i,:]) (+ addend[i,:]) (+ bias) (ReLU)
// (w_e: optional per-edge values, the weighted-mean aggregator of weighted partitions)
//
// The same kernels serve the forward pass (rows of the CSR: destinations gathering their
// in-neighbours) and the backward pass (rows of the CSC: the transposed operator), so no
// floating-point atomics are needed and results are bit-reproducible.
//
// Mapping: a group of G lanes (G = 1..64, a power of two) owns one output row; lane t of
// the group owns columns 4*(t + G*j), j < NJ, as one 16-byte vector, so a group's gather of
// one neighbour row is a single fully coalesced request of F*sizeof(elem) bytes.  The
// group's lanes fetch G column indices with one coalesced load and hand them round with
// wavefront shuffles; four neighbour rows are requested before any is accumulated so that
// several gathers are in flight per lane.
//
// Degree skew: rows longer than SPMM_LONG_ROW edges are cut, when the partition is built,
// into chunks of at most SPMM_CHUNK edges.  A workgroup owns a chunk (its 256/G groups take
// contiguous slices and are summed through LDS in a fixed order) and writes one partial row;
// a third kernel adds a row's partials in chunk order and applies the epilogue.  The split
// depends only on the graph, so results do not depend on scheduling.
#include "common.h"

#include <mutex>
#include <type_traits>

namespace grp {

template <typename T> struct Vec4Load;
template <> struct Vec4Load<float> {
    static __device__ __forceinline__ float4 ld(const float* p) { return *reinterpret_cast<const float4*>(p); }
};
template <> struct Vec4Load<__hip_bfloat16> {
    static __device__ __forceinline__ float4 ld(const __hip_bfloat16* p) {
        uint2 r = *reinterpret_cast<const uint2*>(p);
        float4 v;
        v.x = __uint_as_float(r.x << 16);
        v.y = __uint_as_float(r.x & 0xFFFF0000u);
        v.z = __uint_as_float(r.y << 16);
        v.w = __uint_as_float(r.y & 0xFFFF0000u);
        return v;
    }
};

constexpr int SPMM_DEEP_G = 16;      // groups of this many lanes (rows of 33..64 elements) keep 8 gathers in flight

__device__ __forceinline__ float row_scale(int mode, int64_t deg, int self_term) {
    if (mode == GRP_SCALE_MEAN) return 1.0f / (float)(deg > 1 ? deg : 1);
    if (mode == GRP_SCALE_RSQRT) {
        int64_t d = deg + self_term;
        return 1.0f / sqrtf((float)(d > 1 ? d : 1));
    }
    return 1.0f;
}

__device__ __forceinline__ void axpy4(float4& acc, float s, const float4& v) {
    acc.x = fmaf(s, v.x, acc.x); acc.y = fmaf(s, v.y, acc.y);
    acc.z = fmaf(s, v.z, acc.z); acc.w = fmaf(s, v.w, acc.w);
}
__device__ __forceinline__ void add4(float4& acc, const float4& v) {
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
}

// Sum of X rows over the edges [b, e) for the calling group of G lanes (lane t).
// EV: every edge carries a value val[e] that multiplies its gathered row.
// U neighbour rows are requested before any is accumulated: 4, or 8 for groups of 16 lanes (measured:
// +4 % at F = 47; no gain for wider rows, and narrower groups fetch fewer than 8 indices per batch).
// WIDE (bf16 rows of whole 16-byte units, NJ = 2): a lane owns eight consecutive columns, fetched with one 16-byte load
// and kept as two adjacent 4-column slabs, so a row takes half the lanes and a wavefront gathers twice the rows.
template <int G, bool WIDE> __device__ __forceinline__ int slab_col(int t, int j) { return WIDE ? 8 * t + 4 * j : 4 * (t + G * j); }
__device__ __forceinline__ void bf16x8_to_float4s(const uint4& r, float4& lo, float4& hi) {
    lo = make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u), __uint_as_float(r.y << 16),
                     __uint_as_float(r.y & 0xFFFF0000u));
    hi = make_float4(__uint_as_float(r.z << 16), __uint_as_float(r.z & 0xFFFF0000u), __uint_as_float(r.w << 16),
                     __uint_as_float(r.w & 0xFFFF0000u));
}
template <typename XT, int G, int NJ, bool EV, bool WIDE = false>
__device__ __forceinline__ void gather_rows(const int32_t* __restrict__ idx, const float* __restrict__ val, int64_t b,
                                            int64_t e, const XT* __restrict__ X, int64_t ldx,
                                            const float* __restrict__ colscale, int t, const bool (&live)[NJ],
                                            float4 (&acc)[NJ]) {
    constexpr int U = (G == SPMM_DEEP_G && NJ == 1) ? 8 : 4;       // a batch holds G indices, so U <= G
    for (int64_t base = b; base < e; base += G) {
        const int cnt = (int)((e - base) < (int64_t)G ? (e - base) : (int64_t)G);
        const int mine = (t < cnt) ? idx[base + t] : 0;
        float minew = 1.f;
        if (EV) minew = (t < cnt) ? val[base + t] : 0.f;
        int k = 0;
        for (; k + U <= cnt; k += U) {
            int64_t c[U];
            float sc[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                c[u] = __shfl(mine, k + u, G);
                sc[u] = colscale ? colscale[c[u]] : 1.f;
                if (EV) sc[u] *= __shfl(minew, k + u, G);
            }
            if constexpr (WIDE) {
                static_assert(!WIDE || (NJ == 2 && sizeof(XT) == 2), "eight bf16 columns per lane");
                if (live[0]) {                             // F is a multiple of 8: both slabs are live or neither
                    uint4 r[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) r[u] = *reinterpret_cast<const uint4*>(X + c[u] * ldx + 8 * t);
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        float4 lo, hi;
                        bf16x8_to_float4s(r[u], lo, hi);
                        if (EV || colscale) { axpy4(acc[0], sc[u], lo); axpy4(acc[1], sc[u], hi); }
                        else { add4(acc[0], lo); add4(acc[1], hi); }
                    }
                }
            } else
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (!live[j]) continue;
                const int col = 4 * (t + G * j);
                float4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = Vec4Load<XT>::ld(X + c[u] * ldx + col);
                if (EV || colscale) {
#pragma unroll
                    for (int u = 0; u < U; ++u) axpy4(acc[j], sc[u], v[u]);
                } else {
#pragma unroll
                    for (int u = 0; u < U; ++u) add4(acc[j], v[u]);
                }
            }
        }
        for (; k < cnt; ++k) {
            const int64_t c0 = __shfl(mine, k, G);
            float s0 = colscale ? colscale[c0] : 1.f;
            if (EV) s0 *= __shfl(minew, k, G);
            if constexpr (WIDE) {
                if (live[0]) {
                    float4 lo, hi;
                    bf16x8_to_float4s(*reinterpret_cast<const uint4*>(X + c0 * ldx + 8 * t), lo, hi);
                    axpy4(acc[0], s0, lo); axpy4(acc[1], s0, hi);
                }
            } else
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (!live[j]) continue;
                const float4 v0 = Vec4Load<XT>::ld(X + c0 * ldx + 4 * (t + G * j));
                axpy4(acc[j], s0, v0);
            }
        }
    }
}

struct SpmmEpilogue {
    int scale, self_term, relu, F;
    const float* addend;      // may alias Y
    int64_t ld_add;
    const float* bias;
    float* Y;
    int64_t ldy;
    const float* residual;    // added after the ReLU (residual layers); null otherwise
    int64_t ld_res;
    float* Y2;                // receives the activation before the residual is added; null otherwise
    int64_t ldy2;
    int64_t addend_rows;      // rows >= this have no addend
    const float* mask;        // keep where mask > 0 (after the ReLU); null otherwise
    int64_t ld_mask;
    const float* rowscale;    // a_i given explicitly; null: from `scale` and the row length
    const int64_t* n_rows_dev;       // when set: the real row count and the real addend_rows (device values;
    const int64_t* addend_rows_dev;  //           the launch and addend_rows above are upper bounds)
};

template <typename XT>
__device__ __forceinline__ void finish_row(const SpmmEpilogue& ep, int64_t i, int64_t deg, int col, float4 r,
                                           const XT* __restrict__ X, int64_t ldx) {
    const float a = ep.rowscale ? ep.rowscale[i] : row_scale(ep.scale, deg, ep.self_term);
    if (ep.self_term) add4(r, Vec4Load<XT>::ld(X + i * ldx + col));
    r.x *= a; r.y *= a; r.z *= a; r.w *= a;
    if (ep.addend && i < (ep.addend_rows_dev ? *ep.addend_rows_dev : ep.addend_rows)) add4(r, *reinterpret_cast<const float4*>(ep.addend + i * ep.ld_add + col));
    float o[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (col + q < ep.F) {
            if (ep.bias) o[q] += ep.bias[col + q];
            if (ep.relu) o[q] = o[q] > 0.f ? o[q] : 0.f;
        } else {
            o[q] = 0.f;           // pad columns stay zero
        }
    }
    if (ep.mask) {
        const float4 mk = *reinterpret_cast<const float4*>(ep.mask + i * ep.ld_mask + col);
        o[0] = mk.x > 0.f ? o[0] : 0.f; o[1] = mk.y > 0.f ? o[1] : 0.f;
        o[2] = mk.z > 0.f ? o[2] : 0.f; o[3] = mk.w > 0.f ? o[3] : 0.f;
    }
    if (ep.Y2) *reinterpret_cast<float4*>(ep.Y2 + i * ep.ldy2 + col) = make_float4(o[0], o[1], o[2], o[3]);
    if (ep.residual) {
        const float4 h = *reinterpret_cast<const float4*>(ep.residual + i * ep.ld_res + col);
        o[0] += h.x; o[1] += h.y; o[2] += h.z; o[3] += h.w;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (col + q >= ep.F) o[q] = 0.f;
    }
    *reinterpret_cast<float4*>(ep.Y + i * ep.ldy + col) = make_float4(o[0], o[1], o[2], o[3]);
}

// One workgroup per chunk of a long row -> one partial row.
template <typename XT, int G, int NJ, bool EV, bool WIDE = false>
__device__ __forceinline__ void chunk_body(int64_t cb, int64_t ce, const int32_t* __restrict__ idx,
                                           const float* __restrict__ val, int F,
                                           const XT* __restrict__ X, int64_t ldx, const float* __restrict__ colscale,
                                           float* __restrict__ part_row, float* red) {
    constexpr int NG = 256 / G;
    constexpr int W = 4 * G * NJ;                 // padded row width held by a group
    const int t = threadIdx.x % G, gi = threadIdx.x / G;
    const int64_t per = (ce - cb + NG - 1) / NG;
    int64_t b = cb + gi * per, e = b + per;
    if (b > ce) b = ce;
    if (e > ce) e = ce;
    float4 acc[NJ];
    bool live[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        live[j] = slab_col<G, WIDE>(t, j) < F;
    }
    gather_rows<XT, G, NJ, EV, WIDE>(idx, val, b, e, X, ldx, colscale, t, live, acc);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
        *reinterpret_cast<float4*>(&red[gi * W + slab_col<G, WIDE>(t, j)]) = acc[j];
    __syncthreads();
    const int fpad = (F + 3) & ~3;
    for (int c = threadIdx.x; c < fpad; c += 256) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < NG; ++q) s += red[q * W + c];
        part_row[c] = s;
    }
}

// The first n_chunks workgroups each reduce one chunk of a long row to a partial row (they
// are the heavy ones, so they start first); the others take the rows of at most `long_thr`
// edges, one group per row.  One launch instead of two keeps the few chunk workgroups from
// running on an otherwise idle chip.
template <typename XT, int G, int NJ, bool EV, bool WIDE = false>
__global__ __launch_bounds__(256) void spmm_rows_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx,
                                                        const float* __restrict__ val, int64_t n_rows, int64_t long_thr,
                                                        const XT* __restrict__ X,
                                                        int64_t ldx, const float* __restrict__ colscale,
                                                        SpmmEpilogue ep, int n_chunks,
                                                        const int64_t* __restrict__ chunk_begin,
                                                        const int64_t* __restrict__ chunk_end,
                                                        float* __restrict__ partials, int64_t ld_part) {
    constexpr int ROWS = 256 / G;
    __shared__ __attribute__((aligned(16))) float red[ROWS * 4 * G * NJ];
    if ((int)blockIdx.x < n_chunks) {              // uniform per workgroup
        chunk_body<XT, G, NJ, EV, WIDE>(chunk_begin[blockIdx.x], chunk_end[blockIdx.x], idx, val, ep.F, X, ldx, colscale,
                              partials + (int64_t)blockIdx.x * ld_part, red);
        return;
    }
    const int t = threadIdx.x % G;
    const int64_t i = (int64_t)(blockIdx.x - n_chunks) * ROWS + threadIdx.x / G;
    if (i >= (ep.n_rows_dev ? *ep.n_rows_dev : n_rows)) return;          // whole groups leave together (G divides 64)
    const int64_t b = ptr[i], e = ptr[i + 1];
    if (e - b > long_thr) return;     // its chunks are reduced above, the row is finished by the combine kernel
    float4 acc[NJ];
    bool live[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        live[j] = slab_col<G, WIDE>(t, j) < ep.F;
    }
    gather_rows<XT, G, NJ, EV, WIDE>(idx, val, b, e, X, ldx, colscale, t, live, acc);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
        if (live[j]) finish_row<XT>(ep, i, e - b, slab_col<G, WIDE>(t, j), acc[j], X, ldx);
}

// One group per long row: partial rows added in chunk order, then the epilogue.
template <typename XT, int G, int NJ>
__global__ __launch_bounds__(256) void spmm_combine_kernel(const int32_t* __restrict__ long_row,
                                                           const int32_t* __restrict__ long_first, int n_long,
                                                           const int64_t* __restrict__ ptr,
                                                           const float* __restrict__ partials, int64_t ld_part,
                                                           const XT* __restrict__ X, int64_t ldx, SpmmEpilogue ep) {
    constexpr int ROWS = 256 / G;
    const int t = threadIdx.x % G;
    const int j0 = blockIdx.x * ROWS + threadIdx.x / G;
    if (j0 >= n_long) return;
    const int64_t i = long_row[j0];
    if (i < 0) return;                // an unused slot of a schedule built to its capacity
    const int c0 = long_first[j0], c1 = long_first[j0 + 1];
    const int64_t deg = ptr[i + 1] - ptr[i];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = 4 * (t + G * j);
        if (col >= ep.F) continue;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int c = c0; c < c1; ++c) add4(acc, *reinterpret_cast<const float4*>(partials + (int64_t)c * ld_part + col));
        finish_row<XT>(ep, i, deg, col, acc, X, ldx);
    }
}

// ---- the source-sliced schedule of the long rows (slices.hip): one wavefront per task.
// A task is at most SLICE_TASK_MAX consecutive edges of one long row whose sources lie in one slice of the
// node ids.  The wavefront reads the task's indices with coalesced loads (SLICE_PIECE / 64 per lane), its 64 / G groups
// take consecutive runs of them (handed round with shuffles, up to four gathers in flight per group), the
// groups' sums are added across the wavefront in a fixed butterfly, and the first group writes the partial row.
// VW consecutive elements of a row as floats: the unit a lane owns (16 bytes of fp32, 8 or 16 bytes of bf16).
template <typename XT, int VW> struct LaneVec;
template <> struct LaneVec<float, 4> {
    static __device__ __forceinline__ void ld(const float* p, float (&f)[4]) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
};
template <> struct LaneVec<__hip_bfloat16, 4> {
    static __device__ __forceinline__ void ld(const __hip_bfloat16* p, float (&f)[4]) {
        const uint2 r = *reinterpret_cast<const uint2*>(p);
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
    }
};
template <> struct LaneVec<__hip_bfloat16, 8> {
    static __device__ __forceinline__ void ld(const __hip_bfloat16* p, float (&f)[8]) {
        const uint4 r = *reinterpret_cast<const uint4*>(p);
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
        f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xFFFF0000u);
        f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xFFFF0000u);
    }
};

// G lanes own a row, VW elements each (VW = 8 for bf16 rows that allow 16-byte loads: half the lanes per row,
// so twice the rows in flight per wavefront for the same registers), NJ slabs of G * VW columns.
// SHIFT32 (plain sums only: no edge values, no per-source scale): the rows of X start at multiples of 2^row_shift
// bytes and X is smaller than 4 GiB, so a row's address is a 32-bit shift and add beside the base (the generic
// 64-bit index x pitch product costs three quarter-rate multiplies per gather: a third of the loop's issue cycles),
// and a gathered row is added with one multiply-add per element (times 1, or 0 past the task's end).
template <typename XT, int G, int NJ, int VW, bool EV, bool CS, bool SHIFT32 = false>
__global__ __launch_bounds__(256) void spmm_tasks_kernel(const SliceTask* __restrict__ tasks, int64_t n_tasks, int64_t per_wave,
                                                         const int32_t* __restrict__ idx, const float* __restrict__ val, int F,
                                                         const XT* __restrict__ X, int64_t ldx,
                                                         const float* __restrict__ colscale, float* __restrict__ partials,
                                                         int64_t ld_part, int row_shift) {
    static_assert(!SHIFT32 || (!EV && !CS), "the 32-bit addressing variant is built for plain sums");
    constexpr int IPL = SLICE_PIECE / 64;                 // indices of a task per lane
    static_assert(IPL * 64 == SLICE_PIECE && (IPL & (IPL - 1)) == 0, "a task's indices fill whole registers");
    constexpr int NG = 64 / G;
    constexpr int U = (G * VW >= 64 && NJ == 1) ? 8 : 4;   // gathers in flight per group (measured: 8 loses for narrower rows)
    const int lane = threadIdx.x & 63;
    const int t = lane % G, gi = lane / G;
    // wavefront w takes the tasks [w * per_wave, (w + 1) * per_wave): consecutive wavefronts walk the processing
    // order front to back (a launch holds at most 2^32 work-items, so one task per wavefront does not scale).
    // The loop is software-pipelined: while the gathers of task p are in flight, the indices of task p + 1 and the
    // record of task p + 2 are requested, so a task costs one memory round trip instead of three.
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t p0 = w * per_wave;
    const int64_t p_end = p0 + per_wave < n_tasks ? p0 + per_wave : n_tasks;
    if (p0 >= p_end) return;                               // uniform over the wavefront
    // Every load below is unconditional (an index past a task's end is clamped to its last edge and the gathered
    // row then dropped by a select): a conditional load becomes a branch with a wait behind it, and the gathers
    // of a task would no longer overlap.
    // A task is walked in passes of up to SLICE_PIECE edges; (begin, len) name a pass.
    auto load_indices = [&](int64_t begin, int len, int32_t (&ix)[IPL], float (&wx)[IPL]) {
        const int last = len > 0 ? len - 1 : 0;
#pragma unroll
        for (int q = 0; q < IPL; ++q) {
            const int64_t e = begin + (64 * q + lane < last ? 64 * q + lane : last);
            ix[q] = idx[e];
            if (EV) wx[q] = val[e];
        }
    };
    auto pass_len = [](const SliceTask& tk, int off) { return (int)tk.len - off < SLICE_PIECE ? (int)tk.len - off : SLICE_PIECE; };
    SliceTask cur = tasks[p0];
    SliceTask nxt = tasks[p0 + 1 < p_end ? p0 + 1 : p0];
    int32_t ix[IPL];
    float wx[IPL];
#pragma unroll
    for (int q = 0; q < IPL; ++q) wx[q] = 1.f;
    load_indices(cur.begin, pass_len(cur, 0), ix, wx);
    int col[NJ];                                           // first column of the lane's unit in slab j (a dead unit reads column 0)
    bool live[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        live[j] = VW * (t + G * j) < F;
        col[j] = live[j] ? VW * (t + G * j) : 0;
    }
    float acc[NJ][VW];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int q = 0; q < VW; ++q) acc[j][q] = 0.f;
    int off = 0;                                           // edges of the current task already added
    for (int64_t p = p0; p < p_end;) {
        const int len = pass_len(cur, off);                // >= 1: this pass
        const bool last_pass = off + len == (int)cur.len;
        const int per = (len + NG - 1) / NG;               // the same in every lane
        const int first = gi * per;
        SliceTask nn = nxt;
        int32_t nix[IPL];
        float nwx[IPL];
#pragma unroll
        for (int q = 0; q < IPL; ++q) { nix[q] = 0; nwx[q] = 1.f; }
        for (int k0 = 0; k0 < per; k0 += U) {
            int64_t c[U];
            float sc[U];
            bool on[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int pos = first + k0 + u;
                on[u] = k0 + u < per && pos < len;
                const int src = pos & 63;
                int32_t ci = __shfl(ix[0], src, 64);
#pragma unroll
                for (int q = 1; q < IPL; ++q) {
                    const int32_t o = __shfl(ix[q], src, 64);
                    ci = (pos >> 6) == q ? o : ci;
                }
                c[u] = ci;                                 // a valid index of this task even where `on` is false
                sc[u] = 1.f;
                if (EV) {
                    float wi = __shfl(wx[0], src, 64);
#pragma unroll
                    for (int q = 1; q < IPL; ++q) {
                        const float o = __shfl(wx[q], src, 64);
                        wi = (pos >> 6) == q ? o : wi;
                    }
                    sc[u] = wi;
                }
                if (CS) sc[u] *= colscale[c[u]];
            }
            float v[NJ][U][VW];
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (SHIFT32) {
                        const uint32_t off = ((uint32_t)c[u] << row_shift) + (uint32_t)(col[j] * (int)sizeof(XT));
                        const XT* const src = reinterpret_cast<const XT*>(reinterpret_cast<const char*>(X) + off);
                        LaneVec<XT, VW>::ld(src, v[j][u]);
                    } else {
                        LaneVec<XT, VW>::ld(X + c[u] * ldx + col[j], v[j][u]);
                    }
                }
            if (k0 == 0) {                                 // behind the first gathers: what the next pass and the task after next need
                __builtin_amdgcn_sched_barrier(0);
                if (last_pass) {
                    load_indices(nxt.begin, pass_len(nxt, 0), nix, nwx);
                    nn = tasks[p + 2 < p_end ? p + 2 : p];
                } else {
                    load_indices(cur.begin + off + len, pass_len(cur, off + len), nix, nwx);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int q = 0; q < VW; ++q) {
                        float x = v[j][u][q];
                        if constexpr (SHIFT32) {
                            acc[j][q] = fmaf(x, on[u] ? 1.f : 0.f, acc[j][q]);     // x * 1 + acc rounds once, as x + acc does
                        } else {
                            if (EV || CS) x *= sc[u];
                            acc[j][q] += on[u] ? x : 0.f;
                        }
                    }
        }
        if (last_pass) {                                   // uniform: the task's partial row
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
#pragma unroll
                for (int o = G; o < 64; o <<= 1)
#pragma unroll
                    for (int q = 0; q < VW; ++q) acc[j][q] += __shfl_xor(acc[j][q], o, 64);
                if (gi == 0 && live[j]) {
                    float* out = partials + (int64_t)cur.id * ld_part + col[j];
#pragma unroll
                    for (int q = 0; q < VW; q += 4)
                        *reinterpret_cast<float4*>(out + q) = make_float4(acc[j][q], acc[j][q + 1], acc[j][q + 2], acc[j][q + 3]);
                }
#pragma unroll
                for (int q = 0; q < VW; ++q) acc[j][q] = 0.f;
            }
            cur = nxt; nxt = nn;
            off = 0;
            ++p;
        } else {
            off += len;
        }
#pragma unroll
        for (int q = 0; q < IPL; ++q) { ix[q] = nix[q]; if (EV) wx[q] = nwx[q]; }
    }
}

// One wavefront per long row: group g adds the row's partial rows g, g + 64/G, ... in ascending order, the groups'
// sums are added in a fixed butterfly, then the epilogue.
template <typename XT, int G, int NJ>
__global__ __launch_bounds__(256) void spmm_combine_tasks_kernel(const int32_t* __restrict__ long_row,
                                                                 const int64_t* __restrict__ row_task, int n_long,
                                                                 const int64_t* __restrict__ ptr,
                                                                 const float* __restrict__ partials, int64_t ld_part,
                                                                 const XT* __restrict__ X, int64_t ldx, SpmmEpilogue ep) {
    constexpr int NG = 64 / G;
    const int lane = threadIdx.x & 63;
    const int j0 = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j0 >= n_long) return;
    const int64_t i = long_row[j0];
    if (i < 0) return;
    const int t = lane % G, gi = lane / G;
    const int64_t t0 = row_task[j0], t1 = row_task[j0 + 1];
    const int64_t deg = ptr[i + 1] - ptr[i];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = 4 * (t + G * j);
        const bool live = col < ep.F;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live) {
            int64_t c = t0 + gi;
            for (; c + 3 * NG < t1; c += 4 * NG) {          // four loads in flight, added in ascending order
                const float4 a0 = *reinterpret_cast<const float4*>(partials + c * ld_part + col);
                const float4 a1 = *reinterpret_cast<const float4*>(partials + (c + NG) * ld_part + col);
                const float4 a2 = *reinterpret_cast<const float4*>(partials + (c + 2 * NG) * ld_part + col);
                const float4 a3 = *reinterpret_cast<const float4*>(partials + (c + 3 * NG) * ld_part + col);
                add4(acc, a0); add4(acc, a1); add4(acc, a2); add4(acc, a3);
            }
            for (; c < t1; c += NG) add4(acc, *reinterpret_cast<const float4*>(partials + c * ld_part + col));
        }
#pragma unroll
        for (int o = G; o < 64; o <<= 1) {
            acc.x += __shfl_xor(acc.x, o, 64);
            acc.y += __shfl_xor(acc.y, o, 64);
            acc.z += __shfl_xor(acc.z, o, 64);
            acc.w += __shfl_xor(acc.w, o, 64);
        }
        if (gi == 0 && live) finish_row<XT>(ep, i, deg, col, acc, X, ldx);
    }
}

// Fallback for pitches or pointers that are not 16-byte friendly: one wavefront per row,
// one lane per column (handles rows of any length itself).
template <typename XT>
__global__ __launch_bounds__(256) void spmm_rows_scalar_kernel(
    const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx, int64_t n_rows, int F,
    const XT* __restrict__ X, int64_t ldx, int scale, int self_term, const float* __restrict__ colscale,
    const float* addend, int64_t ld_add, const float* __restrict__ bias, int relu,
    float* Y, int64_t ldy, const float* __restrict__ val, const float* __restrict__ rowscale,
    const int64_t* __restrict__ n_rows_dev /*when set: the real row count; n_rows sized the launch*/) {
    const int64_t i = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (i >= (n_rows_dev ? *n_rows_dev : n_rows)) return;
    const int t = threadIdx.x % 64;
    const int64_t b = ptr[i], e = ptr[i + 1];
    const float a = rowscale ? rowscale[i] : row_scale(scale, e - b, self_term);
    for (int col = t; col < F; col += 64) {
        float acc = 0.f;
        for (int64_t k = b; k < e; ++k)
            acc = fmaf((colscale ? colscale[idx[k]] : 1.f) * (val ? val[k] : 1.f), (float)X[(int64_t)idx[k] * ldx + col], acc);
        if (self_term) acc += (float)X[i * ldx + col];
        acc *= a;
        if (addend) acc += addend[i * ld_add + col];
        if (bias) acc += bias[col];
        if (relu) acc = acc > 0.f ? acc : 0.f;
        Y[i * ldy + col] = acc;
    }
}

template <typename XT, int G, int NJ>
static void launch_one(const SpmmArgs& a, const SpmmEpilogue& ep, hipStream_t st) {
    constexpr int ROWS = 256 / G;
    const LongRows* lr = a.long_rows;
    const bool split = lr && lr->n_long > 0;
    const bool sliced = split && lr->n_tasks > 0;
    const int64_t thr = split ? (int64_t)SPMM_LONG_ROW : INT64_MAX;
    const int n_chunks = split && !sliced ? lr->n_chunks : 0;
    const int64_t ld_part = round_up(a.F, 4);
    if (sliced) {                                          // the long rows' tasks, slice by slice
        // at most 2^19 workgroups of four wavefronts: a wavefront that walks a dozen consecutive tasks keeps its
        // pipeline of index and record prefetches full (2^21 / 2^19 / 2^17 workgroups on the 2^32-edge share: bf16
        // launch 44.3 / 42.9 / 42.4 ms, fp32 F = 16 launch 34.7 / 34.7 / 35.6 ms)
        const int64_t per_wave = cdiv(lr->n_tasks, (int64_t)4 << 19);
        const dim3 tgrid((unsigned)cdiv(lr->n_tasks, 4 * per_wave));
        // plain sums over rows that start at multiples of a power of two inside less than 4 GiB: 32-bit addressing
        int row_shift = -1;
        {
            const int64_t pitch_bytes = a.ldx * (int64_t)sizeof(XT);
            const int64_t x_rows = a.n_src > 0 ? a.n_src : a.n_rows;
            if (!a.val && !a.colscale && pitch_bytes > 0 && (pitch_bytes & (pitch_bytes - 1)) == 0 &&
                x_rows * pitch_bytes <= ((int64_t)1 << 32)) {
                row_shift = 0;
                while (((int64_t)1 << row_shift) < pitch_bytes) ++row_shift;
            }
        }
        auto go = [&](auto kernel) {
            hipLaunchKernelGGL(kernel, tgrid, dim3(256), 0, st, (const SliceTask*)lr->tasks, lr->n_tasks, per_wave, a.idx, a.val, a.F,
                               (const XT*)a.X, a.ldx, a.colscale, a.partials, ld_part, row_shift);
        };
        // bf16 rows of whole 16-byte units: eight elements per lane, half the lanes per row
        constexpr bool bf16 = std::is_same<XT, __hip_bfloat16>::value;
        const bool wide = bf16 && G >= 2 && NJ == 1 && a.F % 8 == 0 && a.ldx % 8 == 0 && ((uintptr_t)a.X % 16) == 0;
        if constexpr (bf16 && G >= 2 && NJ == 1) {
            if (wide) {
                if (a.val && a.colscale) go(spmm_tasks_kernel<XT, G / 2, 1, 8, true, true>);
                else if (a.val) go(spmm_tasks_kernel<XT, G / 2, 1, 8, true, false>);
                else if (a.colscale) go(spmm_tasks_kernel<XT, G / 2, 1, 8, false, true>);
                else if (row_shift >= 0) go(spmm_tasks_kernel<XT, G / 2, 1, 8, false, false, true>);
                else go(spmm_tasks_kernel<XT, G / 2, 1, 8, false, false>);
            }
        }
        if (!wide) {
            if (a.val && a.colscale) go(spmm_tasks_kernel<XT, G, NJ, 4, true, true>);
            else if (a.val) go(spmm_tasks_kernel<XT, G, NJ, 4, true, false>);
            else if (a.colscale) go(spmm_tasks_kernel<XT, G, NJ, 4, false, true>);
            else if (row_shift >= 0) go(spmm_tasks_kernel<XT, G, NJ, 4, false, false, true>);
            else go(spmm_tasks_kernel<XT, G, NJ, 4, false, false>);
        }
    }
    bool rows_done = false;
    if constexpr (std::is_same<XT, __hip_bfloat16>::value && G >= 2 && NJ == 1) {
        // bf16 rows of whole 16-byte units: eight columns per lane, half the lanes per row (twice the rows per wavefront)
        if (a.F % 8 == 0 && a.ldx % 8 == 0 && ((uintptr_t)a.X % 16) == 0 && !a.self_term) {
            constexpr int GW = G / 2;
            const dim3 wgrid((unsigned)(n_chunks + cdiv(a.n_rows, 256 / GW)));
            if (a.val)
                hipLaunchKernelGGL((spmm_rows_kernel<XT, GW, 2, true, true>), wgrid, dim3(256), 0, st, a.ptr, a.idx, a.val, a.n_rows,
                                   thr, (const XT*)a.X, a.ldx, a.colscale, ep, n_chunks, n_chunks ? lr->chunk_begin : nullptr,
                                   n_chunks ? lr->chunk_end : nullptr, a.partials, ld_part);
            else
                hipLaunchKernelGGL((spmm_rows_kernel<XT, GW, 2, false, true>), wgrid, dim3(256), 0, st, a.ptr, a.idx, a.val, a.n_rows,
                                   thr, (const XT*)a.X, a.ldx, a.colscale, ep, n_chunks, n_chunks ? lr->chunk_begin : nullptr,
                                   n_chunks ? lr->chunk_end : nullptr, a.partials, ld_part);
            rows_done = true;
        }
    }
    const dim3 grid((unsigned)(n_chunks + cdiv(a.n_rows, ROWS)));
    if (rows_done) {
    } else if (a.val)
        hipLaunchKernelGGL((spmm_rows_kernel<XT, G, NJ, true>), grid, dim3(256), 0, st, a.ptr, a.idx, a.val, a.n_rows, thr,
                           (const XT*)a.X, a.ldx, a.colscale, ep, n_chunks, n_chunks ? lr->chunk_begin : nullptr,
                           n_chunks ? lr->chunk_end : nullptr, a.partials, ld_part);
    else
        hipLaunchKernelGGL((spmm_rows_kernel<XT, G, NJ, false>), grid, dim3(256), 0, st, a.ptr, a.idx, a.val, a.n_rows, thr,
                           (const XT*)a.X, a.ldx, a.colscale, ep, n_chunks, n_chunks ? lr->chunk_begin : nullptr,
                           n_chunks ? lr->chunk_end : nullptr, a.partials, ld_part);
    if (sliced) {
        hipLaunchKernelGGL((spmm_combine_tasks_kernel<XT, G, NJ>), dim3((unsigned)cdiv(lr->n_long, 4)), dim3(256), 0, st,
                           lr->long_row, (const int64_t*)lr->row_task, lr->n_long, a.ptr, (const float*)a.partials, ld_part,
                           (const XT*)a.X, a.ldx, ep);
    } else if (split) {
        hipLaunchKernelGGL((spmm_combine_kernel<XT, G, NJ>), dim3((unsigned)cdiv(lr->n_long, ROWS)), dim3(256), 0, st,
                           lr->long_row, lr->long_first, lr->n_long, a.ptr, (const float*)a.partials, ld_part,
                           (const XT*)a.X, a.ldx, ep);
    }
}

template <typename XT>
static grp_status dispatch(const SpmmArgs& a, const SpmmEpilogue& ep, hipStream_t st) {
    const int f4 = (a.F + 3) / 4;
    {       // a launch holds fewer than 2^32 work-items: a row per group of f4 lanes (rounded up to a power of two)
        int g = 1;
        while (g < f4 && g < 64) g <<= 1;
        const LongRows* lr = a.long_rows;
        const int64_t chunks = lr && lr->n_long > 0 && lr->n_tasks == 0 ? lr->n_chunks : 0;
        if ((chunks + cdiv(a.n_rows, 256 / g)) * 256 >= ((int64_t)1 << 32))
            return fail(GRP_EUNSUPPORTED, "spmm: %lld rows of %d columns exceed one launch", (long long)a.n_rows, a.F);
    }
    if (f4 <= 1) launch_one<XT, 1, 1>(a, ep, st);
    else if (f4 <= 2) launch_one<XT, 2, 1>(a, ep, st);
    else if (f4 <= 4) launch_one<XT, 4, 1>(a, ep, st);
    else if (f4 <= 8) launch_one<XT, 8, 1>(a, ep, st);
    else if (f4 <= 16) launch_one<XT, 16, 1>(a, ep, st);
    else if (f4 <= 32) launch_one<XT, 32, 1>(a, ep, st);
    else if (f4 <= 64) launch_one<XT, 64, 1>(a, ep, st);
    else if (f4 <= 128) launch_one<XT, 64, 2>(a, ep, st);
    else if (f4 <= 256) launch_one<XT, 64, 4>(a, ep, st);
    else return fail(GRP_EUNSUPPORTED, "spmm: F = %d exceeds 1024", a.F);
    return GRP_OK;
}

size_t spmm_partials_bytes(const LongRows* lr, int32_t F) {
    if (!lr || lr->n_long == 0) return 0;
    const int64_t slots = lr->n_tasks > 0 ? lr->n_tasks : (int64_t)lr->n_chunks;      // one partial row per task or chunk
    return (size_t)slots * round_up(F, 4) * sizeof(float);
}

grp_status launch_spmm(const SpmmArgs& a, hipStream_t st) {
    if (a.n_rows == 0) return GRP_OK;
    if (a.n_rows < 0 || a.F <= 0 || !a.ptr || !a.X || !a.Y)
        return fail(GRP_EINVAL, "spmm: bad arguments");
    const int elem = a.x_bf16 ? 2 : 4;
    const int64_t fpad = round_up(a.F, 4);
    const bool vec_ok = a.ldx >= fpad && a.ldy >= fpad && a.ldx % 4 == 0 && a.ldy % 4 == 0 &&
                        ((uintptr_t)a.X % (4 * elem)) == 0 && ((uintptr_t)a.Y % 16) == 0 &&
                        (!a.addend || (a.ld_add % 4 == 0 && a.ld_add >= fpad && ((uintptr_t)a.addend % 16) == 0));
    // compulsory traffic: the index stream, the row pointers, every source row once, every
    // output row once (+ addend rows)
    const int64_t n_src = a.n_src > 0 ? a.n_src : a.n_rows;
    const double bytes = 4.0 * a.nnz + 8.0 * (a.n_rows + 1) + (double)elem * a.F * n_src +
                         4.0 * a.F * a.n_rows * (1.0 + (a.addend ? 1.0 : 0.0) + (a.mask ? 1.0 : 0.0)) +
                         (a.colscale ? 4.0 * n_src : 0.0) + (a.val ? 4.0 * a.nnz : 0.0);
    prof_detail("[rows=%lld,F=%d,nnz=%lld]", (long long)a.n_rows, a.F, (long long)a.nnz);
    ProfScope ps(a.x_bf16 ? "spmm_rows_bf16" : "spmm_rows_f32", st, 2.0 * a.nnz * a.F, bytes);
    if (vec_ok) {
        if (a.long_rows && a.long_rows->n_long > 0 && (!a.partials || ((uintptr_t)a.partials % 16) != 0))
            return fail(GRP_EINVAL, "spmm: partition has long rows but no scratch for their partial sums");
        if (a.residual && (a.ld_res % 4 != 0 || a.ld_res < fpad || (uintptr_t)a.residual % 16 != 0))
            return fail(GRP_EINVAL, "spmm: residual operand must be 16-byte aligned with a pitch multiple of 4");
        if (a.Y2 && (a.ldy2 % 4 != 0 || a.ldy2 < fpad || (uintptr_t)a.Y2 % 16 != 0))
            return fail(GRP_EINVAL, "spmm: second output must be 16-byte aligned with a pitch multiple of 4");
        if (a.mask && (a.ld_mask % 4 != 0 || a.ld_mask < fpad || (uintptr_t)a.mask % 16 != 0))
            return fail(GRP_EINVAL, "spmm: mask must be 16-byte aligned with a pitch multiple of 4");
        SpmmEpilogue ep{a.scale, a.self_term, a.relu, a.F, a.addend, a.ld_add, a.bias, a.Y, a.ldy,
                        a.residual, a.ld_res, a.Y2, a.ldy2, a.addend_rows > 0 ? a.addend_rows : a.n_rows, a.mask, a.ld_mask,
                        a.rowscale, a.n_rows_dev, a.addend_rows_dev};
        GRP_TRY(a.x_bf16 ? dispatch<__hip_bfloat16>(a, ep, st) : dispatch<float>(a, ep, st));
    } else {
        if (a.residual || a.Y2 || a.mask || a.addend_rows > 0 || a.addend_rows_dev)
            return fail(GRP_EUNSUPPORTED, "spmm: this epilogue needs 16-byte friendly operands");
        const int64_t blocks = cdiv(a.n_rows, 4);
        if (a.x_bf16)
            hipLaunchKernelGGL((spmm_rows_scalar_kernel<__hip_bfloat16>), dim3((unsigned)blocks), dim3(256), 0, st,
                               a.ptr, a.idx, a.n_rows, a.F, (const __hip_bfloat16*)a.X, a.ldx, a.scale,
                               a.self_term, a.colscale, a.addend, a.ld_add, a.bias, a.relu, a.Y, a.ldy, a.val, a.rowscale, a.n_rows_dev);
        else
            hipLaunchKernelGGL((spmm_rows_scalar_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, st, a.ptr,
                               a.idx, a.n_rows, a.F, (const float*)a.X, a.ldx, a.scale, a.self_term, a.colscale, a.addend,
                               a.ld_add, a.bias, a.relu, a.Y, a.ldy, a.val, a.rowscale, a.n_rows_dev);
    }
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

}  // namespace grp

namespace grp {

static grp_status spmm_args_from_call(const grp_partition_t* part, int32_t transposed, int32_t scale, int32_t self_term, int32_t F,
                                      const void* X, int64_t ldx, int32_t x_dtype, float* Y, int64_t ldy, const char* who,
                                      SpmmArgs* out) {
    if (!part || !X || !Y) return fail(GRP_EINVAL, "%s: null argument", who);
    if (F <= 0 || F > 1024 || ldx < F || ldy < F) return fail(GRP_EINVAL, "%s: bad F / pitch", who);
    if (scale < GRP_SCALE_NONE || scale > GRP_SCALE_RSQRT) return fail(GRP_EINVAL, "%s: bad scale", who);
    if (x_dtype != GRP_DTYPE_FP32 && x_dtype != GRP_DTYPE_BF16) return fail(GRP_EINVAL, "%s: bad dtype", who);
    SpmmArgs a;
    a.ptr = transposed ? part->colptr : part->rowptr;
    a.idx = transposed ? part->row : part->col;
    a.long_rows = transposed ? &part->csc_long : &part->csr_long;
    a.n_rows = part->n;
    a.nnz = part->nnz;
    a.F = F;
    a.X = X;
    a.ldx = ldx;
    a.x_bf16 = x_dtype == GRP_DTYPE_BF16;
    a.scale = scale;
    a.self_term = self_term ? 1 : 0;
    a.Y = Y;
    a.ldy = ldy;
    *out = a;
    return GRP_OK;
}

// The partial sums of split rows for callers that cannot allocate: one array per GPU, reserved when the
// library is loaded and kept until the process ends.  The array's name is only a host-side stand-in;
// its device address is looked up once per device and cached.
constexpr size_t SPMM_STATIC_SCRATCH_BYTES = (size_t)32 << 20;
static __device__ __align__(256) unsigned char g_spmm_scratch[SPMM_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_spmm_scratch_ptr[MAX_DEVICES] = {nullptr};
static std::mutex g_spmm_scratch_mu;

static grp_status spmm_static_scratch(void** out) {
    int dev = 0;
    GRP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(GRP_EUNSUPPORTED, "device index %d is outside [0, %d)", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lk(g_spmm_scratch_mu);
    if (!g_spmm_scratch_ptr[dev]) {
        void* p = nullptr;
        GRP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_spmm_scratch)));      // the copy of the array on the current device
        g_spmm_scratch_ptr[dev] = p;
    }
    *out = g_spmm_scratch_ptr[dev];
    return GRP_OK;
}

}  // namespace grp

extern "C" grp_status grp_spmm_workspace_bytes(const grp_partition_t* part, int32_t transposed, int32_t F, size_t* bytes) {
    if (!part || !bytes) return grp::fail(GRP_EINVAL, "grp_spmm_workspace_bytes: null argument");
    if (F <= 0 || F > 1024) return grp::fail(GRP_EINVAL, "grp_spmm_workspace_bytes: bad F");
    *bytes = grp::spmm_partials_bytes(transposed ? &part->csc_long : &part->csr_long, F);
    return GRP_OK;
}

extern "C" grp_status grp_spmm(const grp_partition_t* part, int32_t transposed, int32_t scale,
                               int32_t self_term, int32_t F, const void* X, int64_t ldx, int32_t x_dtype,
                               float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    grp::SpmmArgs a;
    GRP_TRY(grp::spmm_args_from_call(part, transposed, scale, self_term, F, X, ldx, x_dtype, Y, ldy, "grp_spmm", &a));
    const size_t need = grp::spmm_partials_bytes(a.long_rows, F);
    if (need > 0 && (!workspace || workspace_bytes < need))
        return grp::fail(GRP_EWORKSPACE, "grp_spmm: workspace of %zu bytes, %zu needed", workspace_bytes, need);
    if (need > 0 && ((uintptr_t)workspace % 16) != 0) return grp::fail(GRP_EINVAL, "grp_spmm: workspace must be 16-byte aligned");
    a.partials = need ? (float*)workspace : nullptr;
    return grp::launch_spmm(a, (hipStream_t)stream);
}

extern "C" grp_status grp_spmm_static(const grp_partition_t* part, int32_t transposed, int32_t scale,
                                      int32_t self_term, int32_t F, const void* X, int64_t ldx, int32_t x_dtype,
                                      float* Y, int64_t ldy, void* stream) {
    grp::SpmmArgs a;
    GRP_TRY(grp::spmm_args_from_call(part, transposed, scale, self_term, F, X, ldx, x_dtype, Y, ldy, "grp_spmm_static", &a));
    const size_t need = grp::spmm_partials_bytes(a.long_rows, F);
    if (need > grp::SPMM_STATIC_SCRATCH_BYTES)
        return grp::fail(GRP_EWORKSPACE, "grp_spmm_static: the split rows of this partition need %zu bytes of partial sums at F = %d, "
                         "the built-in scratch holds %zu; use grp_spmm with a workspace", need, F, grp::SPMM_STATIC_SCRATCH_BYTES);
    void* scratch = nullptr;
    if (need > 0) GRP_TRY(grp::spmm_static_scratch(&scratch));
    a.partials = (float*)scratch;
    return grp::launch_spmm(a, (hipStream_t)stream);
}
