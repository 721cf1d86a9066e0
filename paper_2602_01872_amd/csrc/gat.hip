// Graph attention layers (one head) for gfx950: attention-weighted neighbour aggregation and its
// reverse pass, around the same MFMA GEMMs as the other models.
//
//   t_u = W^T h_u,  p_u = a_src . t_u,  q_v = a_dst . t_v,
//   e_uv = LeakyReLU_0.2(p_u + q_v) over the in-edges u -> v and the self term u = v,
//   alpha = softmax_u(e_uv),  out_v = sum_u alpha_uv t_u + b,  h'_v = ReLU(out_v) (hidden layers).
//
// Layout.  p and q are two more outputs of the layer's linear map, p = h . (W a_src) and
// q = h . (W a_dst), so the GEMM computes  T_ext = H [W | 0 | W a_src | W a_dst | 0 0]  with the
// two scores at the 16-byte aligned column ld(F); the reverse pass hands the GEMMs
// dT_ext = [dT | 0 | dp | dq | 0 0] in the same layout, and the gradients of W, a_src, a_dst
// follow from dW_ext = H^T dT_ext by the chain rule of the two extra columns.
//
// No per-edge state is kept: alpha_uv is recomputed from four per-node scalars (p_u, q_v, the
// row maximum m_v and the row sum Z_v), so the reverse pass can walk the CSC (rows = sources,
// for dT and dp) and the CSR (rows = destinations, for dq) independently, each row summing in
// its stored edge order: no floating-point atomics, bit-reproducible.
//
// Mapping as in the SpMM: a group of G lanes owns a row, lane t owns columns 4*(t + G*j); rows
// longer than SPMM_LONG_ROW edges are walked in the partition's chunks by whole workgroups.
#include "common.h"

namespace grp {

constexpr float GAT_SLOPE = 0.2f;

__device__ __forceinline__ float leaky(float x) { return x > 0.f ? x : GAT_SLOPE * x; }
__device__ __forceinline__ float leaky_d(float x) { return x > 0.f ? 1.f : GAT_SLOPE; }

template <int G>
__device__ __forceinline__ float group_sum(float x) {
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) x += __shfl_xor(x, o, G);
    return x;
}
template <int G>
__device__ __forceinline__ float group_max(float x) {
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, G));
    return x;
}
__device__ __forceinline__ float dot4(const float4& a, const float4& b) {
    return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
}
__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }

// pq[v] = (p_v, q_v) from the two score columns of T_ext (compact copy: stays in L2).
__global__ __launch_bounds__(256) void gat_extract_pq_kernel(const float* __restrict__ Tx, int64_t ldx, int col_p, int64_t n,
                                                             float2* __restrict__ pq) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < n) pq[v] = make_float2(Tx[v * ldx + col_p], Tx[v * ldx + col_p + 1]);
}

// Row statistics of the attention softmax: rowstat[v] = (m_v, Z_v) = (max_u e_uv, sum_u exp(e_uv - m_v)),
// self term included.  Scalars only (p and q sit in L2).  The first n_long workgroups each take one
// row longer than long_thr edges with all 256 threads (partial results combined through LDS in a
// fixed order); the others give 16 lanes to a row and skip the long ones.
__global__ __launch_bounds__(256) void gat_stats_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx,
                                                        int64_t n, const float2* __restrict__ pq,
                                                        float2* __restrict__ rowstat, const int32_t* __restrict__ long_row,
                                                        int n_long, int64_t long_thr) {
    constexpr int G = 16;
    if ((int)blockIdx.x < n_long) {
        __shared__ float red[4];
        const int64_t v = long_row[blockIdx.x];
        const int64_t b = ptr[v], e = ptr[v + 1];
        const float2 pqv = pq[v];
        const float es = leaky(pqv.x + pqv.y);
        const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
        auto score = [&](int64_t k) { return k < e ? leaky(pq[idx[k]].x + pqv.y) : -INFINITY; };
        float mx = es;
        for (int64_t k = b + tid; k < e; k += 4 * 256) {
            const float s0 = score(k), s1 = score(k + 256), s2 = score(k + 512), s3 = score(k + 768);
            mx = fmaxf(fmaxf(mx, fmaxf(s0, s1)), fmaxf(s2, s3));
        }
        mx = group_max<64>(mx);
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        __syncthreads();
        float sum = 0.f;
        for (int64_t k = b + tid; k < e; k += 4 * 256) {
            const float s0 = score(k), s1 = score(k + 256), s2 = score(k + 512), s3 = score(k + 768);
            sum += __expf(s0 - mx); sum += __expf(s1 - mx); sum += __expf(s2 - mx); sum += __expf(s3 - mx);
        }
        sum = group_sum<64>(sum);
        if (lane == 0) red[wave] = sum;
        __syncthreads();
        if (tid == 0) rowstat[v] = make_float2(mx, ((red[0] + red[1]) + (red[2] + red[3])) + __expf(es - mx));
        return;
    }
    const int t = threadIdx.x % G;
    const int64_t v = ((int64_t)blockIdx.x - n_long) * (256 / G) + threadIdx.x / G;
    if (v >= n) return;               // whole groups leave together
    const int64_t b = ptr[v], e = ptr[v + 1];
    if (e - b > long_thr) return;     // done by one of the first workgroups
    const float2 pqv = pq[v];
    const float es = leaky(pqv.x + pqv.y);
    // four independent index -> score gathers per lane and trip
    auto score = [&](int64_t k) { return k < e ? leaky(pq[idx[k]].x + pqv.y) : -INFINITY; };
    float mx = es;
    for (int64_t k = b + t; k < e; k += 4 * G) {
        const float s0 = score(k), s1 = score(k + G), s2 = score(k + 2 * G), s3 = score(k + 3 * G);
        mx = fmaxf(fmaxf(mx, fmaxf(s0, s1)), fmaxf(s2, s3));
    }
    mx = group_max<G>(mx);
    float sum = 0.f;
    for (int64_t k = b + t; k < e; k += 4 * G) {
        const float s0 = score(k), s1 = score(k + G), s2 = score(k + 2 * G), s3 = score(k + 3 * G);
        sum += __expf(s0 - mx); sum += __expf(s1 - mx); sum += __expf(s2 - mx); sum += __expf(s3 - mx);
    }
    sum = group_sum<G>(sum) + __expf(es - mx);
    if (t == 0) rowstat[v] = make_float2(mx, sum);
}

// The three edge walks share one skeleton.  A walk visits the edges of a row (of the CSR for
// FWD and DST, of the CSC for SRC) and accumulates a feature row `acc` and a scalar `scal`:
//   FWD  acc += alpha_uv T[u,:]                                           (row v, edges u -> v)
//   DST  scal += alpha_uv (dOut_v . T[u,:] - c_v) LeakyReLU'(pre_uv)      (row v; acc unused)
//   SRC  acc += alpha_uv dOut[v,:];  scal += alpha_uv (T_u . dOut[v,:] - c_v) LeakyReLU'(pre_uv)   (row u, edges u -> v)
// Short rows are walked by one group of G lanes.  Rows longer than `long_thr` edges use the
// partition's split schedule: the first workgroups of the launch each walk one chunk (their
// 256/G groups take contiguous slices, summed through LDS in a fixed order) into a partial
// row; a second kernel adds a row's partials in chunk order and finishes it.
enum { GAT_FWD = 0, GAT_DST = 1, GAT_SRC = 2 };

struct GatWalk {
    const int64_t* ptr;
    const int32_t* idx;
    int64_t n;
    int F;
    const float* Tx;  int64_t ldx;
    const float2* pq;
    const float2* rowstat;
    const float* bias;
    int relu;
    float* Hout;      int64_t ldh;       // FWD: output; DST: the layer's stored output
    float hout_scale;                    // DST: out_v = hout_scale * Hout[v,:] where dOut is non-zero (undoes dropout)
    const float* dOut; int64_t ldd;
    float* cvec;                         // DST: written; SRC: read
    float2* dqs;                         // DST: written (dq, self-term score gradient); SRC: read
    float* dTx;                          // SRC: output rows [dT | 0 | dp | dq | 0 0]
    int64_t long_thr;
    int n_chunks;
    const int64_t* chunk_begin;
    const int64_t* chunk_end;
    float* partials;  int64_t ld_part;   // [n_chunks x ld_part]: F columns, the scalar at column ld(F)
};

template <int G, int NJ>
struct GatRow {                          // per-row constants held by every lane of the group
    float4 vec[NJ];                      // DST: dOut[v,:]; SRC: T[u,:]
    float q, mx, inv, c, p;
};

template <int PASS, int G, int NJ>
__device__ __forceinline__ void gat_row_setup(const GatWalk& A, int64_t r, int t, const bool (&live)[NJ], GatRow<G, NJ>& R,
                                              float& dself) {
    const float2 pqr = A.pq[r];
    R.p = pqr.x; R.q = pqr.y;
    R.mx = 0.f; R.inv = 0.f; R.c = 0.f;
    if (PASS != GAT_SRC) {
        const float2 st = A.rowstat[r];
        R.mx = st.x; R.inv = 1.f / st.y;
    }
    dself = 0.f;
    if (PASS == GAT_DST) {
        float cpart = 0.f, spart = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            R.vec[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (!live[j]) continue;
            const int col = 4 * (t + G * j);
            R.vec[j] = ld4(A.dOut + r * A.ldd + col);
            const float4 h = ld4(A.Hout + r * A.ldh + col);
            float bb[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) bb[q] = col + q < A.F ? A.bias[col + q] : 0.f;
            const float hs = A.hout_scale;
            cpart += R.vec[j].x * (h.x * hs - bb[0]) + R.vec[j].y * (h.y * hs - bb[1]) + R.vec[j].z * (h.z * hs - bb[2]) +
                     R.vec[j].w * (h.w * hs - bb[3]);
            spart += dot4(R.vec[j], ld4(A.Tx + r * A.ldx + col));
        }
        R.c = group_sum<G>(cpart);        // c_v = dOut_v . (out_v - b) = sum_u alpha_uv (dOut_v . t_u)
        dself = group_sum<G>(spart);      // dOut_v . t_v
    }
    if (PASS == GAT_SRC) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            R.vec[j] = live[j] ? ld4(A.Tx + r * A.ldx + 4 * (t + G * j)) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

template <int PASS, int G, int NJ>
__device__ __forceinline__ void gat_walk_edges(const GatWalk& A, const GatRow<G, NJ>& R, int64_t b, int64_t e, int t,
                                               const bool (&live)[NJ], float4 (&acc)[NJ], float& scal) {
    for (int64_t base = b; base < e; base += G) {
        const int cnt = (int)(e - base < G ? e - base : G);
        int mine = 0;
        float mya = 0.f, mw = 0.f, mc = R.c;              // alpha, alpha * LeakyReLU', c of the edge's destination
        if (t < cnt) {
            mine = A.idx[base + t];
            float pre, mx, inv;
            if (PASS == GAT_SRC) {
                const float2 sv = A.rowstat[mine];
                pre = R.p + A.pq[mine].y; mx = sv.x; inv = 1.f / sv.y;
                mc = A.cvec[mine];
            } else {
                pre = A.pq[mine].x + R.q; mx = R.mx; inv = R.inv;
            }
            mya = __expf(leaky(pre) - mx) * inv;
            mw = mya * leaky_d(pre);
        }
        for (int k = 0; k < cnt; k += 4) {
            const bool p1 = k + 1 < cnt, p2 = k + 2 < cnt, p3 = k + 3 < cnt;
            const int k1 = p1 ? k + 1 : k, k2 = p2 ? k + 2 : k, k3 = p3 ? k + 3 : k;
            const int64_t c0 = __shfl(mine, k, G), c1 = __shfl(mine, k1, G), c2 = __shfl(mine, k2, G), c3 = __shfl(mine, k3, G);
            const float a0 = __shfl(mya, k, G), a1 = p1 ? __shfl(mya, k1, G) : 0.f;
            const float a2 = p2 ? __shfl(mya, k2, G) : 0.f, a3 = p3 ? __shfl(mya, k3, G) : 0.f;
            float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
            const float* base_ptr = PASS == GAT_SRC ? A.dOut : A.Tx;
            const int64_t ld = PASS == GAT_SRC ? A.ldd : A.ldx;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (!live[j]) continue;
                const int col = 4 * (t + G * j);
                const float4 v0 = ld4(base_ptr + c0 * ld + col), v1 = ld4(base_ptr + c1 * ld + col);
                const float4 v2 = ld4(base_ptr + c2 * ld + col), v3 = ld4(base_ptr + c3 * ld + col);
                if (PASS != GAT_DST) {
                    acc[j].x += a0 * v0.x; acc[j].y += a0 * v0.y; acc[j].z += a0 * v0.z; acc[j].w += a0 * v0.w;
                    acc[j].x += a1 * v1.x; acc[j].y += a1 * v1.y; acc[j].z += a1 * v1.z; acc[j].w += a1 * v1.w;
                    acc[j].x += a2 * v2.x; acc[j].y += a2 * v2.y; acc[j].z += a2 * v2.z; acc[j].w += a2 * v2.w;
                    acc[j].x += a3 * v3.x; acc[j].y += a3 * v3.y; acc[j].z += a3 * v3.z; acc[j].w += a3 * v3.w;
                }
                if (PASS != GAT_FWD) {
                    d0 += dot4(R.vec[j], v0); d1 += dot4(R.vec[j], v1); d2 += dot4(R.vec[j], v2); d3 += dot4(R.vec[j], v3);
                }
            }
            if (PASS != GAT_FWD) {
                d0 = group_sum<G>(d0); d1 = group_sum<G>(d1); d2 = group_sum<G>(d2); d3 = group_sum<G>(d3);
                scal += __shfl(mw, k, G) * (d0 - __shfl(mc, k, G));
                const float w1 = __shfl(mw, k1, G), w2 = __shfl(mw, k2, G), w3 = __shfl(mw, k3, G);
                const float e1 = __shfl(mc, k1, G), e2 = __shfl(mc, k2, G), e3 = __shfl(mc, k3, G);
                if (p1) scal += w1 * (d1 - e1);
                if (p2) scal += w2 * (d2 - e2);
                if (p3) scal += w3 * (d3 - e3);
            }
        }
    }
}

// Adds the self term and writes the row's results.
template <int PASS, int G, int NJ>
__device__ __forceinline__ void gat_row_finish(const GatWalk& A, const GatRow<G, NJ>& R, int64_t r, int t,
                                               const bool (&live)[NJ], float4 (&acc)[NJ], float scal, float dself) {
    if (PASS == GAT_FWD) {
        const float as = __expf(leaky(R.p + R.q) - R.mx) * R.inv;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (!live[j]) continue;
            const int col = 4 * (t + G * j);
            const float4 tv = ld4(A.Tx + r * A.ldx + col);
            float o[4] = {acc[j].x + as * tv.x, acc[j].y + as * tv.y, acc[j].z + as * tv.z, acc[j].w + as * tv.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (col + q < A.F) {
                    o[q] += A.bias[col + q];
                    if (A.relu) o[q] = o[q] > 0.f ? o[q] : 0.f;
                } else {
                    o[q] = 0.f;       // pad columns stay zero
                }
            }
            *reinterpret_cast<float4*>(A.Hout + r * A.ldh + col) = make_float4(o[0], o[1], o[2], o[3]);
        }
    } else if (PASS == GAT_DST) {
        const float pre_s = R.p + R.q;
        const float ds_self = __expf(leaky(pre_s) - R.mx) * R.inv * (dself - R.c) * leaky_d(pre_s);
        if (t == 0) {
            A.cvec[r] = R.c;
            A.dqs[r] = make_float2(scal + ds_self, ds_self);
        }
    } else {
        const float2 st = A.rowstat[r], dq = A.dqs[r];
        const float as = __expf(leaky(R.p + R.q) - st.x) / st.y;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (!live[j]) continue;
            const int col = 4 * (t + G * j);
            const float4 d = ld4(A.dOut + r * A.ldd + col);
            float o[4] = {acc[j].x + as * d.x, acc[j].y + as * d.y, acc[j].z + as * d.z, acc[j].w + as * d.w};
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (col + q >= A.F) o[q] = 0.f;
            *reinterpret_cast<float4*>(A.dTx + r * A.ldx + col) = make_float4(o[0], o[1], o[2], o[3]);
        }
        if (t == 0)
            *reinterpret_cast<float4*>(A.dTx + r * A.ldx + ((A.F + 3) & ~3)) = make_float4(scal + dq.y, dq.x, 0.f, 0.f);
    }
}

template <int PASS, int G, int NJ>
__global__ __launch_bounds__(256) void gat_walk_kernel(GatWalk A) {
    constexpr int ROWS = 256 / G;
    constexpr int W = 4 * G * NJ;                 // padded row width held by a group
    __shared__ __attribute__((aligned(16))) float red[ROWS * (W + 4)];
    __shared__ int64_t chunk_row;
    const int t = threadIdx.x % G, gi = threadIdx.x / G;
    bool live[NJ];
    float4 acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        live[j] = 4 * (t + G * j) < A.F;
        acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    GatRow<G, NJ> R;
    float scal = 0.f, dself = 0.f;
    if ((int)blockIdx.x < A.n_chunks) {           // uniform per workgroup: one chunk of a long row
        const int64_t cb = A.chunk_begin[blockIdx.x], ce = A.chunk_end[blockIdx.x];
        if (threadIdx.x == 0) {                   // the row that owns edge cb: last r with ptr[r] <= cb
            int64_t lo = 0, hi = A.n;
            while (hi - lo > 1) {
                const int64_t mid = (lo + hi) >> 1;
                if (A.ptr[mid] <= cb) lo = mid; else hi = mid;
            }
            chunk_row = lo;
        }
        __syncthreads();
        const int64_t r = chunk_row;
        gat_row_setup<PASS, G, NJ>(A, r, t, live, R, dself);
        const int64_t per = (ce - cb + ROWS - 1) / ROWS;
        int64_t b = cb + gi * per, e = b + per;
        if (b > ce) b = ce;
        if (e > ce) e = ce;
        gat_walk_edges<PASS, G, NJ>(A, R, b, e, t, live, acc, scal);
#pragma unroll
        for (int j = 0; j < NJ; ++j) *reinterpret_cast<float4*>(&red[gi * (W + 4) + 4 * (t + G * j)]) = acc[j];
        if (t == 0) red[gi * (W + 4) + W] = scal;
        __syncthreads();
        float* prow = A.partials + (int64_t)blockIdx.x * A.ld_part;
        const int fpad = (A.F + 3) & ~3;
        for (int c = threadIdx.x; c <= fpad; c += 256) {
            const int cc = c < fpad ? c : W;      // the last one is the scalar
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < ROWS; ++q) s += red[q * (W + 4) + cc];
            prow[c] = s;
        }
        return;
    }
    const int64_t r = (int64_t)(blockIdx.x - A.n_chunks) * ROWS + gi;
    if (r >= A.n) return;                         // whole groups leave together
    const int64_t b = A.ptr[r], e = A.ptr[r + 1];
    if (e - b > A.long_thr) return;               // walked in chunks above, finished by the combine kernel
    gat_row_setup<PASS, G, NJ>(A, r, t, live, R, dself);
    gat_walk_edges<PASS, G, NJ>(A, R, b, e, t, live, acc, scal);
    gat_row_finish<PASS, G, NJ>(A, R, r, t, live, acc, scal, dself);
}

template <int PASS, int G, int NJ>
__global__ __launch_bounds__(256) void gat_combine_kernel(GatWalk A, const int32_t* __restrict__ long_row,
                                                          const int32_t* __restrict__ long_first, int n_long) {
    constexpr int ROWS = 256 / G;
    const int t = threadIdx.x % G;
    const int j0 = blockIdx.x * ROWS + threadIdx.x / G;
    if (j0 >= n_long) return;
    const int64_t r = long_row[j0];
    const int c0 = long_first[j0], c1 = long_first[j0 + 1];
    bool live[NJ];
    float4 acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        live[j] = 4 * (t + G * j) < A.F;
        acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    GatRow<G, NJ> R;
    float scal = 0.f, dself = 0.f;
    gat_row_setup<PASS, G, NJ>(A, r, t, live, R, dself);
    const int fpad = (A.F + 3) & ~3;
    for (int c = c0; c < c1; ++c) {
        const float* prow = A.partials + (int64_t)c * A.ld_part;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (!live[j]) continue;
            const float4 v = ld4(prow + 4 * (t + G * j));
            acc[j].x += v.x; acc[j].y += v.y; acc[j].z += v.z; acc[j].w += v.w;
        }
        scal += prow[fpad];
    }
    gat_row_finish<PASS, G, NJ>(A, R, r, t, live, acc, scal, dself);
}

// Packed weights of one layer: Wp[Fin x ldx] = wp_scale [W | 0 | W a_src | W a_dst | 0 0] (rows of the
// product dT_ext -> dH; wp_scale = 1 / (1 - rate) when the layer's input went through dropout) and the
// unscaled transpose Wt[ldx x ld(Fin)] (rows of the product H -> T_ext).
__global__ __launch_bounds__(256) void gat_pack_kernel(const float* __restrict__ W, const float* __restrict__ a_s,
                                                       const float* __restrict__ a_d, int fin, int fout, int fin_pad, int ldx,
                                                       float wp_scale, float* __restrict__ Wp, float* __restrict__ Wt) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)fin_pad * ldx) return;
    const int i = (int)(e / ldx), c = (int)(e % ldx);
    const int cp = (fout + 3) & ~3;
    float val = 0.f;
    if (i < fin) {
        if (c < fout) {
            val = W[(int64_t)i * fout + c];
        } else if (c == cp || c == cp + 1) {
            const float* a = c == cp ? a_s : a_d;
            for (int j = 0; j < fout; ++j) val = fmaf(W[(int64_t)i * fout + j], a[j], val);
        }
        Wp[(int64_t)i * ldx + c] = val * wp_scale;
    }
    Wt[(int64_t)c * fin_pad + i] = val;
}

// Gradients of W, a_src, a_dst from dWx = H^T dT_ext [Fin x ldx]:
//   dW = dWx[:, :F] + dWx[:, cp] a_src^T + dWx[:, cp+1] a_dst^T,  da_src = W^T dWx[:, cp],  da_dst = W^T dWx[:, cp+1].
__global__ __launch_bounds__(256) void gat_param_grad_kernel(const float* __restrict__ dWx, int ldx, const float* __restrict__ W,
                                                             const float* __restrict__ a_s, const float* __restrict__ a_d,
                                                             int fin, int fout, float* __restrict__ gW,
                                                             float* __restrict__ ga_s, float* __restrict__ ga_d) {
    // workgroup j < fout: column j of dW and the two attention-vector gradients of index j
    __shared__ float sm[8];
    const int cp = (fout + 3) & ~3;
    const int j = blockIdx.x;
    float s = 0.f, d = 0.f;
    const float asj = a_s[j], adj = a_d[j];
    for (int i = threadIdx.x; i < fin; i += 256) {
        const float ds = dWx[(int64_t)i * ldx + cp], dd = dWx[(int64_t)i * ldx + cp + 1];
        const float w = W[(int64_t)i * fout + j];
        gW[(int64_t)i * fout + j] = dWx[(int64_t)i * ldx + j] + ds * asj + dd * adj;
        s = fmaf(w, ds, s);
        d = fmaf(w, dd, d);
    }
    for (int o = 32; o > 0; o >>= 1) { s += __shfl_down(s, o, 64); d += __shfl_down(d, o, 64); }
    if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = s; sm[4 + (threadIdx.x >> 6)] = d; }
    __syncthreads();
    if (threadIdx.x == 0) {
        ga_s[j] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
        ga_d[j] = (sm[4] + sm[5]) + (sm[6] + sm[7]);
    }
}

// ------------------------------------------------------------------ launchers
struct GatLayer {
    int fin, fout;
    int64_t ldx, ldh, ldin_pad;      // ld(Fout) + 4; ld(Fout); ld(Fin)
    int64_t off_w, off_as, off_ad, off_b;
    float *Wp, *Wt, *Tx, *Hout;
    float2 *pq, *rowstat;
};

struct GatPlan {
    std::vector<GatLayer> L;
    float *dZa, *dZb, *dTx, *cvec, *dWx, *partials;
    float2* dqs;
    void *tn_ws, *colsum_ws, *stats_ws;
    size_t tn_ws_bytes, total;
};

static inline int64_t ldp4(int64_t f) { return round_up(f, 4); }

static GatPlan gat_plan(const grp_partition_t* part, const grp_model_desc* m, void* ws, size_t ws_bytes) {
    GatPlan p;
    Bump b(ws, ws_bytes);
    const int64_t n = part->n;
    const int k = m->n_layers;
    p.L.resize(k);
    int64_t off = 0, ldmax = 4, ldxmax = 8, wxmax = 1;
    size_t tn_bytes = 0, cs_bytes = 0;
    for (int l = 0; l < k; ++l) {
        GatLayer& L = p.L[l];
        L.fin = m->dims[l]; L.fout = m->dims[l + 1];
        L.ldh = ldp4(L.fout); L.ldx = L.ldh + 4; L.ldin_pad = ldp4(L.fin);
        L.off_w = off; off += (int64_t)L.fin * L.fout;
        L.off_as = off; off += L.fout;
        L.off_ad = off; off += L.fout;
        L.off_b = off; off += L.fout;
        L.Wp = b.take<float>((size_t)L.ldin_pad * L.ldx);
        L.Wt = b.take<float>((size_t)L.ldx * L.ldin_pad);
        L.Tx = b.take<float>((size_t)n * L.ldx);
        L.Hout = b.take<float>((size_t)n * L.ldh);
        L.pq = b.take<float2>((size_t)n);
        L.rowstat = b.take<float2>((size_t)n);
        if (L.ldh > ldmax) ldmax = L.ldh;
        if (L.ldx > ldxmax) ldxmax = L.ldx;
        if ((int64_t)L.fin * L.ldx > wxmax) wxmax = (int64_t)L.fin * L.ldx;
        const size_t t = gemm_tn_workspace_bytes(n, L.fin, (int32_t)L.ldx);
        if (t > tn_bytes) tn_bytes = t;
        const size_t c = colsum_workspace_bytes(n, L.fout);
        if (c > cs_bytes) cs_bytes = c;
    }
    p.dZa = b.take<float>((size_t)n * ldmax);
    p.dZb = b.take<float>((size_t)n * ldmax);
    p.dTx = b.take<float>((size_t)n * ldxmax);
    p.cvec = b.take<float>((size_t)n);
    p.dqs = b.take<float2>((size_t)n);
    p.dWx = b.take<float>((size_t)wxmax);
    const int64_t chunks_cap = part->csr_long.n_chunks > part->csc_long.n_chunks ? part->csr_long.n_chunks : part->csc_long.n_chunks;
    p.partials = b.take<float>((size_t)chunks_cap * ldxmax);
    p.tn_ws = b.take<char>(tn_bytes);
    p.tn_ws_bytes = tn_bytes;
    p.colsum_ws = b.take<char>(cs_bytes);
    p.stats_ws = b.take<char>(stats_workspace_bytes(n));
    p.total = b.total();
    return p;
}

size_t gat_step_workspace_bytes(const grp_partition_t* part, const grp_model_desc* m) {
    return gat_plan(part, m, nullptr, 0).total;
}

void gat_step_activation(const grp_partition_t* part, const grp_model_desc* m, void* ws, size_t ws_bytes, int layer,
                         const float** out, int64_t* ld) {
    const GatPlan p = gat_plan(part, m, ws, ws_bytes);
    *out = p.L[layer].Hout;
    *ld = p.L[layer].ldh;
}

template <int PASS, int G, int NJ>
static void gat_walk_one(const GatWalk& A, const LongRows* lr, hipStream_t st) {
    constexpr int ROWS = 256 / G;
    hipLaunchKernelGGL((gat_walk_kernel<PASS, G, NJ>), dim3((unsigned)(A.n_chunks + cdiv(A.n, ROWS))), dim3(256), 0, st, A);
    if (A.n_chunks > 0)
        hipLaunchKernelGGL((gat_combine_kernel<PASS, G, NJ>), dim3((unsigned)cdiv(lr->n_long, ROWS)), dim3(256), 0, st, A,
                           (const int32_t*)lr->long_row, (const int32_t*)lr->long_first, lr->n_long);
}

template <int PASS>
static grp_status launch_gat_walk(GatWalk A, const LongRows* lr, float* partials, hipStream_t st) {
    const bool split = lr && lr->n_long > 0;
    A.long_thr = split ? (int64_t)SPMM_LONG_ROW : INT64_MAX;
    A.n_chunks = split ? lr->n_chunks : 0;
    A.chunk_begin = split ? lr->chunk_begin : nullptr;
    A.chunk_end = split ? lr->chunk_end : nullptr;
    A.partials = partials;
    A.ld_part = round_up(A.F, 4) + 4;
    const int f4 = (A.F + 3) / 4;
    if (f4 <= 1) gat_walk_one<PASS, 1, 1>(A, lr, st);
    else if (f4 <= 2) gat_walk_one<PASS, 2, 1>(A, lr, st);
    else if (f4 <= 4) gat_walk_one<PASS, 4, 1>(A, lr, st);
    else if (f4 <= 8) gat_walk_one<PASS, 8, 1>(A, lr, st);
    else if (f4 <= 16) gat_walk_one<PASS, 16, 1>(A, lr, st);
    else if (f4 <= 32) gat_walk_one<PASS, 32, 1>(A, lr, st);
    else if (f4 <= 64) gat_walk_one<PASS, 64, 1>(A, lr, st);
    else if (f4 <= 128) gat_walk_one<PASS, 64, 2>(A, lr, st);
    else gat_walk_one<PASS, 64, 4>(A, lr, st);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

grp_status gat_step(const grp_partition_t* g, const grp_model_desc* m, const grp_step_opts* o, const void* X,
                    const int32_t* labels, const uint8_t* mask, const float* theta, void* ws, size_t ws_bytes,
                    hipStream_t st, float* grad, grp_step_stats* stats) {
    GatPlan p = gat_plan(g, m, ws, ws_bytes);
    const int64_t n = g->n;
    const int k = m->n_layers;
    GRP_TRY(launch_stats(n, nullptr, mask, g->d_local_in, g->d_global_in, nullptr, g->nnz, nullptr, 0, p.stats_ws, stats, st));
    if (n == 0) {                                       // nothing to train on: zero gradient
        int64_t P = 0;
        for (int l = 0; l < k; ++l) P += (int64_t)m->dims[l] * m->dims[l + 1] + 3 * m->dims[l + 1];
        GRP_TRY(launch_fill_zero(grad, (size_t)P * sizeof(float), st));      // a kernel, so the step can be captured in a graph
        return launch_softmax_xent(0, m->dims[k], nullptr, 4, labels, nullptr, mask, o->estimator == GRP_EST_NODE_LEVEL,
                                   g->d_local_in, g->d_global_in, nullptr, p.dZa, 4, p.stats_ws, stats, st);
    }
    const DropoutPlan drop = dropout_plan(o);
    // ---------------- packed weights
    for (int l = 0; l < k; ++l) {
        const GatLayer& L = p.L[l];
        ProfScope ps("gat_pack_weights", st);
        hipLaunchKernelGGL(gat_pack_kernel, dim3((unsigned)cdiv((int64_t)L.ldin_pad * L.ldx, 256)), dim3(256), 0, st,
                           theta + L.off_w, theta + L.off_as, theta + L.off_ad, L.fin, L.fout, (int)L.ldin_pad, (int)L.ldx,
                           l > 0 ? drop.scale : 1.f, L.Wp, L.Wt);
        GRP_LAUNCH_CHECK();
    }
    // ---------------- forward
    const void* H = X;
    int64_t ldh = m->dims[0];
    int h_bf16 = m->feat_dtype == GRP_DTYPE_BF16;
    for (int l = 0; l < k; ++l) {
        const GatLayer& L = p.L[l];
        GemmNNArgs a;          // T_ext = H [W | 0 | W a_src | W a_dst | 0 0]
        a.M = n; a.N = (int)L.ldx; a.K = L.fin; a.A = H; a.lda = ldh; a.a_bf16 = h_bf16; a.Bt = L.Wt; a.ldbt = L.ldin_pad;
        a.C = L.Tx; a.ldc = L.ldx;
        GRP_TRY(launch_gemm_nn(a, st));
        {
            ProfScope ps("gat_forward", st, 2.0 * g->nnz * L.fout, 4.0 * g->nnz + 8.0 * L.fout * n);
            hipLaunchKernelGGL(gat_extract_pq_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, L.Tx, L.ldx, (int)L.ldh, n, L.pq);
            hipLaunchKernelGGL(gat_stats_kernel, dim3((unsigned)(cdiv(n, 16) + g->csr_long.n_long)), dim3(256), 0, st,
                               g->rowptr, g->col, n, (const float2*)L.pq, L.rowstat, g->csr_long.long_row,
                               g->csr_long.n_long, (int64_t)SPMM_LONG_ROW);
            GRP_LAUNCH_CHECK();
            GatWalk A{};
            A.ptr = g->rowptr; A.idx = g->col; A.n = n; A.F = L.fout; A.Tx = L.Tx; A.ldx = L.ldx; A.pq = L.pq;
            A.rowstat = L.rowstat; A.bias = theta + L.off_b; A.relu = l < k - 1 ? 1 : 0; A.Hout = L.Hout; A.ldh = L.ldh;
            GRP_TRY(launch_gat_walk<GAT_FWD>(A, &g->csr_long, p.partials, st));
        }
        if (l < k - 1) GRP_TRY(launch_dropout(drop, l, g->l2g, n, L.fout, L.Hout, L.ldh, nullptr, 0, nullptr, 0, st));
        H = L.Hout; ldh = L.ldh; h_bf16 = 0;
    }
    // ---------------- loss
    const int C = m->dims[k];
    float* dZ = p.dZa;
    float* dZ_other = p.dZb;
    GRP_TRY(launch_softmax_xent(n, C, p.L[k - 1].Hout, ldp4(C), labels, nullptr, mask, o->estimator == GRP_EST_NODE_LEVEL,
                                g->d_local_in, g->d_global_in, nullptr, dZ, ldp4(C), p.stats_ws, stats, st));
    // ---------------- backward
    for (int l = k - 1; l >= 0; --l) {
        const GatLayer& L = p.L[l];
        const void* Hin = l == 0 ? X : (const void*)p.L[l - 1].Hout;
        const int64_t ldin = l == 0 ? m->dims[0] : p.L[l - 1].ldh;
        const int in_bf16 = l == 0 && m->feat_dtype == GRP_DTYPE_BF16;
        GRP_TRY(launch_colsum(dZ, n, L.fout, L.ldh, grad + L.off_b, p.colsum_ws, st));
        {
            ProfScope ps("gat_backward", st, 6.0 * g->nnz * L.fout, 8.0 * g->nnz + 16.0 * L.fout * n);
            GatWalk A{};
            A.ptr = g->rowptr; A.idx = g->col; A.n = n; A.F = L.fout; A.Tx = L.Tx; A.ldx = L.ldx; A.pq = L.pq;
            A.rowstat = L.rowstat; A.bias = theta + L.off_b; A.Hout = L.Hout; A.ldh = L.ldh; A.dOut = dZ; A.ldd = L.ldh;
            A.cvec = p.cvec; A.dqs = p.dqs; A.dTx = p.dTx;
            A.hout_scale = (drop.on && l < k - 1) ? 1.0f - o->dropout_rate : 1.f;
            GRP_TRY(launch_gat_walk<GAT_DST>(A, &g->csr_long, p.partials, st));
            A.ptr = g->colptr; A.idx = g->row;
            GRP_TRY(launch_gat_walk<GAT_SRC>(A, &g->csc_long, p.partials, st));
        }
        GemmTNArgs t;          // dW_ext = H_in^T dT_ext
        t.M = n; t.K = L.fin; t.N = (int)L.ldx; t.A = Hin; t.lda = ldin; t.a_bf16 = in_bf16; t.B = p.dTx; t.ldb = L.ldx;
        t.C = p.dWx; t.ldc = L.ldx; t.workspace = p.tn_ws; t.workspace_bytes = p.tn_ws_bytes;
        GRP_TRY(launch_gemm_tn(t, st));
        {
            ProfScope ps("gat_param_grad", st);
            hipLaunchKernelGGL(gat_param_grad_kernel, dim3((unsigned)L.fout), dim3(256), 0, st, (const float*)p.dWx,
                               (int)L.ldx, theta + L.off_w, theta + L.off_as, theta + L.off_ad, L.fin, L.fout,
                               grad + L.off_w, grad + L.off_as, grad + L.off_ad);
            GRP_LAUNCH_CHECK();
        }
        if (l > 0) {
            GemmNNArgs c;      // dZ_prev = (H_in > 0) * (dT_ext W_ext^T)
            c.M = n; c.N = L.fin; c.K = (int)L.ldx; c.A = p.dTx; c.lda = L.ldx; c.Bt = L.Wp; c.ldbt = L.ldx;
            c.mask = p.L[l - 1].Hout; c.ld_mask = p.L[l - 1].ldh;
            c.C = dZ_other; c.ldc = p.L[l - 1].ldh; c.zero_pad_to = (int)p.L[l - 1].ldh;
            GRP_TRY(launch_gemm_nn(c, st));
        }
        float* sw = dZ; dZ = dZ_other; dZ_other = sw;
    }
    return GRP_OK;
}

}  // namespace grp
