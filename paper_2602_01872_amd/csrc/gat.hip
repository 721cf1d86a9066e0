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
// Mapping as in the SpMM: a group of G lanes owns a row, lane t owns columns 4*(t + G*j).
// Rows of any length are walked by their group (no long-row splitting here).
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

// Forward: row statistics (m_v, Z_v) and H_out[v,:] = act(sum_u alpha_uv T[u,:] + b).
template <int G, int NJ>
__global__ __launch_bounds__(256) void gat_forward_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx,
                                                          int64_t n, int F, const float* __restrict__ Tx, int64_t ldx,
                                                          const float2* __restrict__ pq, const float* __restrict__ bias,
                                                          int relu, float* __restrict__ Hout, int64_t ldh,
                                                          float2* __restrict__ rowstat) {
    constexpr int ROWS = 256 / G;
    const int t = threadIdx.x % G;
    const int64_t v = (int64_t)blockIdx.x * ROWS + threadIdx.x / G;
    if (v >= n) return;               // whole groups leave together
    const int64_t b = ptr[v], e = ptr[v + 1];
    const float2 pqv = pq[v];
    const float es = leaky(pqv.x + pqv.y);
    float mx = es;
    for (int64_t k = b + t; k < e; k += G) mx = fmaxf(mx, leaky(pq[idx[k]].x + pqv.y));
    mx = group_max<G>(mx);
    float sum = 0.f;
    for (int64_t k = b + t; k < e; k += G) sum += __expf(leaky(pq[idx[k]].x + pqv.y) - mx);
    sum = group_sum<G>(sum) + __expf(es - mx);
    const float inv = 1.f / sum;
    if (t == 0) rowstat[v] = make_float2(mx, sum);

    float4 acc[NJ];
    bool live[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        live[j] = 4 * (t + G * j) < F;
    }
    for (int64_t base = b; base < e; base += G) {
        const int cnt = (int)(e - base < G ? e - base : G);
        int mine = 0;
        float mya = 0.f;
        if (t < cnt) {
            mine = idx[base + t];
            mya = __expf(leaky(pq[mine].x + pqv.y) - mx) * inv;
        }
        for (int k = 0; k < cnt; k += 4) {
            const bool p1 = k + 1 < cnt, p2 = k + 2 < cnt, p3 = k + 3 < cnt;
            const int64_t c0 = __shfl(mine, k, G), c1 = __shfl(mine, p1 ? k + 1 : k, G);
            const int64_t c2 = __shfl(mine, p2 ? k + 2 : k, G), c3 = __shfl(mine, p3 ? k + 3 : k, G);
            const float a0 = __shfl(mya, k, G), a1 = p1 ? __shfl(mya, k + 1, G) : 0.f;
            const float a2 = p2 ? __shfl(mya, k + 2, G) : 0.f, a3 = p3 ? __shfl(mya, k + 3, G) : 0.f;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (!live[j]) continue;
                const int col = 4 * (t + G * j);
                const float4 v0 = ld4(Tx + c0 * ldx + col), v1 = ld4(Tx + c1 * ldx + col);
                const float4 v2 = ld4(Tx + c2 * ldx + col), v3 = ld4(Tx + c3 * ldx + col);
                acc[j].x += a0 * v0.x; acc[j].y += a0 * v0.y; acc[j].z += a0 * v0.z; acc[j].w += a0 * v0.w;
                acc[j].x += a1 * v1.x; acc[j].y += a1 * v1.y; acc[j].z += a1 * v1.z; acc[j].w += a1 * v1.w;
                acc[j].x += a2 * v2.x; acc[j].y += a2 * v2.y; acc[j].z += a2 * v2.z; acc[j].w += a2 * v2.w;
                acc[j].x += a3 * v3.x; acc[j].y += a3 * v3.y; acc[j].z += a3 * v3.z; acc[j].w += a3 * v3.w;
            }
        }
    }
    const float as = __expf(es - mx) * inv;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (!live[j]) continue;
        const int col = 4 * (t + G * j);
        const float4 tv = ld4(Tx + v * ldx + col);
        float o[4] = {acc[j].x + as * tv.x, acc[j].y + as * tv.y, acc[j].z + as * tv.z, acc[j].w + as * tv.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (col + q < F) {
                o[q] += bias[col + q];
                if (relu) o[q] = o[q] > 0.f ? o[q] : 0.f;
            } else {
                o[q] = 0.f;       // pad columns stay zero
            }
        }
        *reinterpret_cast<float4*>(Hout + v * ldh + col) = make_float4(o[0], o[1], o[2], o[3]);
    }
}

// Reverse pass over the CSR (row v = a destination): c_v = sum_u alpha_uv dalpha_uv, which equals
// dOut_v . (out_v - b), then dq_v = sum_u de_uv LeakyReLU'(.) with de_uv = alpha_uv (dOut_v . t_u - c_v),
// the self term included; the self term's score gradient is also stored for the source side.
template <int G, int NJ>
__global__ __launch_bounds__(256) void gat_backward_dst_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx,
                                                               int64_t n, int F, const float* __restrict__ Tx, int64_t ldx,
                                                               const float2* __restrict__ pq, const float2* __restrict__ rowstat,
                                                               const float* __restrict__ bias, const float* __restrict__ Hout,
                                                               int64_t ldh, const float* __restrict__ dOut, int64_t ldd,
                                                               float* __restrict__ cvec, float2* __restrict__ dqs) {
    constexpr int ROWS = 256 / G;
    const int t = threadIdx.x % G;
    const int64_t v = (int64_t)blockIdx.x * ROWS + threadIdx.x / G;
    if (v >= n) return;
    const int64_t b = ptr[v], e = ptr[v + 1];
    float4 dO[NJ];
    bool live[NJ];
    float cpart = 0.f, spart = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = 4 * (t + G * j);
        live[j] = col < F;
        dO[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!live[j]) continue;
        dO[j] = ld4(dOut + v * ldd + col);
        const float4 h = ld4(Hout + v * ldh + col);
        float bb[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) bb[q] = col + q < F ? bias[col + q] : 0.f;
        cpart += dO[j].x * (h.x - bb[0]) + dO[j].y * (h.y - bb[1]) + dO[j].z * (h.z - bb[2]) + dO[j].w * (h.w - bb[3]);
        spart += dot4(dO[j], ld4(Tx + v * ldx + col));
    }
    const float c = group_sum<G>(cpart);
    const float dself = group_sum<G>(spart);
    const float2 pqv = pq[v], st = rowstat[v];
    const float inv = 1.f / st.y;
    const float pre_s = pqv.x + pqv.y;
    const float ds_self = __expf(leaky(pre_s) - st.x) * inv * (dself - c) * leaky_d(pre_s);
    float dq = ds_self;
    for (int64_t base = b; base < e; base += G) {
        const int cnt = (int)(e - base < G ? e - base : G);
        int mine = 0;
        float mpre = 0.f;
        if (t < cnt) {
            mine = idx[base + t];
            mpre = pq[mine].x + pqv.y;
        }
        for (int k = 0; k < cnt; k += 4) {
            const bool p1 = k + 1 < cnt, p2 = k + 2 < cnt, p3 = k + 3 < cnt;
            const int64_t c0 = __shfl(mine, k, G), c1 = __shfl(mine, p1 ? k + 1 : k, G);
            const int64_t c2 = __shfl(mine, p2 ? k + 2 : k, G), c3 = __shfl(mine, p3 ? k + 3 : k, G);
            float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (!live[j]) continue;
                const int col = 4 * (t + G * j);
                const float4 v0 = ld4(Tx + c0 * ldx + col), v1 = ld4(Tx + c1 * ldx + col);
                const float4 v2 = ld4(Tx + c2 * ldx + col), v3 = ld4(Tx + c3 * ldx + col);
                d0 += dot4(dO[j], v0); d1 += dot4(dO[j], v1); d2 += dot4(dO[j], v2); d3 += dot4(dO[j], v3);
            }
            d0 = group_sum<G>(d0); d1 = group_sum<G>(d1); d2 = group_sum<G>(d2); d3 = group_sum<G>(d3);
            const float r0 = __shfl(mpre, k, G), r1 = __shfl(mpre, p1 ? k + 1 : k, G);
            const float r2 = __shfl(mpre, p2 ? k + 2 : k, G), r3 = __shfl(mpre, p3 ? k + 3 : k, G);
            dq += __expf(leaky(r0) - st.x) * inv * (d0 - c) * leaky_d(r0);
            if (p1) dq += __expf(leaky(r1) - st.x) * inv * (d1 - c) * leaky_d(r1);
            if (p2) dq += __expf(leaky(r2) - st.x) * inv * (d2 - c) * leaky_d(r2);
            if (p3) dq += __expf(leaky(r3) - st.x) * inv * (d3 - c) * leaky_d(r3);
        }
    }
    if (t == 0) {
        cvec[v] = c;
        dqs[v] = make_float2(dq, ds_self);
    }
}

// Reverse pass over the CSC (row u = a source): dT_u = sum_v alpha_uv dOut_v and
// dp_u = sum_v de_uv LeakyReLU'(.), self terms included; writes the row [dT_u | 0 | dp_u | dq_u | 0 0].
template <int G, int NJ>
__global__ __launch_bounds__(256) void gat_backward_src_kernel(const int64_t* __restrict__ ptrT, const int32_t* __restrict__ idxT,
                                                               int64_t n, int F, const float* __restrict__ Tx, int64_t ldx,
                                                               const float2* __restrict__ pq, const float2* __restrict__ rowstat,
                                                               const float* __restrict__ dOut, int64_t ldd,
                                                               const float* __restrict__ cvec, const float2* __restrict__ dqs,
                                                               float* __restrict__ dTx) {
    constexpr int ROWS = 256 / G;
    const int t = threadIdx.x % G;
    const int64_t u = (int64_t)blockIdx.x * ROWS + threadIdx.x / G;
    if (u >= n) return;
    const int64_t b = ptrT[u], e = ptrT[u + 1];
    float4 tu[NJ], acc[NJ];
    bool live[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = 4 * (t + G * j);
        live[j] = col < F;
        acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        tu[j] = live[j] ? ld4(Tx + u * ldx + col) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const float2 pqu = pq[u], stu = rowstat[u], dqu = dqs[u];
    float dp = dqu.y;                                  // the self term's score gradient
    {
        const float as = __expf(leaky(pqu.x + pqu.y) - stu.x) / stu.y;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            if (!live[j]) continue;
            const float4 d = ld4(dOut + u * ldd + 4 * (t + G * j));
            acc[j].x += as * d.x; acc[j].y += as * d.y; acc[j].z += as * d.z; acc[j].w += as * d.w;
        }
    }
    for (int64_t base = b; base < e; base += G) {
        const int cnt = (int)(e - base < G ? e - base : G);
        int mine = 0;
        float mya = 0.f, mw = 0.f, mc = 0.f;             // alpha, alpha * LeakyReLU', c of the destination
        if (t < cnt) {
            mine = idxT[base + t];
            const float2 sv = rowstat[mine];
            const float pre = pqu.x + pq[mine].y;
            mya = __expf(leaky(pre) - sv.x) / sv.y;
            mw = mya * leaky_d(pre);
            mc = cvec[mine];
        }
        for (int k = 0; k < cnt; k += 4) {
            const bool p1 = k + 1 < cnt, p2 = k + 2 < cnt, p3 = k + 3 < cnt;
            const int64_t c0 = __shfl(mine, k, G), c1 = __shfl(mine, p1 ? k + 1 : k, G);
            const int64_t c2 = __shfl(mine, p2 ? k + 2 : k, G), c3 = __shfl(mine, p3 ? k + 3 : k, G);
            const float a0 = __shfl(mya, k, G), a1 = p1 ? __shfl(mya, k + 1, G) : 0.f;
            const float a2 = p2 ? __shfl(mya, k + 2, G) : 0.f, a3 = p3 ? __shfl(mya, k + 3, G) : 0.f;
            float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (!live[j]) continue;
                const int col = 4 * (t + G * j);
                const float4 v0 = ld4(dOut + c0 * ldd + col), v1 = ld4(dOut + c1 * ldd + col);
                const float4 v2 = ld4(dOut + c2 * ldd + col), v3 = ld4(dOut + c3 * ldd + col);
                acc[j].x += a0 * v0.x; acc[j].y += a0 * v0.y; acc[j].z += a0 * v0.z; acc[j].w += a0 * v0.w;
                acc[j].x += a1 * v1.x; acc[j].y += a1 * v1.y; acc[j].z += a1 * v1.z; acc[j].w += a1 * v1.w;
                acc[j].x += a2 * v2.x; acc[j].y += a2 * v2.y; acc[j].z += a2 * v2.z; acc[j].w += a2 * v2.w;
                acc[j].x += a3 * v3.x; acc[j].y += a3 * v3.y; acc[j].z += a3 * v3.z; acc[j].w += a3 * v3.w;
                d0 += dot4(tu[j], v0); d1 += dot4(tu[j], v1); d2 += dot4(tu[j], v2); d3 += dot4(tu[j], v3);
            }
            d0 = group_sum<G>(d0); d1 = group_sum<G>(d1); d2 = group_sum<G>(d2); d3 = group_sum<G>(d3);
            dp += __shfl(mw, k, G) * (d0 - __shfl(mc, k, G));
            if (p1) dp += __shfl(mw, k + 1, G) * (d1 - __shfl(mc, k + 1, G));
            if (p2) dp += __shfl(mw, k + 2, G) * (d2 - __shfl(mc, k + 2, G));
            if (p3) dp += __shfl(mw, k + 3, G) * (d3 - __shfl(mc, k + 3, G));
        }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (!live[j]) continue;
        const int col = 4 * (t + G * j);
        float o[4] = {acc[j].x, acc[j].y, acc[j].z, acc[j].w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (col + q >= F) o[q] = 0.f;
        *reinterpret_cast<float4*>(dTx + u * ldx + col) = make_float4(o[0], o[1], o[2], o[3]);
    }
    if (t == 0) *reinterpret_cast<float4*>(dTx + u * ldx + ((F + 3) & ~3)) = make_float4(dp, dqu.x, 0.f, 0.f);
}

// Packed weights of one layer: Wp[Fin x ldx] = [W | 0 | W a_src | W a_dst | 0 0] (rows of the
// product dT_ext -> dH) and its transpose Wt[ldx x ld(Fin)] (rows of the product H -> T_ext).
__global__ __launch_bounds__(256) void gat_pack_kernel(const float* __restrict__ W, const float* __restrict__ a_s,
                                                       const float* __restrict__ a_d, int fin, int fout, int fin_pad, int ldx,
                                                       float* __restrict__ Wp, float* __restrict__ Wt) {
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
        Wp[(int64_t)i * ldx + c] = val;
    }
    Wt[(int64_t)c * fin_pad + i] = val;
}

// Gradients of W, a_src, a_dst from dWx = H^T dT_ext [Fin x ldx]:
//   dW = dWx[:, :F] + dWx[:, cp] a_src^T + dWx[:, cp+1] a_dst^T,  da_src = W^T dWx[:, cp],  da_dst = W^T dWx[:, cp+1].
__global__ __launch_bounds__(256) void gat_param_grad_kernel(const float* __restrict__ dWx, int ldx, const float* __restrict__ W,
                                                             const float* __restrict__ a_s, const float* __restrict__ a_d,
                                                             int fin, int fout, float* __restrict__ gW,
                                                             float* __restrict__ ga_s, float* __restrict__ ga_d) {
    const int cp = (fout + 3) & ~3;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < (int64_t)fin * fout) {
        const int i = (int)(e / fout), j = (int)(e % fout);
        gW[e] = dWx[(int64_t)i * ldx + j] + dWx[(int64_t)i * ldx + cp] * a_s[j] + dWx[(int64_t)i * ldx + cp + 1] * a_d[j];
    }
    if (e < fout) {
        float s = 0.f, d = 0.f;
        for (int i = 0; i < fin; ++i) {
            const float w = W[(int64_t)i * fout + e];
            s = fmaf(w, dWx[(int64_t)i * ldx + cp], s);
            d = fmaf(w, dWx[(int64_t)i * ldx + cp + 1], d);
        }
        ga_s[e] = s;
        ga_d[e] = d;
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
    float *dZa, *dZb, *dTx, *cvec, *dWx;
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

#define GRP_GAT_DISPATCH(KERNEL, F, ...)                                                                       \
    do {                                                                                                       \
        const int f4_ = ((F) + 3) / 4;                                                                         \
        if (f4_ <= 1) GRP_GAT_ONE(KERNEL, 1, 1, __VA_ARGS__);                                                  \
        else if (f4_ <= 2) GRP_GAT_ONE(KERNEL, 2, 1, __VA_ARGS__);                                             \
        else if (f4_ <= 4) GRP_GAT_ONE(KERNEL, 4, 1, __VA_ARGS__);                                             \
        else if (f4_ <= 8) GRP_GAT_ONE(KERNEL, 8, 1, __VA_ARGS__);                                             \
        else if (f4_ <= 16) GRP_GAT_ONE(KERNEL, 16, 1, __VA_ARGS__);                                           \
        else if (f4_ <= 32) GRP_GAT_ONE(KERNEL, 32, 1, __VA_ARGS__);                                           \
        else if (f4_ <= 64) GRP_GAT_ONE(KERNEL, 64, 1, __VA_ARGS__);                                           \
        else if (f4_ <= 128) GRP_GAT_ONE(KERNEL, 64, 2, __VA_ARGS__);                                          \
        else GRP_GAT_ONE(KERNEL, 64, 4, __VA_ARGS__);                                                          \
    } while (0)
#define GRP_GAT_ONE(KERNEL, G_, NJ_, ...) \
    hipLaunchKernelGGL((KERNEL<G_, NJ_>), dim3((unsigned)cdiv(n, 256 / G_)), dim3(256), 0, st, __VA_ARGS__)

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
        GRP_HIP(hipMemsetAsync(grad, 0, (size_t)P * sizeof(float), st));
        return launch_softmax_xent(0, m->dims[k], nullptr, 4, labels, nullptr, mask, o->estimator == GRP_EST_NODE_LEVEL,
                                   g->d_local_in, g->d_global_in, nullptr, p.dZa, 4, p.stats_ws, stats, st);
    }
    // ---------------- packed weights
    for (int l = 0; l < k; ++l) {
        const GatLayer& L = p.L[l];
        ProfScope ps("gat_pack_weights", st);
        hipLaunchKernelGGL(gat_pack_kernel, dim3((unsigned)cdiv((int64_t)L.ldin_pad * L.ldx, 256)), dim3(256), 0, st,
                           theta + L.off_w, theta + L.off_as, theta + L.off_ad, L.fin, L.fout, (int)L.ldin_pad, (int)L.ldx,
                           L.Wp, L.Wt);
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
            GRP_GAT_DISPATCH(gat_forward_kernel, L.fout, g->rowptr, g->col, n, L.fout, (const float*)L.Tx, L.ldx,
                             (const float2*)L.pq, theta + L.off_b, l < k - 1 ? 1 : 0, L.Hout, L.ldh, L.rowstat);
            GRP_LAUNCH_CHECK();
        }
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
            GRP_GAT_DISPATCH(gat_backward_dst_kernel, L.fout, g->rowptr, g->col, n, L.fout, (const float*)L.Tx, L.ldx,
                             (const float2*)L.pq, (const float2*)L.rowstat, theta + L.off_b, (const float*)L.Hout, L.ldh,
                             (const float*)dZ, L.ldh, p.cvec, p.dqs);
            GRP_GAT_DISPATCH(gat_backward_src_kernel, L.fout, g->colptr, g->row, n, L.fout, (const float*)L.Tx, L.ldx,
                             (const float2*)L.pq, (const float2*)L.rowstat, (const float*)dZ, L.ldh, (const float*)p.cvec,
                             (const float2*)p.dqs, p.dTx);
            GRP_LAUNCH_CHECK();
        }
        GemmTNArgs t;          // dW_ext = H_in^T dT_ext
        t.M = n; t.K = L.fin; t.N = (int)L.ldx; t.A = Hin; t.lda = ldin; t.a_bf16 = in_bf16; t.B = p.dTx; t.ldb = L.ldx;
        t.C = p.dWx; t.ldc = L.ldx; t.workspace = p.tn_ws; t.workspace_bytes = p.tn_ws_bytes;
        GRP_TRY(launch_gemm_tn(t, st));
        {
            ProfScope ps("gat_param_grad", st);
            const int64_t work = (int64_t)L.fin * L.fout > L.fout ? (int64_t)L.fin * L.fout : L.fout;
            hipLaunchKernelGGL(gat_param_grad_kernel, dim3((unsigned)cdiv(work, 256)), dim3(256), 0, st, (const float*)p.dWx,
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
