// Row-parallel neighbour aggregation (SpMM) for gfx950.
//
// Y[i,:] = a_i (sum_{e in row i} X[idx[e],:] + self * X[i,:]) (+ addend[i,:]) (+ bias) (ReLU)
//
// The same kernel serves the forward pass (rows of the CSR, i.e. destinations gathering
// their in-neighbours) and the backward pass (rows of the CSC: the transposed operator),
// so no floating-point atomics are needed and results are bit-reproducible.
//
// Mapping: a group of G lanes (G = 1..64, a power of two) owns one output row; lane t of
// the group owns columns 4*(t + G*j), j < NJ, as one 16-byte vector, so a group's gather of
// one neighbour row is a single fully coalesced request of F*sizeof(elem) bytes.  The
// group's lanes fetch G column indices with one coalesced load and hand them round with
// wavefront shuffles; four neighbour rows are requested before any is accumulated so that
// several gathers are in flight per lane.
#include "common.h"

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

__device__ __forceinline__ float row_scale(int mode, int64_t deg, int self_term) {
    if (mode == GRP_SCALE_MEAN) return 1.0f / (float)(deg > 1 ? deg : 1);
    if (mode == GRP_SCALE_RSQRT) {
        int64_t d = deg + self_term;
        return 1.0f / sqrtf((float)(d > 1 ? d : 1));
    }
    return 1.0f;
}

template <typename XT, int G, int NJ>
__global__ __launch_bounds__(256) void spmm_rows_kernel(
    const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx, int64_t n_rows, int F,
    const XT* __restrict__ X, int64_t ldx, int scale, int self_term, const float* __restrict__ colscale,
    const float* addend, int64_t ld_add, const float* __restrict__ bias, int relu,
    float* Y, int64_t ldy) {
    constexpr int ROWS = 256 / G;
    const int t = threadIdx.x % G;
    const int64_t i = (int64_t)blockIdx.x * ROWS + threadIdx.x / G;
    if (i >= n_rows) return;          // whole groups leave together (G divides 64)
    const int64_t b = ptr[i], e = ptr[i + 1];

    float4 acc[NJ];
    bool live[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        live[j] = 4 * (t + G * j) < F;
    }

    for (int64_t base = b; base < e; base += G) {
        const int cnt = (int)((e - base) < (int64_t)G ? (e - base) : (int64_t)G);
        const int mine = (t < cnt) ? idx[base + t] : 0;
        int k = 0;
        for (; k + 4 <= cnt; k += 4) {
            const int64_t c0 = __shfl(mine, k, G), c1 = __shfl(mine, k + 1, G);
            const int64_t c2 = __shfl(mine, k + 2, G), c3 = __shfl(mine, k + 3, G);
            float s0 = 1.f, s1 = 1.f, s2 = 1.f, s3 = 1.f;
            if (colscale) { s0 = colscale[c0]; s1 = colscale[c1]; s2 = colscale[c2]; s3 = colscale[c3]; }
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (!live[j]) continue;
                const int col = 4 * (t + G * j);
                const float4 v0 = Vec4Load<XT>::ld(X + c0 * ldx + col);
                const float4 v1 = Vec4Load<XT>::ld(X + c1 * ldx + col);
                const float4 v2 = Vec4Load<XT>::ld(X + c2 * ldx + col);
                const float4 v3 = Vec4Load<XT>::ld(X + c3 * ldx + col);
                if (colscale) {
                    acc[j].x = fmaf(s0, v0.x, acc[j].x); acc[j].y = fmaf(s0, v0.y, acc[j].y);
                    acc[j].z = fmaf(s0, v0.z, acc[j].z); acc[j].w = fmaf(s0, v0.w, acc[j].w);
                    acc[j].x = fmaf(s1, v1.x, acc[j].x); acc[j].y = fmaf(s1, v1.y, acc[j].y);
                    acc[j].z = fmaf(s1, v1.z, acc[j].z); acc[j].w = fmaf(s1, v1.w, acc[j].w);
                    acc[j].x = fmaf(s2, v2.x, acc[j].x); acc[j].y = fmaf(s2, v2.y, acc[j].y);
                    acc[j].z = fmaf(s2, v2.z, acc[j].z); acc[j].w = fmaf(s2, v2.w, acc[j].w);
                    acc[j].x = fmaf(s3, v3.x, acc[j].x); acc[j].y = fmaf(s3, v3.y, acc[j].y);
                    acc[j].z = fmaf(s3, v3.z, acc[j].z); acc[j].w = fmaf(s3, v3.w, acc[j].w);
                } else {
                    acc[j].x += v0.x; acc[j].y += v0.y; acc[j].z += v0.z; acc[j].w += v0.w;
                    acc[j].x += v1.x; acc[j].y += v1.y; acc[j].z += v1.z; acc[j].w += v1.w;
                    acc[j].x += v2.x; acc[j].y += v2.y; acc[j].z += v2.z; acc[j].w += v2.w;
                    acc[j].x += v3.x; acc[j].y += v3.y; acc[j].z += v3.z; acc[j].w += v3.w;
                }
            }
        }
        for (; k < cnt; ++k) {
            const int64_t c0 = __shfl(mine, k, G);
            const float s0 = colscale ? colscale[c0] : 1.f;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if (!live[j]) continue;
                const float4 v0 = Vec4Load<XT>::ld(X + c0 * ldx + 4 * (t + G * j));
                acc[j].x = fmaf(s0, v0.x, acc[j].x); acc[j].y = fmaf(s0, v0.y, acc[j].y);
                acc[j].z = fmaf(s0, v0.z, acc[j].z); acc[j].w = fmaf(s0, v0.w, acc[j].w);
            }
        }
    }

    const float a = row_scale(scale, e - b, self_term);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (!live[j]) continue;
        const int col = 4 * (t + G * j);
        float4 r = acc[j];
        if (self_term) {
            const float4 s = Vec4Load<XT>::ld(X + i * ldx + col);
            r.x += s.x; r.y += s.y; r.z += s.z; r.w += s.w;
        }
        r.x *= a; r.y *= a; r.z *= a; r.w *= a;
        if (addend) {
            const float4 s = *reinterpret_cast<const float4*>(addend + i * ld_add + col);
            r.x += s.x; r.y += s.y; r.z += s.z; r.w += s.w;
        }
        float o[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (col + q < F) {
                if (bias) o[q] += bias[col + q];
                if (relu) o[q] = o[q] > 0.f ? o[q] : 0.f;
            } else {
                o[q] = 0.f;           // pad columns stay zero
            }
        }
        *reinterpret_cast<float4*>(Y + i * ldy + col) = make_float4(o[0], o[1], o[2], o[3]);
    }
}

// Fallback for pitches or pointers that are not 16-byte friendly: one lane per column.
template <typename XT>
__global__ __launch_bounds__(256) void spmm_rows_scalar_kernel(
    const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx, int64_t n_rows, int F,
    const XT* __restrict__ X, int64_t ldx, int scale, int self_term, const float* __restrict__ colscale,
    const float* addend, int64_t ld_add, const float* __restrict__ bias, int relu,
    float* Y, int64_t ldy) {
    const int64_t i = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (i >= n_rows) return;
    const int t = threadIdx.x % 64;
    const int64_t b = ptr[i], e = ptr[i + 1];
    const float a = row_scale(scale, e - b, self_term);
    for (int col = t; col < F; col += 64) {
        float acc = 0.f;
        for (int64_t k = b; k < e; ++k) acc += (colscale ? colscale[idx[k]] : 1.f) * (float)X[(int64_t)idx[k] * ldx + col];
        if (self_term) acc += (float)X[i * ldx + col];
        acc *= a;
        if (addend) acc += addend[i * ld_add + col];
        if (bias) acc += bias[col];
        if (relu) acc = acc > 0.f ? acc : 0.f;
        Y[i * ldy + col] = acc;
    }
}

template <typename XT, int G, int NJ>
static void launch_one(const SpmmArgs& a, hipStream_t st) {
    constexpr int ROWS = 256 / G;
    const int64_t blocks = cdiv(a.n_rows, ROWS);
    hipLaunchKernelGGL((spmm_rows_kernel<XT, G, NJ>), dim3((unsigned)blocks), dim3(256), 0, st, a.ptr, a.idx,
                       a.n_rows, a.F, (const XT*)a.X, a.ldx, a.scale, a.self_term, a.colscale, a.addend, a.ld_add,
                       a.bias, a.relu, a.Y, a.ldy);
}

template <typename XT>
static grp_status dispatch(const SpmmArgs& a, hipStream_t st) {
    const int f4 = (a.F + 3) / 4;
    if (f4 <= 1) launch_one<XT, 1, 1>(a, st);
    else if (f4 <= 2) launch_one<XT, 2, 1>(a, st);
    else if (f4 <= 4) launch_one<XT, 4, 1>(a, st);
    else if (f4 <= 8) launch_one<XT, 8, 1>(a, st);
    else if (f4 <= 16) launch_one<XT, 16, 1>(a, st);
    else if (f4 <= 32) launch_one<XT, 32, 1>(a, st);
    else if (f4 <= 64) launch_one<XT, 64, 1>(a, st);
    else if (f4 <= 128) launch_one<XT, 64, 2>(a, st);
    else if (f4 <= 256) launch_one<XT, 64, 4>(a, st);
    else return fail(GRP_EUNSUPPORTED, "spmm: F = %d exceeds 1024", a.F);
    return GRP_OK;
}

grp_status launch_spmm(const SpmmArgs& a, hipStream_t st) {
    if (a.n_rows == 0) return GRP_OK;
    if (a.n_rows < 0 || a.F <= 0 || !a.ptr || !a.X || !a.Y)
        return fail(GRP_EINVAL, "spmm: bad arguments");
    const int elem = a.x_bf16 ? 2 : 4;
    const int64_t fpad = round_up(a.F, 4);
    const bool vec_ok = a.ldx >= fpad && a.ldy >= fpad && (a.ldx * elem) % (4 * elem) == 0 &&
                        a.ldx % 4 == 0 && a.ldy % 4 == 0 &&
                        ((uintptr_t)a.X % (4 * elem)) == 0 && ((uintptr_t)a.Y % 16) == 0 &&
                        (!a.addend || (a.ld_add % 4 == 0 && a.ld_add >= fpad && ((uintptr_t)a.addend % 16) == 0));
    // compulsory traffic: the index stream, the row pointers, every source row once, every
    // output row once (+ addend rows)
    const int64_t n_src = a.n_src > 0 ? a.n_src : a.n_rows;
    const double bytes = 4.0 * a.nnz + 8.0 * (a.n_rows + 1) + (double)elem * a.F * n_src +
                         4.0 * a.F * a.n_rows * (a.addend ? 2.0 : 1.0) + (a.colscale ? 4.0 * n_src : 0.0);
    ProfScope ps(a.x_bf16 ? "spmm_rows_bf16" : "spmm_rows_f32", st, 2.0 * a.nnz * a.F, bytes);
    if (vec_ok) {
        GRP_TRY(a.x_bf16 ? dispatch<__hip_bfloat16>(a, st) : dispatch<float>(a, st));
    } else {
        const int64_t blocks = cdiv(a.n_rows, 4);
        if (a.x_bf16)
            hipLaunchKernelGGL((spmm_rows_scalar_kernel<__hip_bfloat16>), dim3((unsigned)blocks), dim3(256), 0, st,
                               a.ptr, a.idx, a.n_rows, a.F, (const __hip_bfloat16*)a.X, a.ldx, a.scale,
                               a.self_term, a.colscale, a.addend, a.ld_add, a.bias, a.relu, a.Y, a.ldy);
        else
            hipLaunchKernelGGL((spmm_rows_scalar_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, st, a.ptr,
                               a.idx, a.n_rows, a.F, (const float*)a.X, a.ldx, a.scale, a.self_term, a.colscale, a.addend,
                               a.ld_add, a.bias, a.relu, a.Y, a.ldy);
    }
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

}  // namespace grp

extern "C" grp_status grp_spmm(const grp_partition_t* part, int32_t transposed, int32_t scale,
                               int32_t self_term, int32_t F, const void* X, int64_t ldx, int32_t x_dtype,
                               float* Y, int64_t ldy, void* stream) {
    if (!part || !X || !Y) return grp::fail(GRP_EINVAL, "grp_spmm: null argument");
    if (F <= 0 || ldx < F || ldy < F) return grp::fail(GRP_EINVAL, "grp_spmm: bad F / pitch");
    if (scale < GRP_SCALE_NONE || scale > GRP_SCALE_RSQRT) return grp::fail(GRP_EINVAL, "grp_spmm: bad scale");
    if (x_dtype != GRP_DTYPE_FP32 && x_dtype != GRP_DTYPE_BF16) return grp::fail(GRP_EINVAL, "grp_spmm: bad dtype");
    grp::SpmmArgs a;
    a.ptr = transposed ? part->colptr : part->rowptr;
    a.idx = transposed ? part->row : part->col;
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
    return grp::launch_spmm(a, (hipStream_t)stream);
}
