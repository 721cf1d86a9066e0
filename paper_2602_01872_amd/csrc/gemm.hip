// Dense feature transforms on the gfx950 matrix cores (fp32 MFMA, fp32 accumulate).
//
//   gemm_nn:  C[M x N] = epilogue(A[M x K] B[K x N] + A2[M x K2] B2[K2 x N])   (X W, dY W^T)
//   gemm_tn:  C[K x N] = A[M x K]^T B[M x N]                                   (X^T dY)
//
// M is the number of nodes (10^5..10^7); K and N are layer widths (<= a few hundred), so
// both products are tall-and-skinny: a workgroup owns a 128-row slab of nodes (nn) or a
// slice of the node dimension (tn, partial sums reduced afterwards in a fixed order, so
// the result does not depend on scheduling).
//
// Tiling: 256 threads = 4 wavefronts laid out WM x WN; a wavefront owns TM x TN tiles of
// 32x32 computed with v_mfma_f32_32x32x2_f32.  Operand layout of that instruction on a
// 64-lane wavefront: lane l supplies A[i = l%32][k = l/32] and B[k = l/32][j = l%32]; of
// the 16 accumulator registers, register r of lane l holds D[8*(r/4) + 4*(l/32) + r%4][l%32].
// Both operands are staged in LDS k-major (the 32 lanes of a half-wave read 32 consecutive
// floats: no bank conflicts); the next k-tile is fetched from HBM into registers while the
// current one is multiplied.
#include "common.h"

namespace grp {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 32;      // k-tile depth

template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<__hip_bfloat16>(__hip_bfloat16 v) { return __bfloat162float(v); }

// Four consecutive elements row[k..k+3] as floats; elements at k+q >= K read as zero.
template <typename T, bool VEC>
__device__ __forceinline__ void load4(const T* __restrict__ row, int k, int K, float o[4]) {
    o[0] = o[1] = o[2] = o[3] = 0.f;
    if (k >= K) return;
    if constexpr (VEC) {
        if constexpr (sizeof(T) == 4) {
            const float4 v = *reinterpret_cast<const float4*>(row + k);
            o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
        } else {
            const uint2 r = *reinterpret_cast<const uint2*>(row + k);
            o[0] = __uint_as_float(r.x << 16);
            o[1] = __uint_as_float(r.x & 0xFFFF0000u);
            o[2] = __uint_as_float(r.y << 16);
            o[3] = __uint_as_float(r.y & 0xFFFF0000u);
        }
#pragma unroll
        for (int q = 1; q < 4; ++q)
            if (k + q >= K) o[q] = 0.f;
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (k + q < K) o[q] = to_f<T>(row[k + q]);
    }
}

// One BK-deep step of the wavefront's TM x TN block from k-major LDS tiles.
template <int TM, int TN, int PA, int PB>
__device__ __forceinline__ void mma_step(const float* __restrict__ As, const float* __restrict__ Bs, int a_off,
                                         int b_off, floatx16 (&acc)[TM][TN]) {
    const int lane = threadIdx.x & 63;
    const int li = lane & 31, lk = lane >> 5;
#pragma unroll
    for (int k = 0; k < BK; k += 2) {
        float a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = As[(k + lk) * PA + a_off + 32 * i + li];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = Bs[(k + lk) * PB + b_off + 32 * j + li];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

// ------------------------------------------------------------------------------- NN
template <typename AT, bool VECA, bool VECB, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_nn_kernel(GemmNNArgs g) {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int PA = BM + 4, PB = BN + 4;
    constexpr int A_REPS = BM * BK / 4 / 256;        // float4 loads per thread for the A tile
    constexpr int B_REPS = (BN * BK / 4 + 255) / 256;
    __shared__ float As[BK * PA];
    __shared__ float Bs[BK * PB];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int n_store = g.zero_pad_to > g.N ? g.zero_pad_to : g.N;
    const int n_tiles = (n_store + BN - 1) / BN;
    const int64_t m0 = (int64_t)(blockIdx.x / n_tiles) * BM;
    const int n0 = (blockIdx.x % n_tiles) * BN;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk1 = (g.K + BK - 1) / BK;
    const int nk2 = (g.K2 + BK - 1) / BK;
    const int nk = nk1 + nk2;

    float ra[A_REPS][4], rb[B_REPS][4];

    auto fetch = [&](int kt) {
        const bool second = kt >= nk1;
        const int k0 = (second ? kt - nk1 : kt) * BK;
        const int Kc = second ? g.K2 : g.K;
#pragma unroll
        for (int r = 0; r < A_REPS; ++r) {
            const int f = tid + 256 * r;                 // float4 slot in the BM x BK tile
            const int m = f / (BK / 4), kq = f % (BK / 4);
            const int64_t gm = m0 + m;
            if (gm < g.M) {
                if (second) load4<float, true>(g.A2 + gm * g.lda2, k0 + 4 * kq, Kc, ra[r]);
                else load4<AT, VECA>((const AT*)g.A + gm * g.lda, k0 + 4 * kq, Kc, ra[r]);
            } else {
                ra[r][0] = ra[r][1] = ra[r][2] = ra[r][3] = 0.f;
            }
        }
        const float* Bp = second ? g.B2 : g.B;
        const int64_t ldb = second ? g.ldb2 : g.ldb;
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            const int f = tid + 256 * r;
            const int k = f / (BN / 4), nq = f % (BN / 4);
            rb[r][0] = rb[r][1] = rb[r][2] = rb[r][3] = 0.f;
            if (f < BN * BK / 4 && k0 + k < Kc) load4<float, VECB>(Bp + (int64_t)(k0 + k) * ldb, n0 + 4 * nq, g.N, rb[r]);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int r = 0; r < A_REPS; ++r) {
            const int f = tid + 256 * r;
            const int m = f / (BK / 4), kq = f % (BK / 4);
#pragma unroll
            for (int q = 0; q < 4; ++q) As[(4 * kq + q) * PA + m] = ra[r][q];
        }
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            const int f = tid + 256 * r;
            const int k = f / (BN / 4), nq = f % (BN / 4);
            if (f < BN * BK / 4)
                *reinterpret_cast<float4*>(&Bs[k * PB + 4 * nq]) = make_float4(rb[r][0], rb[r][1], rb[r][2], rb[r][3]);
        }
    };

    fetch(0);
    stage();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) fetch(kt + 1);
        mma_step<TM, TN, PA, PB>(As, Bs, wm * TM * 32, wn * TN * 32, acc);
        __syncthreads();
        if (kt + 1 < nk) {
            stage();
            __syncthreads();
        }
    }

    const int li = lane & 31, lk = lane >> 5;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + (wn * TN + j) * 32 + li;
            if (col >= n_store) continue;
            const float bv = (g.bias && col < g.N) ? g.bias[col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (m >= g.M) continue;
                float v = 0.f;
                if (col < g.N) {
                    v = acc[i][j][r] + bv;
                    if (g.addend) v += g.addend[m * g.ld_add + col];
                    if (g.rowscale) v *= g.rowscale[m];
                    if (g.relu) v = v > 0.f ? v : 0.f;
                    if (g.mask) v = g.mask[m * g.ld_mask + col] > 0.f ? v : 0.f;
                }
                g.C[m * g.ldc + col] = v;
            }
        }
}

template <typename AT, bool VECA, bool VECB>
static void nn_pick(const GemmNNArgs& a, hipStream_t st) {
    const int n_eff = a.zero_pad_to > a.N ? a.zero_pad_to : a.N;
    if (n_eff > 64) {
        const int64_t blocks = cdiv(a.M, 128) * cdiv(n_eff, 128);
        hipLaunchKernelGGL((gemm_nn_kernel<AT, VECA, VECB, 2, 2, 2, 2>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    } else if (n_eff > 32) {
        const int64_t blocks = cdiv(a.M, 128) * cdiv(n_eff, 64);
        hipLaunchKernelGGL((gemm_nn_kernel<AT, VECA, VECB, 4, 1, 1, 2>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    } else {
        const int64_t blocks = cdiv(a.M, 128) * cdiv(n_eff, 32);
        hipLaunchKernelGGL((gemm_nn_kernel<AT, VECA, VECB, 4, 1, 1, 1>), dim3((unsigned)blocks), dim3(256), 0, st, a);
    }
}

grp_status launch_gemm_nn(const GemmNNArgs& a, hipStream_t st) {
    if (a.M == 0 || a.N == 0) return GRP_OK;
    if (a.M < 0 || a.N < 0 || a.K <= 0 || !a.A || !a.B || !a.C) return fail(GRP_EINVAL, "gemm_nn: bad arguments");
    if (a.K2 > 0 && (!a.A2 || !a.B2 || a.lda2 % 4 != 0 || (uintptr_t)a.A2 % 16 != 0))
        return fail(GRP_EINVAL, "gemm_nn: second operand must be 16-byte aligned with a pitch multiple of 4");
    const int elem = a.a_bf16 ? 2 : 4;
    const bool veca = a.lda % 4 == 0 && a.lda >= round_up(a.K, 4) && (uintptr_t)a.A % (4 * elem) == 0;
    const bool vecb = a.ldb % 4 == 0 && a.ldb >= round_up(a.N, 4) && (uintptr_t)a.B % 16 == 0 &&
                      (a.K2 == 0 || (a.ldb2 % 4 == 0 && a.ldb2 >= round_up(a.N, 4) && (uintptr_t)a.B2 % 16 == 0));
    const double nn_flops = 2.0 * a.M * a.N * ((double)a.K + a.K2);
    const double nn_bytes = (double)a.M * a.K * elem + 4.0 * a.M * a.K2 + 4.0 * a.N * ((double)a.K + a.K2) +
                            4.0 * a.M * a.N * (1.0 + (a.addend ? 1.0 : 0.0) + (a.mask ? 1.0 : 0.0));
    ProfScope ps(a.a_bf16 ? "gemm_nn_bf16a" : "gemm_nn_f32", st, nn_flops, nn_bytes);
    if (a.a_bf16) {
        if (veca && vecb) nn_pick<__hip_bfloat16, true, true>(a, st);
        else nn_pick<__hip_bfloat16, false, false>(a, st);
    } else {
        if (veca && vecb) nn_pick<float, true, true>(a, st);
        else nn_pick<float, false, false>(a, st);
    }
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// ------------------------------------------------------------------------------- TN
constexpr int TN_ROWS_PER_SPLIT_MIN = 2048;   // node rows per split (multiple of BK)
constexpr int TN_MAX_SPLITS = 256;

struct TnPlan {
    int tiles_k, tiles_n, splits;
    int64_t chunk;
    int bk_tile, bn_tile;
};

static TnPlan tn_plan(int64_t M, int K, int N) {
    TnPlan p;
    p.bk_tile = 128;
    p.bn_tile = N > 64 ? 128 : (N > 32 ? 64 : 32);
    p.tiles_k = (int)cdiv(K, p.bk_tile);
    p.tiles_n = (int)cdiv(N, p.bn_tile);
    int64_t s = cdiv(M, TN_ROWS_PER_SPLIT_MIN);
    if (s > TN_MAX_SPLITS) s = TN_MAX_SPLITS;
    if (s < 1) s = 1;
    p.chunk = round_up(cdiv(M, s), BK);
    if (p.chunk < BK) p.chunk = BK;
    p.splits = (int)cdiv(M, p.chunk);
    if (p.splits < 1) p.splits = 1;
    return p;
}

size_t gemm_tn_workspace_bytes(int64_t M, int32_t K, int32_t N) {
    TnPlan p = tn_plan(M, K, N);
    return p.splits > 1 ? (size_t)p.splits * K * N * sizeof(float) : 0;
}

template <typename AT, bool VECA, bool VECB, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_tn_kernel(GemmTNArgs g, int tiles_n, int64_t chunk, float* __restrict__ out,
                                                      int64_t out_ld, int64_t out_split_stride) {
    constexpr int BKA = WM * TM * 32, BN = WN * TN * 32;   // output tile: BKA (rows of C) x BN
    constexpr int PA = BKA + 4, PB = BN + 4;
    constexpr int A_REPS = BKA * BK / 4 / 256;
    constexpr int B_REPS = (BN * BK / 4 + 255) / 256;
    __shared__ float As[BK * PA];
    __shared__ float Bs[BK * PB];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int ka0 = (blockIdx.x / tiles_n) * BKA;
    const int n0 = (blockIdx.x % tiles_n) * BN;
    const int64_t m_begin = (int64_t)blockIdx.y * chunk;
    const int64_t m_end = m_begin + chunk < g.M ? m_begin + chunk : g.M;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float ra[A_REPS][4], rb[B_REPS][4];
    auto fetch = [&](int64_t mt) {
#pragma unroll
        for (int r = 0; r < A_REPS; ++r) {
            const int f = tid + 256 * r;
            const int m = f / (BKA / 4), cq = f % (BKA / 4);
            const int64_t gm = mt + m;
            ra[r][0] = ra[r][1] = ra[r][2] = ra[r][3] = 0.f;
            if (gm < m_end) load4<AT, VECA>((const AT*)g.A + gm * g.lda, ka0 + 4 * cq, g.K, ra[r]);
        }
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            const int f = tid + 256 * r;
            const int m = f / (BN / 4), cq = f % (BN / 4);
            const int64_t gm = mt + m;
            rb[r][0] = rb[r][1] = rb[r][2] = rb[r][3] = 0.f;
            if (f < BN * BK / 4 && gm < m_end) load4<float, VECB>(g.B + gm * g.ldb, n0 + 4 * cq, g.N, rb[r]);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int r = 0; r < A_REPS; ++r) {
            const int f = tid + 256 * r;
            const int m = f / (BKA / 4), cq = f % (BKA / 4);
            *reinterpret_cast<float4*>(&As[m * PA + 4 * cq]) = make_float4(ra[r][0], ra[r][1], ra[r][2], ra[r][3]);
        }
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            const int f = tid + 256 * r;
            const int m = f / (BN / 4), cq = f % (BN / 4);
            if (f < BN * BK / 4)
                *reinterpret_cast<float4*>(&Bs[m * PB + 4 * cq]) = make_float4(rb[r][0], rb[r][1], rb[r][2], rb[r][3]);
        }
    };

    if (m_begin < m_end) {
        fetch(m_begin);
        stage();
        __syncthreads();
        for (int64_t mt = m_begin; mt < m_end; mt += BK) {
            const bool more = mt + BK < m_end;
            if (more) fetch(mt + BK);
            mma_step<TM, TN, PA, PB>(As, Bs, wm * TM * 32, wn * TN * 32, acc);
            __syncthreads();
            if (more) {
                stage();
                __syncthreads();
            }
        }
    }

    const int li = lane & 31, lk = lane >> 5;
    float* o = out + (int64_t)blockIdx.y * out_split_stride;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + (wn * TN + j) * 32 + li;
            if (col >= g.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ka = ka0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (ka < g.K) o[(int64_t)ka * out_ld + col] = acc[i][j][r];
            }
        }
}

__global__ __launch_bounds__(256) void tn_reduce_kernel(const float* __restrict__ part, int splits, int K, int N,
                                                        float* __restrict__ C, int64_t ldc) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)K * N) return;
    float s = 0.f;
    for (int p = 0; p < splits; ++p) s += part[(int64_t)p * K * N + e];
    C[(e / N) * ldc + (e % N)] = s;
}

template <typename AT, bool VECA, bool VECB>
static void tn_pick(const GemmTNArgs& a, const TnPlan& p, float* out, int64_t out_ld, int64_t stride, hipStream_t st) {
    dim3 grid((unsigned)(p.tiles_k * p.tiles_n), (unsigned)p.splits);
    if (p.bn_tile == 128)
        hipLaunchKernelGGL((gemm_tn_kernel<AT, VECA, VECB, 2, 2, 2, 2>), grid, dim3(256), 0, st, a, p.tiles_n, p.chunk, out, out_ld, stride);
    else if (p.bn_tile == 64)
        hipLaunchKernelGGL((gemm_tn_kernel<AT, VECA, VECB, 4, 1, 1, 2>), grid, dim3(256), 0, st, a, p.tiles_n, p.chunk, out, out_ld, stride);
    else
        hipLaunchKernelGGL((gemm_tn_kernel<AT, VECA, VECB, 4, 1, 1, 1>), grid, dim3(256), 0, st, a, p.tiles_n, p.chunk, out, out_ld, stride);
}

grp_status launch_gemm_tn(const GemmTNArgs& a, hipStream_t st) {
    if (a.K <= 0 || a.N <= 0 || a.M < 0 || !a.C) return fail(GRP_EINVAL, "gemm_tn: bad arguments");
    if (a.M > 0 && (!a.A || !a.B)) return fail(GRP_EINVAL, "gemm_tn: null operand");
    const TnPlan p = tn_plan(a.M, a.K, a.N);
    const size_t need = p.splits > 1 ? (size_t)p.splits * a.K * a.N * sizeof(float) : 0;
    if (need > a.workspace_bytes || (need && !a.workspace))
        return fail(GRP_EWORKSPACE, "gemm_tn: workspace %zu < %zu bytes", a.workspace_bytes, need);
    const int elem = a.a_bf16 ? 2 : 4;
    const bool veca = a.lda % 4 == 0 && a.lda >= round_up(a.K, 4) && (uintptr_t)a.A % (4 * elem) == 0;
    const bool vecb = a.ldb % 4 == 0 && a.ldb >= round_up(a.N, 4) && (uintptr_t)a.B % 16 == 0;
    float* out = p.splits > 1 ? (float*)a.workspace : a.C;
    const int64_t out_ld = p.splits > 1 ? a.N : a.ldc;
    const int64_t stride = p.splits > 1 ? (int64_t)a.K * a.N : 0;
    {
        ProfScope ps(a.a_bf16 ? "gemm_tn_bf16a" : "gemm_tn_f32", st, 2.0 * a.M * a.K * a.N,
                     (double)a.M * a.K * elem + 4.0 * a.M * a.N + 4.0 * a.K * a.N);
        if (a.a_bf16) {
            if (veca && vecb) tn_pick<__hip_bfloat16, true, true>(a, p, out, out_ld, stride, st);
            else tn_pick<__hip_bfloat16, false, false>(a, p, out, out_ld, stride, st);
        } else {
            if (veca && vecb) tn_pick<float, true, true>(a, p, out, out_ld, stride, st);
            else tn_pick<float, false, false>(a, p, out, out_ld, stride, st);
        }
        GRP_LAUNCH_CHECK();
    }
    if (p.splits > 1) {
        ProfScope ps("gemm_tn_reduce", st, 0.0, 4.0 * a.K * a.N * (p.splits + 1.0));
        const int64_t blocks = cdiv((int64_t)a.K * a.N, 256);
        hipLaunchKernelGGL(tn_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const float*)a.workspace,
                           p.splits, a.K, a.N, a.C, a.ldc);
        GRP_LAUNCH_CHECK();
    }
    return GRP_OK;
}

}  // namespace grp

extern "C" grp_status grp_gemm_nn(int64_t M, int32_t N, int32_t K, const void* A, int64_t lda, int32_t a_dtype,
                                  const float* B, int64_t ldb, float* C, int64_t ldc, void* stream) {
    if (!A || !B || !C) return grp::fail(GRP_EINVAL, "grp_gemm_nn: null argument");
    if (M < 0 || N <= 0 || K <= 0 || lda < K || ldb < N || ldc < N) return grp::fail(GRP_EINVAL, "grp_gemm_nn: bad shape");
    grp::GemmNNArgs a;
    a.M = M; a.N = N; a.K = K; a.A = A; a.lda = lda; a.a_bf16 = a_dtype == GRP_DTYPE_BF16;
    a.B = B; a.ldb = ldb; a.C = C; a.ldc = ldc;
    return grp::launch_gemm_nn(a, (hipStream_t)stream);
}

extern "C" size_t grp_gemm_tn_workspace_bytes(int64_t M, int32_t K, int32_t N) {
    if (M < 0 || K <= 0 || N <= 0) return 0;
    return grp::gemm_tn_workspace_bytes(M, K, N);
}

extern "C" grp_status grp_gemm_tn(int64_t M, int32_t K, int32_t N, const void* A, int64_t lda, int32_t a_dtype,
                                  const float* B, int64_t ldb, float* C, int64_t ldc, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    if (!C || (M > 0 && (!A || !B))) return grp::fail(GRP_EINVAL, "grp_gemm_tn: null argument");
    if (M < 0 || N <= 0 || K <= 0 || lda < K || ldb < N || ldc < N) return grp::fail(GRP_EINVAL, "grp_gemm_tn: bad shape");
    grp::GemmTNArgs a;
    a.M = M; a.K = K; a.N = N; a.A = A; a.lda = lda; a.a_bf16 = a_dtype == GRP_DTYPE_BF16;
    a.B = B; a.ldb = ldb; a.C = C; a.ldc = ldc; a.workspace = workspace; a.workspace_bytes = workspace_bytes;
    return grp::launch_gemm_tn(a, (hipStream_t)stream);
}
