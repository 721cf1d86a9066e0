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
// floats: no bank conflicts).  The next k-tile is requested from HBM into raw registers
// before the current one is multiplied and is only touched (converted, masked, written to
// LDS) after the multiply, so the loads overlap the matrix instructions; addresses are
// clamped into the operand instead of branching, and out-of-range elements are zeroed when
// they are written to LDS.
#include "common.h"

#include <algorithm>

#include <type_traits>

namespace grp {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 32;      // k-tile depth
constexpr int NXCD = 8;     // L2 domains; consecutive workgroup ids go round them

template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<__hip_bfloat16>(__hip_bfloat16 v) { return __bfloat162float(v); }

// Four consecutive elements as raw bits (fp32: 16 bytes, bf16: 8 bytes in .x/.y).
template <typename T>
__device__ __forceinline__ uint4 ldg_raw4(const T* __restrict__ p) {
    if constexpr (sizeof(T) == 4) {
        return *reinterpret_cast<const uint4*>(p);
    } else {
        const uint2 r = *reinterpret_cast<const uint2*>(p);
        return make_uint4(r.x, r.y, 0u, 0u);
    }
}
__device__ __forceinline__ void unpack4(const uint4& r, bool bf16, float o[4]) {
    if (bf16) {
        o[0] = __uint_as_float(r.x << 16);
        o[1] = __uint_as_float(r.x & 0xFFFF0000u);
        o[2] = __uint_as_float(r.y << 16);
        o[3] = __uint_as_float(r.y & 0xFFFF0000u);
    } else {
        o[0] = __uint_as_float(r.x); o[1] = __uint_as_float(r.y);
        o[2] = __uint_as_float(r.z); o[3] = __uint_as_float(r.w);
    }
}

// Slow, always-safe element loads for operands whose pitch or base is not 16-byte friendly.
template <typename T>
__device__ __forceinline__ uint4 ldg_safe4(const T* __restrict__ row, bool row_ok, int k, int K) {
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    if (row_ok) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (k + q < K) o[q] = to_f<T>(row[k + q]);
    }
    return make_uint4(__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3]));
}

__device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }
__device__ __forceinline__ int64_t lmin(int64_t a, int64_t b) { return a < b ? a : b; }

// One BKT-deep step of the wavefront's TM x TN block from k-major LDS tiles.  The operands of
// the next k-pair are read from LDS before the matrix instructions of the current one are
// issued, so the LDS latency hides behind them.
template <int TM, int TN, int PA, int PB, int BKT>
__device__ __forceinline__ void mma_step(const float* __restrict__ As, const float* __restrict__ Bs, int a_off,
                                         int b_off, floatx16 (&acc)[TM][TN]) {
    const int lane = threadIdx.x & 63;
    const int li = lane & 31, lk = lane >> 5;
    const float* ap = As + lk * PA + a_off + li;
    const float* bp = Bs + lk * PB + b_off + li;
    float a[2][TM], b[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) a[0][i] = ap[32 * i];
#pragma unroll
    for (int j = 0; j < TN; ++j) b[0][j] = bp[32 * j];
#pragma unroll
    for (int k = 0; k < BKT; k += 2) {
        const int cur = (k >> 1) & 1, nxt = cur ^ 1;
        if (k + 2 < BKT) {
#pragma unroll
            for (int i = 0; i < TM; ++i) a[nxt][i] = ap[(k + 2) * PA + 32 * i];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[nxt][j] = bp[(k + 2) * PB + 32 * j];
        }
        __builtin_amdgcn_sched_barrier(0);    // keep the next operands' LDS reads ahead of these MFMAs
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Variant for the tn kernel, whose LDS tiles keep the output dimension contiguous: tile t of
// a wavefront's TM (or TN) tiles takes the interleaved columns TM*l + t of its 32*TM-wide
// block, so that one 4*TM-byte LDS read per lane feeds all TM tiles.  Accumulator register r
// of tile (i, j) then holds row TM*(8*(r/4) + 4*(lane/32) + r%4) + i, column TN*(lane%32) + j
// of the wavefront's block.
template <int TM, int TN, int PA, int PB, int BKT>
__device__ __forceinline__ void mma_step_interleaved(const float* __restrict__ As, const float* __restrict__ Bs, int a_off,
                                                     int b_off, floatx16 (&acc)[TM][TN]) {
    static_assert((TM == 1 || TM == 2) && (TN == 1 || TN == 2), "one LDS read of at most 8 bytes per operand");
    const int lane = threadIdx.x & 63;
    const int li = lane & 31, lk = lane >> 5;
    const float* ap = As + lk * PA + a_off + TM * li;
    const float* bp = Bs + lk * PB + b_off + TN * li;
    float a[2][TM], b[2][TN];
    auto rd = [&](int k, int buf) {
        if constexpr (TM == 2) { const float2 t = *reinterpret_cast<const float2*>(ap + k * PA); a[buf][0] = t.x; a[buf][1] = t.y; }
        else a[buf][0] = ap[k * PA];
        if constexpr (TN == 2) { const float2 t = *reinterpret_cast<const float2*>(bp + k * PB); b[buf][0] = t.x; b[buf][1] = t.y; }
        else b[buf][0] = bp[k * PB];
    };
    rd(0, 0);
#pragma unroll
    for (int k = 0; k < BKT; k += 2) {
        const int cur = (k >> 1) & 1, nxt = cur ^ 1;
        if (k + 2 < BKT) rd(k + 2, nxt);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Epilogue shared by the nn kernels: (+ addend) (+ bias) -> C_raw; (* rowscale) (ReLU) (mask) -> C.
// When every operand allows 16-byte accesses the accumulators go through LDS, 32 tile rows
// per wavefront row at a time, so that addend / mask are read and the results written as
// whole 16-byte vectors along rows (one 512-byte run per 32 lanes).  `lds` must hold
// WM*32*(BN+4) floats and must no longer be read by the main loop.
template <bool VEC, int WM, int WN, int TM, int TN>
__device__ __forceinline__ void nn_epilogue(const GemmNNArgs& g, floatx16 (&acc)[TM][TN], float* lds, int64_t m0, int n0,
                                            int n_store) {
    constexpr int BN = WN * TN * 32;
    constexpr int PC = BN + 4;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lk = lane >> 5;
    // Epilogue.  When every operand allows 16-byte accesses the accumulators go through LDS,
    // 32 tile rows per wavefront row at a time, so that bias / addend / mask are read and the
    // results written as whole 16-byte vectors along rows (one 512-byte run per 32 lanes).
    const bool vec_epi = VEC && (n_store % 4 == 0) && g.ldc % 4 == 0 && ((uintptr_t)g.C % 16) == 0 &&
                         (!g.addend || (g.ld_add % 4 == 0 && ((uintptr_t)g.addend % 16) == 0)) &&
                         (!g.mask || (g.ld_mask % 4 == 0 && ((uintptr_t)g.mask % 16) == 0)) &&
                         (!g.C_raw || (g.ld_raw % 4 == 0 && ((uintptr_t)g.C_raw % 16) == 0));
    const int bias_n = g.bias_n > 0 ? g.bias_n : g.N - g.bias_col0;
    const int rs_cols = g.rowscale_cols > 0 ? g.rowscale_cols : g.N;   // a multiple of 4 when set
    if (vec_epi) {
        float* Cs = lds;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (i > 0) __syncthreads();               // the previous pass has been read out
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    Cs[(wm * 32 + 8 * (r / 4) + 4 * lk + (r % 4)) * PC + (wn * TN + j) * 32 + li] = acc[i][j][r];
            __syncthreads();
            constexpr int C4 = BN / 4;                // 16-byte columns per tile row
            for (int f = tid; f < WM * 32 * C4; f += 256) {
                const int lr = f / C4, c4 = f % C4;
                const int col = n0 + 4 * c4;
                const int64_t m = m0 + ((lr >> 5) * TM + i) * 32 + (lr & 31);
                if (m >= g.M || col >= n_store) continue;
                const float4 a4 = *reinterpret_cast<const float4*>(&Cs[lr * PC + 4 * c4]);
                float v[4] = {a4.x, a4.y, a4.z, a4.w};
                if (g.addend) {
                    const float4 t = *reinterpret_cast<const float4*>(g.addend + m * g.ld_add + col);
                    v[0] += t.x; v[1] += t.y; v[2] += t.z; v[3] += t.w;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int cb = col + q - g.bias_col0;
                    if (col + q < g.N) { if (g.bias && cb >= 0 && cb < bias_n) v[q] += g.bias[cb]; }
                    else v[q] = 0.f;
                }
                if (g.C_raw) *reinterpret_cast<float4*>(g.C_raw + m * g.ld_raw + col) = make_float4(v[0], v[1], v[2], v[3]);
                const float rs = (g.rowscale && col < rs_cols) ? g.rowscale[m] : 1.f;
                float4 mk = make_float4(1.f, 1.f, 1.f, 1.f);
                if (g.mask) mk = *reinterpret_cast<const float4*>(g.mask + m * g.ld_mask + col);
                const float mv[4] = {mk.x, mk.y, mk.z, mk.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float t = v[q] * rs;
                    if (g.relu) t = t > 0.f ? t : 0.f;
                    if (g.mask) t = mv[q] > 0.f ? t : 0.f;
                    v[q] = col + q < g.N ? t : 0.f;
                }
                *reinterpret_cast<float4*>(g.C + m * g.ldc + col) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + (wn * TN + j) * 32 + li;
            if (col >= n_store) continue;
            const int cb = col - g.bias_col0;
            const float bv = (g.bias && col < g.N && cb >= 0 && cb < bias_n) ? g.bias[cb] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (m >= g.M) continue;
                float v = 0.f;
                if (col < g.N) {
                    v = acc[i][j][r] + bv;
                    if (g.addend) v += g.addend[m * g.ld_add + col];
                }
                if (g.C_raw) g.C_raw[m * g.ld_raw + col] = v;
                if (col < g.N) {
                    if (g.rowscale && col < rs_cols) v *= g.rowscale[m];
                    if (g.relu) v = v > 0.f ? v : 0.f;
                    if (g.mask) v = g.mask[m * g.ld_mask + col] > 0.f ? v : 0.f;
                }
                g.C[m * g.ldc + col] = v;
            }
        }
}

// ------------------------------------------------------------------------------- NN
template <typename AT, bool VEC, int WM, int WN, int TM, int TN, int BK, int NBUF>
__global__ __launch_bounds__(256) void gemm_nn_kernel(GemmNNArgs g) {
    if (g.M_dev) {                                    // the launch was sized by upper bounds
        g.M = *g.M_dev;
        if (g.a_valid_rows_dev) g.a_valid_rows = *g.a_valid_rows_dev;
    }
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int PA = BM + 2, PB = BN + 4;          // PA = 2 mod 8 spreads the transposing writes
    constexpr int A_REPS = BM * BK / 4 / 256;        // 4-element loads per thread for the A tile
    constexpr int B_REPS = (BN * BK / 4 + 255) / 256;
    constexpr bool A_BF16 = sizeof(AT) == 2;
    static_assert(BM * BK / 4 % 256 == 0, "A tile must fill the workgroup");
    constexpr int PC = BN + 4;                        // pitch of the staged output tile
    constexpr int A_FLOATS = ((BK * PA + 3) / 4) * 4; // keeps the B tiles 16-byte aligned
    constexpr int MAIN_FLOATS = NBUF * (A_FLOATS + BK * PB);
    constexpr int EPI_FLOATS = WM * 32 * PC;
    constexpr int LDS_FLOATS = MAIN_FLOATS > EPI_FLOATS ? MAIN_FLOATS : EPI_FLOATS;
    __shared__ __attribute__((aligned(16))) float lds[LDS_FLOATS];
    float* const As0 = lds;
    float* const Bs0 = lds + NBUF * A_FLOATS;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int n_store = g.zero_pad_to > g.N ? g.zero_pad_to : g.N;
    const int n_tiles = (n_store + BN - 1) / BN;
    // Workgroup ids go round the NXCD L2 domains; the column tiles of one row slab get ids
    // that differ by NXCD, so they run on the same domain and the slab's second read hits L2.
    const int64_t hq = blockIdx.x / NXCD;
    const int64_t slab = (hq / n_tiles) * NXCD + blockIdx.x % NXCD;
    const int64_t m0 = slab * BM;
    const int n0 = (int)(hq % n_tiles) * BN;
    if (m0 >= g.M) return;

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
    const int npad = (g.N + 3) & ~3;

    uint4 ra[A_REPS], rb[B_REPS];

    // rows of the first product's A: optional indirection and a limit on the valid rows
    const int64_t a_valid = g.a_valid_rows > 0 ? g.a_valid_rows : g.M;
    int64_t arow[A_REPS];
#pragma unroll
    for (int r = 0; r < A_REPS; ++r) {
        const int64_t gm = lmin(m0 + (tid + 256 * r) / (BK / 4), a_valid - 1);
        arow[r] = g.a_rows ? (int64_t)g.a_rows[gm] : gm;
    }

    auto fetch = [&](int kt) {
        const bool second = kt >= nk1;
        const int k0 = (second ? kt - nk1 : kt) * BK;
        const int Kc = second ? g.K2 : g.K;
        const int kpad = (Kc + 3) & ~3;
        const float* Bp = second ? g.B2 : g.B;
        const int64_t ldb = second ? g.ldb2 : g.ldb;
#pragma unroll
        for (int r = 0; r < A_REPS; ++r) {
            const int f = tid + 256 * r;                 // 4-element slot in the BM x BK tile
            const int m = f / (BK / 4), kq = f % (BK / 4);
            if constexpr (VEC) {
                const int64_t gm = lmin(m0 + m, g.M - 1);
                const int kk = imin(k0 + 4 * kq, kpad - 4);
                ra[r] = second ? ldg_raw4<float>(g.A2 + gm * g.lda2 + kk)
                               : ldg_raw4<AT>((const AT*)g.A + arow[r] * g.lda + kk);
            } else {
                const int64_t gm = m0 + m;
                const bool ok2 = gm < g.M, ok1 = gm < a_valid;
                ra[r] = second ? ldg_safe4<float>(g.A2 + (ok2 ? gm : 0) * g.lda2, ok2, k0 + 4 * kq, Kc)
                               : ldg_safe4<AT>((const AT*)g.A + arow[r] * g.lda, ok1, k0 + 4 * kq, Kc);
            }
        }
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            const int f = tid + 256 * r;
            const int k = f / (BN / 4), nq = f % (BN / 4);
            if (BN * BK / 4 % 256 != 0 && f >= BN * BK / 4) { rb[r] = make_uint4(0u, 0u, 0u, 0u); continue; }
            if constexpr (VEC) {
                const int kb = imin(k0 + k, Kc - 1);
                const int nc = imin(n0 + 4 * nq, npad - 4);
                rb[r] = ldg_raw4<float>(Bp + (int64_t)kb * ldb + nc);
            } else if (g.Bt) {                           // B given transposed: element (k, n) is Bt[n][k]
                const float* Btp = second ? g.Bt2 : g.Bt;
                const int64_t ldbt = second ? g.ldbt2 : g.ldbt;
                float o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + 4 * nq + q;
                    o[q] = (k0 + k < Kc && n < g.N) ? Btp[(int64_t)n * ldbt + k0 + k] : 0.f;
                }
                rb[r] = make_uint4(__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3]));
            } else {
                const bool ok = k0 + k < Kc;
                rb[r] = ldg_safe4<float>(Bp + (int64_t)(ok ? k0 + k : 0) * ldb, ok, n0 + 4 * nq, g.N);
            }
        }
    };
    auto stage = [&](int kt) {
        const bool second = kt >= nk1;
        const int k0 = (second ? kt - nk1 : kt) * BK;
        const int Kc = second ? g.K2 : g.K;
        float* As = As0 + (NBUF == 1 ? 0 : (kt & 1)) * A_FLOATS;
        float* Bs = Bs0 + (NBUF == 1 ? 0 : (kt & 1)) * (BK * PB);
#pragma unroll
        for (int r = 0; r < A_REPS; ++r) {
            const int f = tid + 256 * r;
            const int m = f / (BK / 4), kq = f % (BK / 4);
            float v[4];
            unpack4(ra[r], VEC && A_BF16 && !second, v);
            const bool row_ok = m0 + m < (second ? g.M : a_valid);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                As[(4 * kq + q) * PA + m] = (!VEC || (row_ok && k0 + 4 * kq + q < Kc)) ? v[q] : 0.f;
        }
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            const int f = tid + 256 * r;
            const int k = f / (BN / 4), nq = f % (BN / 4);
            if (BN * BK / 4 % 256 != 0 && f >= BN * BK / 4) continue;
            float v[4];
            unpack4(rb[r], false, v);
            const bool k_ok = k0 + k < Kc;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (VEC && !(k_ok && n0 + 4 * nq + q < g.N)) v[q] = 0.f;
            *reinterpret_cast<float4*>(&Bs[k * PB + 4 * nq]) = make_float4(v[0], v[1], v[2], v[3]);
        }
    };

    fetch(0);
    stage(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) fetch(kt + 1);
        mma_step<TM, TN, PA, PB, BK>(As0 + (NBUF == 1 ? 0 : (kt & 1)) * A_FLOATS,
                                     Bs0 + (NBUF == 1 ? 0 : (kt & 1)) * (BK * PB), wm * TM * 32, wn * TN * 32, acc);
        if (NBUF == 1) __syncthreads();
        if (kt + 1 < nk) stage(kt + 1);
        __syncthreads();
    }

    nn_epilogue<VEC, WM, WN, TM, TN>(g, acc, lds, m0, n0, n_store);
}

// ------------------------------------------------------------------------------- NT (fast path of nn)
// Epilogue of an interior tile (all 128 rows < M, all columns < N, bias and row scale either
// cover the whole tile or none of it, every pointer and pitch 16-byte friendly).  A waiting
// wavefront issues an instruction only every few cycles while another one feeds the matrix
// pipe, so what counts here is the instruction count: uniform bases, 32-bit per-thread
// offsets, immediate LDS offsets, the options applied without branches (neutral operands),
// and all loads of a pass issued before its first store.
template <int WM, int WN, int TM, int TN>
__device__ __forceinline__ void nn_epilogue_interior(const GemmNNArgs& g, floatx16 (&acc)[TM][TN], float* lds, int64_t m0,
                                                     int n0, bool use_bias, bool use_rs) {
    constexpr int BN = WN * TN * 32;
    constexpr int PC = BN + 4;
    constexpr int C4 = BN / 4;                        // 16-byte columns per tile row
    // tile rows covered by one pass of the workgroup: a power of two (a pass must not straddle
    // two 32-row blocks); with BN = 96 only 192 of the 256 threads take part
    constexpr int RPI = 256 / C4 >= 32 ? 32 : 256 / C4 >= 16 ? 16 : 256 / C4 >= 8 ? 8 : 4;
    constexpr int ITS = WM * 32 / RPI;
    constexpr int ITB = ITS < 8 ? ITS : 8;            // passes whose loads are in flight together
    static_assert(32 % RPI == 0 && ITS % ITB == 0, "a pass must not straddle two 32-row blocks");
    const int tid = threadIdx.x;
    const bool active = tid < RPI * C4;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lk = lane >> 5;
    const uint32_t c4 = tid % C4, r0 = tid / C4;
    const float* const rd = lds + r0 * PC + 4 * c4;
    float* const wr = lds + (wm * 32 + 4 * lk) * PC + wn * TN * 32 + li;
    float4 b4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (use_bias && active) b4 = *reinterpret_cast<const float4*>(g.bias + (n0 - g.bias_col0) + 4 * c4);
    const float floor_v = g.relu ? 0.f : -INFINITY;
    float* const Cb = g.C + m0 * g.ldc + n0;
    float* const Rb = g.C_raw ? g.C_raw + m0 * g.ld_raw + n0 : nullptr;
    const float* const Ab = g.addend ? g.addend + m0 * g.ld_add + n0 : nullptr;
    const float* const Mb = g.mask ? g.mask + m0 * g.ld_mask + n0 : nullptr;
    const float* const Sb = use_rs ? g.rowscale + m0 : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (i > 0) __syncthreads();                   // the previous pass has been read out
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) wr[(8 * (r / 4) + (r % 4)) * PC + 32 * j] = acc[i][j][r];
        __syncthreads();
        if (!active) continue;                        // (uniform barriers above: nothing below synchronises)
#pragma unroll
        for (int it0 = 0; it0 < ITS; it0 += ITB) {
            float4 av[ITB], mv[ITB];
            float rs[ITB];
#pragma unroll
            for (int u = 0; u < ITB; ++u) {
                const int it = it0 + u;
                const uint32_t row = ((RPI * it) / 32 * TM + i) * 32 + (RPI * it) % 32 + r0;
                av[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                mv[u] = make_float4(1.f, 1.f, 1.f, 1.f);
                rs[u] = 1.f;
                if (Ab) av[u] = *reinterpret_cast<const float4*>(Ab + (row * (uint32_t)g.ld_add + 4 * c4));
                if (Mb) mv[u] = *reinterpret_cast<const float4*>(Mb + (row * (uint32_t)g.ld_mask + 4 * c4));
                if (Sb) rs[u] = Sb[row];
            }
#pragma unroll
            for (int u = 0; u < ITB; ++u) {
                const int it = it0 + u;
                const uint32_t row = ((RPI * it) / 32 * TM + i) * 32 + (RPI * it) % 32 + r0;
                float4 v = *reinterpret_cast<const float4*>(rd + RPI * it * PC);
                v.x += av[u].x + b4.x; v.y += av[u].y + b4.y; v.z += av[u].z + b4.z; v.w += av[u].w + b4.w;
                if (Rb) *reinterpret_cast<float4*>(Rb + (row * (uint32_t)g.ld_raw + 4 * c4)) = v;
                v.x = fmaxf(v.x * rs[u], floor_v); v.y = fmaxf(v.y * rs[u], floor_v);
                v.z = fmaxf(v.z * rs[u], floor_v); v.w = fmaxf(v.w * rs[u], floor_v);
                v.x = mv[u].x > 0.f ? v.x : 0.f; v.y = mv[u].y > 0.f ? v.y : 0.f;
                v.z = mv[u].z > 0.f ? v.z : 0.f; v.w = mv[u].w > 0.f ? v.w : 0.f;
                *reinterpret_cast<float4*>(Cb + (row * (uint32_t)g.ldc + 4 * c4)) = v;
            }
        }
    }
}

// Same product as gemm_nn with B supplied transposed (Bt[N x K], k contiguous), which is how
// the step keeps its weight matrices.  Both operands are then loaded along k as 16-byte
// vectors and written to LDS unchanged (row-major [row][k], pitch 36 floats: the 16-byte
// writes and reads of eight consecutive lanes fall in distinct banks).  A lane of the MFMA
// reads its four consecutive k values with one 16-byte LDS read and uses them in four
// consecutive MFMAs: within a k-tile, step (s, t) multiplies k = 8s + 4*(lane/32) + t from
// both operands, a permutation of the tile's 32 k values.  Loads use a uniform base that
// advances along k plus 32-bit per-thread offsets fixed before the loop; rows past the end of
// an operand are clamped to its last row (their products land in rows or columns the epilogue
// does not store, or zero-fills); only the last, ragged k-tile of a product is masked.
// IRREG selects the variant with gathered (a_rows) or limited (a_valid_rows) A rows.
template <typename AT, int WM, int WN, int TM, int TN, bool IRREG, int BKT, int NBUF>
__global__ __launch_bounds__(256) void gemm_nt_kernel(GemmNNArgs g) {
    if (g.M_dev) {                                    // the launch was sized by upper bounds
        g.M = *g.M_dev;
        if (g.a_valid_rows_dev) g.a_valid_rows = *g.a_valid_rows_dev;
    }
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int PK = BKT + 4;
    constexpr int KQ = BKT / 4;                       // 16-byte slots per tile row
    constexpr int RSTEP = 256 / KQ;                   // tile rows covered by one pass of the workgroup
    constexpr int A_REPS = BM * BKT / 4 / 256, B_REPS = (BN * BKT / 4 + 255) / 256;
    constexpr bool B_FULL = BN * BKT / 4 % 256 == 0;  // else the last pass over the B tile is partial (BN = 96, BKT = 16)
    constexpr bool A_BF16 = sizeof(AT) == 2;
    static_assert(BM * BKT / 4 % 256 == 0 && BKT % 8 == 0, "the A tile must fill the workgroup");
    constexpr int PC = BN + 4;
    constexpr int MAIN_FLOATS = NBUF * (BM + BN) * PK;
    constexpr int EPI_FLOATS = WM * 32 * PC;
    constexpr int LDS_FLOATS = MAIN_FLOATS > EPI_FLOATS ? MAIN_FLOATS : EPI_FLOATS;
    __shared__ __attribute__((aligned(16))) float lds[LDS_FLOATS];
    float* const As0 = lds;
    float* const Bs0 = lds + NBUF * BM * PK;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lk = lane >> 5;
    const int n_store = g.zero_pad_to > g.N ? g.zero_pad_to : g.N;
    const int n_tiles = (n_store + BN - 1) / BN;
    const int64_t hq = blockIdx.x / NXCD;
    const int64_t slab = (hq / n_tiles) * NXCD + blockIdx.x % NXCD;
    const int64_t m0 = slab * BM;
    const int n0 = (int)(hq % n_tiles) * BN;
    if (m0 >= g.M) return;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Per-thread offsets of its 16-byte slots (k offset 4*kq included).  Regular variant: 32-bit
    // offsets from the slab's first row; irregular variant: 64-bit offsets from the operand base.
    const int kq4 = 4 * (tid % KQ);
    const int trow = tid / KQ;
    const int rows_here = (int)lmin((int64_t)BM, g.M - m0);
    using aoff_t = typename std::conditional<IRREG, int64_t, uint32_t>::type;
    aoff_t aoff[A_REPS];
    uint32_t aoff2[A_REPS], boff[B_REPS], boff2[B_REPS];
    bool a_zero[A_REPS];
    const AT* a_base = (const AT*)g.A;
    if (!IRREG) a_base += m0 * g.lda;
#pragma unroll
    for (int r = 0; r < A_REPS; ++r) {
        const int lr = imin(trow + RSTEP * r, rows_here - 1);
        if (IRREG) {
            const int64_t a_valid = g.a_valid_rows > 0 ? g.a_valid_rows : g.M;
            const int64_t r1 = lmin(m0 + lr, a_valid - 1);
            aoff[r] = (aoff_t)((g.a_rows ? (int64_t)g.a_rows[r1] : r1) * g.lda + kq4);
            a_zero[r] = m0 + lr >= a_valid;
        } else {
            aoff[r] = (aoff_t)((uint32_t)lr * (uint32_t)g.lda + kq4);
            a_zero[r] = false;
        }
        aoff2[r] = (uint32_t)lr * (uint32_t)g.lda2 + kq4;
    }
#pragma unroll
    for (int r = 0; r < B_REPS; ++r) {
        const uint32_t nc = imin(n0 + trow + RSTEP * r, g.N - 1);
        boff[r] = nc * (uint32_t)g.ldbt + kq4;
        boff2[r] = nc * (uint32_t)g.ldbt2 + kq4;
    }
    const float* const a2_base = g.A2 + m0 * g.lda2;

    const int nk1 = (g.K + BKT - 1) / BKT;
    const int nk2 = (g.K2 + BKT - 1) / BKT;
    const int nk = nk1 + nk2;
    uint4 ra[A_REPS], rb[B_REPS];

    auto fetch = [&](int kt) {
        const bool second = kt >= nk1;
        const int k0 = (second ? kt - nk1 : kt) * BKT;
        const int Kc = second ? g.K2 : g.K;
        // a ragged last tile reads the operand's last whole 16-byte slot again (masked when staged)
        const int d = k0 + BKT > Kc ? imin(0, ((Kc + 3) & ~3) - 4 - k0 - kq4) : 0;
        if (second) {
            const float* pa = a2_base + k0;
            const float* pb = g.Bt2 + k0;
#pragma unroll
            for (int r = 0; r < A_REPS; ++r) ra[r] = ldg_raw4<float>(pa + (aoff2[r] + d));
#pragma unroll
            for (int r = 0; r < B_REPS; ++r) rb[r] = ldg_raw4<float>(pb + (boff2[r] + d));
        } else {
            const AT* pa = a_base + k0;
            const float* pb = g.Bt + k0;
#pragma unroll
            for (int r = 0; r < A_REPS; ++r) ra[r] = ldg_raw4<AT>(pa + (aoff[r] + d));
#pragma unroll
            for (int r = 0; r < B_REPS; ++r) rb[r] = ldg_raw4<float>(pb + (boff[r] + d));
        }
    };
    float* const as_w = As0 + trow * PK + kq4;
    float* const bs_w = Bs0 + trow * PK + kq4;
    auto stage = [&](int kt) {
        const bool second = kt >= nk1;
        const int k0 = (second ? kt - nk1 : kt) * BKT;
        const int Kc = second ? g.K2 : g.K;
        const bool ragged = k0 + BKT > Kc;                // uniform: only the last k-tile of a product
        const int kbase = k0 + kq4;
        const int buf = NBUF == 1 ? 0 : (kt & 1);
        float* As = as_w + buf * BM * PK;
        float* Bs = bs_w + buf * BN * PK;
        if (!ragged && !(A_BF16 && !second) && !IRREG) {  // common case: registers go to LDS as loaded
#pragma unroll
            for (int r = 0; r < A_REPS; ++r) *reinterpret_cast<uint4*>(As + RSTEP * r * PK) = ra[r];
#pragma unroll
            for (int r = 0; r < B_REPS; ++r)
                if (B_FULL || trow + RSTEP * r < BN) *reinterpret_cast<uint4*>(Bs + RSTEP * r * PK) = rb[r];
            return;
        }
#pragma unroll
        for (int r = 0; r < A_REPS; ++r) {
            float v[4];
            unpack4(ra[r], A_BF16 && !second, v);
            if (ragged) {
#pragma unroll
                for (int q = 0; q < 4; ++q) v[q] = kbase + q < Kc ? v[q] : 0.f;
            }
            if (IRREG && !second && a_zero[r]) { v[0] = v[1] = v[2] = v[3] = 0.f; }
            *reinterpret_cast<float4*>(As + RSTEP * r * PK) = make_float4(v[0], v[1], v[2], v[3]);
        }
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            float v[4];
            unpack4(rb[r], false, v);
            if (ragged) {
#pragma unroll
                for (int q = 0; q < 4; ++q) v[q] = kbase + q < Kc ? v[q] : 0.f;
            }
            if (B_FULL || trow + RSTEP * r < BN)
                *reinterpret_cast<float4*>(Bs + RSTEP * r * PK) = make_float4(v[0], v[1], v[2], v[3]);
        }
    };

    const float* const ap0 = As0 + (wm * TM * 32 + li) * PK + 4 * lk;
    const float* const bp0 = Bs0 + (wn * TN * 32 + li) * PK + 4 * lk;
    auto mma = [&](int kt) {
        const float* ap = ap0 + (NBUF == 1 ? 0 : (kt & 1)) * BM * PK;
        const float* bp = bp0 + (NBUF == 1 ? 0 : (kt & 1)) * BN * PK;
        float4 a4[2][TM], b4[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a4[0][i] = *reinterpret_cast<const float4*>(ap + 32 * i * PK);
#pragma unroll
        for (int j = 0; j < TN; ++j) b4[0][j] = *reinterpret_cast<const float4*>(bp + 32 * j * PK);
#pragma unroll
        for (int s = 0; s < BKT / 8; ++s) {
            const int cur = s & 1, nxt = cur ^ 1;
            if (s + 1 < BKT / 8) {
#pragma unroll
                for (int i = 0; i < TM; ++i) a4[nxt][i] = *reinterpret_cast<const float4*>(ap + 32 * i * PK + 8 * (s + 1));
#pragma unroll
                for (int j = 0; j < TN; ++j) b4[nxt][j] = *reinterpret_cast<const float4*>(bp + 32 * j * PK + 8 * (s + 1));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const float av = t == 0 ? a4[cur][i].x : t == 1 ? a4[cur][i].y : t == 2 ? a4[cur][i].z : a4[cur][i].w;
                        const float bv = t == 0 ? b4[cur][j].x : t == 1 ? b4[cur][j].y : t == 2 ? b4[cur][j].z : b4[cur][j].w;
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    fetch(0);
    stage(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) fetch(kt + 1);
        mma(kt);
        if (NBUF == 1) __syncthreads();
        if (kt + 1 < nk) stage(kt + 1);
        __syncthreads();
    }
    // interior tiles take the lean epilogue; edge tiles and awkward operands the general one
    const int bias_n = g.bias_n > 0 ? g.bias_n : g.N - g.bias_col0;
    const int rs_cols = g.rowscale_cols > 0 ? g.rowscale_cols : g.N;
    const bool bias_in = g.bias && n0 >= g.bias_col0 && n0 + BN <= g.bias_col0 + bias_n;
    const bool bias_out = !g.bias || n0 + BN <= g.bias_col0 || n0 >= g.bias_col0 + bias_n;
    const bool rs_in = g.rowscale && n0 + BN <= rs_cols;
    const bool rs_out = !g.rowscale || n0 >= rs_cols;
    const bool interior = m0 + BM <= g.M && n0 + BN <= g.N && (bias_in || bias_out) && (rs_in || rs_out) &&
                          g.ldc % 4 == 0 && ((uintptr_t)g.C % 16) == 0 &&
                          (!g.addend || (g.ld_add % 4 == 0 && ((uintptr_t)g.addend % 16) == 0)) &&
                          (!g.mask || (g.ld_mask % 4 == 0 && ((uintptr_t)g.mask % 16) == 0)) &&
                          (!g.C_raw || (g.ld_raw % 4 == 0 && ((uintptr_t)g.C_raw % 16) == 0)) &&
                          (!bias_in || (g.bias_col0 % 4 == 0 && ((uintptr_t)g.bias % 16) == 0));
    if (interior) nn_epilogue_interior<WM, WN, TM, TN>(g, acc, lds, m0, n0, bias_in, rs_in);
    else nn_epilogue<true, WM, WN, TM, TN>(g, acc, lds, m0, n0, n_store);
}

// Tile choice (measured on MI355X at M = 3e5; the nt path adds a 128 x 96 tile for 64 < N <= 96,
// e.g. two stacked 47-wide weight blocks): 128 x 128 output tiles at three workgroups per
// CU beat 128 x 256 at one; a 32-deep single-buffered k-tile is best for long reductions, a
// 16-deep double-buffered one wastes less on short or ragged K.
template <typename AT, bool VEC>
static void nn_pick(const GemmNNArgs& a, hipStream_t st) {
    const int n_eff = a.zero_pad_to > a.N ? a.zero_pad_to : a.N;
    const bool short_k = a.K <= 128 || (a.K2 > 0 && a.K2 <= 128);
    const int64_t slabs = round_up(cdiv(a.M, 128), NXCD);
    if (n_eff > 64) {
        const unsigned blocks = (unsigned)(slabs * cdiv(n_eff, 128));
        if (short_k) hipLaunchKernelGGL((gemm_nn_kernel<AT, VEC, 2, 2, 2, 2, 16, 2>), dim3(blocks), dim3(256), 0, st, a);
        else hipLaunchKernelGGL((gemm_nn_kernel<AT, VEC, 2, 2, 2, 2, 32, 1>), dim3(blocks), dim3(256), 0, st, a);
    } else if (n_eff > 32) {
        hipLaunchKernelGGL((gemm_nn_kernel<AT, VEC, 4, 1, 1, 2, 32, 1>), dim3((unsigned)slabs), dim3(256), 0, st, a);
    } else {
        hipLaunchKernelGGL((gemm_nn_kernel<AT, VEC, 4, 1, 1, 1, 32, 1>), dim3((unsigned)slabs), dim3(256), 0, st, a);
    }
}

grp_status launch_gemm_nn(const GemmNNArgs& a, hipStream_t st) {
    if (a.M == 0 || a.N == 0) return GRP_OK;
    if (a.M < 0 || a.N < 0 || a.K <= 0 || !a.A || (!a.B && !a.Bt) || !a.C) return fail(GRP_EINVAL, "gemm_nn: bad arguments");
    if (a.K2 > 0 && (!a.A2 || (!a.B2 && !a.Bt2) || a.lda2 % 4 != 0 || a.lda2 < round_up(a.K2, 4) || (uintptr_t)a.A2 % 16 != 0))
        return fail(GRP_EINVAL, "gemm_nn: second operand must be 16-byte aligned with a pitch multiple of 4");
    const int elem = a.a_bf16 ? 2 : 4;
    const bool veca = a.lda % 4 == 0 && a.lda >= round_up(a.K, 4) && (uintptr_t)a.A % (4 * elem) == 0;
    const bool vecb = a.B && a.ldb % 4 == 0 && a.ldb >= round_up(a.N, 4) && (uintptr_t)a.B % 16 == 0 &&
                      (a.K2 == 0 || (a.ldb2 % 4 == 0 && a.ldb2 >= round_up(a.N, 4) && (uintptr_t)a.B2 % 16 == 0));
    const double nn_flops = 2.0 * a.M * a.N * ((double)a.K + a.K2);
    const double nn_bytes = (double)a.M * a.K * elem + 4.0 * a.M * a.K2 + 4.0 * a.N * ((double)a.K + a.K2) +
                            4.0 * a.M * a.N * (1.0 + (a.addend ? 1.0 : 0.0) + (a.mask ? 1.0 : 0.0));
    prof_detail("[M=%lld,N=%d,K=%d+%d%s%s%s]", (long long)a.M, a.N, a.K, a.K2, a.addend ? ",add" : "", a.mask ? ",mask" : "",
                a.rowscale ? ",rs" : "");
    if (a.Bt) {
        // 32-bit element offsets inside a slab and inside Bt
        const bool small = a.lda < (1 << 23) && a.lda2 < (1 << 23) && (int64_t)a.N * a.ldbt < (1ll << 31) &&
                           (int64_t)a.N * a.ldbt2 < (1ll << 31);
        const bool ok = small && veca && a.ldbt % 4 == 0 && a.ldbt >= round_up(a.K, 4) && (uintptr_t)a.Bt % 16 == 0 &&
                        (a.K2 == 0 || (a.Bt2 && a.ldbt2 % 4 == 0 && a.ldbt2 >= round_up(a.K2, 4) && (uintptr_t)a.Bt2 % 16 == 0));
        const int n_eff = a.zero_pad_to > a.N ? a.zero_pad_to : a.N;
        const bool short_k = a.K <= 128 || (a.K2 > 0 && a.K2 <= 128);
        // one profiling name per kernel variant, so that the names line up with a kernel trace
        char pname[64];
        snprintf(pname, sizeof pname, "gemm_%s_%s_%s%s", ok ? "nt" : "nn", a.a_bf16 ? "bf16a" : "f32",
                 ok ? (a.M > 0 && n_eff > 32 && (cdiv(a.M_dev ? (a.M + 1) / 2 : a.M, 128) * cdiv(n_eff, n_eff > 96 ? 128 : n_eff > 64 ? 96 : 64) < 384 || a.K + a.K2 <= 64)
                           ? "64x64" : n_eff > 96 ? "128x128" : n_eff > 64 ? "128x96" : "128x64")
                    : (n_eff > 64 ? "128x128" : n_eff > 32 ? "128x64" : "128x32"),
                 short_k ? "_k16" : "_k32");
        ProfScope ps(pname, st, nn_flops, nn_bytes);
        if (!ok) {                                       // slow, always-safe kernel
            if (a.a_bf16) nn_pick<__hip_bfloat16, false>(a, st); else nn_pick<float, false>(a, st);
            GRP_LAUNCH_CHECK();
            return GRP_OK;
        }
        const bool rowlimit = a.a_rows != nullptr || a.a_valid_rows_dev != nullptr || (a.a_valid_rows > 0 && a.a_valid_rows < a.M);
        int tile_n = n_eff > 96 ? 128 : n_eff > 64 ? 96 : 64;
        // A product whose 128-row tiles would leave half the chip idle (mini-batch blocks) is cut into
        // 64 x 64 tiles instead: four times the workgroups, each a quarter of the work.
        // (an upper bound of M that the device will cut down counts half: sampled blocks fill about that much)
        const int64_t m_plan = a.M_dev ? (a.M + 1) / 2 : a.M;
        // A product with almost no reduction (K + K2 <= 64) is its epilogue: eight resident 64 x 64 workgroups per CU
        // overlap their loads and stores better than three of 128 x 128 (K = 16 + 16, N = 128 over 1.7e7 rows: 3.73 -> 3.32 ms).
        const bool small_tiles = n_eff > 32 && (cdiv(m_plan, 128) * cdiv(n_eff, tile_n) < 384 || a.K + a.K2 <= 64);
        if (small_tiles) tile_n = 64;
        const int64_t slabs = round_up(cdiv(a.M, small_tiles ? 64 : 128), NXCD);
        const unsigned blocks = (unsigned)(slabs * cdiv(n_eff, tile_n));
#define GRP_NT_LAUNCH2(AT, WM_, WN_, TM_, TN_, RL)                                                                        \
    do {                                                                                                                  \
        if (short_k) hipLaunchKernelGGL((gemm_nt_kernel<AT, WM_, WN_, TM_, TN_, RL, 16, 2>), dim3(blocks), dim3(256), 0, st, a); \
        else hipLaunchKernelGGL((gemm_nt_kernel<AT, WM_, WN_, TM_, TN_, RL, 32, 1>), dim3(blocks), dim3(256), 0, st, a);         \
    } while (0)
#define GRP_NT_LAUNCH(AT, WM_, WN_, TM_, TN_)                                                                       \
    do {                                                                                                            \
        if (rowlimit) GRP_NT_LAUNCH2(AT, WM_, WN_, TM_, TN_, true);                                                 \
        else GRP_NT_LAUNCH2(AT, WM_, WN_, TM_, TN_, false);                                                         \
    } while (0)
        if (small_tiles) {
            if (a.a_bf16) GRP_NT_LAUNCH(__hip_bfloat16, 2, 2, 1, 1); else GRP_NT_LAUNCH(float, 2, 2, 1, 1);
        } else if (n_eff > 96) {
            if (a.a_bf16) GRP_NT_LAUNCH(__hip_bfloat16, 2, 2, 2, 2); else GRP_NT_LAUNCH(float, 2, 2, 2, 2);
        } else if (n_eff > 64) {
            if (a.a_bf16) GRP_NT_LAUNCH(__hip_bfloat16, 4, 1, 1, 3); else GRP_NT_LAUNCH(float, 4, 1, 1, 3);
        } else {
            if (a.a_bf16) GRP_NT_LAUNCH(__hip_bfloat16, 4, 1, 1, 2); else GRP_NT_LAUNCH(float, 4, 1, 1, 2);
        }
#undef GRP_NT_LAUNCH
#undef GRP_NT_LAUNCH2
        GRP_LAUNCH_CHECK();
        return GRP_OK;
    }
    ProfScope ps(a.a_bf16 ? "gemm_nn_bf16a" : "gemm_nn_f32", st, nn_flops, nn_bytes);
    if (a.a_bf16) {
        if (veca && vecb) nn_pick<__hip_bfloat16, true>(a, st);
        else nn_pick<__hip_bfloat16, false>(a, st);
    } else {
        if (veca && vecb) nn_pick<float, true>(a, st);
        else nn_pick<float, false>(a, st);
    }
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// ------------------------------------------------------------------------------- TN
constexpr int TN_ROWS_PER_SPLIT_MIN = 128;    // node rows per split (multiple of BK): a lone workgroup spends ~3 us per 32 rows
constexpr int TN_MAX_SPLITS = 256;
constexpr int TN_TARGET_WGS = 768;            // 256 CUs x 3 resident workgroups: one full round

struct TnPlan {
    int tiles_k, tiles_n, splits;
    int64_t chunk;
    int bk_tile, bn_tile;
};

static TnPlan tn_plan(int64_t M, int K, int N, int products = 1) {
    TnPlan p;
    p.bn_tile = N > 64 ? 128 : (N > 32 ? 64 : 32);
    p.bk_tile = (K <= 64 && p.bn_tile >= 64) ? 64 : 128;      // a short K fills a 64-row tile
    p.tiles_k = (int)cdiv(K, p.bk_tile);
    p.tiles_n = (int)cdiv(N, p.bn_tile);
    // Products over very many rows are streams (a few output tiles, each workgroup a long run of rows): they want more
    // loads in flight than one round of workgroups holds, and the partial tiles cost nothing beside 10^7 rows
    // (K = 128, N = 16 over 1.7e7 rows: 3.84 -> 2.88 ms; bf16 K = 64 + 64, N = 128: 5.9 -> 5.2 ms; at 3e5 rows four times
    // the slices cost 4 %).
    const bool stream = M >= ((int64_t)1 << 23);
    int64_t s = (stream ? 4 * TN_TARGET_WGS : TN_TARGET_WGS) / (p.tiles_k * p.tiles_n * products);
    if (s > cdiv(M, TN_ROWS_PER_SPLIT_MIN)) s = cdiv(M, TN_ROWS_PER_SPLIT_MIN);
    if (s > (stream ? 8 * TN_MAX_SPLITS : TN_MAX_SPLITS)) s = stream ? 8 * TN_MAX_SPLITS : TN_MAX_SPLITS;
    if (s < 1) s = 1;
    p.chunk = round_up(cdiv(M, s), BK);
    if (p.chunk < BK) p.chunk = BK;
    p.splits = (int)cdiv(M, p.chunk);
    if (p.splits < 1) p.splits = 1;
    return p;
}

size_t gemm_tn_workspace_bytes(int64_t M, int32_t K, int32_t N) {
    // room for one product, or for two from one launch: (2K + 1) rows of N, or (K + 1) rows of 2N
    size_t need = 0;
    for (int products = 1; products <= 2; ++products) {
        const TnPlan p = tn_plan(M, K, N, products);
        if (p.splits <= 1) continue;
        const size_t rows_n = products == 1 ? (size_t)(K + 1) * N : std::max((size_t)(2 * (size_t)K + 1) * N, (size_t)(K + 1) * 2 * N);
        need = std::max(need, (size_t)p.splits * rows_n * sizeof(float));
    }
    return need;
}

// Grid: x = NXCD * tiles * ceil(splits / NXCD).  Workgroup ids are mapped so that the output
// tiles of one slice of the node dimension run on the same L2 domain (they read the same rows).
// Whole 32-row steps (all but the last of a slice) load through a uniform base plus 32-bit
// per-thread offsets and go to LDS as loaded; columns past K or N are read from clamped
// addresses and never masked, since they only reach output rows / columns that are not stored.
// GATHER: rows of A are taken through g.a_rows.  cs_out (optional): the workgroups of the
// first row of output tiles also add up the columns of B they stream (times colsum_scale).
template <typename AT, bool VEC, bool GATHER, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_tn_kernel(GemmTNArgs g, int tiles_k, int tiles_n, int dual, int splits, int64_t chunk,
                                                      float* __restrict__ out, float* __restrict__ out2, int64_t out_ld,
                                                      int64_t out_split_stride, float* __restrict__ cs_out,
                                                      int64_t cs_split_stride) {
    if (g.M_dev) {                                         // the launch was sized by an upper bound of M:
        g.M = *g.M_dev;                                    // the real rows are dealt evenly to its slices
        chunk = (g.M + splits - 1) / splits;
        chunk = (chunk + BK - 1) / BK * BK;
        if (chunk < BK) chunk = BK;
    }
    constexpr int BKA = WM * TM * 32, BN = WN * TN * 32;   // output tile: BKA (rows of C) x BN
    constexpr int PA = BKA + 4, PB = BN + 4;
    constexpr int QA = BKA / 4, QB = BN / 4;               // 16-byte slots per tile row
    constexpr int RA = 256 / QA, RB = 256 / QB;            // tile rows per pass of the workgroup
    constexpr int A_REPS = BK / RA, B_REPS = BK / RB;
    constexpr bool A_BF16 = sizeof(AT) == 2;
    static_assert(BK % RA == 0 && BK % RB == 0 && B_REPS >= 1, "tiles must fill the workgroup");
    __shared__ __attribute__((aligned(16))) float As[BK * PA];
    __shared__ __attribute__((aligned(16))) float Bs[BK * PB];

    // dual = 1: the second half of the tiles multiplies A2 instead of A; dual = 2: B2 instead of B
    const int tiles1 = tiles_k * tiles_n;
    const int tiles = tiles1 * (dual ? 2 : 1);
    const int hq = blockIdx.x / NXCD;
    const int tile_all = hq % tiles;
    const bool op2 = tile_all >= tiles1;
    const int tile = tile_all % tiles1;
    const int split = (hq / tiles) * NXCD + blockIdx.x % NXCD;
    if (split >= splits) return;
    const bool a2 = op2 && dual == 1, b2 = op2 && dual == 2;
    const void* const Aop = a2 ? (const void*)g.A2 : g.A;
    const int64_t lda = a2 ? g.lda2 : g.lda;
    const int32_t* const a_rows = a2 ? nullptr : g.a_rows;
    const float* const Bop = b2 ? g.B2 : g.B;
    const int64_t ldb = b2 ? g.ldb2 : g.ldb;
    const bool a_is_bf16 = sizeof(AT) == 2 && !a2;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int ka0 = (tile / tiles_n) * BKA;
    const int n0 = (tile % tiles_n) * BN;
    const int64_t m_begin = (int64_t)split * chunk;
    const int64_t m_end = m_begin + chunk < g.M ? m_begin + chunk : g.M;
    const int kpad = (g.K + 3) & ~3, npad = (g.N + 3) & ~3;
    const bool do_cs = cs_out != nullptr && ka0 == 0 && !op2;
    const float* const cs_scale = do_cs ? g.colsum_scale : nullptr;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int cqa = tid % QA, ma = tid / QA, cqb = tid % QB, mb = tid / QB;
    const int ca = imin(ka0 + 4 * cqa, kpad - 4), cb = imin(n0 + 4 * cqb, npad - 4);
    uint32_t aoff[A_REPS], boff[B_REPS];
#pragma unroll
    for (int r = 0; r < A_REPS; ++r) aoff[r] = (uint32_t)(ma + RA * r) * (uint32_t)lda + ca;
#pragma unroll
    for (int r = 0; r < B_REPS; ++r) boff[r] = (uint32_t)(mb + RB * r) * (uint32_t)ldb + cb;
    float* const as_w = As + ma * PA + 4 * cqa;
    float* const bs_w = Bs + mb * PB + 4 * cqb;
    float csum[4] = {0.f, 0.f, 0.f, 0.f};

    uint4 ra[A_REPS], rb[B_REPS];
    float rsc[B_REPS];
    auto fetch = [&](int64_t mt) {
        const bool full = mt + BK <= m_end;
        if (cs_scale) {
#pragma unroll
            for (int r = 0; r < B_REPS; ++r) rsc[r] = cs_scale[lmin(mt + mb + RB * r, g.M - 1)];
        }
        if (VEC && (!GATHER || !a_rows) && full) {
            const float* pb = Bop + mt * ldb;
            if (A_BF16 && !a_is_bf16) {               // the second operand of a bf16 launch is fp32
                const float* pa = (const float*)Aop + mt * lda;
#pragma unroll
                for (int r = 0; r < A_REPS; ++r) ra[r] = ldg_raw4<float>(pa + aoff[r]);
            } else {
                const AT* pa = (const AT*)Aop + mt * lda;
#pragma unroll
                for (int r = 0; r < A_REPS; ++r) ra[r] = ldg_raw4<AT>(pa + aoff[r]);
            }
#pragma unroll
            for (int r = 0; r < B_REPS; ++r) rb[r] = ldg_raw4<float>(pb + boff[r]);
            return;
        }
#pragma unroll
        for (int r = 0; r < A_REPS; ++r) {
            const int m = ma + RA * r;
            if constexpr (VEC) {
                const int64_t gm = lmin(mt + m, g.M - 1);
                const int64_t row = a_rows ? (int64_t)a_rows[gm] : gm;
                if (A_BF16 && !a_is_bf16) ra[r] = ldg_raw4<float>((const float*)Aop + row * lda + ca);
                else ra[r] = ldg_raw4<AT>((const AT*)Aop + row * lda + ca);
            } else {
                const bool ok = mt + m < m_end;
                const int64_t gm = ok ? mt + m : 0;
                const int64_t row = (a_rows && ok) ? (int64_t)a_rows[gm] : gm;
                if (A_BF16 && !a_is_bf16) ra[r] = ldg_safe4<float>((const float*)Aop + row * lda, ok, ka0 + 4 * cqa, g.K);
                else ra[r] = ldg_safe4<AT>((const AT*)Aop + row * lda, ok, ka0 + 4 * cqa, g.K);
            }
        }
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            const int m = mb + RB * r;
            if constexpr (VEC) {
                rb[r] = ldg_raw4<float>(Bop + lmin(mt + m, g.M - 1) * ldb + cb);
            } else {
                const bool ok = mt + m < m_end;
                rb[r] = ldg_safe4<float>(Bop + (ok ? mt + m : 0) * ldb, ok, n0 + 4 * cqb, g.N);
            }
        }
    };
    auto stage = [&](int64_t mt) {
        const bool full = mt + BK <= m_end;
        if (VEC && full && !a_is_bf16) {
#pragma unroll
            for (int r = 0; r < A_REPS; ++r) *reinterpret_cast<uint4*>(as_w + RA * r * PA) = ra[r];
        } else {
#pragma unroll
            for (int r = 0; r < A_REPS; ++r) {
                float v[4];
                unpack4(ra[r], VEC && a_is_bf16, v);
                if (VEC && mt + ma + RA * r >= m_end) { v[0] = v[1] = v[2] = v[3] = 0.f; }
                *reinterpret_cast<float4*>(as_w + RA * r * PA) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
#pragma unroll
        for (int r = 0; r < B_REPS; ++r) {
            float v[4];
            unpack4(rb[r], false, v);
            if (VEC && !full && mt + mb + RB * r >= m_end) { v[0] = v[1] = v[2] = v[3] = 0.f; }
            *reinterpret_cast<float4*>(bs_w + RB * r * PB) = make_float4(v[0], v[1], v[2], v[3]);
            if (do_cs) {
                const float sc = cs_scale ? rsc[r] : 1.f;
#pragma unroll
                for (int q = 0; q < 4; ++q) csum[q] += v[q] * sc;
            }
        }
    };

    if (m_begin < m_end) {
        fetch(m_begin);
        stage(m_begin);
        __syncthreads();
        for (int64_t mt = m_begin; mt < m_end; mt += BK) {
            const bool more = mt + BK < m_end;
            if (more) fetch(mt + BK);
            mma_step_interleaved<TM, TN, PA, PB, BK>(As, Bs, wm * TM * 32, wn * TN * 32, acc);
            __syncthreads();
            if (more) {
                stage(mt + BK);
                __syncthreads();
            }
        }
    }

    const int li = lane & 31, lk = lane >> 5;
    // Partial tiles (out2 null): the second product's rows follow the first's K rows (dual = 1) or its
    // columns follow the first's N columns (dual = 2).  Direct output: out2 is the second matrix.
    float* o = (op2 && out2 ? out2 : out) + (int64_t)split * out_split_stride;
    if (op2 && !out2) o += a2 ? (int64_t)g.K * out_ld : (int64_t)g.N;
    const int colb = n0 + wn * TN * 32 + TN * li;     // first of this lane's TN interleaved columns
    const bool pair = TN == 2 && out_ld % 2 == 0 && ((uintptr_t)o % 8) == 0 && colb + 1 < g.N;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ka = ka0 + wm * TM * 32 + TM * (8 * (r / 4) + 4 * lk + (r % 4)) + i;
            if (ka >= g.K) continue;
            float* orow = o + (int64_t)ka * out_ld + colb;
            if constexpr (TN == 2) {
                if (pair) { *reinterpret_cast<float2*>(orow) = make_float2(acc[i][0][r], acc[i][1][r]); continue; }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j)
                if (colb + j < g.N) orow[j] = acc[i][j][r];
        }
    if (do_cs) {                                      // the main loop ended on a barrier: As is free
        float* red = As;
#pragma unroll
        for (int q = 0; q < 4; ++q) red[mb * BN + 4 * cqb + q] = csum[q];
        __syncthreads();
        if (tid < BN) {
            float t = 0.f;
            for (int u = 0; u < RB; ++u) t += red[u * BN + tid];
            if (n0 + tid < g.N) cs_out[(int64_t)split * cs_split_stride + n0 + tid] = t;
        }
    }
}

// Where element (row, col) of the reduced partials goes: rows [0, K) x cols [0, N) -> C; with two
// products the second one's rows [K, 2K) (dual = 1) or columns [N, 2N) (dual = 2) -> C2; the last row
// holds the column sums of B (its first N columns).
__device__ __forceinline__ void tn_store(int64_t e, float val, int K, int N, int dual, float* __restrict__ C,
                                         float* __restrict__ C2, int64_t ldc, float* __restrict__ colsum_out) {
    const int width = dual == 2 ? 2 * N : N;
    const int64_t row = e / width;
    const int col = (int)(e % width);
    const int krows = dual == 1 ? 2 * K : K;
    if (row >= krows) {
        if (colsum_out && col < N) colsum_out[col] = val;
    } else if (dual == 1 && row >= K) {
        C2[(row - K) * ldc + col] = val;
    } else if (dual == 2 && col >= N) {
        C2[row * ldc + (col - N)] = val;
    } else {
        C[row * ldc + col] = val;
    }
}

// C[e] = sum_p part[p][e], p ascending.  Four partial tiles are requested before the first is
// added (the adds stay in split order, so the result is the plain sequential sum).
__global__ __launch_bounds__(256) void tn_reduce_kernel(const float* __restrict__ part, int splits, int K, int N,
                                                        int64_t part_stride, float* __restrict__ C, int64_t ldc,
                                                        float* __restrict__ colsum_out, int dual, float* __restrict__ C2,
                                                        int64_t total) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;                           // total = (rows of products + the column-sum row) x width
    const float* p0 = part + e;
    float s = 0.f;
    int p = 0;
    for (; p + 4 <= splits; p += 4) {
        const float a = p0[(int64_t)p * part_stride], b = p0[(int64_t)(p + 1) * part_stride];
        const float c = p0[(int64_t)(p + 2) * part_stride], d = p0[(int64_t)(p + 3) * part_stride];
        s += a; s += b; s += c; s += d;
    }
    for (; p < splits; ++p) s += p0[(int64_t)p * part_stride];
    tn_store(e, s, K, N, dual, C, C2, ldc, colsum_out);
}

// The same sum for partials whose stride allows 16-byte loads: a workgroup owns 64 elements,
// 16 groups of threads each add a contiguous range of splits in ascending order, and the 16
// group sums are then added in ascending order: a fixed association, so still deterministic.
__global__ __launch_bounds__(256) void tn_reduce_vec_kernel(const float* __restrict__ part, int splits, int K, int N,
                                                            int64_t part_stride, float* __restrict__ C, int64_t ldc,
                                                            float* __restrict__ colsum_out, int dual, float* __restrict__ C2,
                                                            int64_t total) {           // total: a multiple of 4
    __shared__ float4 red[16][16];
    const int c = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int64_t e = ((int64_t)blockIdx.x * 16 + c) * 4;
    const int per = (splits + 15) / 16;
    const int p_begin = grp * per, p_end = p_begin + per < splits ? p_begin + per : splits;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (e < total) {
        const float* p0 = part + e;
        int p = p_begin;
        for (; p + 4 <= p_end; p += 4) {
            const float4 a = *reinterpret_cast<const float4*>(p0 + (int64_t)p * part_stride);
            const float4 b = *reinterpret_cast<const float4*>(p0 + (int64_t)(p + 1) * part_stride);
            const float4 c4 = *reinterpret_cast<const float4*>(p0 + (int64_t)(p + 2) * part_stride);
            const float4 d = *reinterpret_cast<const float4*>(p0 + (int64_t)(p + 3) * part_stride);
            s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
            s.x += b.x; s.y += b.y; s.z += b.z; s.w += b.w;
            s.x += c4.x; s.y += c4.y; s.z += c4.z; s.w += c4.w;
            s.x += d.x; s.y += d.y; s.z += d.z; s.w += d.w;
        }
        for (; p < p_end; ++p) {
            const float4 a = *reinterpret_cast<const float4*>(p0 + (int64_t)p * part_stride);
            s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
        }
    }
    red[grp][c] = s;
    __syncthreads();
    if (grp == 0 && e < total) {
        float4 t = red[0][c];
        for (int u = 1; u < 16; ++u) { const float4 v = red[u][c]; t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w; }
        const float tv[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) tn_store(e + q, tv[q], K, N, dual, C, C2, ldc, colsum_out);
    }
}

// Scalar variant of the same scheme for strides that rule out 16-byte loads: a workgroup owns
// 64 elements, 4 groups of threads each add a contiguous quarter of the splits in ascending
// order, the 4 group sums are added in ascending order.
__global__ __launch_bounds__(256) void tn_reduce_4way_kernel(const float* __restrict__ part, int splits, int K, int N,
                                                             int64_t part_stride, float* __restrict__ C, int64_t ldc,
                                                             float* __restrict__ colsum_out, int dual, float* __restrict__ C2,
                                                             int64_t total) {
    __shared__ float red[4][64];
    const int c = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int64_t e = (int64_t)blockIdx.x * 64 + c;
    const int per = (splits + 3) / 4;
    const int p_begin = grp * per, p_end = p_begin + per < splits ? p_begin + per : splits;
    float s = 0.f;
    if (e < total) {
        const float* p0 = part + e;
        int p = p_begin;
        for (; p + 4 <= p_end; p += 4) {
            const float a = p0[(int64_t)p * part_stride], b = p0[(int64_t)(p + 1) * part_stride];
            const float c2 = p0[(int64_t)(p + 2) * part_stride], d = p0[(int64_t)(p + 3) * part_stride];
            s += a; s += b; s += c2; s += d;
        }
        for (; p < p_end; ++p) s += p0[(int64_t)p * part_stride];
    }
    red[grp][c] = s;
    __syncthreads();
    if (grp == 0 && e < total) {
        const float t = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
        tn_store(e, t, K, N, dual, C, C2, ldc, colsum_out);
    }
}

template <typename AT, bool VEC, bool GATHER>
static void tn_pick(const GemmTNArgs& a, const TnPlan& p, int dual, float* out, float* out2, int64_t out_ld, int64_t stride,
                    float* cs_out, hipStream_t st) {
    const unsigned blocks = (unsigned)(NXCD * p.tiles_k * p.tiles_n * (dual ? 2 : 1) * cdiv(p.splits, NXCD));
    dim3 grid(blocks);
#define GRP_TN_LAUNCH(WM_, WN_, TM_, TN_)                                                                              \
    hipLaunchKernelGGL((gemm_tn_kernel<AT, VEC, GATHER, WM_, WN_, TM_, TN_>), grid, dim3(256), 0, st, a, p.tiles_k,     \
                       p.tiles_n, dual, p.splits, p.chunk, out, out2, out_ld, stride, cs_out, stride)
    if (p.bk_tile == 64 && p.bn_tile == 128) GRP_TN_LAUNCH(2, 2, 1, 2);
    else if (p.bk_tile == 64) GRP_TN_LAUNCH(2, 2, 1, 1);
    else if (p.bn_tile == 128) GRP_TN_LAUNCH(2, 2, 2, 2);
    else if (p.bn_tile == 64) GRP_TN_LAUNCH(4, 1, 1, 2);
    else GRP_TN_LAUNCH(4, 1, 1, 1);
#undef GRP_TN_LAUNCH
}

// One launch computes C = A^T B and, when a second operand is given, C2 = A2^T B (a.A2) or
// C2 = A^T B2 (a.B2); C2 has C's shape and leading dimension.  A2 is fp32 and never gathered.
grp_status launch_gemm_tn(const GemmTNArgs& a, hipStream_t st) {
    if (a.K <= 0 || a.N <= 0 || a.M < 0 || !a.C) return fail(GRP_EINVAL, "gemm_tn: bad arguments");
    if (a.M > 0 && (!a.A || !a.B)) return fail(GRP_EINVAL, "gemm_tn: null operand");
    if (a.A2 && a.B2) return fail(GRP_EINVAL, "gemm_tn: at most one second operand");
    const int dual = a.A2 ? 1 : (a.B2 ? 2 : 0);
    if (dual && !a.C2) return fail(GRP_EINVAL, "gemm_tn: second product without an output");
    const TnPlan p = tn_plan(a.M, a.K, a.N, dual ? 2 : 1);
    // partial tiles of one slice: the products' rows (dual = 1: 2K) by their columns (dual = 2: 2N), then
    // one more row for the column sums of B
    const int64_t krows = dual == 1 ? 2 * (int64_t)a.K : a.K;
    const int64_t width = dual == 2 ? 2 * (int64_t)a.N : a.N;
    const int64_t stride = p.splits > 1 ? (krows + 1) * width : 0;
    const size_t need = (size_t)p.splits * stride * sizeof(float);
    if (need > a.workspace_bytes || (need && !a.workspace))
        return fail(GRP_EWORKSPACE, "gemm_tn: workspace %zu < %zu bytes", a.workspace_bytes, need);
    const int elem = a.a_bf16 ? 2 : 4;
    // vector path: 16-byte friendly operands whose 32-row steps fit 32-bit element offsets
    const bool veca = a.M > 0 && a.lda % 4 == 0 && a.lda >= round_up(a.K, 4) && (uintptr_t)a.A % (4 * elem) == 0 && a.lda < (1 << 25);
    const bool vecb = a.M > 0 && a.ldb % 4 == 0 && a.ldb >= round_up(a.N, 4) && (uintptr_t)a.B % 16 == 0 && a.ldb < (1 << 25);
    const bool veca2 = !a.A2 || (a.lda2 % 4 == 0 && a.lda2 >= round_up(a.K, 4) && (uintptr_t)a.A2 % 16 == 0 && a.lda2 < (1 << 25));
    const bool vecb2 = !a.B2 || (a.ldb2 % 4 == 0 && a.ldb2 >= round_up(a.N, 4) && (uintptr_t)a.B2 % 16 == 0 && a.ldb2 < (1 << 25));
    float* out = p.splits > 1 ? (float*)a.workspace : a.C;
    float* out2 = p.splits > 1 ? nullptr : a.C2;
    const int64_t out_ld = p.splits > 1 ? width : a.ldc;
    float* cs_out = !a.colsum_out ? nullptr : (p.splits > 1 ? (float*)a.workspace + krows * width : a.colsum_out);
    {
        prof_detail("[M=%lld,K=%d,N=%d%s%s]", (long long)a.M, a.K, a.N, a.colsum_out ? ",colsum" : "",
                    dual == 1 ? ",A2" : (dual == 2 ? ",B2" : ""));
        const double prods = dual ? 2.0 : 1.0;
        ProfScope ps(a.a_bf16 ? "gemm_tn_bf16a" : "gemm_tn_f32", st, 2.0 * prods * a.M * a.K * a.N,
                     (double)a.M * a.K * (elem + (dual == 1 ? 4 : 0)) + 4.0 * a.M * a.N * (dual == 2 ? 2 : 1) + 4.0 * prods * a.K * a.N);
        const bool vec = veca && vecb && veca2 && vecb2;
        if (a.a_bf16) {
            if (vec && !a.a_rows) tn_pick<__hip_bfloat16, true, false>(a, p, dual, out, out2, out_ld, stride, cs_out, st);
            else if (vec) tn_pick<__hip_bfloat16, true, true>(a, p, dual, out, out2, out_ld, stride, cs_out, st);
            else tn_pick<__hip_bfloat16, false, true>(a, p, dual, out, out2, out_ld, stride, cs_out, st);
        } else {
            if (vec && !a.a_rows) tn_pick<float, true, false>(a, p, dual, out, out2, out_ld, stride, cs_out, st);
            else if (vec) tn_pick<float, true, true>(a, p, dual, out, out2, out_ld, stride, cs_out, st);
            else tn_pick<float, false, true>(a, p, dual, out, out2, out_ld, stride, cs_out, st);
        }
        GRP_LAUNCH_CHECK();
    }
    if (p.splits > 1) {
        const int64_t total = krows * width + (a.colsum_out ? a.N : 0);
        ProfScope ps("gemm_tn_reduce", st, 0.0, 4.0 * total * (p.splits + 1.0));
        const float* part = (const float*)a.workspace;
        if (stride % 4 == 0 && total % 4 == 0 && (uintptr_t)a.workspace % 16 == 0 && p.splits >= 16) {
            hipLaunchKernelGGL(tn_reduce_vec_kernel, dim3((unsigned)cdiv(total, 64)), dim3(256), 0, st, part, p.splits, a.K,
                               a.N, stride, a.C, a.ldc, a.colsum_out, dual, a.C2, total);
        } else if (p.splits >= 16) {
            hipLaunchKernelGGL(tn_reduce_4way_kernel, dim3((unsigned)cdiv(total, 64)), dim3(256), 0, st, part, p.splits, a.K,
                               a.N, stride, a.C, a.ldc, a.colsum_out, dual, a.C2, total);
        } else {
            hipLaunchKernelGGL(tn_reduce_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, st, part, p.splits, a.K,
                               a.N, stride, a.C, a.ldc, a.colsum_out, dual, a.C2, total);
        }
        GRP_LAUNCH_CHECK();
    }
    return GRP_OK;
}

}  // namespace grp

extern "C" grp_status grp_gemm_nn(int64_t M, int32_t N, int32_t K, const void* A, int64_t lda, int32_t a_dtype,
                                  const float* B, int64_t ldb, float* C, int64_t ldc, void* stream) {
    if (M < 0 || N <= 0 || K <= 0 || lda < K || ldb < N || ldc < N) return grp::fail(GRP_EINVAL, "grp_gemm_nn: bad shape");
    if (!B || (M > 0 && (!A || !C))) return grp::fail(GRP_EINVAL, "grp_gemm_nn: null argument");
    if (M == 0) return GRP_OK;                          // no rows: nothing to compute
    grp::GemmNNArgs a;
    a.M = M; a.N = N; a.K = K; a.A = A; a.lda = lda; a.a_bf16 = a_dtype == GRP_DTYPE_BF16;
    a.B = B; a.ldb = ldb; a.C = C; a.ldc = ldc;
    return grp::launch_gemm_nn(a, (hipStream_t)stream);
}

extern "C" grp_status grp_gemm_nt(int64_t M, int32_t N, int32_t K, const void* A, int64_t lda, int32_t a_dtype,
                                  const float* Bt, int64_t ldbt, float* C, int64_t ldc, void* stream) {
    if (!Bt || (M > 0 && (!A || !C))) return grp::fail(GRP_EINVAL, "grp_gemm_nt: null argument");
    if (M < 0 || N <= 0 || K <= 0 || lda < K || ldbt < K || ldc < N) return grp::fail(GRP_EINVAL, "grp_gemm_nt: bad shape");
    if (M == 0) return GRP_OK;                          // no rows: nothing to compute
    grp::GemmNNArgs a;
    a.M = M; a.N = N; a.K = K; a.A = A; a.lda = lda; a.a_bf16 = a_dtype == GRP_DTYPE_BF16;
    a.Bt = Bt; a.ldbt = ldbt; a.C = C; a.ldc = ldc;
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
