// Isolated k-hop neighbour sampling inside one partition (mini-batch mode), on the GPU.
//
// Per destination node: all local in-edges if there are at most `fanout`, otherwise the
// `fanout` in-edges with the smallest 64-bit key (ties by position), kept in position order.
//   key = M(M(M(M(M(sampler_seed) ^ batch_id) ^ layer) ^ global_id(v)) ^ j),
//   M(x) = SplitMix64 finaliser of x + 0x9E3779B97F4A7C15, j = position in v's CSR row.
// The keys depend only on (seed, batch, layer, node, position), so the selection is
// independent of scheduling and bit-reproducible.
//
// Selection for a row of d > fanout edges (one wavefront per row, four for very long rows): keys are uniform, so the
// fanout-th smallest is near fanout/d * 2^64; edges with key <= T (T = 4x that) are compacted
// into an LDS candidate list, T is doubled / halved until the list holds between fanout and
// SAMPLE_CAND entries (it does at the first try with overwhelming probability), and the
// fanout smallest candidates are extracted by repeated wave-wide minimum.  Any edge outside
// the list has a key above every listed one, so the result is exact.
//
// Layers are built from the seeds inwards.  Above the input layer, new source nodes are
// found with a per-node flag array and a prefix sum (ascending local id), sources are
// relabelled to block-local indices and the block is also stored transposed (by radix
// sort) for the backward pass.  The input layer keeps partition-local ids: they index the
// feature matrix directly, so no feature rows are copied.
#include "common.h"

#include <vector>

namespace grp {

constexpr int SAMPLE_CAND = 512;
constexpr int SAMPLE_MAX_FANOUT = 64;

__host__ __device__ __forceinline__ uint64_t mixM(uint64_t x) {
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct KeyJ {
    uint64_t key;
    int32_t j;
};
__device__ __forceinline__ bool less_kj(uint64_t k1, int32_t j1, uint64_t k2, int32_t j2) {
    return k1 < k2 || (k1 == k2 && j1 < j2);
}

__device__ __forceinline__ void wave_min_kj(uint64_t& k, int32_t& j) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t ok = __shfl_xor(k, o, 64);
        const int32_t oj = __shfl_xor(j, o, 64);
        if (less_kj(ok, oj, k, j)) { k = ok; j = oj; }
    }
}

__global__ __launch_bounds__(256) void sample_count_kernel(const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ dst_nodes, int64_t n_dst,
                                                           int fanout, int64_t* __restrict__ cnt /*[n_dst+1]*/,
                                                           int32_t* __restrict__ cnt32 /*[n_dst] or null*/) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i > n_dst) return;
    if (i == n_dst) { cnt[i] = 0; return; }
    const int64_t v = dst_nodes[i];
    const int64_t d = rowptr[v + 1] - rowptr[v];
    const int64_t c = d < fanout ? d : fanout;
    cnt[i] = c;
    if (cnt32) cnt32[i] = (int32_t)c;
}

// One workgroup of SAMPLE_WAVES wavefronts per destination row.  Rows of at most SAMPLE_MULTI edges
// are handled by the first wavefront alone (the others leave at once); longer rows (the hubs of a
// skewed graph, 10^5 edges and more) are scanned by the whole workgroup, which appends its
// candidates to the LDS list through an LDS counter.  The list's order then depends on timing,
// the selection does not: it is the `fanout` smallest (key, position) pairs.
constexpr int SAMPLE_WAVES = 4;
constexpr int SAMPLE_MULTI = 2048;

__global__ __launch_bounds__(64 * SAMPLE_WAVES) void sample_select_kernel(const int64_t* __restrict__ rowptr,
                                                                          const int32_t* __restrict__ col,
                                                                          const int64_t* __restrict__ l2g,
                                                                          const int32_t* __restrict__ dst_nodes,
                                                                          int fanout, uint64_t h2,
                                                                          const int64_t* __restrict__ out_ptr,
                                                                          int32_t* __restrict__ out_idx) {
    __shared__ uint64_t ckey[SAMPLE_CAND];
    __shared__ int32_t cj[SAMPLE_CAND];
    __shared__ int32_t sel[SAMPLE_MAX_FANOUT];
    __shared__ int cand_count;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t v = dst_nodes[blockIdx.x];
    const int64_t b = rowptr[v];
    const int64_t d = rowptr[v + 1] - b;
    const int64_t o = out_ptr[blockIdx.x];
    const bool multi = d > SAMPLE_MULTI;                 // uniform over the workgroup
    if (!multi && wave > 0) return;
    if (d <= fanout) {
        for (int64_t j = lane; j < d; j += 64) out_idx[o + j] = col[b + j];
        return;
    }
    const uint64_t h3 = mixM(h2 ^ (uint64_t)l2g[v]);

    uint64_t T = ~0ull;
    if (d > SAMPLE_CAND) T = (uint64_t)((4.0 * (double)fanout / (double)d) * 18446744073709551615.0);
    int count = 0;
    bool have = false;
    for (int iter = 0; iter < 96 && !have; ++iter) {
        if (multi) {
            if (tid == 0) cand_count = 0;
            __syncthreads();
            for (int64_t j = tid; j < d; j += 64 * SAMPLE_WAVES) {
                const uint64_t key = mixM(h3 ^ (uint64_t)j);
                if (key <= T) {
                    const int pos = atomicAdd(&cand_count, 1);
                    if (pos < SAMPLE_CAND) { ckey[pos] = key; cj[pos] = (int32_t)j; }
                }
            }
            __syncthreads();
            count = cand_count;
            __syncthreads();                             // everyone has read it before the next reset
        } else {
            count = 0;
            for (int64_t base = 0; base < d; base += 64) {
                const int64_t j = base + lane;
                const bool valid = j < d;
                const uint64_t key = valid ? mixM(h3 ^ (uint64_t)j) : ~0ull;
                const bool take = valid && key <= T;
                const unsigned long long m = __ballot(take);
                const int pos = count + __popcll(m & ((1ull << lane) - 1ull));
                if (take && pos < SAMPLE_CAND) { ckey[pos] = key; cj[pos] = (int32_t)j; }
                count += __popcll(m);
            }
        }
        if (count < fanout) T = T > (~0ull >> 1) ? ~0ull : (T << 1) | 1ull;
        else if (count > SAMPLE_CAND) T >>= 1;
        else have = true;
    }
    // The first wavefront finishes the row.  No workgroup barrier from here on (the others have
    // left); the candidates were published by the scan's last barrier, and a single wavefront's
    // LDS accesses complete in program order.
    if (wave > 0) return;
    __builtin_amdgcn_wave_barrier();

    uint64_t last_k = 0;
    int32_t last_j = -1;
    for (int r = 0; r < fanout; ++r) {
        uint64_t bk = ~0ull;
        int32_t bj = 0x7FFFFFFF;
        if (have) {
            for (int c = lane; c < count; c += 64) {
                const uint64_t k = ckey[c];
                const int32_t j = cj[c];
                if ((r == 0 || less_kj(last_k, last_j, k, j)) && less_kj(k, j, bk, bj)) { bk = k; bj = j; }
            }
        } else {                                         // exact fallback: rescan the whole row
            for (int64_t j = lane; j < d; j += 64) {
                const uint64_t k = mixM(h3 ^ (uint64_t)j);
                if ((r == 0 || less_kj(last_k, last_j, k, (int32_t)j)) && less_kj(k, (int32_t)j, bk, bj)) { bk = k; bj = (int32_t)j; }
            }
        }
        wave_min_kj(bk, bj);
        last_k = bk;
        last_j = bj;
        if (lane == 0) sel[r] = bj;
    }
    __builtin_amdgcn_wave_barrier();
    if (lane < fanout) {                                 // positions are distinct: rank = output slot
        const int32_t myj = sel[lane];
        int rank = 0;
        for (int u = 0; u < fanout; ++u) rank += sel[u] < myj ? 1 : 0;
        out_idx[o + rank] = col[b + myj];
    }
}

__global__ __launch_bounds__(256) void mark_dst_kernel(const int32_t* __restrict__ dst_nodes, int64_t n_dst,
                                                       int32_t* __restrict__ mark, int32_t* __restrict__ src_nodes) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_dst) return;
    mark[dst_nodes[i]] = (int32_t)i + 1;
    src_nodes[i] = dst_nodes[i];
}

__global__ __launch_bounds__(256) void flag_new_kernel(const int32_t* __restrict__ idx_local,
                                                       const int64_t* __restrict__ nnz_dev,
                                                       const int32_t* __restrict__ mark, int32_t* __restrict__ newflag) {
    const int64_t nnz = *nnz_dev;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * 256) {
        const int32_t u = idx_local[e];
        if (mark[u] == 0) newflag[u] = 1;                // idempotent plain store
    }
}

__global__ __launch_bounds__(256) void assign_new_kernel(int64_t n, const int32_t* __restrict__ newflag,
                                                         const int32_t* __restrict__ newpos, int64_t n_dst,
                                                         int32_t* __restrict__ mark, int32_t* __restrict__ src_nodes) {
    const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= n || !newflag[u]) return;
    const int32_t p = (int32_t)n_dst + newpos[u];
    src_nodes[p] = (int32_t)u;
    mark[u] = p + 1;
}

// idx_blk[e] = block-local index of the source; keyT[e] = (source index << 32) | destination index
__global__ __launch_bounds__(256) void relabel_kernel(const int64_t* __restrict__ ptr, int64_t n_dst,
                                                      const int32_t* __restrict__ idx_local,
                                                      const int32_t* __restrict__ mark, int32_t* __restrict__ idx_blk,
                                                      uint64_t* __restrict__ keyT) {
    const int64_t i = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (i >= n_dst) return;
    const int lane = threadIdx.x & 63;
    for (int64_t e = ptr[i] + lane; e < ptr[i + 1]; e += 64) {
        const int32_t s = mark[idx_local[e]] - 1;
        idx_blk[e] = s;
        keyT[e] = ((uint64_t)(uint32_t)s << 32) | (uint64_t)i;
    }
}

__global__ __launch_bounds__(256) void clear_marks_kernel(const int32_t* __restrict__ src_nodes, int64_t n_src,
                                                          int32_t* __restrict__ mark, int32_t* __restrict__ newflag) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_src) return;
    const int32_t u = src_nodes[i];
    mark[u] = 0;
    newflag[u] = 0;
}

__global__ __launch_bounds__(256) void inv_count_kernel(const int64_t* __restrict__ ptr, int64_t n_dst,
                                                        float* __restrict__ inv) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_dst) return;
    const int64_t c = ptr[i + 1] - ptr[i];
    inv[i] = 1.0f / (float)(c > 1 ? c : 1);
}

void sampler_bounds(int64_t n, int64_t n_seeds, const int32_t* fanouts, int k, SamplerBounds* out) {
    int64_t nd = n_seeds;
    for (int l = k - 1; l >= 0; --l) {
        out->dst[l] = nd;
        out->nnz[l] = nd * fanouts[l];
        int64_t ns = nd + out->nnz[l];
        if (ns > n) ns = n;
        out->src[l] = ns;
        nd = ns;
    }
}

struct SamplerLayerBufs {
    int64_t* cnt;        // [dst+1] counts, then in place the block row pointer
    int64_t* ptr;        // [dst+1]
    int32_t* cnt32;      // [dst]
    int32_t* idx_local;  // [nnz] partition-local source ids
    int32_t* idx_blk;    // [nnz] block-local (layers >= 1)
    int32_t* src_nodes;  // [src] (layers >= 1)
    uint64_t *keys, *keys_sorted;  // [nnz] (layers >= 1)
    int64_t* ptrT;       // [src+1]
    int32_t* idxT;       // [nnz]
    float* inv_in;       // [dst]
    int32_t *lr_row, *lr_first;    // long rows of the transposed block
    int64_t *lr_cb, *lr_ce;
    int64_t lr_cap_long, lr_cap_chunks;
};

struct SamplerBufs {
    SamplerLayerBufs L[GRP_MAX_LAYERS];
    int32_t *mark, *newflag, *newpos;   // [n], [n+1], [n+1]
    void *scan_tmp, *sort_tmp;
    size_t scan_bytes, sort_bytes;
    size_t total;
};

static SamplerBufs carve_sampler(int64_t n, const SamplerBounds& b, int k, void* ws, size_t ws_bytes) {
    SamplerBufs s;
    Bump bump(ws, ws_bytes);
    int64_t max_nnz = 1, max_dst = 1;
    for (int l = 0; l < k; ++l) {
        SamplerLayerBufs& L = s.L[l];
        L.cnt = bump.take<int64_t>((size_t)b.dst[l] + 1);
        L.ptr = bump.take<int64_t>((size_t)b.dst[l] + 1);
        L.cnt32 = bump.take<int32_t>((size_t)b.dst[l]);
        L.idx_local = bump.take<int32_t>((size_t)b.nnz[l]);
        L.inv_in = bump.take<float>((size_t)b.dst[l]);
        if (b.dst[l] > max_dst) max_dst = b.dst[l];
        if (l > 0) {
            L.idx_blk = bump.take<int32_t>((size_t)b.nnz[l]);
            L.src_nodes = bump.take<int32_t>((size_t)b.src[l]);
            L.keys = bump.take<uint64_t>((size_t)b.nnz[l]);
            L.keys_sorted = bump.take<uint64_t>((size_t)b.nnz[l]);
            L.ptrT = bump.take<int64_t>((size_t)b.src[l] + 1);
            L.idxT = bump.take<int32_t>((size_t)b.nnz[l]);
            L.lr_cap_long = b.nnz[l] / SPMM_LONG_ROW + 1;
            L.lr_cap_chunks = b.nnz[l] / SPMM_CHUNK + L.lr_cap_long + 1;
            L.lr_row = bump.take<int32_t>((size_t)L.lr_cap_long);
            L.lr_first = bump.take<int32_t>((size_t)L.lr_cap_long + 1);
            L.lr_cb = bump.take<int64_t>((size_t)L.lr_cap_chunks);
            L.lr_ce = bump.take<int64_t>((size_t)L.lr_cap_chunks);
            if (b.nnz[l] > max_nnz) max_nnz = b.nnz[l];
        } else {
            L.idx_blk = nullptr; L.src_nodes = nullptr; L.keys = L.keys_sorted = nullptr;
            L.ptrT = nullptr; L.idxT = nullptr; L.lr_row = L.lr_first = nullptr; L.lr_cb = L.lr_ce = nullptr;
            L.lr_cap_long = L.lr_cap_chunks = 0;
        }
    }
    s.mark = bump.take<int32_t>((size_t)n);
    s.newflag = bump.take<int32_t>((size_t)n + 1);
    s.newpos = bump.take<int32_t>((size_t)n + 1);
    s.scan_bytes = scan_temp_bytes(n + 1 > max_dst + 1 ? n + 1 : max_dst + 1);
    s.scan_tmp = bump.take<char>(s.scan_bytes);
    s.sort_bytes = k > 1 ? sort_keys_temp_bytes(max_nnz) : 0;
    s.sort_tmp = bump.take<char>(s.sort_bytes);
    s.total = bump.total();
    return s;
}

size_t sampler_workspace_bytes(int64_t n, const SamplerBounds& b, int k) { return carve_sampler(n, b, k, nullptr, 0).total; }

static unsigned blocks_for(int64_t work) {
    int64_t b = cdiv(work > 0 ? work : 1, 256);
    return (unsigned)(b > 65536 ? 65536 : b);
}

grp_status sample_blocks(const grp_partition_t* part, const grp_step_opts* o, int k, void* ws, size_t ws_bytes,
                         Block* blocks, LongRows* long_bwd_store, const int64_t** nnz_parts_dev,
                         const int32_t** seed_counts_dev, hipStream_t st) {
    const int64_t n = part->n;
    if (o->n_seeds < 1 || !o->seeds) return fail(GRP_EINVAL, "mini-batch: need at least one seed node");
    for (int l = 0; l < k; ++l)
        if (o->fanouts[l] < 1 || o->fanouts[l] > SAMPLE_MAX_FANOUT)
            return fail(GRP_EINVAL, "mini-batch: fanout %d outside [1, %d]", o->fanouts[l], SAMPLE_MAX_FANOUT);
    SamplerBounds bd;
    sampler_bounds(n, o->n_seeds, o->fanouts, k, &bd);
    SamplerBufs s = carve_sampler(n, bd, k, ws, ws_bytes);
    if (s.total > ws_bytes) return fail(GRP_EWORKSPACE, "mini-batch: sampler workspace %zu < %zu", ws_bytes, s.total);

    if (k > 1) {                                         // the flag arrays start at zero
        GRP_TRY(launch_fill_zero(s.mark, (size_t)n * sizeof(int32_t), st));
        GRP_TRY(launch_fill_zero(s.newflag, ((size_t)n + 1) * sizeof(int32_t), st));
    }
    const uint64_t h1 = mixM(mixM(o->sampler_seed) ^ o->batch_id);
    const int32_t* dst_nodes = o->seeds;
    int64_t n_dst = o->n_seeds;
    for (int l = k - 1; l >= 0; --l) {
        SamplerLayerBufs& L = s.L[l];
        const int f = o->fanouts[l];
        hipLaunchKernelGGL(sample_count_kernel, dim3(blocks_for(n_dst + 1)), dim3(256), 0, st, part->rowptr, dst_nodes, n_dst,
                           f, L.cnt, L.cnt32);
        GRP_LAUNCH_CHECK();
        GRP_TRY(exclusive_scan_i64(s.scan_tmp, s.scan_bytes, L.cnt, L.ptr, n_dst + 1, st));
        {
            ProfScope ps("sample_select", st);
            hipLaunchKernelGGL(sample_select_kernel, dim3((unsigned)n_dst), dim3(64 * SAMPLE_WAVES), 0, st, part->rowptr, part->col, part->l2g,
                               dst_nodes, f, mixM(h1 ^ (uint64_t)l), (const int64_t*)L.ptr, L.idx_local);
            GRP_LAUNCH_CHECK();
        }
        hipLaunchKernelGGL(inv_count_kernel, dim3(blocks_for(n_dst)), dim3(256), 0, st, (const int64_t*)L.ptr, n_dst, L.inv_in);
        GRP_LAUNCH_CHECK();

        Block& B = blocks[l];
        B.n_dst = n_dst;
        B.dst_nodes = dst_nodes;
        B.ptr = L.ptr;
        B.inv_in = L.inv_in;
        B.long_fwd = nullptr;                            // rows hold at most `fanout` edges
        nnz_parts_dev[l] = L.ptr + n_dst;
        if (l == k - 1) *seed_counts_dev = L.cnt32;
        if (l == 0) {
            B.idx = L.idx_local;
            B.n_in = n;
            B.self_rows = dst_nodes;
            B.ptrT = nullptr; B.idxT = nullptr; B.long_bwd = nullptr;
            B.nnz = bd.nnz[0];                           // upper bound; only the profiler reads it
            break;
        }
        // new source nodes in ascending local id, block-local relabelling, transposed block
        hipLaunchKernelGGL(mark_dst_kernel, dim3(blocks_for(n_dst)), dim3(256), 0, st, dst_nodes, n_dst, s.mark, L.src_nodes);
        GRP_LAUNCH_CHECK();
        hipLaunchKernelGGL(flag_new_kernel, dim3(blocks_for(bd.nnz[l])), dim3(256), 0, st, (const int32_t*)L.idx_local,
                           (const int64_t*)(L.ptr + n_dst), (const int32_t*)s.mark, s.newflag);
        GRP_LAUNCH_CHECK();
        GRP_TRY(exclusive_scan_i32(s.scan_tmp, s.scan_bytes, s.newflag, s.newpos, n + 1, st));
        hipLaunchKernelGGL(assign_new_kernel, dim3(blocks_for(n)), dim3(256), 0, st, n, (const int32_t*)s.newflag,
                           (const int32_t*)s.newpos, n_dst, s.mark, L.src_nodes);
        GRP_LAUNCH_CHECK();
        hipLaunchKernelGGL(relabel_kernel, dim3((unsigned)cdiv(n_dst, 4)), dim3(256), 0, st, (const int64_t*)L.ptr, n_dst,
                           (const int32_t*)L.idx_local, (const int32_t*)s.mark, L.idx_blk, L.keys);
        GRP_LAUNCH_CHECK();
        int64_t host_nnz = 0;
        int32_t host_new = 0;
        GRP_HIP(hipMemcpyAsync(&host_nnz, L.ptr + n_dst, sizeof(int64_t), hipMemcpyDeviceToHost, st));
        GRP_HIP(hipMemcpyAsync(&host_new, s.newpos + n, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
        const int64_t n_src = n_dst + host_new;
        if (host_nnz > bd.nnz[l] || n_src > bd.src[l]) return fail(GRP_EHIP, "mini-batch: sampled block exceeds its bounds");
        hipLaunchKernelGGL(clear_marks_kernel, dim3(blocks_for(n_src)), dim3(256), 0, st, (const int32_t*)L.src_nodes, n_src,
                           s.mark, s.newflag);
        GRP_LAUNCH_CHECK();
        int bits = 1;
        while (bits < 32 && ((int64_t)1 << bits) < n_src) ++bits;
        GRP_TRY(sort_keys_u64(s.sort_tmp, s.sort_bytes, L.keys, L.keys_sorted, host_nnz, 32u + (unsigned)bits, st));
        GRP_TRY(launch_csr_from_sorted_keys(L.keys_sorted, host_nnz, n_src, L.ptrT, L.idxT, st));
        LongRows& lr = long_bwd_store[l];
        lr.long_row = L.lr_row; lr.long_first = L.lr_first; lr.chunk_begin = L.lr_cb; lr.chunk_end = L.lr_ce;
        GRP_TRY(build_long_rows_into(L.ptrT, n_src, &lr, L.lr_cap_long, L.lr_cap_chunks, st));
        B.idx = L.idx_blk;
        B.n_in = n_src;
        B.nnz = host_nnz;
        B.self_rows = nullptr;
        B.ptrT = L.ptrT;
        B.idxT = L.idxT;
        B.long_bwd = &lr;
        dst_nodes = L.src_nodes;
        n_dst = n_src;
    }
    return GRP_OK;
}

}  // namespace grp
