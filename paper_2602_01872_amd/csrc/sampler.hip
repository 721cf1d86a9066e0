// Isolated k-hop neighbour sampling inside one partition (mini-batch mode), on the GPU.
//
// Per destination node v with d local in-edges: all of them if d <= fanout, otherwise a uniformly
// random fanout-subset of the positions 0..d-1 of its CSR row, grown one element at a time:
//   for t = 0..fanout-1:  top = d - fanout + t,  r = floor(u_t * (top + 1) / 2^64),
//                         the subset gains r if it does not hold r yet, else top;
//   u_t = M(M(M(M(M(sampler_seed) ^ batch_id) ^ layer) ^ global_id(v)) ^ t),
//   M(x) = SplitMix64 finaliser of x + 0x9E3779B97F4A7C15.
// Every subset is equally likely; the draws depend only on (seed, batch, layer, node, t), so the
// selection is independent of scheduling and bit-reproducible; and a row costs O(fanout) whatever
// its length (the hub rows of a skewed graph hold 10^5..10^6 edges).  The chosen edges are kept
// in position order.
//
// Layers are built from the seeds inwards.  Above the input layer, new source nodes are
// found with a node bitmap and a prefix sum over its words (ascending local id), sources are
// relabelled to block-local indices and the block is also stored transposed (by radix
// sort) for the backward pass.  The input layer keeps partition-local ids: they index the
// feature matrix directly, so no feature rows are copied.
//
// The host never learns a block's sizes.  They depend on the draws, so they exist on the device only
// (`sizes`, four numbers per layer); every launch is sized by the upper bounds that follow from the seeds
// and fanouts, reads the real sizes from device memory and leaves the slots between the two in a state
// that is harmless to read (empty rows, sentinel keys).  A step is therefore queued without waiting for
// the device, and can be captured in a graph.
#include "common.h"

#include <vector>

namespace grp {

constexpr int SAMPLE_MAX_FANOUT = 64;         // one lane of a wavefront per chosen edge
// A layer's sizes on the device: destinations, sources (destinations first, then the newly reached nodes),
// edges, newly reached nodes.
enum { SZ_DST = 0, SZ_SRC = 1, SZ_NNZ = 2, SZ_NEW = 3, SZ_PER_LAYER = 4 };

// Per destination row: the number of edges it keeps and 1 / max(that, 1); above the input layer also
// the row's place in the block's source list (destinations come first, in order) and in the node -> block
// index map.  The elements of `cnt` from n_dst to the bound are zero and close the prefix sum.
__global__ __launch_bounds__(256) void sample_count_kernel(const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ dst_nodes,
                                                           const int64_t* __restrict__ n_dst_dev, int64_t bound,
                                                           int fanout, int64_t* __restrict__ cnt /*[bound+1]*/,
                                                           int32_t* __restrict__ cnt32 /*[n_dst] or null*/,
                                                           float* __restrict__ inv /*[n_dst]*/,
                                                           int32_t* __restrict__ mark /*[n] or null*/,
                                                           int32_t* __restrict__ src_nodes /*[>= n_dst] or null*/) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i > bound) return;
    if (i >= *n_dst_dev) { cnt[i] = 0; return; }          // rows between the real count and the bound are empty
    const int32_t v = dst_nodes[i];
    const int64_t d = rowptr[v + 1] - rowptr[v];
    const int64_t c = d < fanout ? d : fanout;
    cnt[i] = c;
    if (cnt32) cnt32[i] = (int32_t)c;
    inv[i] = 1.0f / (float)(c > 1 ? c : 1);
    if (mark) {
        mark[v] = (int32_t)i + 1;
        src_nodes[i] = v;
    }
}

// Seeds outside [0, n) are counted (`bad`, zero on entry; the step's statistics report it) and replaced by
// node 0 in the copy the sampler works on, so that no kernel reads outside the partition.  Also states the
// seed-side block's number of destinations.
__global__ __launch_bounds__(256) void check_seeds_kernel(const int32_t* __restrict__ seeds, int64_t n_seeds, int64_t n,
                                                          int32_t* __restrict__ safe, int64_t* __restrict__ bad,
                                                          int64_t* __restrict__ n_dst_out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i == 0) *n_dst_out = n_seeds;
    if (i >= n_seeds) return;
    const int32_t v = seeds[i];
    const bool ok = v >= 0 && (int64_t)v < n;
    safe[i] = ok ? v : 0;
    if (!ok) atomicAdd((unsigned long long*)bad, 1ull);
}

// One wavefront per destination row.  Lane t computes draw t; the subset is grown in `fanout`
// wave-uniform steps with lane t keeping the t-th element; each lane then finds the rank of its
// element (they are distinct) and writes the edge to that output slot.
constexpr int SAMPLE_ROWS_PER_WG = 4;

__global__ __launch_bounds__(64 * SAMPLE_ROWS_PER_WG) void sample_select_kernel(const int64_t* __restrict__ rowptr,
                                                                                const int32_t* __restrict__ col,
                                                                                const int64_t* __restrict__ l2g,
                                                                                const int32_t* __restrict__ dst_nodes,
                                                                                int64_t* __restrict__ sizes /*of this layer*/,
                                                                                int fanout, uint64_t h0 /*M(sampler_seed)*/,
                                                                                uint64_t batch_id,
                                                                                const uint64_t* __restrict__ batch_id_dev,
                                                                                int layer,
                                                                                const int64_t* __restrict__ out_ptr,
                                                                                int32_t* __restrict__ out_idx) {
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * SAMPLE_ROWS_PER_WG + (threadIdx.x >> 6);
    const int64_t n_dst = sizes[SZ_DST];
    if (blockIdx.x == 0 && threadIdx.x == 0) sizes[SZ_NNZ] = out_ptr[n_dst];      // the block's number of edges
    if (i >= n_dst) return;                              // uniform over the wavefront
    const int64_t v = dst_nodes[i];
    const int64_t b = rowptr[v];
    const int64_t d = rowptr[v + 1] - b;
    const int64_t o = out_ptr[i];
    if (d <= fanout) {
        for (int64_t j = lane; j < d; j += 64) out_idx[o + j] = col[b + j];
        return;
    }
    const uint64_t h2 = mixM(mixM(h0 ^ (batch_id_dev ? *batch_id_dev : batch_id)) ^ (uint64_t)layer);
    const uint64_t h3 = mixM(h2 ^ (uint64_t)l2g[v]);
    const uint64_t my_bits = mixM(h3 ^ (uint64_t)lane);
    int64_t mine = -1;                                   // lane t < fanout: the t-th element of the subset
    for (int t = 0; t < fanout; ++t) {
        const uint64_t u = __shfl(my_bits, t, 64);
        const int64_t top = d - fanout + t;
        int64_t r = (int64_t)__umul64hi(u, (uint64_t)(top + 1));
        if (__ballot(lane < t && mine == r)) r = top;    // r is taken: top cannot be (earlier elements are below it)
        if (lane == t) mine = r;
    }
    int rank = 0;
    for (int t = 0; t < fanout; ++t) rank += __shfl(mine, t, 64) < mine ? 1 : 0;
    if (lane < fanout) out_idx[o + rank] = col[b + mine];
}

// New source nodes are collected in a bitmap over the partition's nodes (one bit each): the words'
// population counts are prefix-summed and every non-empty word then numbers its own nodes, which
// yields them in ascending local id while touching n / 8 bytes instead of per-node flag arrays.
__global__ __launch_bounds__(256) void flag_new_kernel(const int32_t* __restrict__ idx_local,
                                                       const int64_t* __restrict__ nnz_dev,
                                                       const int32_t* __restrict__ mark, uint32_t* __restrict__ bits) {
    const int64_t nnz = *nnz_dev;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * 256) {
        const int32_t u = idx_local[e];
        if (mark[u] == 0) atomicOr(&bits[u >> 5], 1u << (u & 31));
    }
}

// Also clears the bitmap for the next layer.
__global__ __launch_bounds__(256) void assign_new_kernel(int64_t n_words, uint32_t* __restrict__ bits,
                                                         const int32_t* __restrict__ wpos,
                                                         const int64_t* __restrict__ n_dst_dev,
                                                         int32_t* __restrict__ mark, int32_t* __restrict__ src_nodes) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_words) return;
    uint32_t w = bits[i];
    if (!w) return;
    bits[i] = 0;
    int32_t p = (int32_t)*n_dst_dev + wpos[i];
    while (w) {
        const int32_t u = (int32_t)(i * 32) + (__ffs(w) - 1);
        src_nodes[p] = u;
        mark[u] = ++p;
        w &= w - 1;
    }
}

// idx_blk[e] = block-local index of the source; keyT[e] = (source index << 32) | destination index.  The key
// slots from the real number of edges to the bound receive `sentinel` (a source index above every real
// one), so that the sort of the whole bound leaves them at the end.  Also completes the layer's sizes and
// states the next layer's number of destinations (this layer's sources).
__global__ __launch_bounds__(256) void relabel_kernel(const int64_t* __restrict__ ptr, int64_t* __restrict__ sizes,
                                                      int64_t* __restrict__ next_n_dst, const int32_t* __restrict__ idx_local,
                                                      const int32_t* __restrict__ mark, int32_t* __restrict__ idx_blk,
                                                      uint64_t* __restrict__ keyT, int64_t nnz_bound, uint64_t sentinel,
                                                      const int32_t* __restrict__ n_new) {
    const int64_t n_dst = sizes[SZ_DST];
    const int64_t nnz = sizes[SZ_NNZ];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sizes[SZ_NEW] = *n_new;
        sizes[SZ_SRC] = n_dst + *n_new;
        *next_n_dst = n_dst + *n_new;
    }
    for (int64_t e = nnz + (int64_t)blockIdx.x * 256 + threadIdx.x; e < nnz_bound; e += (int64_t)gridDim.x * 256)
        keyT[e] = sentinel;
    const int64_t i = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (i >= n_dst) return;
    const int lane = threadIdx.x & 63;
    for (int64_t e = ptr[i] + lane; e < ptr[i + 1]; e += 64) {
        const int32_t s = mark[idx_local[e]] - 1;
        idx_blk[e] = s;
        keyT[e] = ((uint64_t)(uint32_t)s << 32) | (uint64_t)i;
    }
}

__global__ __launch_bounds__(256) void clear_marks_kernel(const int32_t* __restrict__ src_nodes,
                                                          const int64_t* __restrict__ n_src_dev, int32_t* __restrict__ mark) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= *n_src_dev) return;
    mark[src_nodes[i]] = 0;
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
    int64_t* lr_scan;              // [src+1] scratch of the schedule's construction
    int64_t lr_cap_long, lr_cap_chunks;
};

struct SamplerBufs {
    SamplerLayerBufs L[GRP_MAX_LAYERS];
    int32_t* seeds;                     // [n_seeds] the caller's seeds, range-checked
    int64_t* sizes;                     // [SZ_PER_LAYER * GRP_MAX_LAYERS] the blocks' real sizes (see the enum)
    int64_t* bad;                       // [2] seeds outside the partition (carved just before `mark`: one fill clears all)
    int32_t* mark;                      // [n] block-local index + 1 of the current layer's nodes, else 0
    uint32_t* bits;                     // [n_words + 1] bitmap of newly reached nodes (the last word stays 0)
    int32_t* wpos;                      // [n_words + 1] set bits in the words before each word
    int64_t n_words;
    void *scan_tmp, *sort_tmp;
    void* scan_tmp_side;                // the prefix sums of the transposed blocks (built on a helper stream)
    size_t scan_bytes, sort_bytes;
    size_t total;
};

static SamplerBufs carve_sampler(int64_t n, const SamplerBounds& b, int k, void* ws, size_t ws_bytes) {
    SamplerBufs s;
    Bump bump(ws, ws_bytes);
    int64_t max_nnz = 1, max_dst = 1;
    s.sizes = bump.take<int64_t>(SZ_PER_LAYER * GRP_MAX_LAYERS);
    s.seeds = bump.take<int32_t>((size_t)b.dst[k - 1]);
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
            L.lr_scan = bump.take<int64_t>((size_t)b.src[l] + 1);
            if (b.nnz[l] > max_nnz) max_nnz = b.nnz[l];
        } else {
            L.idx_blk = nullptr; L.src_nodes = nullptr; L.keys = L.keys_sorted = nullptr;
            L.ptrT = nullptr; L.idxT = nullptr; L.lr_row = L.lr_first = nullptr; L.lr_cb = L.lr_ce = nullptr;
            L.lr_scan = nullptr;
            L.lr_cap_long = L.lr_cap_chunks = 0;
        }
    }
    s.bad = bump.take<int64_t>(2);
    s.mark = bump.take<int32_t>((size_t)n);
    s.n_words = cdiv(n, 32);
    s.bits = bump.take<uint32_t>((size_t)s.n_words + 1);
    s.wpos = bump.take<int32_t>((size_t)s.n_words + 1);
    s.scan_bytes = scan_temp_bytes(s.n_words + 1 > max_dst + 1 ? s.n_words + 1 : max_dst + 1);
    s.scan_tmp = bump.take<char>(s.scan_bytes);
    s.scan_tmp_side = k > 1 ? bump.take<char>(s.scan_bytes) : nullptr;
    s.sort_bytes = k > 1 ? sort_keys_temp_bytes(max_nnz) : 0;
    s.sort_tmp = bump.take<char>(s.sort_bytes);
    s.total = bump.total();
    return s;
}

size_t sampler_workspace_bytes(int64_t n, const SamplerBounds& b, int k) { return carve_sampler(n, b, k, nullptr, 0).total; }

// One thread per item (item counts here stay below 2^31, so the grid fits).
static unsigned blocks_for(int64_t work) { return (unsigned)cdiv(work > 0 ? work : 1, 256); }

grp_status sample_blocks(const grp_partition_t* part, const grp_step_opts* o, int k, void* ws, size_t ws_bytes,
                         Block* blocks, LongRows* long_bwd_store, const int64_t** nnz_parts_dev,
                         const int32_t** seed_counts_dev, const int64_t** bad_seeds_dev, hipStream_t st,
                         hipEvent_t* transposed_ready) {
    const int64_t n = part->n;
    *transposed_ready = nullptr;
    if (o->n_seeds < 1 || !o->seeds) return fail(GRP_EINVAL, "mini-batch: need at least one seed node");
    if (n == 0) return fail(GRP_ERANGE, "mini-batch: seeds given for a partition without nodes");
    for (int l = 0; l < k; ++l)
        if (o->fanouts[l] < 1 || o->fanouts[l] > SAMPLE_MAX_FANOUT)
            return fail(GRP_EINVAL, "mini-batch: fanout %d outside [1, %d]", o->fanouts[l], SAMPLE_MAX_FANOUT);
    SamplerBounds bd;
    sampler_bounds(n, o->n_seeds, o->fanouts, k, &bd);
    SamplerBufs s = carve_sampler(n, bd, k, ws, ws_bytes);
    if (s.total > ws_bytes) return fail(GRP_EWORKSPACE, "mini-batch: sampler workspace %zu < %zu", ws_bytes, s.total);

    {   // the bad-seed counter and, with more than one layer, the node map and the bitmap start at zero
        // (carved back to back: one fill covers them)
        char* const lo = (char*)s.bad;
        char* const hi = k > 1 ? (char*)(s.bits + s.n_words + 1) : (char*)(s.bad + 2);
        GRP_TRY(launch_fill_zero(lo, (size_t)(hi - lo), st));
    }
    hipLaunchKernelGGL(check_seeds_kernel, dim3(blocks_for(o->n_seeds)), dim3(256), 0, st, o->seeds, (int64_t)o->n_seeds, n,
                       s.seeds, s.bad, s.sizes + SZ_PER_LAYER * (k - 1) + SZ_DST);
    GRP_LAUNCH_CHECK();
    *bad_seeds_dev = s.bad;
    SideLane* const lane = (k > 1 && !(o->flags & GRP_STEP_ONE_STREAM)) ? side_lane(st) : nullptr;
    const uint64_t h0 = mixM(o->sampler_seed);
    const int32_t* dst_nodes = s.seeds;
    for (int l = k - 1; l >= 0; --l) {
        SamplerLayerBufs& L = s.L[l];
        int64_t* const D = s.sizes + SZ_PER_LAYER * l;   // this layer's sizes; D[SZ_DST] is already there
        const int64_t dst_bound = bd.dst[l];
        const int f = o->fanouts[l];
        hipLaunchKernelGGL(sample_count_kernel, dim3(blocks_for(dst_bound + 1)), dim3(256), 0, st, part->rowptr, dst_nodes,
                           (const int64_t*)(D + SZ_DST), dst_bound, f, L.cnt, L.cnt32, L.inv_in, l > 0 ? s.mark : nullptr,
                           l > 0 ? L.src_nodes : nullptr);
        GRP_LAUNCH_CHECK();
        GRP_TRY(exclusive_scan_i64(s.scan_tmp, s.scan_bytes, L.cnt, L.ptr, dst_bound + 1, st));
        {
            ProfScope ps("sample_select", st);
            hipLaunchKernelGGL(sample_select_kernel, dim3((unsigned)cdiv(dst_bound, SAMPLE_ROWS_PER_WG)),
                               dim3(64 * SAMPLE_ROWS_PER_WG), 0, st, part->rowptr, part->col, part->l2g, dst_nodes, D, f,
                               h0, (uint64_t)o->batch_id, o->batch_id_dev, l, (const int64_t*)L.ptr, L.idx_local);
            GRP_LAUNCH_CHECK();
        }

        Block& B = blocks[l];
        B.n_dst = dst_bound;
        B.n_dst_dev = D + SZ_DST;
        B.nnz = bd.nnz[l];
        B.dst_nodes = dst_nodes;
        B.ptr = L.ptr;
        B.inv_in = L.inv_in;
        B.long_fwd = nullptr;                            // rows hold at most `fanout` edges
        nnz_parts_dev[l] = D + SZ_NNZ;
        if (l == k - 1) *seed_counts_dev = L.cnt32;
        if (l == 0) {
            B.idx = L.idx_local;
            B.n_in = n;
            B.n_in_dev = nullptr;                        // the inputs are the partition's nodes
            B.self_rows = dst_nodes;
            B.ptrT = nullptr; B.idxT = nullptr; B.long_bwd = nullptr;
            break;
        }
        // new source nodes in ascending local id, block-local relabelling, transposed block
        const int64_t src_bound = bd.src[l], nnz_bound = bd.nnz[l];
        hipLaunchKernelGGL(flag_new_kernel, dim3(blocks_for(nnz_bound)), dim3(256), 0, st, (const int32_t*)L.idx_local,
                           (const int64_t*)(D + SZ_NNZ), (const int32_t*)s.mark, s.bits);
        GRP_LAUNCH_CHECK();
        GRP_TRY(exclusive_scan_popcount(s.scan_tmp, s.scan_bytes, s.bits, s.wpos, s.n_words + 1, st));
        hipLaunchKernelGGL(assign_new_kernel, dim3(blocks_for(s.n_words)), dim3(256), 0, st, s.n_words, s.bits,
                           (const int32_t*)s.wpos, (const int64_t*)(D + SZ_DST), s.mark, L.src_nodes);
        GRP_LAUNCH_CHECK();
        // Keys are (source << 32 | destination); the unused slots up to the bound get the source index
        // src_bound, which no real source reaches, and the sort covers the bits of that value.
        int bits = 1;
        while (bits < 32 && ((int64_t)1 << bits) <= src_bound) ++bits;
        hipLaunchKernelGGL(relabel_kernel, dim3((unsigned)cdiv(dst_bound, 4)), dim3(256), 0, st, (const int64_t*)L.ptr, D,
                           s.sizes + SZ_PER_LAYER * (l - 1) + SZ_DST, (const int32_t*)L.idx_local, (const int32_t*)s.mark,
                           L.idx_blk, L.keys, nnz_bound, (uint64_t)src_bound << 32, (const int32_t*)(s.wpos + s.n_words));
        GRP_LAUNCH_CHECK();
        // The transposed block is read by the backward pass only: it is built on the helper stream, beside the
        // sampling of the next layers and the forward pass.
        hipStream_t bst = st;
        void* scan_tmp_t = s.scan_tmp;
        if (lane) {
            GRP_HIP(hipEventRecord(lane->fork[l], st));
            GRP_HIP(hipStreamWaitEvent(lane->stream, lane->fork[l], 0));
            bst = lane->stream;
            scan_tmp_t = s.scan_tmp_side;
        }
        hipLaunchKernelGGL(clear_marks_kernel, dim3(blocks_for(src_bound)), dim3(256), 0, st, (const int32_t*)L.src_nodes,
                           (const int64_t*)(D + SZ_SRC), s.mark);
        GRP_LAUNCH_CHECK();
        GRP_TRY(sort_keys_u64(s.sort_tmp, s.sort_bytes, L.keys, L.keys_sorted, nnz_bound, 32u + (unsigned)bits, bst));
        // Over src_bound rows: those past the real sources come out empty (their pointer is the real number
        // of edges, where the sentinels begin), and the entries of idxT past that number are never read.
        GRP_TRY(launch_csr_from_sorted_keys(L.keys_sorted, nnz_bound, src_bound, L.ptrT, L.idxT, bst));
        LongRows& lr = long_bwd_store[l];
        lr.long_row = L.lr_row; lr.long_first = L.lr_first; lr.chunk_begin = L.lr_cb; lr.chunk_end = L.lr_ce;
        GRP_TRY(build_long_rows_device(L.ptrT, src_bound, &lr, L.lr_cap_long, L.lr_cap_chunks, L.lr_scan, scan_tmp_t,
                                       s.scan_bytes, bst));
        B.idx = L.idx_blk;
        B.n_in = src_bound;
        B.n_in_dev = D + SZ_SRC;
        B.self_rows = nullptr;
        B.ptrT = L.ptrT;
        B.idxT = L.idxT;
        B.long_bwd = &lr;
        dst_nodes = L.src_nodes;
    }
    if (lane) {
        GRP_HIP(hipEventRecord(lane->join, lane->stream));
        *transposed_ready = lane->join;
    }
    return GRP_OK;
}

// Where a finished step left block `layer` inside its sampler workspace (same partition size, seeds count,
// fanouts and depth).  Copies the block sizes from the device: synchronises the device.
grp_status sampler_block_view(const grp_partition_t* part, const grp_step_opts* o, int k, void* ws, size_t ws_bytes, int layer,
                              grp_block_view_t* out) {
    SamplerBounds bd;
    sampler_bounds(part->n, o->n_seeds, o->fanouts, k, &bd);
    const SamplerBufs s = carve_sampler(part->n, bd, k, ws, ws_bytes);
    if (s.total > ws_bytes) return fail(GRP_EWORKSPACE, "grp_step_block: sampler workspace %zu < %zu", ws_bytes, s.total);
    int64_t sizes[SZ_PER_LAYER * GRP_MAX_LAYERS] = {0};
    GRP_HIP(hipDeviceSynchronize());
    GRP_HIP(hipMemcpy(sizes, s.sizes, sizeof sizes, hipMemcpyDeviceToHost));
    const int64_t* const D = sizes + SZ_PER_LAYER * layer;
    const SamplerLayerBufs& L = s.L[layer];
    if (D[SZ_DST] < 0 || D[SZ_DST] > bd.dst[layer] || D[SZ_NNZ] < 0 || D[SZ_NNZ] > bd.nnz[layer])
        return fail(GRP_EINVAL, "grp_step_block: the workspace does not hold a step of this shape");
    out->n_dst = D[SZ_DST];
    out->nnz = D[SZ_NNZ];
    out->rowptr = L.ptr;
    out->dst_nodes = layer == k - 1 ? s.seeds : s.L[layer + 1].src_nodes;
    if (layer == 0) {
        out->n_src = part->n;
        out->col = L.idx_local;
        out->src_nodes = nullptr;
    } else {
        if (D[SZ_SRC] < D[SZ_DST] || D[SZ_SRC] > bd.src[layer])
            return fail(GRP_EINVAL, "grp_step_block: the workspace does not hold a step of this shape");
        out->n_src = D[SZ_SRC];
        out->col = L.idx_blk;
        out->src_nodes = L.src_nodes;
    }
    return GRP_OK;
}

}  // namespace grp
