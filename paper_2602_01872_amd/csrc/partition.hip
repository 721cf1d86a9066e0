// Random node assignment and the isolated local subgraph, built on the GPU.
//
// owner(v) = SplitMix64_output(seed, v) mod K.  A partition keeps the edges whose two
// endpoints it owns, renumbers nodes by ascending global id and stores the edge multiset
// twice in canonical order: CSR by destination (sources ascending) and CSC by source
// (destinations ascending).  Canonical order comes from a radix sort of the 64-bit keys
// (row << 32 | column); equal keys are indistinguishable, so the arrays are unique and can
// be compared bit for bit.  Everything is integer work: counters use integer atomics only.
//
// The device-wide radix sort and prefix sum are rocPRIM's; the hashing, filtering,
// relabelling and pointer construction are the kernels below.
#include "common.h"

#include <cstring>
#include <new>
#include <vector>

#include <rocprim/rocprim.hpp>

namespace grp {

__device__ __forceinline__ uint64_t splitmix64_output(uint64_t seed, uint64_t index) {
    uint64_t z = seed + (index + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void owner_flag_kernel(int64_t N, uint32_t K, uint64_t seed, uint32_t part,
                                                         int32_t* __restrict__ flag) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < N) flag[v] = (splitmix64_output(seed, (uint64_t)v) % K) == part ? 1 : 0;
}

// owner[v] for every node and (optionally) the number of nodes per partition.
__global__ __launch_bounds__(256) void node_owners_kernel(int64_t N, uint32_t K, uint64_t seed, int32_t* __restrict__ owner,
                                                          unsigned long long* __restrict__ hist) {
    constexpr int LDS_BINS = 1024;
    __shared__ unsigned int bins[LDS_BINS];
    const bool local = hist && K <= LDS_BINS;
    if (local) {
        for (int i = threadIdx.x; i < (int)K; i += 256) bins[i] = 0u;
        __syncthreads();
    }
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < N; v += (int64_t)gridDim.x * 256) {
        const uint32_t o = (uint32_t)(splitmix64_output(seed, (uint64_t)v) % K);
        owner[v] = (int32_t)o;
        if (local) atomicAdd(&bins[o], 1u);
        else if (hist) atomicAdd(&hist[o], 1ull);
    }
    if (local) {
        __syncthreads();
        for (int i = threadIdx.x; i < (int)K; i += 256)
            if (bins[i]) atomicAdd(&hist[i], (unsigned long long)bins[i]);
    }
}

__global__ __launch_bounds__(256) void scatter_l2g_kernel(int64_t N, const int32_t* __restrict__ flag,
                                                          const int64_t* __restrict__ pos, int64_t* __restrict__ l2g) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < N && flag[v]) l2g[pos[v]] = v;
}

// Edges e and e + 1 (e even) of an id array with one 16-byte load when the array allows it; `fill` past the end.
typedef int64_t i64x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void load_edge_pair(const int64_t* __restrict__ p, int64_t e, int64_t E, bool vec, int64_t fill,
                                               int64_t& a, int64_t& b) {
    if (vec && e + 1 < E) {
        const i64x2 t = *reinterpret_cast<const i64x2*>(p + e);
        a = t.x;
        b = t.y;
    } else {
        a = e < E ? p[e] : fill;
        b = e + 1 < E ? p[e + 1] : fill;
    }
}

// A node set as a bitmap plus the number of members before each 32-node word: membership and the
// member's rank (its local id) from two small arrays that stay in the L2 caches (N / 4 bytes in all),
// where per-node flag and position arrays (12 bytes per node) cost a cache line from HBM per lookup.
struct NodeSet {
    const uint32_t* bits;
    const int32_t* before;
};
__device__ __forceinline__ bool set_has(const NodeSet& s, int64_t v) { return (s.bits[v >> 5] >> (v & 31)) & 1u; }
__device__ __forceinline__ int32_t set_rank(const NodeSet& s, int64_t v) {
    return s.before[v >> 5] + __popc(s.bits[v >> 5] & ((1u << (v & 31)) - 1u));
}

// ---- weighted partitions: the selected edges are compacted in edge-list order, so that equal
// (dst, src) pairs keep their order through the stable sorts and the result does not depend on
// scheduling.  A tile is 2048 consecutive edges, eight consecutive edges per thread; a first pass counts
// the selected edges of every tile, a prefix sum over the tiles gives each its first slot, a second pass
// repeats the selection and places every edge at the tile's slot plus its rank inside the tile.
// WHICH = 0: edges with both endpoints in the set; WHICH = 1: edges whose destination is in the set.
constexpr int OC_PER = 8;
constexpr int OC_TILE = 256 * OC_PER;

template <int WHICH>
__device__ __forceinline__ int oc_select(const int64_t* __restrict__ src, const int64_t* __restrict__ dst, int64_t E,
                                         bool vec, const NodeSet& own, int64_t e0, int64_t (&us)[OC_PER],
                                         int64_t (&vs)[OC_PER], bool (&on)[OC_PER]) {
#pragma unroll
    for (int i = 0; i < OC_PER; i += 2) {
        load_edge_pair(src, e0 + i, E, vec, 0, us[i], us[i + 1]);
        load_edge_pair(dst, e0 + i, E, vec, -1, vs[i], vs[i + 1]);       // -1: past the end
    }
    int count = 0;
#pragma unroll
    for (int i = 0; i < OC_PER; ++i) {
        on[i] = vs[i] >= 0 && set_has(own, vs[i]) && (WHICH == 1 || set_has(own, us[i]));
        count += on[i] ? 1 : 0;
    }
    return count;
}

template <int WHICH>
__global__ __launch_bounds__(256) void ordered_count_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                            int64_t E, NodeSet own, int64_t n_tiles,
                                                            int64_t* __restrict__ tile_count /*[n_tiles + 1]*/) {
    __shared__ int wave_count[4];
    const bool vec = (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        int64_t us[OC_PER], vs[OC_PER];
        bool on[OC_PER];
        int c = oc_select<WHICH>(src, dst, E, vec, own, tile * OC_TILE + (int64_t)threadIdx.x * OC_PER, us, vs, on);
        for (int o = 32; o > 0; o >>= 1) c += __shfl_down(c, o, 64);
        if (lane == 0) wave_count[wave] = c;
        __syncthreads();
        if (threadIdx.x == 0) tile_count[tile] = wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
        __syncthreads();
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) tile_count[n_tiles] = 0;
}

template <int WHICH>
__global__ __launch_bounds__(256) void ordered_emit_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                           const float* __restrict__ w, int64_t E, NodeSet own,
                                                           int64_t n_tiles, const int64_t* __restrict__ tile_base,
                                                           uint64_t* __restrict__ keys, uint32_t* __restrict__ keys32,
                                                           float* __restrict__ vals) {
    __shared__ int wave_count[4];
    const bool vec = (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t e0 = tile * OC_TILE + (int64_t)threadIdx.x * OC_PER;
        int64_t us[OC_PER], vs[OC_PER];
        bool on[OC_PER];
        const int mine = oc_select<WHICH>(src, dst, E, vec, own, e0, us, vs, on);
        int incl = mine;                                 // inclusive prefix over the wavefront, then over the four
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wave_count[wave] = incl;
        __syncthreads();
        int before = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (q < wave) before += wave_count[q];
        int64_t slot = tile_base[tile] + before + incl - mine;
#pragma unroll
        for (int i = 0; i < OC_PER; ++i) {
            if (!on[i]) continue;
            if (WHICH == 0) keys[slot] = ((uint64_t)(uint32_t)set_rank(own, vs[i]) << 32) | (uint64_t)(uint32_t)set_rank(own, us[i]);
            else keys32[slot] = (uint32_t)set_rank(own, vs[i]);
            vals[slot] = w[e0 + i];
            ++slot;
        }
        __syncthreads();                                 // wave_count is reused by the next tile
    }
}

// bits[w] = flags of nodes 32w .. 32w+31; the grid covers n_words * 32 nodes
__global__ __launch_bounds__(256) void pack_bits_kernel(const int32_t* __restrict__ flag, int64_t N, int64_t n_words,
                                                        uint32_t* __restrict__ bits) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const unsigned long long m = __ballot(v < N && flag[v] != 0);
    const int64_t w = v >> 5;
    if ((threadIdx.x & 63) == 0 && w < n_words) {
        bits[w] = (uint32_t)m;
        if (w + 1 < n_words) bits[w + 1] = (uint32_t)(m >> 32);
    }
}

// Pass 1 over the edges: id range check, global in-degree of owned destinations, count of kept edges.
// The in-degree counts go through a table in LDS first (open addressing on the local id, a few probes,
// LDS atomics) and reach memory once per workgroup and node: a hub of a skewed graph receives 10^5..10^6
// edges, and that many atomics on one address serialise in the L2 (they set the time of this pass before).
// An edge that finds no slot adds to memory directly.
constexpr int DG_SLOTS = 4096;
constexpr int DG_PROBES = 4;
constexpr int EDGE_SCAN_GRID = 4096;      // fat workgroups: more edges of a hub meet in one table

__device__ __forceinline__ void dg_table_add(int32_t* slot_key, uint32_t* slot_count, unsigned long long* __restrict__ dg,
                                             int32_t r) {
    uint32_t h = (uint32_t)r * 2654435761u >> 20;        // top 12 bits of a multiplicative hash
    for (int probe = 0; probe < DG_PROBES; ++probe, h = (h + 1) & (DG_SLOTS - 1)) {
        const int32_t seen = atomicCAS(&slot_key[h], -1, r);
        if (seen == -1 || seen == r) {
            atomicAdd(&slot_count[h], 1u);
            return;
        }
    }
    atomicAdd(&dg[r], 1ull);
}

__global__ __launch_bounds__(256) void edge_scan_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                        int64_t E, int64_t N, NodeSet own,
                                                        unsigned long long* __restrict__ dg,
                                                        unsigned long long* __restrict__ counters /*[0]=kept,[1]=bad*/) {
    const bool vec = (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
    __shared__ int32_t slot_key[DG_SLOTS];
    __shared__ uint32_t slot_count[DG_SLOTS];
    for (int i = threadIdx.x; i < DG_SLOTS; i += 256) { slot_key[i] = -1; slot_count[i] = 0u; }
    __syncthreads();
    unsigned long long kept = 0, bad = 0;
    constexpr int PER = 8;                               // edges per thread and tile: their loads are in flight together
    const int64_t n_tiles = (E + 256 * PER - 1) / (256 * PER);
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t e0 = tile * (256 * PER) + 2 * threadIdx.x;
        int64_t us[PER], vs[PER];
#pragma unroll
        for (int i = 0; i < PER; i += 2) {               // a thread takes pairs of consecutive edges
            const int64_t e = e0 + (int64_t)i * 256;
            load_edge_pair(src, e, E, vec, 0, us[i], us[i + 1]);
            load_edge_pair(dst, e, E, vec, -2, vs[i], vs[i + 1]);     // -2: past the end, neither counted nor an error
        }
        bool mine[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int64_t u = us[i], v = vs[i];
            mine[i] = false;
            if (v == -2) continue;
            if (u < 0 || v < 0 || u >= N || v >= N) { bad++; continue; }
            mine[i] = set_has(own, v);
        }
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (!mine[i]) continue;
            dg_table_add(slot_key, slot_count, dg, set_rank(own, vs[i]));
            if (set_has(own, us[i])) kept++;
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < DG_SLOTS; i += 256)
        if (slot_key[i] >= 0) atomicAdd(&dg[slot_key[i]], (unsigned long long)slot_count[i]);
    for (int o = 32; o > 0; o >>= 1) {
        kept += __shfl_down(kept, o, 64);
        bad += __shfl_down(bad, o, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        if (kept) atomicAdd(&counters[0], kept);
        if (bad) atomicAdd(&counters[1], bad);
    }
}

// Which edges a partition keeps and their key (dst_local << 32 | src_local).
struct SetSelect {                        // both endpoints in the node set
    NodeSet own;
    __device__ __forceinline__ bool operator()(int64_t u, int64_t v, uint64_t& key) const {
        if (!set_has(own, v) || !set_has(own, u)) return false;
        key = ((uint64_t)(uint32_t)set_rank(own, v) << 32) | (uint64_t)(uint32_t)set_rank(own, u);
        return true;
    }
};
struct ArraySelect {                      // per-node flag and position arrays
    const int32_t* flag;
    const int64_t* pos;
    int dst_only;                         // keep every edge whose destination is flagged (halo partitions), whatever its source
    __device__ __forceinline__ bool operator()(int64_t u, int64_t v, uint64_t& key) const {
        if (!flag[v] || !(dst_only || flag[u])) return false;
        key = ((uint64_t)pos[v] << 32) | (uint64_t)pos[u];
        return true;
    }
};

// Pass 2: write the key of every kept edge.  The slot order is
// arbitrary; the sort that follows makes the result canonical.  A workgroup takes tiles of
// 256 x 8 edges, counts its kept edges through LDS and reserves their slots with one atomic
// per tile (one atomic per kept edge on a single address would serialise the whole pass).
template <typename Select>
__global__ __launch_bounds__(256) void edge_keys_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                        int64_t E, Select select,
                                                        unsigned long long* __restrict__ cursor,
                                                        uint64_t* __restrict__ keys) {
    constexpr int PER = 8;
    const bool vec = (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
    __shared__ int wave_count[4];
    __shared__ unsigned long long tile_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n_tiles = (E + 256 * PER - 1) / (256 * PER);
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t e0 = tile * (256 * PER) + 2 * tid;
        int64_t us[PER], vs[PER];
#pragma unroll
        for (int i = 0; i < PER; i += 2) {               // a thread takes pairs of consecutive edges
            const int64_t e = e0 + (int64_t)i * 256;
            load_edge_pair(src, e, E, vec, 0, us[i], us[i + 1]);
            load_edge_pair(dst, e, E, vec, -1, vs[i], vs[i + 1]);     // -1: past the end
        }
        uint64_t key[PER];
        int mine = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            key[i] = ~0ull;
            uint64_t k;
            if (vs[i] >= 0 && select(us[i], vs[i], k)) { key[i] = k; ++mine; }
        }
        // exclusive prefix of `mine` over the workgroup: inside the wavefront by shuffles, across the four by LDS
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wave_count[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) before += wave_count[w];
            total += wave_count[w];
        }
        if (tid == 0) tile_base = total ? atomicAdd(cursor, (unsigned long long)total) : 0ull;
        __syncthreads();
        unsigned long long slot = tile_base + (unsigned long long)(before + incl - mine);
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (key[i] != ~0ull) keys[slot++] = key[i];
        __syncthreads();                                 // wave_count / tile_base are reused by the next tile
    }
}

// Both passes in one (unweighted builds): range check, global in-degrees of owned destinations and the keys of
// the kept edges, written into a buffer of `cap` keys.  counters: [1] += bad ids, [2] += kept edges (the
// slot cursor).  If the cursor ends above cap the keys are incomplete and the caller runs edge_keys_kernel
// with a buffer of the exact size (the in-degrees and the count are complete either way).
__global__ __launch_bounds__(256) void edge_scan_keys_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                             int64_t E, int64_t N, NodeSet own,
                                                             unsigned long long* __restrict__ dg,
                                                             unsigned long long* __restrict__ counters,
                                                             uint64_t* __restrict__ keys, unsigned long long cap) {
    constexpr int PER = 8;
    const bool vec = (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
    __shared__ int32_t slot_key[DG_SLOTS];
    __shared__ uint32_t slot_count[DG_SLOTS];
    __shared__ int wave_count[4];
    __shared__ unsigned long long tile_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < DG_SLOTS; i += 256) { slot_key[i] = -1; slot_count[i] = 0u; }
    __syncthreads();
    unsigned long long bad = 0;
    const int64_t n_tiles = (E + 256 * PER - 1) / (256 * PER);
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t e0 = tile * (256 * PER) + 2 * tid;
        int64_t us[PER], vs[PER];
#pragma unroll
        for (int i = 0; i < PER; i += 2) {
            const int64_t e = e0 + (int64_t)i * 256;
            load_edge_pair(src, e, E, vec, 0, us[i], us[i + 1]);
            load_edge_pair(dst, e, E, vec, -2, vs[i], vs[i + 1]);     // -2: past the end, neither counted nor an error
        }
        uint64_t key[PER];
        int mine = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int64_t u = us[i], v = vs[i];
            key[i] = ~0ull;
            if (v == -2) continue;
            if (u < 0 || v < 0 || u >= N || v >= N) { bad++; continue; }
            if (!set_has(own, v)) continue;
            const int32_t rv = set_rank(own, v);
            dg_table_add(slot_key, slot_count, dg, rv);
            if (set_has(own, u)) {
                key[i] = ((uint64_t)(uint32_t)rv << 32) | (uint64_t)(uint32_t)set_rank(own, u);
                ++mine;
            }
        }
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wave_count[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) before += wave_count[w];
            total += wave_count[w];
        }
        if (tid == 0) tile_base = total ? atomicAdd(&counters[2], (unsigned long long)total) : 0ull;
        __syncthreads();
        unsigned long long slot = tile_base + (unsigned long long)(before + incl - mine);
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (key[i] != ~0ull) {
                if (slot < cap) keys[slot] = key[i];
                ++slot;
            }
        __syncthreads();                                 // wave_count / tile_base are reused by the next tile
    }
    for (int i = tid; i < DG_SLOTS; i += 256)
        if (slot_key[i] >= 0) atomicAdd(&dg[slot_key[i]], (unsigned long long)slot_count[i]);
    for (int o = 32; o > 0; o >>= 1) bad += __shfl_down(bad, o, 64);
    if (lane == 0 && bad) atomicAdd(&counters[1], bad);
}

// Local edge list: range check + keys in place order.
__global__ __launch_bounds__(256) void local_keys_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                         int64_t E, int64_t n, uint64_t* __restrict__ keys,
                                                         unsigned long long* __restrict__ bad) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < E; e += (int64_t)gridDim.x * 256) {
        const int64_t u = src[e], v = dst[e];
        if (u < 0 || v < 0 || u >= n || v >= n) {
            atomicAdd(bad, 1ull);
            keys[e] = 0;
        } else {
            keys[e] = ((uint64_t)v << 32) | (uint64_t)u;
        }
    }
}

__global__ __launch_bounds__(256) void swap_halves_kernel(const uint64_t* __restrict__ in, int64_t nnz,
                                                          uint64_t* __restrict__ out) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nnz; i += (int64_t)gridDim.x * 256)
        out[i] = (in[i] << 32) | (in[i] >> 32);
}

// From sorted keys: idx[i] = low half; ptr[r] = first position whose high half is >= r.
__global__ __launch_bounds__(256) void csr_from_keys_kernel(const uint64_t* __restrict__ keys, int64_t nnz, int64_t n,
                                                            int64_t* __restrict__ ptr, int32_t* __restrict__ idx) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i <= nnz; i += (int64_t)gridDim.x * 256) {
        const int64_t hi = i < nnz ? (int64_t)(keys[i] >> 32) : n;
        const int64_t prev = i > 0 ? (int64_t)(keys[i - 1] >> 32) : -1;
        for (int64_t r = prev + 1; r <= hi; ++r) ptr[r] = i;
        if (i < nnz) idx[i] = (int32_t)(keys[i] & 0xFFFFFFFFull);
    }
}

__global__ __launch_bounds__(256) void degree_from_ptr_kernel(const int64_t* __restrict__ ptr, int64_t n,
                                                              int32_t* __restrict__ deg) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < n) deg[v] = (int32_t)(ptr[v + 1] - ptr[v]);
}

__global__ __launch_bounds__(256) void iota_kernel(int64_t n, int64_t* __restrict__ out) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < n) out[v] = v;
}

__global__ __launch_bounds__(256) void widen_kernel(const int32_t* __restrict__ in, int64_t n, int64_t* __restrict__ out) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < n) out[v] = in[v];
}

__global__ __launch_bounds__(256) void weight_check_kernel(const float* __restrict__ w, int64_t E,
                                                           unsigned long long* __restrict__ bad) {
    unsigned long long b = 0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < E; e += (int64_t)gridDim.x * 256)
        if (!(w[e] > 0.f) || !(w[e] <= 3.402823466e+38f)) b++;
    if (b) atomicAdd(bad, b);
}

// mass[r] = sum of vals over [ptr[r], ptr[r+1]) in fp64.  Rows of at most ROW_MASS_SERIAL entries are added in
// stored order by one thread.  Longer rows (hubs: 10^5 entries and more, which one thread would take
// milliseconds over) are left to row_mass_long_kernel: one workgroup per row, every thread adds a contiguous
// run in stored order and the 256 partial sums are added in thread order, a fixed order that does not depend
// on scheduling (and the same value as the serial sum whenever the partial sums are exact in fp64, as they
// are for float weights of similar magnitude).
constexpr int ROW_MASS_SERIAL = 1024;

__global__ __launch_bounds__(256) void row_mass_kernel(const int64_t* __restrict__ ptr, const float* __restrict__ vals,
                                                       int64_t n, double* __restrict__ mass,
                                                       int32_t* __restrict__ long_rows, int32_t* __restrict__ n_long) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= n) return;
    const int64_t b = ptr[r], e = ptr[r + 1];
    if (e - b > ROW_MASS_SERIAL) {
        long_rows[atomicAdd(n_long, 1)] = (int32_t)r;    // any order: each row is summed on its own
        return;
    }
    double s = 0.0;
    for (int64_t k = b; k < e; ++k) s += (double)vals[k];
    mass[r] = s;
}

__global__ __launch_bounds__(256) void row_mass_long_kernel(const int64_t* __restrict__ ptr, const float* __restrict__ vals,
                                                            const int32_t* __restrict__ long_rows,
                                                            const int32_t* __restrict__ n_long, double* __restrict__ mass) {
    __shared__ double part[256];
    const int count = *n_long;
    for (int j = blockIdx.x; j < count; j += gridDim.x) {
        const int64_t r = long_rows[j];
        const int64_t b = ptr[r], e = ptr[r + 1];
        const int64_t per = (e - b + 255) / 256;
        int64_t lo = b + threadIdx.x * per, hi = lo + per;
        if (lo > e) lo = e;
        if (hi > e) hi = e;
        double s = 0.0;
        for (int64_t k = lo; k < hi; ++k) s += (double)vals[k];
        part[threadIdx.x] = s;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int q = 0; q < 256; ++q) t += part[q];
            mass[r] = t;
        }
        __syncthreads();
    }
}

// Row masses of a CSR-like (ptr, vals) pair; `scratch`: [n + 1] int32 device words (list of long rows + their count).
static grp_status launch_row_mass(const int64_t* ptr, const float* vals, int64_t n, double* mass, int32_t* scratch,
                                  hipStream_t st) {
    if (n == 0) return GRP_OK;
    GRP_HIP(hipMemsetAsync(scratch + n, 0, sizeof(int32_t), st));
    hipLaunchKernelGGL(row_mass_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, ptr, vals, n, mass, scratch, scratch + n);
    GRP_LAUNCH_CHECK();
    hipLaunchKernelGGL(row_mass_long_kernel, dim3(1024), dim3(256), 0, st, ptr, vals, (const int32_t*)scratch,
                       (const int32_t*)(scratch + n), mass);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

static unsigned grid_for(int64_t work) {
    int64_t b = cdiv(work > 0 ? work : 1, 256);
    return (unsigned)(b > 16384 ? 16384 : b);
}

struct DevBuf {
    void* p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    grp_status alloc(size_t bytes) {
        if (hipMalloc(&p, bytes ? bytes : 4) != hipSuccess) {
            p = nullptr;
            (void)hipGetLastError();
            return fail(GRP_ENOMEM, "device allocation of %zu bytes failed", bytes);
        }
        return GRP_OK;
    }
    template <typename T> T* as() { return (T*)p; }
};

struct DevView {                          // a typed look at part of an allocation (same accessors as DevBuf)
    void* p;
    template <typename T> T* as() { return (T*)p; }
};

static void free_partition(grp_partition_t* h) {
    if (!h) return;
    if (h->borrowed_csr) { h->rowptr = nullptr; h->col = nullptr; }
    void* ptrs[] = {h->l2g, h->rowptr, h->col, h->colptr, h->row, h->d_local_in, h->d_local_out, h->d_global_in,
                    h->csr_long.long_row, h->csr_long.long_first, h->csr_long.chunk_begin, h->csr_long.chunk_end,
                    h->csc_long.long_row, h->csc_long.long_first, h->csc_long.chunk_begin, h->csc_long.chunk_end,
                    h->base_mask, h->csr_long.tasks, h->csr_long.row_task, h->csc_long.tasks, h->csc_long.row_task, h->csr_w, h->csc_w, h->w_local_in, h->w_global_in};
    const char* lo = (const char*)h->slab;
    for (void* q : ptrs)
        if (q && !(lo && (const char*)q >= lo && (const char*)q < lo + h->slab_bytes)) (void)hipFree(q);
    if (h->slab) (void)hipFree(h->slab);
    delete h;
}

template <typename T>
static grp_status halloc(T** out, int64_t count) {
    void* p = nullptr;
    const size_t bytes = (size_t)(count > 0 ? count : 1) * sizeof(T);
    if (hipMalloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(GRP_ENOMEM, "device allocation of %zu bytes failed", bytes);
    }
    *out = (T*)p;
    return GRP_OK;
}

static int bits_for(int64_t n) {
    int b = 1;
    while (b < 32 && ((int64_t)1 << b) < n) ++b;
    return b;
}

// Split schedule of the rows longer than SPMM_LONG_ROW edges (a function of the pointer
// array only), built on the device into arrays sized for the worst case (out->long_row .. chunk_end,
// cap_long / cap_chunks entries); the two counts come back to the host (the launches that use the
// schedule are sized by them).  scanned: [n + 1] int64 scratch.
static grp_status build_long_rows(const int64_t* ptr_dev, int64_t n, LongRows* out, int64_t cap_long, int64_t cap_chunks,
                                  int64_t* scanned, void* tmp, size_t tmp_bytes, hipStream_t st) {
    out->n_long = out->n_chunks = 0;
    if (n == 0 || cap_long == 0) return GRP_OK;          // no row can be long
    GRP_TRY(build_long_rows_device(ptr_dev, n, out, cap_long, cap_chunks, scanned, tmp, tmp_bytes, st));
    int64_t total = 0;
    GRP_HIP(hipMemcpyAsync(&total, scanned + n, sizeof total, hipMemcpyDeviceToHost, st));
    GRP_HIP(hipStreamSynchronize(st));
    out->n_long = (int32_t)(total >> 32);
    out->n_chunks = (int32_t)(total & 0xFFFFFFFFll);
    return GRP_OK;
}

// The arrays build_csr_csc fills, carved from one allocation (base null: only measures).
static size_t carve_csr_csc(grp_partition_t* h, bool weighted, int64_t cap_long, int64_t cap_chunks, void* base, size_t cap) {
    Bump b(base, cap);
    const size_t n1 = (size_t)(h->n > 0 ? h->n : 1), z1 = (size_t)(h->nnz > 0 ? h->nnz : 1);
    if (weighted) {
        h->csr_w = b.take<float>(z1);
        h->csc_w = b.take<float>(z1);
    }
    h->rowptr = b.take<int64_t>(n1 + 1);
    h->colptr = b.take<int64_t>(n1 + 1);
    h->col = b.take<int32_t>(z1);
    h->row = b.take<int32_t>(z1);
    h->d_local_in = b.take<int32_t>(n1);
    h->d_local_out = b.take<int32_t>(n1);
    for (LongRows* lr : {&h->csr_long, &h->csc_long}) {
        if (cap_long == 0) continue;
        lr->long_row = b.take<int32_t>((size_t)cap_long);
        lr->long_first = b.take<int32_t>((size_t)cap_long + 1);
        lr->chunk_begin = b.take<int64_t>((size_t)cap_chunks);
        lr->chunk_end = b.take<int64_t>((size_t)cap_chunks);
    }
    return b.total();
}

// keys (unsorted, nnz of them; clobbered) -> h->rowptr/col/d_local_in and h->colptr/row/d_local_out.
// vals / vals_alt (optional, nnz floats each; clobbered): a value per key that travels through the
// (stable) sorts into h->csr_w and h->csc_w.
static grp_status build_csr_csc(grp_partition_t* h, uint64_t* keys, uint64_t* keys_alt, hipStream_t st,
                                float* vals = nullptr, float* vals_alt = nullptr) {
    const int64_t n = h->n, nnz = h->nnz;
    const int64_t cap_long = nnz > SPMM_LONG_ROW ? nnz / SPMM_LONG_ROW + 1 : 0;
    const int64_t cap_chunks = cap_long ? nnz / SPMM_CHUNK + cap_long + 1 : 0;
    if (cap_chunks >= ((int64_t)1 << 31)) return fail(GRP_ERANGE, "more than 2^31 row chunks");
    h->slab_bytes = carve_csr_csc(h, vals != nullptr, cap_long, cap_chunks, nullptr, 0);
    if (hipMalloc(&h->slab, h->slab_bytes) != hipSuccess) {
        (void)hipGetLastError();
        h->slab = nullptr;
        return fail(GRP_ENOMEM, "device allocation of %zu bytes failed", h->slab_bytes);
    }
    (void)carve_csr_csc(h, vals != nullptr, cap_long, cap_chunks, h->slab, h->slab_bytes);
    const unsigned end_bit = 32 + bits_for(n > 1 ? n : 2);
    // one scratch allocation: the sorts' temporary storage, later the long-row pass's prefix sums
    size_t sort_bytes = 0;
    if (nnz > 0 && !vals)
        GRP_HIP(rocprim::radix_sort_keys(nullptr, sort_bytes, keys, keys_alt, (size_t)nnz, 0u, end_bit, st));
    else if (nnz > 0)
        GRP_HIP(rocprim::radix_sort_pairs(nullptr, sort_bytes, keys, keys_alt, vals, vals_alt, (size_t)nnz, 0u, end_bit, st));
    const size_t scan_bytes = cap_long ? scan_temp_bytes(n + 1) : 0;
    const size_t scanned_bytes = cap_long ? (((size_t)n + 1) * sizeof(int64_t) + 255) & ~(size_t)255 : 0;
    size_t tmp_bytes = sort_bytes > scanned_bytes + scan_bytes ? sort_bytes : scanned_bytes + scan_bytes;
    DevBuf tmp;
    GRP_TRY(tmp.alloc(tmp_bytes));
    if (nnz > 0 && !vals) {
        GRP_HIP(rocprim::radix_sort_keys(tmp.p, sort_bytes, keys, keys_alt, (size_t)nnz, 0u, end_bit, st));
    } else if (nnz > 0) {
        GRP_HIP(rocprim::radix_sort_pairs(tmp.p, sort_bytes, keys, keys_alt, vals, vals_alt, (size_t)nnz, 0u, end_bit, st));
        GRP_HIP(hipMemcpyAsync(h->csr_w, vals_alt, (size_t)nnz * sizeof(float), hipMemcpyDeviceToDevice, st));
    }
    hipLaunchKernelGGL(csr_from_keys_kernel, dim3(grid_for(nnz + 1)), dim3(256), 0, st, keys_alt, nnz, n, h->rowptr, h->col);
    GRP_LAUNCH_CHECK();
    if (nnz > 0) {
        hipLaunchKernelGGL(swap_halves_kernel, dim3(grid_for(nnz)), dim3(256), 0, st, keys_alt, nnz, keys);
        GRP_LAUNCH_CHECK();
        if (!vals) {
            GRP_HIP(rocprim::radix_sort_keys(tmp.p, sort_bytes, keys, keys_alt, (size_t)nnz, 0u, end_bit, st));
        } else {      // from CSR order (vals_alt) to CSC order (vals)
            GRP_HIP(rocprim::radix_sort_pairs(tmp.p, sort_bytes, keys, keys_alt, vals_alt, vals, (size_t)nnz, 0u, end_bit, st));
            GRP_HIP(hipMemcpyAsync(h->csc_w, vals, (size_t)nnz * sizeof(float), hipMemcpyDeviceToDevice, st));
        }
    }
    hipLaunchKernelGGL(csr_from_keys_kernel, dim3(grid_for(nnz + 1)), dim3(256), 0, st, keys_alt, nnz, n, h->colptr, h->row);
    GRP_LAUNCH_CHECK();
    if (n > 0) {
        hipLaunchKernelGGL(degree_from_ptr_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, h->rowptr, n, h->d_local_in);
        GRP_LAUNCH_CHECK();
        hipLaunchKernelGGL(degree_from_ptr_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, h->colptr, n, h->d_local_out);
        GRP_LAUNCH_CHECK();
    }
    int64_t* const scanned = (int64_t*)tmp.p;            // the sorts are done (stream order): their scratch is free
    void* const scan_tmp = (char*)tmp.p + scanned_bytes;
    GRP_TRY(build_long_rows(h->rowptr, n, &h->csr_long, cap_long, cap_chunks, scanned, scan_tmp, scan_bytes, st));
    GRP_TRY(build_long_rows(h->colptr, n, &h->csc_long, cap_long, cap_chunks, scanned, scan_tmp, scan_bytes, st));
    GRP_HIP(hipStreamSynchronize(st));
    if (!vals) {                                          // weighted partitions keep the chunk schedule
        GRP_TRY(build_slice_tasks(h->rowptr, h->col, n, h->nnz, &h->csr_long, st));
        GRP_TRY(build_slice_tasks(h->colptr, h->row, n, h->nnz, &h->csc_long, st));
    }
    return GRP_OK;
}

static grp_status weighted_build(const int64_t* src, const int64_t* dst, const float* w, int64_t E, NodeSet own,
                                 hipStream_t st, grp_partition_t* h);

static grp_status partition_impl(const int64_t* src, const int64_t* dst, int64_t E, int64_t N, int32_t K, uint64_t seed,
                                 int32_t part_id, hipStream_t st, grp_partition_t* h, const float* w = nullptr,
                                 bool weighted = false) {
    // every N-sized temporary from one allocation: flags, positions, the node set, counters, scan scratch
    const int64_t n_words = cdiv(N > 0 ? N : 1, 32);
    size_t pos_scan_bytes = 0;
    if (N > 0)
        GRP_HIP(rocprim::exclusive_scan(nullptr, pos_scan_bytes, (const int32_t*)nullptr, (int64_t*)nullptr, (int64_t)0, (size_t)N,
                                        rocprim::plus<int64_t>(), st));
    const size_t set_scan_bytes = scan_temp_bytes(n_words + 1);
    const size_t scratch_bytes = pos_scan_bytes > set_scan_bytes ? pos_scan_bytes : set_scan_bytes;
    DevBuf slab;
    struct { int32_t* flag; int64_t* pos; unsigned long long* counters; uint32_t* bits; int32_t* before; char* scratch; } t{};
    for (int pass = 0; pass < 2; ++pass) {
        Bump b(slab.p, 0);
        t.counters = b.take<unsigned long long>(4);
        t.flag = b.take<int32_t>((size_t)(N > 0 ? N : 1));
        t.pos = b.take<int64_t>((size_t)(N > 0 ? N : 1));
        t.bits = b.take<uint32_t>((size_t)n_words + 1);
        t.before = b.take<int32_t>((size_t)n_words + 1);
        t.scratch = b.take<char>(scratch_bytes);
        if (pass == 0) GRP_TRY(slab.alloc(b.total()));
    }
    DevView flag{t.flag}, pos{t.pos}, counters{t.counters};
    GRP_HIP(hipMemsetAsync(counters.p, 0, 3 * sizeof(unsigned long long), st));

    int64_t n = 0;
    if (N > 0) {
        hipLaunchKernelGGL(owner_flag_kernel, dim3((unsigned)cdiv(N, 256)), dim3(256), 0, st, N, (uint32_t)K, seed,
                           (uint32_t)part_id, flag.as<int32_t>());
        GRP_LAUNCH_CHECK();
        GRP_HIP(rocprim::exclusive_scan(t.scratch, pos_scan_bytes, flag.as<int32_t>(), pos.as<int64_t>(), (int64_t)0, (size_t)N,
                                        rocprim::plus<int64_t>(), st));
        int64_t last_pos = 0;
        int32_t last_flag = 0;
        GRP_HIP(hipMemcpyAsync(&last_pos, pos.as<int64_t>() + (N - 1), sizeof(int64_t), hipMemcpyDeviceToHost, st));
        GRP_HIP(hipMemcpyAsync(&last_flag, flag.as<int32_t>() + (N - 1), sizeof(int32_t), hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
        n = last_pos + last_flag;
    }
    if (n >= ((int64_t)1 << 31)) return fail(GRP_ERANGE, "partition has %lld >= 2^31 local nodes", (long long)n);
    h->n = n;
    GRP_TRY(halloc(&h->l2g, n));
    GRP_TRY(halloc(&h->d_global_in, n));
    GRP_HIP(hipMemsetAsync(h->d_global_in, 0, (size_t)(n > 0 ? n : 1) * sizeof(int64_t), st));
    if (N > 0) {
        hipLaunchKernelGGL(scatter_l2g_kernel, dim3((unsigned)cdiv(N, 256)), dim3(256), 0, st, N, flag.as<int32_t>(),
                           pos.as<int64_t>(), h->l2g);
        GRP_LAUNCH_CHECK();
    }
    unsigned long long host_counters[3] = {0, 0, 0};
    NodeSet own{nullptr, nullptr};
    if (E > 0 && N > 0) {
        hipLaunchKernelGGL(pack_bits_kernel, dim3((unsigned)cdiv(n_words * 32, 256)), dim3(256), 0, st,
                           (const int32_t*)flag.as<int32_t>(), N, n_words, t.bits);
        GRP_LAUNCH_CHECK();
        GRP_HIP(hipMemsetAsync(t.bits + n_words, 0, sizeof(uint32_t), st));
        GRP_TRY(exclusive_scan_popcount(t.scratch, set_scan_bytes, t.bits, t.before, n_words + 1, st));
        own = NodeSet{t.bits, t.before};
    }
    const unsigned scan_grid = grid_for(E) < (unsigned)EDGE_SCAN_GRID ? grid_for(E) : (unsigned)EDGE_SCAN_GRID;
    // unweighted: one pass writes the keys too, into a buffer sized for twice the expected E / K^2 kept edges
    int64_t cap = weighted ? 0 : 2 * (E / K / K) + (1 << 20);
    if (cap > E) cap = E;
    DevBuf keybuf;                                       // both key arrays
    size_t key_pitch = (((size_t)(cap > 0 ? cap : 1) * sizeof(uint64_t)) + 255) & ~(size_t)255;
    if (!weighted) GRP_TRY(keybuf.alloc(2 * key_pitch));
    if (E > 0) {
        if (weighted) {
            ProfScope ps("partition_edge_scan", st, 0.0, 16.0 * (double)E);
            hipLaunchKernelGGL(edge_scan_kernel, dim3(scan_grid), dim3(256), 0, st, src, dst, E, N, own,
                               (unsigned long long*)h->d_global_in, counters.as<unsigned long long>());
            GRP_LAUNCH_CHECK();
        } else {
            ProfScope ps("partition_edge_scan_keys", st, 0.0, 16.0 * (double)E);
            hipLaunchKernelGGL(edge_scan_keys_kernel, dim3(scan_grid), dim3(256), 0, st, src, dst, E, N, own,
                               (unsigned long long*)h->d_global_in, counters.as<unsigned long long>(), keybuf.as<uint64_t>(),
                               (unsigned long long)cap);
            GRP_LAUNCH_CHECK();
        }
        GRP_HIP(hipMemcpyAsync(host_counters, counters.p, sizeof host_counters, hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
    }
    if (host_counters[1] != 0)
        return fail(GRP_ERANGE, "%llu edges have an endpoint outside [0, %lld)", host_counters[1], (long long)N);
    const int64_t nnz = (int64_t)(weighted ? host_counters[0] : host_counters[2]);
    h->nnz = nnz;
    if (weighted) return weighted_build(src, dst, w, E, own, st, h);
    DevBuf exact;                                        // only if the first buffer was too small
    uint64_t* keys = keybuf.as<uint64_t>();
    if (nnz > cap) {
        key_pitch = (((size_t)nnz * sizeof(uint64_t)) + 255) & ~(size_t)255;
        GRP_TRY(exact.alloc(2 * key_pitch));
        keys = exact.as<uint64_t>();
        GRP_HIP(hipMemsetAsync(counters.as<unsigned long long>() + 2, 0, sizeof(unsigned long long), st));
        ProfScope ps("partition_edge_keys", st, 0.0, 16.0 * (double)E + 8.0 * (double)nnz);
        hipLaunchKernelGGL(edge_keys_kernel<SetSelect>, dim3(grid_for(E)), dim3(256), 0, st, src, dst, E, SetSelect{own},
                           counters.as<unsigned long long>() + 2, keys);
        GRP_LAUNCH_CHECK();
    }
    uint64_t* const keys_alt = (uint64_t*)((char*)keys + key_pitch);
    return build_csr_csc(h, keys, keys_alt, st);
}

// ------------------------------------------------------------------ halo partitions
// One hop outwards: the source of every edge whose destination is already inside joins.
// The rest of a weighted partition build (h->n, h->nnz, h->l2g, h->d_global_in are set; the ids are
// range-checked): CSR/CSC with the edge weights carried along, then the weight masses.
static grp_status weighted_build(const int64_t* src, const int64_t* dst, const float* w, int64_t E, NodeSet own,
                                 hipStream_t st, grp_partition_t* h) {
    const int64_t n = h->n, nnz = h->nnz;
    DevBuf bad, tiles, scan_tmp;
    GRP_TRY(bad.alloc(sizeof(unsigned long long)));
    GRP_HIP(hipMemsetAsync(bad.p, 0, sizeof(unsigned long long), st));
    unsigned long long host_bad = 0;
    if (E > 0) {
        hipLaunchKernelGGL(weight_check_kernel, dim3(grid_for(E)), dim3(256), 0, st, w, E, bad.as<unsigned long long>());
        GRP_LAUNCH_CHECK();
        GRP_HIP(hipMemcpyAsync(&host_bad, bad.p, sizeof host_bad, hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
    }
    if (host_bad) return fail(GRP_EINVAL, "%llu edge weights are not positive finite numbers", host_bad);
    const int64_t n_tiles = cdiv(E, OC_TILE);
    const size_t tile_pitch = (((size_t)n_tiles + 1) * sizeof(int64_t) + 255) & ~(size_t)255;
    GRP_TRY(tiles.alloc(2 * tile_pitch));                 // per-tile counts, then their prefix sums
    int64_t* const tile_count = tiles.as<int64_t>();
    int64_t* const tile_base = (int64_t*)((char*)tiles.p + tile_pitch);
    const size_t scan_bytes = scan_temp_bytes(n_tiles + 1);
    GRP_TRY(scan_tmp.alloc(scan_bytes));
    const unsigned oc_grid = (unsigned)(n_tiles < 16384 ? (n_tiles > 0 ? n_tiles : 1) : 16384);
    // the slots of the selected edges, in edge-list order (which = 0: local edges, 1: every in-edge of an owned node)
    auto place = [&](int which) -> grp_status {
        if (E <= 0) return GRP_OK;
        if (which == 0)
            hipLaunchKernelGGL(ordered_count_kernel<0>, dim3(oc_grid), dim3(256), 0, st, src, dst, E, own, n_tiles, tile_count);
        else
            hipLaunchKernelGGL(ordered_count_kernel<1>, dim3(oc_grid), dim3(256), 0, st, src, dst, E, own, n_tiles, tile_count);
        GRP_LAUNCH_CHECK();
        return exclusive_scan_i64(scan_tmp.p, scan_bytes, tile_count, tile_base, n_tiles + 1, st);
    };
    // ---- local edges with their weights
    DevBuf keys, keys_alt, vals, vals_alt;
    GRP_TRY(keys.alloc((size_t)nnz * sizeof(uint64_t)));
    GRP_TRY(keys_alt.alloc((size_t)nnz * sizeof(uint64_t)));
    GRP_TRY(vals.alloc((size_t)nnz * sizeof(float)));
    GRP_TRY(vals_alt.alloc((size_t)nnz * sizeof(float)));
    if (nnz > 0) {
        GRP_TRY(place(0));
        hipLaunchKernelGGL(ordered_emit_kernel<0>, dim3(oc_grid), dim3(256), 0, st, src, dst, w, E, own, n_tiles,
                           (const int64_t*)tile_base, keys.as<uint64_t>(), (uint32_t*)nullptr, vals.as<float>());
        GRP_LAUNCH_CHECK();
    }
    GRP_TRY(build_csr_csc(h, keys.as<uint64_t>(), keys_alt.as<uint64_t>(), st, vals.as<float>(), vals_alt.as<float>()));
    GRP_TRY(halloc(&h->w_local_in, n));
    GRP_TRY(halloc(&h->w_global_in, n));
    if (n == 0) return GRP_OK;
    DevBuf mass_scratch;
    GRP_TRY(mass_scratch.alloc(((size_t)n + 1) * sizeof(int32_t)));
    GRP_TRY(launch_row_mass(h->rowptr, h->csr_w, n, h->w_local_in, mass_scratch.as<int32_t>(), st));
    // ---- every in-edge of an owned node, grouped by destination in edge-list order
    DevBuf cnt, off;
    GRP_TRY(cnt.alloc((size_t)(n + 1) * sizeof(int64_t)));
    GRP_TRY(off.alloc((size_t)(n + 1) * sizeof(int64_t)));
    GRP_HIP(hipMemsetAsync(cnt.p, 0, (size_t)(n + 1) * sizeof(int64_t), st));
    GRP_HIP(hipMemcpyAsync(cnt.p, h->d_global_in, (size_t)n * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
    {
        size_t bytes = 0;
        DevBuf tmp;
        GRP_HIP(rocprim::exclusive_scan(nullptr, bytes, cnt.as<int64_t>(), off.as<int64_t>(), (int64_t)0, (size_t)(n + 1),
                                        rocprim::plus<int64_t>(), st));
        GRP_TRY(tmp.alloc(bytes));
        GRP_HIP(rocprim::exclusive_scan(tmp.p, bytes, cnt.as<int64_t>(), off.as<int64_t>(), (int64_t)0, (size_t)(n + 1),
                                        rocprim::plus<int64_t>(), st));
        GRP_HIP(hipStreamSynchronize(st));        // tmp is released at the end of this scope
    }
    int64_t total = 0;
    GRP_HIP(hipMemcpy(&total, off.as<int64_t>() + n, sizeof(int64_t), hipMemcpyDeviceToHost));
    DevBuf k32, k32_alt, vin, vin_alt, sort_tmp;
    GRP_TRY(k32.alloc((size_t)total * sizeof(uint32_t)));
    GRP_TRY(k32_alt.alloc((size_t)total * sizeof(uint32_t)));
    GRP_TRY(vin.alloc((size_t)total * sizeof(float)));
    GRP_TRY(vin_alt.alloc((size_t)total * sizeof(float)));
    if (total > 0) {
        GRP_TRY(place(1));
        hipLaunchKernelGGL(ordered_emit_kernel<1>, dim3(oc_grid), dim3(256), 0, st, src, dst, w, E, own, n_tiles,
                           (const int64_t*)tile_base, (uint64_t*)nullptr, k32.as<uint32_t>(), vin.as<float>());
        GRP_LAUNCH_CHECK();
        const unsigned end_bit = (unsigned)bits_for(n > 1 ? n : 2);
        size_t bytes = 0;
        GRP_HIP(rocprim::radix_sort_pairs(nullptr, bytes, k32.as<uint32_t>(), k32_alt.as<uint32_t>(), vin.as<float>(),
                                          vin_alt.as<float>(), (size_t)total, 0u, end_bit, st));
        GRP_TRY(sort_tmp.alloc(bytes));
        GRP_HIP(rocprim::radix_sort_pairs(sort_tmp.p, bytes, k32.as<uint32_t>(), k32_alt.as<uint32_t>(), vin.as<float>(),
                                          vin_alt.as<float>(), (size_t)total, 0u, end_bit, st));
    }
    GRP_TRY(launch_row_mass(off.as<int64_t>(), vin_alt.as<float>(), n, h->w_global_in, mass_scratch.as<int32_t>(), st));
    GRP_HIP(hipStreamSynchronize(st));
    return GRP_OK;
}

__global__ __launch_bounds__(256) void halo_grow_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                        int64_t E, int64_t N, const int32_t* __restrict__ inner,
                                                        int32_t* __restrict__ member, unsigned long long* __restrict__ bad) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < E; e += (int64_t)gridDim.x * 256) {
        const int64_t u = src[e], v = dst[e];
        if (u < 0 || v < 0 || u >= N || v >= N) { atomicAdd(bad, 1ull); continue; }
        if (inner[v]) member[u] = 1;              // every writer stores the same value
    }
}

// Global in-degree of the members and the number of kept edges (destination in `inner`).
__global__ __launch_bounds__(256) void halo_scan_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                        int64_t E, const int32_t* __restrict__ member,
                                                        const int32_t* __restrict__ inner, const int64_t* __restrict__ pos,
                                                        unsigned long long* __restrict__ dg,
                                                        unsigned long long* __restrict__ kept_out) {
    __shared__ int32_t slot_key[DG_SLOTS];               // in-degree counts go through an LDS table (see edge_scan_kernel)
    __shared__ uint32_t slot_count[DG_SLOTS];
    for (int i = threadIdx.x; i < DG_SLOTS; i += 256) { slot_key[i] = -1; slot_count[i] = 0u; }
    __syncthreads();
    unsigned long long kept = 0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < E; e += (int64_t)gridDim.x * 256) {
        const int64_t v = dst[e];
        if (member[v]) dg_table_add(slot_key, slot_count, dg, (int32_t)pos[v]);
        if (inner[v]) kept++;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < DG_SLOTS; i += 256)
        if (slot_key[i] >= 0) atomicAdd(&dg[slot_key[i]], (unsigned long long)slot_count[i]);
    for (int o = 32; o > 0; o >>= 1) kept += __shfl_down(kept, o, 64);
    if ((threadIdx.x & 63) == 0 && kept) atomicAdd(kept_out, kept);
}

__global__ __launch_bounds__(256) void halo_nodes_kernel(int64_t N, const int32_t* __restrict__ member,
                                                         const int32_t* __restrict__ owned, const int64_t* __restrict__ pos,
                                                         int64_t* __restrict__ l2g, uint8_t* __restrict__ owned_mask) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < N && member[v]) {
        l2g[pos[v]] = v;
        owned_mask[pos[v]] = owned[v] ? 1 : 0;
    }
}

static grp_status halo_partition_impl(const int64_t* src, const int64_t* dst, int64_t E, int64_t N, int32_t K, uint64_t seed,
                                      int32_t part_id, int32_t hops, hipStream_t st, grp_partition_t* h) {
    DevBuf owned, member, inner, pos, counters, scan_tmp;
    GRP_TRY(owned.alloc((size_t)N * sizeof(int32_t)));
    GRP_TRY(member.alloc((size_t)N * sizeof(int32_t)));
    GRP_TRY(inner.alloc((size_t)N * sizeof(int32_t)));
    GRP_TRY(pos.alloc((size_t)N * sizeof(int64_t)));
    GRP_TRY(counters.alloc(3 * sizeof(unsigned long long)));          // [0] kept, [1] bad ids, [2] key cursor
    GRP_HIP(hipMemsetAsync(counters.p, 0, 3 * sizeof(unsigned long long), st));
    int64_t n = 0;
    if (N > 0) {
        hipLaunchKernelGGL(owner_flag_kernel, dim3((unsigned)cdiv(N, 256)), dim3(256), 0, st, N, (uint32_t)K, seed,
                           (uint32_t)part_id, owned.as<int32_t>());
        GRP_LAUNCH_CHECK();
        GRP_HIP(hipMemcpyAsync(member.p, owned.p, (size_t)N * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        for (int hop = 0; hop < hops; ++hop) {
            GRP_HIP(hipMemcpyAsync(inner.p, member.p, (size_t)N * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
            if (E > 0) {
                hipLaunchKernelGGL(halo_grow_kernel, dim3(grid_for(E)), dim3(256), 0, st, src, dst, E, N, inner.as<int32_t>(),
                                   member.as<int32_t>(), counters.as<unsigned long long>() + 1);
                GRP_LAUNCH_CHECK();
            }
        }
        size_t bytes = 0;
        GRP_HIP(rocprim::exclusive_scan(nullptr, bytes, member.as<int32_t>(), pos.as<int64_t>(), (int64_t)0, (size_t)N,
                                        rocprim::plus<int64_t>(), st));
        GRP_TRY(scan_tmp.alloc(bytes));
        GRP_HIP(rocprim::exclusive_scan(scan_tmp.p, bytes, member.as<int32_t>(), pos.as<int64_t>(), (int64_t)0, (size_t)N,
                                        rocprim::plus<int64_t>(), st));
        int64_t last_pos = 0;
        int32_t last_flag = 0;
        unsigned long long nbad = 0;
        GRP_HIP(hipMemcpyAsync(&last_pos, pos.as<int64_t>() + (N - 1), sizeof(int64_t), hipMemcpyDeviceToHost, st));
        GRP_HIP(hipMemcpyAsync(&last_flag, member.as<int32_t>() + (N - 1), sizeof(int32_t), hipMemcpyDeviceToHost, st));
        GRP_HIP(hipMemcpyAsync(&nbad, counters.as<unsigned long long>() + 1, sizeof nbad, hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
        if (nbad) return fail(GRP_ERANGE, "edges have an endpoint outside [0, %lld)", (long long)N);
        n = last_pos + last_flag;
    }
    if (n >= ((int64_t)1 << 31)) return fail(GRP_ERANGE, "partition has %lld >= 2^31 local nodes", (long long)n);
    h->n = n;
    GRP_TRY(halloc(&h->l2g, n));
    GRP_TRY(halloc(&h->d_global_in, n));
    GRP_TRY(halloc(&h->base_mask, n));
    GRP_HIP(hipMemsetAsync(h->d_global_in, 0, (size_t)(n > 0 ? n : 1) * sizeof(int64_t), st));
    unsigned long long kept = 0;
    if (N > 0) {
        hipLaunchKernelGGL(halo_nodes_kernel, dim3((unsigned)cdiv(N, 256)), dim3(256), 0, st, N, member.as<int32_t>(),
                           owned.as<int32_t>(), pos.as<int64_t>(), h->l2g, h->base_mask);
        GRP_LAUNCH_CHECK();
    }
    if (E > 0) {
        const unsigned scan_grid = grid_for(E) < (unsigned)EDGE_SCAN_GRID ? grid_for(E) : (unsigned)EDGE_SCAN_GRID;
        hipLaunchKernelGGL(halo_scan_kernel, dim3(scan_grid), dim3(256), 0, st, src, dst, E, member.as<int32_t>(),
                           inner.as<int32_t>(), pos.as<int64_t>(), (unsigned long long*)h->d_global_in,
                           counters.as<unsigned long long>());
        GRP_LAUNCH_CHECK();
        GRP_HIP(hipMemcpyAsync(&kept, counters.p, sizeof kept, hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
    }
    const int64_t nnz = (int64_t)kept;
    h->nnz = nnz;
    DevBuf keys, keys_alt;
    GRP_TRY(keys.alloc((size_t)nnz * sizeof(uint64_t)));
    GRP_TRY(keys_alt.alloc((size_t)nnz * sizeof(uint64_t)));
    if (nnz > 0) {
        hipLaunchKernelGGL(edge_keys_kernel<ArraySelect>, dim3(grid_for(E)), dim3(256), 0, st, src, dst, E,
                           ArraySelect{inner.as<int32_t>(), pos.as<int64_t>(), 1}, counters.as<unsigned long long>() + 2,
                           keys.as<uint64_t>());
        GRP_LAUNCH_CHECK();
    }
    return build_csr_csc(h, keys.as<uint64_t>(), keys_alt.as<uint64_t>(), st);
}

// ------------------------------------------------------------------ chunks
constexpr int MAX_CHUNKS = 64;        // n_chunks^2 bucket counters must fit a workgroup's LDS

// Node -> chunk: the random split, or a caller-supplied assignment (any partitioner's output).
struct ChunkMap {
    uint64_t seed;
    uint32_t c;
    const int32_t* assign;            // [N] chunk ids in [0, c), or null
};
__device__ __forceinline__ uint32_t chunk_of(const ChunkMap& m, int64_t v) {
    return m.assign ? (uint32_t)m.assign[v] : (uint32_t)(splitmix64_output(m.seed, (uint64_t)v) % m.c);
}

__global__ __launch_bounds__(256) void assignment_check_kernel(const int32_t* __restrict__ assign, int64_t N, int32_t c,
                                                               unsigned long long* __restrict__ bad) {
    unsigned long long b = 0;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < N; v += (int64_t)gridDim.x * 256)
        if (assign[v] < 0 || assign[v] >= c) b++;
    if (b) atomicAdd(bad, b);
}

// Pass 1: range check, global in-degrees, size of every (chunk(dst), chunk(src)) bucket.
__global__ __launch_bounds__(256) void chunk_count_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                          int64_t E, int64_t N, ChunkMap cm,
                                                          unsigned long long* __restrict__ dg,
                                                          unsigned long long* __restrict__ bucket_count,
                                                          unsigned long long* __restrict__ bad) {
    extern __shared__ unsigned int hist[];            // c*c counters of this workgroup
    const uint32_t c = cm.c;
    for (int i = threadIdx.x; i < (int)(c * c); i += 256) hist[i] = 0;
    __syncthreads();
    unsigned long long nbad = 0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < E; e += (int64_t)gridDim.x * 256) {
        const int64_t u = src[e], v = dst[e];
        if (u < 0 || v < 0 || u >= N || v >= N) { nbad++; continue; }
        atomicAdd(&dg[v], 1ull);
        atomicAdd(&hist[chunk_of(cm, v) * c + chunk_of(cm, u)], 1u);
    }
    if (nbad) atomicAdd(bad, nbad);
    __syncthreads();
    for (int i = threadIdx.x; i < (int)(c * c); i += 256)
        if (hist[i]) atomicAdd(&bucket_count[i], (unsigned long long)hist[i]);
}

// Pass 2: every workgroup reserves a run in each bucket for the edges it holds, then writes
// them (the order inside a bucket is arbitrary; partitions are sorted when they are built).
__global__ __launch_bounds__(256) void chunk_scatter_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                            int64_t E, ChunkMap cm,
                                                            unsigned long long* __restrict__ cursor,
                                                            int64_t* __restrict__ out_src, int64_t* __restrict__ out_dst) {
    extern __shared__ unsigned int lds_u32[];         // [0, c*c): counts, then run starts (low / high words)
    const uint32_t c = cm.c;
    unsigned int* cnt = lds_u32;
    unsigned long long* start = (unsigned long long*)(lds_u32 + ((c * c + 1) & ~1u));
    const int64_t per = (E + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * per, hi = lo + per < E ? lo + per : E;
    for (int i = threadIdx.x; i < (int)(c * c); i += 256) cnt[i] = 0;
    __syncthreads();
    for (int64_t e = lo + threadIdx.x; e < hi; e += 256)
        atomicAdd(&cnt[chunk_of(cm, dst[e]) * c + chunk_of(cm, src[e])], 1u);
    __syncthreads();
    for (int i = threadIdx.x; i < (int)(c * c); i += 256) {
        start[i] = cnt[i] ? atomicAdd(&cursor[i], (unsigned long long)cnt[i]) : 0ull;
        cnt[i] = 0;
    }
    __syncthreads();
    for (int64_t e = lo + threadIdx.x; e < hi; e += 256) {
        const int64_t u = src[e], v = dst[e];
        const uint32_t b = chunk_of(cm, v) * c + chunk_of(cm, u);
        const unsigned long long slot = start[b] + atomicAdd(&cnt[b], 1u);
        out_src[slot] = u;
        out_dst[slot] = v;
    }
}

__global__ __launch_bounds__(256) void pair_flag_kernel(int64_t N, ChunkMap cm, uint32_t base, uint32_t swept,
                                                        int32_t* __restrict__ flag) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < N) {
        const uint32_t ch = chunk_of(cm, v);
        flag[v] = (ch == base || ch == swept) ? 1 : 0;
    }
}

__global__ __launch_bounds__(256) void pair_nodes_kernel(int64_t N, ChunkMap cm, uint32_t base,
                                                         const int32_t* __restrict__ flag, const int64_t* __restrict__ pos,
                                                         const int64_t* __restrict__ dg_all, int64_t* __restrict__ l2g,
                                                         int64_t* __restrict__ dg, uint8_t* __restrict__ base_mask) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < N && flag[v]) {
        const int64_t i = pos[v];
        l2g[i] = v;
        dg[i] = dg_all[v];
        base_mask[i] = chunk_of(cm, v) == base ? 1 : 0;
    }
}

// Keys of one bucket's edges (both endpoints are members by construction).
__global__ __launch_bounds__(256) void bucket_keys_kernel(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                          int64_t count, const int64_t* __restrict__ pos,
                                                          uint64_t* __restrict__ keys) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256)
        keys[e] = ((uint64_t)pos[dst[e]] << 32) | (uint64_t)pos[src[e]];
}

static void free_chunks(grp_chunks_t* h) {
    if (!h) return;
    for (void* q : {(void*)h->src, (void*)h->dst, (void*)h->d_global_all, (void*)h->assign})
        if (q) (void)hipFree(q);
    delete h;
}

static grp_status chunks_impl(const int64_t* src, const int64_t* dst, int64_t E, int64_t N, int32_t c, uint64_t seed,
                              const int32_t* assignment, hipStream_t st, grp_chunks_t* h) {
    const int nb = c * c;
    h->n_chunks = c; h->seed = seed; h->N = N; h->E = E;
    h->bucket_ptr.assign((size_t)nb + 1, 0);
    if (assignment) {                                  // keep a checked copy: partitions are built from it later
        GRP_TRY(halloc(&h->assign, N));
        GRP_HIP(hipMemcpyAsync(h->assign, assignment, (size_t)N * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        DevBuf bad;
        GRP_TRY(bad.alloc(sizeof(unsigned long long)));
        GRP_HIP(hipMemsetAsync(bad.p, 0, sizeof(unsigned long long), st));
        unsigned long long host_bad = 0;
        if (N > 0) {
            hipLaunchKernelGGL(assignment_check_kernel, dim3(grid_for(N)), dim3(256), 0, st, (const int32_t*)h->assign, N, c,
                               bad.as<unsigned long long>());
            GRP_LAUNCH_CHECK();
        }
        GRP_HIP(hipMemcpyAsync(&host_bad, bad.p, sizeof host_bad, hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
        if (host_bad) return fail(GRP_ERANGE, "%llu nodes are assigned to a chunk outside [0, %d)", host_bad, c);
    }
    const ChunkMap cm{seed, (uint32_t)c, h->assign};
    GRP_TRY(halloc(&h->src, E));
    GRP_TRY(halloc(&h->dst, E));
    GRP_TRY(halloc(&h->d_global_all, N));
    GRP_HIP(hipMemsetAsync(h->d_global_all, 0, (size_t)(N > 0 ? N : 1) * sizeof(int64_t), st));
    DevBuf counters;                                   // [0, nb): counts then cursors; [nb]: bad ids
    GRP_TRY(counters.alloc((size_t)(nb + 1) * sizeof(unsigned long long)));
    GRP_HIP(hipMemsetAsync(counters.p, 0, (size_t)(nb + 1) * sizeof(unsigned long long), st));
    if (E == 0) { GRP_HIP(hipStreamSynchronize(st)); return GRP_OK; }
    const unsigned grid = grid_for(E) > 2048 ? 2048 : grid_for(E);
    hipLaunchKernelGGL(chunk_count_kernel, dim3(grid), dim3(256), (size_t)nb * sizeof(unsigned int), st, src, dst, E, N,
                       cm, (unsigned long long*)h->d_global_all, counters.as<unsigned long long>(),
                       counters.as<unsigned long long>() + nb);
    GRP_LAUNCH_CHECK();
    std::vector<unsigned long long> host((size_t)nb + 1);
    GRP_HIP(hipMemcpyAsync(host.data(), counters.p, host.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    GRP_HIP(hipStreamSynchronize(st));
    if (host[nb] != 0) return fail(GRP_ERANGE, "%llu edges have an endpoint outside [0, %lld)", host[nb], (long long)N);
    for (int b = 0; b < nb; ++b) h->bucket_ptr[b + 1] = h->bucket_ptr[b] + (int64_t)host[b];
    std::vector<unsigned long long> cur((size_t)nb);
    for (int b = 0; b < nb; ++b) cur[b] = (unsigned long long)h->bucket_ptr[b];
    GRP_HIP(hipMemcpyAsync(counters.p, cur.data(), cur.size() * sizeof(unsigned long long), hipMemcpyHostToDevice, st));
    const size_t lds = (size_t)((nb + 1) & ~1) * sizeof(unsigned int) + (size_t)nb * sizeof(unsigned long long);
    hipLaunchKernelGGL(chunk_scatter_kernel, dim3(grid), dim3(256), lds, st, src, dst, E, cm,
                       counters.as<unsigned long long>(), h->src, h->dst);
    GRP_LAUNCH_CHECK();
    GRP_HIP(hipStreamSynchronize(st));
    return GRP_OK;
}

static grp_status pair_partition_impl(const grp_chunks_t* ck, int32_t base, int32_t swept, hipStream_t st,
                                      grp_partition_t* h) {
    const int64_t N = ck->N;
    const int c = ck->n_chunks;
    DevBuf flag, pos, scan_tmp;
    GRP_TRY(flag.alloc((size_t)N * sizeof(int32_t)));
    GRP_TRY(pos.alloc((size_t)N * sizeof(int64_t)));
    int64_t n = 0;
    if (N > 0) {
        hipLaunchKernelGGL(pair_flag_kernel, dim3((unsigned)cdiv(N, 256)), dim3(256), 0, st, N, ChunkMap{ck->seed, (uint32_t)c, ck->assign},
                           (uint32_t)base, (uint32_t)swept, flag.as<int32_t>());
        GRP_LAUNCH_CHECK();
        size_t bytes = 0;
        GRP_HIP(rocprim::exclusive_scan(nullptr, bytes, flag.as<int32_t>(), pos.as<int64_t>(), (int64_t)0, (size_t)N,
                                        rocprim::plus<int64_t>(), st));
        GRP_TRY(scan_tmp.alloc(bytes));
        GRP_HIP(rocprim::exclusive_scan(scan_tmp.p, bytes, flag.as<int32_t>(), pos.as<int64_t>(), (int64_t)0, (size_t)N,
                                        rocprim::plus<int64_t>(), st));
        int64_t last_pos = 0;
        int32_t last_flag = 0;
        GRP_HIP(hipMemcpyAsync(&last_pos, pos.as<int64_t>() + (N - 1), sizeof(int64_t), hipMemcpyDeviceToHost, st));
        GRP_HIP(hipMemcpyAsync(&last_flag, flag.as<int32_t>() + (N - 1), sizeof(int32_t), hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
        n = last_pos + last_flag;
    }
    if (n >= ((int64_t)1 << 31)) return fail(GRP_ERANGE, "partition has %lld >= 2^31 local nodes", (long long)n);
    h->n = n;
    GRP_TRY(halloc(&h->l2g, n));
    GRP_TRY(halloc(&h->d_global_in, n));
    GRP_TRY(halloc(&h->base_mask, n));
    if (N > 0) {
        hipLaunchKernelGGL(pair_nodes_kernel, dim3((unsigned)cdiv(N, 256)), dim3(256), 0, st, N, ChunkMap{ck->seed, (uint32_t)c, ck->assign},
                           (uint32_t)base, flag.as<int32_t>(), pos.as<int64_t>(), ck->d_global_all, h->l2g, h->d_global_in,
                           h->base_mask);
        GRP_LAUNCH_CHECK();
    }
    // the partition's edges are exactly the buckets (x, y) with x, y in {base, swept}
    int chunks2[2] = {base, swept};
    const int nc = base == swept ? 1 : 2;
    int64_t nnz = 0;
    for (int a = 0; a < nc; ++a)
        for (int b = 0; b < nc; ++b) {
            const int bk = chunks2[a] * c + chunks2[b];
            nnz += ck->bucket_ptr[bk + 1] - ck->bucket_ptr[bk];
        }
    h->nnz = nnz;
    DevBuf keys, keys_alt;
    GRP_TRY(keys.alloc((size_t)nnz * sizeof(uint64_t)));
    GRP_TRY(keys_alt.alloc((size_t)nnz * sizeof(uint64_t)));
    int64_t off = 0;
    for (int a = 0; a < nc; ++a)
        for (int b = 0; b < nc; ++b) {
            const int bk = chunks2[a] * c + chunks2[b];
            const int64_t lo = ck->bucket_ptr[bk], cnt = ck->bucket_ptr[bk + 1] - lo;
            if (cnt > 0) {
                hipLaunchKernelGGL(bucket_keys_kernel, dim3(grid_for(cnt)), dim3(256), 0, st, ck->src + lo, ck->dst + lo, cnt,
                                   pos.as<int64_t>(), keys.as<uint64_t>() + off);
                GRP_LAUNCH_CHECK();
            }
            off += cnt;
        }
    return build_csr_csc(h, keys.as<uint64_t>(), keys_alt.as<uint64_t>(), st);
}

}  // namespace grp

extern "C" grp_status grp_chunks_build(const int64_t* src, const int64_t* dst, int64_t E, int64_t N, int32_t n_chunks,
                                       uint64_t seed, void* stream, grp_chunks_t** out) {
    using namespace grp;
    if (!out) return fail(GRP_EINVAL, "grp_chunks_build: out is null");
    *out = nullptr;
    if (E < 0 || N < 0) return fail(GRP_EINVAL, "grp_chunks_build: negative size");
    if (E > 0 && (!src || !dst)) return fail(GRP_EINVAL, "grp_chunks_build: null edge arrays");
    if (n_chunks < 1 || n_chunks > MAX_CHUNKS)
        return fail(GRP_EINVAL, "grp_chunks_build: n_chunks = %d outside [1, %d]", n_chunks, MAX_CHUNKS);
    grp_chunks_t* h = new (std::nothrow) grp_chunks_t();
    if (!h) return fail(GRP_ENOMEM, "grp_chunks_build: host allocation failed");
    (void)hipGetDevice(&h->device);
    const grp_status s = chunks_impl(src, dst, E, N, n_chunks, seed, nullptr, (hipStream_t)stream, h);
    if (s != GRP_OK) {
        free_chunks(h);
        return s;
    }
    *out = h;
    return GRP_OK;
}

extern "C" grp_status grp_chunks_build_assigned(const int64_t* src, const int64_t* dst, int64_t E, int64_t N,
                                                int32_t n_chunks, const int32_t* chunk_of_node, void* stream,
                                                grp_chunks_t** out) {
    using namespace grp;
    if (!out) return fail(GRP_EINVAL, "grp_chunks_build_assigned: out is null");
    *out = nullptr;
    if (E < 0 || N < 0) return fail(GRP_EINVAL, "grp_chunks_build_assigned: negative size");
    if (E > 0 && (!src || !dst)) return fail(GRP_EINVAL, "grp_chunks_build_assigned: null edge arrays");
    if (N > 0 && !chunk_of_node) return fail(GRP_EINVAL, "grp_chunks_build_assigned: null assignment");
    if (n_chunks < 1 || n_chunks > MAX_CHUNKS)
        return fail(GRP_EINVAL, "grp_chunks_build_assigned: n_chunks = %d outside [1, %d]", n_chunks, MAX_CHUNKS);
    grp_chunks_t* h = new (std::nothrow) grp_chunks_t();
    if (!h) return fail(GRP_ENOMEM, "grp_chunks_build_assigned: host allocation failed");
    (void)hipGetDevice(&h->device);
    const grp_status s = chunks_impl(src, dst, E, N, n_chunks, 0, chunk_of_node, (hipStream_t)stream, h);
    if (s != GRP_OK) {
        free_chunks(h);
        return s;
    }
    *out = h;
    return GRP_OK;
}

extern "C" grp_status grp_chunks_destroy(grp_chunks_t* chunks) {
    grp::free_chunks(chunks);
    return GRP_OK;
}

extern "C" grp_status grp_partition_from_chunks(const grp_chunks_t* chunks, int32_t base, int32_t swept, void* stream,
                                                grp_partition_t** out) {
    using namespace grp;
    if (!out) return fail(GRP_EINVAL, "grp_partition_from_chunks: out is null");
    *out = nullptr;
    if (!chunks) return fail(GRP_EINVAL, "grp_partition_from_chunks: chunks is null");
    if (base < 0 || base >= chunks->n_chunks || swept < 0 || swept >= chunks->n_chunks)
        return fail(GRP_EINVAL, "grp_partition_from_chunks: chunk ids (%d, %d) outside [0, %d)", base, swept, chunks->n_chunks);
    grp_partition_t* h = new (std::nothrow) grp_partition_t();
    if (!h) return fail(GRP_ENOMEM, "grp_partition_from_chunks: host allocation failed");
    (void)hipGetDevice(&h->device);
    const grp_status s = pair_partition_impl(chunks, base, swept, (hipStream_t)stream, h);
    if (s != GRP_OK) {
        free_partition(h);
        return s;
    }
    *out = h;
    return GRP_OK;
}

extern "C" grp_status grp_partition_halo(const int64_t* src, const int64_t* dst, int64_t E, int64_t N, int32_t K, uint64_t seed,
                                         int32_t part_id, int32_t hops, void* stream, grp_partition_t** out) {
    using namespace grp;
    if (!out) return fail(GRP_EINVAL, "grp_partition_halo: out is null");
    *out = nullptr;
    if (E < 0 || N < 0) return fail(GRP_EINVAL, "grp_partition_halo: negative size");
    if (E > 0 && (!src || !dst)) return fail(GRP_EINVAL, "grp_partition_halo: null edge arrays");
    if (K < 1) return fail(GRP_EINVAL, "grp_partition_halo: K = %d < 1", K);
    if (part_id < 0 || part_id >= K) return fail(GRP_EINVAL, "grp_partition_halo: part_id %d outside [0, %d)", part_id, K);
    if (hops < 1 || hops > GRP_MAX_LAYERS) return fail(GRP_EINVAL, "grp_partition_halo: hops = %d outside [1, %d]", hops, GRP_MAX_LAYERS);
    grp_partition_t* h = new (std::nothrow) grp_partition_t();
    if (!h) return fail(GRP_ENOMEM, "grp_partition_halo: host allocation failed");
    (void)hipGetDevice(&h->device);
    const grp_status s = halo_partition_impl(src, dst, E, N, K, seed, part_id, hops, (hipStream_t)stream, h);
    if (s != GRP_OK) {
        free_partition(h);
        return s;
    }
    *out = h;
    return GRP_OK;
}

extern "C" grp_status grp_partition_base_mask(const grp_partition_t* part, const uint8_t** mask) {
    if (!part || !mask) return grp::fail(GRP_EINVAL, "grp_partition_base_mask: null argument");
    *mask = part->base_mask;
    return GRP_OK;
}

extern "C" grp_status grp_partition(const int64_t* src, const int64_t* dst, int64_t E, int64_t N, int32_t K, uint64_t seed,
                                    int32_t part_id, void* stream, grp_partition_t** out) {
    using namespace grp;
    if (!out) return fail(GRP_EINVAL, "grp_partition: out is null");
    *out = nullptr;
    if (E < 0 || N < 0) return fail(GRP_EINVAL, "grp_partition: negative size");
    if (E > 0 && (!src || !dst)) return fail(GRP_EINVAL, "grp_partition: null edge arrays");
    if (K < 1) return fail(GRP_EINVAL, "grp_partition: K = %d < 1", K);
    if (part_id < 0 || part_id >= K) return fail(GRP_EINVAL, "grp_partition: part_id %d outside [0, %d)", part_id, K);
    grp_partition_t* h = new (std::nothrow) grp_partition_t();
    if (!h) return fail(GRP_ENOMEM, "grp_partition: host allocation failed");
    (void)hipGetDevice(&h->device);
    const grp_status s = partition_impl(src, dst, E, N, K, seed, part_id, (hipStream_t)stream, h);
    if (s != GRP_OK) {
        free_partition(h);
        return s;
    }
    *out = h;
    return GRP_OK;
}

extern "C" grp_status grp_node_owners(int64_t N, int32_t K, uint64_t seed, int32_t* owner_out, int64_t* count_out,
                                      void* stream) {
    using namespace grp;
    if (N < 0 || K < 1) return fail(GRP_EINVAL, "grp_node_owners: N = %lld, K = %d", (long long)N, K);
    if (N > 0 && !owner_out) return fail(GRP_EINVAL, "grp_node_owners: null output");
    hipStream_t st = (hipStream_t)stream;
    if (count_out) GRP_TRY(launch_fill_zero(count_out, (size_t)K * sizeof(int64_t), st));    // a kernel: the call can be captured in a graph
    if (N == 0) return GRP_OK;
    int64_t blocks = cdiv(N, 256 * 8);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(node_owners_kernel, dim3((unsigned)blocks), dim3(256), 0, st, N, (uint32_t)K, seed, owner_out,
                       (unsigned long long*)count_out);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

namespace grp {
// ---- seed order of an epoch: the training nodes sorted by M(M(M(seed) ^ epoch) ^ global id), ties by local id
__global__ __launch_bounds__(256) void train_flag_kernel(const uint8_t* __restrict__ mask, int64_t n,
                                                         int32_t* __restrict__ flag /*[n+1]*/) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v > n) return;
    flag[v] = v < n && (!mask || mask[v] != 0) ? 1 : 0;
}

__global__ __launch_bounds__(256) void seed_keys_kernel(const int32_t* __restrict__ flag, const int32_t* __restrict__ pos,
                                                        const int64_t* __restrict__ l2g, int64_t n, uint64_t h,
                                                        uint64_t* __restrict__ keys, int32_t* __restrict__ ids) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n || !flag[v]) return;
    keys[pos[v]] = mixM(h ^ (uint64_t)l2g[v]);           // slots ascend with the local id: the stable sort keeps ties in that order
    ids[pos[v]] = (int32_t)v;
}
}  // namespace grp

extern "C" grp_status grp_epoch_seeds(const grp_partition_t* part, const uint8_t* train_mask, uint64_t sampler_seed,
                                      uint64_t epoch, void* stream, int32_t* seeds_out, int64_t* n_seeds_out) {
    using namespace grp;
    if (!part || !n_seeds_out) return fail(GRP_EINVAL, "grp_epoch_seeds: null argument");
    *n_seeds_out = 0;
    const int64_t n = part->n;
    if (n == 0) return GRP_OK;
    if (!seeds_out) return fail(GRP_EINVAL, "grp_epoch_seeds: null output");
    hipStream_t st = (hipStream_t)stream;
    DevBuf flag, pos, keys, keys_alt, ids, tmp;
    GRP_TRY(flag.alloc(((size_t)n + 1) * sizeof(int32_t)));
    GRP_TRY(pos.alloc(((size_t)n + 1) * sizeof(int32_t)));
    GRP_TRY(keys.alloc((size_t)n * sizeof(uint64_t)));
    GRP_TRY(keys_alt.alloc((size_t)n * sizeof(uint64_t)));
    GRP_TRY(ids.alloc((size_t)n * sizeof(int32_t)));
    size_t sort_bytes = 0;
    GRP_HIP(rocprim::radix_sort_pairs(nullptr, sort_bytes, keys.as<uint64_t>(), keys_alt.as<uint64_t>(), ids.as<int32_t>(),
                                      seeds_out, (size_t)n, 0u, 64u, st));
    const size_t scan_bytes = scan_temp_bytes(n + 1);
    GRP_TRY(tmp.alloc(sort_bytes > scan_bytes ? sort_bytes : scan_bytes));
    hipLaunchKernelGGL(train_flag_kernel, dim3((unsigned)cdiv(n + 1, 256)), dim3(256), 0, st, train_mask, n, flag.as<int32_t>());
    GRP_LAUNCH_CHECK();
    GRP_TRY(exclusive_scan_i32(tmp.p, scan_bytes, flag.as<int32_t>(), pos.as<int32_t>(), n + 1, st));
    hipLaunchKernelGGL(seed_keys_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, (const int32_t*)flag.as<int32_t>(),
                       (const int32_t*)pos.as<int32_t>(), part->l2g, n, mixM(mixM(sampler_seed) ^ epoch), keys.as<uint64_t>(),
                       ids.as<int32_t>());
    GRP_LAUNCH_CHECK();
    int32_t total = 0;
    GRP_HIP(hipMemcpyAsync(&total, pos.as<int32_t>() + n, sizeof total, hipMemcpyDeviceToHost, st));
    GRP_HIP(hipStreamSynchronize(st));
    if (total > 0) {
        GRP_HIP(rocprim::radix_sort_pairs(tmp.p, sort_bytes, keys.as<uint64_t>(), keys_alt.as<uint64_t>(), ids.as<int32_t>(),
                                          seeds_out, (size_t)total, 0u, 64u, st));
        GRP_HIP(hipStreamSynchronize(st));               // the temporaries are released on return
    }
    *n_seeds_out = total;
    return GRP_OK;
}

extern "C" grp_status grp_partition_weighted(const int64_t* src, const int64_t* dst, const float* w, int64_t E, int64_t N,
                                             int32_t K, uint64_t seed, int32_t part_id, void* stream,
                                             grp_partition_t** out) {
    using namespace grp;
    if (!out) return fail(GRP_EINVAL, "grp_partition_weighted: out is null");
    *out = nullptr;
    if (E < 0 || N < 0) return fail(GRP_EINVAL, "grp_partition_weighted: negative size");
    if (E > 0 && (!src || !dst)) return fail(GRP_EINVAL, "grp_partition_weighted: null edge arrays");
    if (E > 0 && !w) return fail(GRP_EINVAL, "grp_partition_weighted: null weights");
    if (K < 1) return fail(GRP_EINVAL, "grp_partition_weighted: K = %d < 1", K);
    if (part_id < 0 || part_id >= K)
        return fail(GRP_EINVAL, "grp_partition_weighted: part_id %d outside [0, %d)", part_id, K);
    grp_partition_t* h = new (std::nothrow) grp_partition_t();
    if (!h) return fail(GRP_ENOMEM, "grp_partition_weighted: host allocation failed");
    (void)hipGetDevice(&h->device);
    const grp_status s = partition_impl(src, dst, E, N, K, seed, part_id, (hipStream_t)stream, h, w, true);
    if (s != GRP_OK) {
        free_partition(h);
        return s;
    }
    *out = h;
    return GRP_OK;
}

extern "C" grp_status grp_partition_weights(const grp_partition_t* part, grp_partition_weights_t* view) {
    if (!part || !view) return grp::fail(GRP_EINVAL, "grp_partition_weights: null argument");
    view->csr_w = part->csr_w;
    view->csc_w = part->csc_w;
    view->w_local_in = part->w_local_in;
    view->w_global_in = part->w_global_in;
    return GRP_OK;
}

extern "C" grp_status grp_partition_from_local_coo(const int64_t* src_local, const int64_t* dst_local, int64_t E, int64_t n,
                                                   const int64_t* d_global_in, const int64_t* l2g, void* stream,
                                                   grp_partition_t** out) {
    using namespace grp;
    if (!out) return fail(GRP_EINVAL, "grp_partition_from_local_coo: out is null");
    *out = nullptr;
    if (E < 0 || n < 0) return fail(GRP_EINVAL, "grp_partition_from_local_coo: negative size");
    if (E > 0 && (!src_local || !dst_local)) return fail(GRP_EINVAL, "grp_partition_from_local_coo: null edge arrays");
    if (n >= ((int64_t)1 << 31)) return fail(GRP_ERANGE, "n = %lld >= 2^31", (long long)n);
    hipStream_t st = (hipStream_t)stream;
    grp_partition_t* h = new (std::nothrow) grp_partition_t();
    if (!h) return fail(GRP_ENOMEM, "host allocation failed");
    (void)hipGetDevice(&h->device);
    h->n = n;
    h->nnz = E;
    auto body = [&]() -> grp_status {
        DevBuf keys, keys_alt, bad;
        GRP_TRY(keys.alloc((size_t)E * sizeof(uint64_t)));
        GRP_TRY(keys_alt.alloc((size_t)E * sizeof(uint64_t)));
        GRP_TRY(bad.alloc(sizeof(unsigned long long)));
        GRP_HIP(hipMemsetAsync(bad.p, 0, sizeof(unsigned long long), st));
        if (E > 0) {
            hipLaunchKernelGGL(local_keys_kernel, dim3(grid_for(E)), dim3(256), 0, st, src_local, dst_local, E, n,
                               keys.as<uint64_t>(), bad.as<unsigned long long>());
            GRP_LAUNCH_CHECK();
        }
        unsigned long long nbad = 0;
        GRP_HIP(hipMemcpyAsync(&nbad, bad.p, sizeof nbad, hipMemcpyDeviceToHost, st));
        GRP_HIP(hipStreamSynchronize(st));
        if (nbad) return fail(GRP_ERANGE, "%llu edges have an endpoint outside [0, %lld)", nbad, (long long)n);
        GRP_TRY(build_csr_csc(h, keys.as<uint64_t>(), keys_alt.as<uint64_t>(), st));
        GRP_TRY(halloc(&h->l2g, n));
        GRP_TRY(halloc(&h->d_global_in, n));
        if (n > 0) {
            const unsigned g = (unsigned)cdiv(n, 256);
            if (l2g) GRP_HIP(hipMemcpyAsync(h->l2g, l2g, (size_t)n * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
            else hipLaunchKernelGGL(iota_kernel, dim3(g), dim3(256), 0, st, n, h->l2g);
            if (d_global_in)
                GRP_HIP(hipMemcpyAsync(h->d_global_in, d_global_in, (size_t)n * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
            else hipLaunchKernelGGL(widen_kernel, dim3(g), dim3(256), 0, st, h->d_local_in, n, h->d_global_in);
            GRP_LAUNCH_CHECK();
        }
        GRP_HIP(hipStreamSynchronize(st));
        return GRP_OK;
    };
    const grp_status s = body();
    if (s != GRP_OK) {
        free_partition(h);
        return s;
    }
    *out = h;
    return GRP_OK;
}

extern "C" grp_status grp_partition_view(const grp_partition_t* part, grp_partition_view_t* view) {
    if (!part || !view) return grp::fail(GRP_EINVAL, "grp_partition_view: null argument");
    view->n = part->n;
    view->nnz = part->nnz;
    view->l2g = part->l2g;
    view->rowptr = part->rowptr;
    view->col = part->col;
    view->colptr = part->colptr;
    view->row = part->row;
    view->d_local_in = part->d_local_in;
    view->d_local_out = part->d_local_out;
    view->d_global_in = part->d_global_in;
    return GRP_OK;
}

extern "C" grp_status grp_partition_destroy(grp_partition_t* part) {
    grp::free_partition(part);
    return GRP_OK;
}

// ------------------------------------------------------------------ shared device primitives
namespace grp {

size_t sort_keys_temp_bytes(int64_t count) {
    size_t bytes = 0;
    (void)rocprim::radix_sort_keys(nullptr, bytes, (const uint64_t*)nullptr, (uint64_t*)nullptr,
                                   (size_t)(count > 0 ? count : 1), 0u, 64u, (hipStream_t)0);
    return bytes + 256;
}

grp_status sort_keys_u64(void* temp, size_t temp_bytes, const uint64_t* in, uint64_t* out, int64_t count,
                         unsigned end_bit, hipStream_t st) {
    if (count <= 0) return GRP_OK;
    size_t need = 0;
    GRP_HIP(rocprim::radix_sort_keys(nullptr, need, in, out, (size_t)count, 0u, end_bit, st));
    if (need > temp_bytes) return fail(GRP_EWORKSPACE, "sort temp %zu < %zu", temp_bytes, need);
    GRP_HIP(rocprim::radix_sort_keys(temp, need, in, out, (size_t)count, 0u, end_bit, st));
    return GRP_OK;
}

size_t scan_temp_bytes(int64_t count) {
    size_t bytes = 0;
    (void)rocprim::exclusive_scan(nullptr, bytes, (const int64_t*)nullptr, (int64_t*)nullptr, (int64_t)0,
                                  (size_t)(count > 0 ? count : 1), rocprim::plus<int64_t>(), (hipStream_t)0);
    return bytes + 256;
}

grp_status exclusive_scan_i64(void* temp, size_t temp_bytes, const int64_t* in, int64_t* out, int64_t count,
                              hipStream_t st) {
    if (count <= 0) return GRP_OK;
    size_t need = 0;
    GRP_HIP(rocprim::exclusive_scan(nullptr, need, in, out, (int64_t)0, (size_t)count, rocprim::plus<int64_t>(), st));
    if (need > temp_bytes) return fail(GRP_EWORKSPACE, "scan temp %zu < %zu", temp_bytes, need);
    GRP_HIP(rocprim::exclusive_scan(temp, need, in, out, (int64_t)0, (size_t)count, rocprim::plus<int64_t>(), st));
    return GRP_OK;
}

grp_status exclusive_scan_i32(void* temp, size_t temp_bytes, const int32_t* in, int32_t* out, int64_t count,
                              hipStream_t st) {
    if (count <= 0) return GRP_OK;
    size_t need = 0;
    GRP_HIP(rocprim::exclusive_scan(nullptr, need, in, out, (int32_t)0, (size_t)count, rocprim::plus<int32_t>(), st));
    if (need > temp_bytes) return fail(GRP_EWORKSPACE, "scan temp %zu < %zu", temp_bytes, need);
    GRP_HIP(rocprim::exclusive_scan(temp, need, in, out, (int32_t)0, (size_t)count, rocprim::plus<int32_t>(), st));
    return GRP_OK;
}

struct PopcountOf {
    __host__ __device__ int32_t operator()(uint32_t w) const {
#if defined(__HIP_DEVICE_COMPILE__)
        return __popc(w);
#else
        return __builtin_popcount(w);
#endif
    }
};

// out[i] = number of set bits in words[0 .. i), for i in [0, count)
grp_status exclusive_scan_popcount(void* temp, size_t temp_bytes, const uint32_t* words, int32_t* out, int64_t count,
                                   hipStream_t st) {
    if (count <= 0) return GRP_OK;
    auto in = rocprim::make_transform_iterator(words, PopcountOf());
    size_t need = 0;
    GRP_HIP(rocprim::exclusive_scan(nullptr, need, in, out, (int32_t)0, (size_t)count, rocprim::plus<int32_t>(), st));
    if (need > temp_bytes) return fail(GRP_EWORKSPACE, "scan temp %zu < %zu", temp_bytes, need);
    GRP_HIP(rocprim::exclusive_scan(temp, need, in, out, (int32_t)0, (size_t)count, rocprim::plus<int32_t>(), st));
    return GRP_OK;
}

// Same result as csr_from_keys_kernel for matrices with many empty rows (a sampled block has more
// rows than most of them have entries): every row pointer is found by binary search instead of by
// the thread at the end of the previous row walking over the gap.
__global__ __launch_bounds__(256) void csr_from_keys_search_kernel(const uint64_t* __restrict__ keys, int64_t nnz, int64_t n,
                                                                   int64_t* __restrict__ ptr, int32_t* __restrict__ idx) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < nnz) idx[i] = (int32_t)(keys[i] & 0xFFFFFFFFull);
    if (i <= n) {
        int64_t lo = 0, hi = nnz;                        // first position whose row is >= i
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if ((int64_t)(keys[mid] >> 32) < i) lo = mid + 1; else hi = mid;
        }
        ptr[i] = lo;
    }
}

grp_status launch_csr_from_sorted_keys(const uint64_t* keys, int64_t nnz, int64_t n, int64_t* ptr, int32_t* idx,
                                       hipStream_t st) {
    const int64_t work = nnz > n + 1 ? nnz : n + 1;
    hipLaunchKernelGGL(csr_from_keys_search_kernel, dim3((unsigned)cdiv(work, 256)), dim3(256), 0, st, keys, nnz, n, ptr, idx);
    GRP_LAUNCH_CHECK();
    return GRP_OK;
}

// ---- split schedule of the long rows, built on the device (no host pass, no synchronisation).
// The exclusive prefix sum of (1 << 32 | chunks of row r) for a long row, 0 otherwise, gives every
// long row its slot (high half) and first chunk (low half), in ascending row order.
struct LongRowPack {
    const int64_t* ptr;
    int64_t n;
    __host__ __device__ int64_t operator()(int64_t r) const {
        if (r >= n) return 0;
        const int64_t len = ptr[r + 1] - ptr[r];
        return len > SPMM_LONG_ROW ? (((int64_t)1 << 32) | ((len + SPMM_CHUNK - 1) / SPMM_CHUNK)) : 0;
    }
};

// Slots past the real counts are made harmless: row -1 (skipped by the combine pass), empty chunks.
__global__ __launch_bounds__(256) void long_rows_emit_kernel(const int64_t* __restrict__ ptr, int64_t n,
                                                             const int64_t* __restrict__ scanned /*[n+1]*/,
                                                             int64_t cap_long, int64_t cap_chunks,
                                                             int32_t* __restrict__ long_row, int32_t* __restrict__ long_first,
                                                             int64_t* __restrict__ chunk_begin, int64_t* __restrict__ chunk_end) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = scanned[n];
    const int64_t n_long = total >> 32, n_chunks = total & 0xFFFFFFFFll;
    if (r < n) {
        const int64_t b = ptr[r], e = ptr[r + 1];
        if (e - b > SPMM_LONG_ROW) {
            const int64_t slot = scanned[r] >> 32;
            int64_t c = scanned[r] & 0xFFFFFFFFll;
            if (slot < cap_long) {
                long_row[slot] = (int32_t)r;
                long_first[slot] = (int32_t)c;
            }
            for (int64_t at = b; at < e; at += SPMM_CHUNK, ++c) {
                if (c >= cap_chunks) break;
                chunk_begin[c] = at;
                chunk_end[c] = at + SPMM_CHUNK < e ? at + SPMM_CHUNK : e;
            }
        }
    }
    if (r >= n_long && r <= cap_long) {
        if (r < cap_long) long_row[r] = -1;
        long_first[r] = (int32_t)(n_chunks < cap_chunks ? n_chunks : cap_chunks);
    }
    if (r >= n_chunks && r < cap_chunks) { chunk_begin[r] = 0; chunk_end[r] = 0; }
}

grp_status build_long_rows_device(const int64_t* ptr_dev, int64_t n, LongRows* out, int64_t cap_long, int64_t cap_chunks,
                                  int64_t* scanned, void* scan_tmp, size_t scan_bytes, hipStream_t st) {
    {
        auto in = rocprim::make_transform_iterator(rocprim::make_counting_iterator<int64_t>(0), LongRowPack{ptr_dev, n});
        size_t need = 0;
        GRP_HIP(rocprim::exclusive_scan(nullptr, need, in, scanned, (int64_t)0, (size_t)(n + 1), rocprim::plus<int64_t>(), st));
        if (need > scan_bytes) return fail(GRP_EWORKSPACE, "scan temp %zu < %zu", scan_bytes, need);
        GRP_HIP(rocprim::exclusive_scan(scan_tmp, need, in, scanned, (int64_t)0, (size_t)(n + 1), rocprim::plus<int64_t>(), st));
    }
    int64_t work = n;
    if (cap_long + 1 > work) work = cap_long + 1;
    if (cap_chunks > work) work = cap_chunks;
    hipLaunchKernelGGL(long_rows_emit_kernel, dim3((unsigned)cdiv(work, 256)), dim3(256), 0, st, ptr_dev, n,
                       (const int64_t*)scanned, cap_long, cap_chunks, out->long_row, out->long_first, out->chunk_begin,
                       out->chunk_end);
    GRP_LAUNCH_CHECK();
    out->n_long = (int32_t)cap_long;          // upper bounds: the launches cover them, the device arrays say which are real
    out->n_chunks = (int32_t)cap_chunks;
    return GRP_OK;
}

}  // namespace grp
