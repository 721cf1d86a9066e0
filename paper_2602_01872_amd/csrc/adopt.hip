// Adopting a local subgraph that already exists as a CSR in device memory (a partition's share
// generated or loaded directly as rows of in-edges): the handle borrows the caller's row
// pointers and column indices, and only the transposed structure (the CSC the reverse pass walks),
// the two degree arrays and the long-row schedules are built here.
//
// The transpose never holds more than `slice_edges` edges outside the two structures themselves: the
// sources are cut into consecutive ranges of at most that many edges (from a histogram of the column
// indices over 4096 equal ranges of source ids), and for one range at a time the edges whose source lies
// in it are written as keys (source << 32 | destination), sorted (rocPRIM radix sort) and unpacked
// into their final places in `row`, with `colptr` found by binary search in the sorted keys.  Equal keys
// are indistinguishable, so the result is the canonical CSC whatever order the keys were emitted in.
// A share of 2^32 edges therefore needs its 36 GB of indices plus a few GB of temporaries, where sorting
// an edge list of the same share would hold the list, two key buffers and the sort's scratch at once.
#include "common.h"

#include <new>
#include <vector>

#include <rocprim/rocprim.hpp>

namespace grp {

constexpr int AD_BINS = 4096;        // histogram resolution over the source ids
constexpr int AD_TILE = 4096;        // edges per workgroup tile of the emit pass
constexpr int AD_PER = AD_TILE / 256;
constexpr int AD_WIN = 2048;         // row pointers of a tile kept in LDS (more rows: search in global memory)

// counters: [0] malformed row pointers, [1] column indices outside [0, n), [2] positions e > 0 with
// col[e] < col[e-1], [3] non-empty rows that start at such a position (rows are ascending iff [2] == [3])
__global__ __launch_bounds__(256) void adopt_check_ptr_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ col,
                                                              int64_t n, int64_t nnz,
                                                              unsigned long long* __restrict__ counters) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool bad = false, starts_low = false;
    if (r <= n) {
        const int64_t b = ptr[r];
        bad = b < 0 || b > nnz || (r == 0 && b != 0) || (r == n && b != nnz);
        if (r < n) {
            const int64_t e = ptr[r + 1];
            if (e < b) bad = true;
            starts_low = !bad && e <= nnz && e > b && b > 0 && col[b] < col[b - 1];
        }
    }
    // nearly every row of a real graph starts below the end of the row before it: one atomic per wavefront,
    // not per row (16 M atomics on one address took 106 ms on a 2^24-node share)
    const unsigned long long low = __ballot(starts_low), bads = __ballot(bad);
    if ((threadIdx.x & 63) == 0) {
        if (low) atomicAdd(&counters[3], (unsigned long long)__popcll(low));
        if (bads) atomicAdd(&counters[0], (unsigned long long)__popcll(bads));
    }
}

// Range check, order check and the histogram of the sources over bins of 2^shift ids.
__global__ __launch_bounds__(256) void adopt_check_col_kernel(const int32_t* __restrict__ col, int64_t nnz, int64_t n,
                                                              int shift, unsigned long long* __restrict__ counters,
                                                              unsigned long long* __restrict__ hist) {
    __shared__ unsigned int bins[AD_BINS];
    for (int i = threadIdx.x; i < AD_BINS; i += 256) bins[i] = 0u;
    __syncthreads();
    unsigned long long bad = 0, desc = 0;
    // a workgroup takes runs of 2^20 consecutive edges, so that a bin counter in LDS cannot overflow
    const int64_t run = (int64_t)1 << 20;
    for (int64_t r0 = (int64_t)blockIdx.x * run; r0 < nnz; r0 += (int64_t)gridDim.x * run) {
        const int64_t r1 = r0 + run < nnz ? r0 + run : nnz;
        for (int64_t e = r0 + threadIdx.x; e < r1; e += 256) {
            const int32_t c = col[e];
            if (c < 0 || (int64_t)c >= n) { ++bad; continue; }
            if (e > 0 && c < col[e - 1]) ++desc;
            atomicAdd(&bins[c >> shift], 1u);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < AD_BINS; i += 256) {
            if (bins[i]) atomicAdd(&hist[i], (unsigned long long)bins[i]);
            bins[i] = 0u;
        }
        __syncthreads();
    }
    for (int o = 32; o > 0; o >>= 1) {
        bad += __shfl_down(bad, o, 64);
        desc += __shfl_down(desc, o, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        if (bad) atomicAdd(&counters[1], bad);
        if (desc) atomicAdd(&counters[2], desc);
    }
}

// The row that holds edge e: the largest r in [lo, hi] with ptr[r] <= e (ptr[lo] <= e < ptr[hi + 1]).
template <typename P>
__device__ __forceinline__ int64_t row_of_edge(const P& ptr, int64_t lo, int64_t hi, int64_t e) {
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (ptr(mid) <= e) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Keys (source << 32 | destination) of the edges whose source lies in [lo, hi), in any order.
// cursor: the number of keys written so far (one atomic per tile that has any).
__global__ __launch_bounds__(256) void adopt_slice_keys_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ col,
                                                               int64_t n, int64_t nnz, int32_t lo, int32_t hi,
                                                               uint64_t* __restrict__ keys, unsigned long long cap,
                                                               unsigned long long* __restrict__ cursor) {
    __shared__ int64_t win[AD_WIN + 2];
    __shared__ uint64_t stage[AD_TILE];
    __shared__ int64_t edge_row[2];
    __shared__ int count;
    __shared__ unsigned long long base;
    const int tid = threadIdx.x;
    const int64_t n_tiles = (nnz + AD_TILE - 1) / AD_TILE;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t t0 = tile * AD_TILE, t1 = t0 + AD_TILE < nnz ? t0 + AD_TILE : nnz;
        int32_t c[AD_PER];
        int any = 0;
#pragma unroll
        for (int i = 0; i < AD_PER; ++i) {
            const int64_t e = t0 + (int64_t)i * 256 + tid;
            c[i] = e < t1 ? col[e] : -1;
            any |= (c[i] >= lo && c[i] < hi) ? 1 : 0;
        }
        if (tid == 0) count = 0;
        if (!__syncthreads_or(any)) continue;              // the same answer in every thread
        auto gptr = [&](int64_t r) { return ptr[r]; };
        if (tid == 0) edge_row[0] = row_of_edge(gptr, 0, n - 1, t0);
        if (tid == 64) edge_row[1] = row_of_edge(gptr, 0, n - 1, t1 - 1);
        __syncthreads();
        const int64_t r_lo = edge_row[0], r_hi = edge_row[1];
        const bool in_lds = r_hi - r_lo + 2 <= AD_WIN + 2;
        if (in_lds)
            for (int64_t i = tid; i < r_hi - r_lo + 2; i += 256) win[i] = ptr[r_lo + i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < AD_PER; ++i) {
            if (!(c[i] >= lo && c[i] < hi)) continue;
            const int64_t e = t0 + (int64_t)i * 256 + tid;
            int64_t r;
            if (in_lds) {
                auto lptr = [&](int64_t k) { return win[k]; };
                r = r_lo + row_of_edge(lptr, 0, r_hi - r_lo, e);
            } else {
                r = row_of_edge(gptr, r_lo, r_hi, e);
            }
            const int at = atomicAdd(&count, 1);
            stage[at] = ((uint64_t)(uint32_t)c[i] << 32) | (uint64_t)(uint32_t)r;
        }
        __syncthreads();
        if (tid == 0) base = atomicAdd(cursor, (unsigned long long)count);
        __syncthreads();
        for (int i = tid; i < count; i += 256)
            if (base + (unsigned long long)i < cap) keys[base + i] = stage[i];
        __syncthreads();                                   // stage / count are reused by the next tile
    }
}

// Sorted keys of the sources [lo, hi) -> their part of the CSC: row[at + i] = destination of key i,
// colptr[s] = at + the first key whose source is >= s.
__global__ __launch_bounds__(256) void adopt_slice_csc_kernel(const uint64_t* __restrict__ keys, int64_t count, int64_t at,
                                                              int32_t lo, int32_t hi, int64_t* __restrict__ colptr,
                                                              int32_t* __restrict__ row) {
    const int64_t span = (int64_t)hi - lo;
    const int64_t work = count > span ? count : span;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < work; i += (int64_t)gridDim.x * 256) {
        if (i < count) row[at + i] = (int32_t)(keys[i] & 0xFFFFFFFFull);
        if (i < span) {
            const uint64_t want = (uint64_t)(uint32_t)(lo + i) << 32;
            int64_t a = 0, b = count;
            while (a < b) {
                const int64_t mid = (a + b) >> 1;
                if (keys[mid] < want) a = mid + 1; else b = mid;
            }
            colptr[lo + i] = at + a;
        }
    }
}

__global__ __launch_bounds__(256) void adopt_finish_kernel(const int64_t* __restrict__ rowptr, int64_t* __restrict__ colptr,
                                                           int64_t n, int64_t nnz, int32_t* __restrict__ d_in,
                                                           int32_t* __restrict__ d_out, const int64_t* __restrict__ d_global_src,
                                                           int64_t* __restrict__ d_global, const int64_t* __restrict__ l2g_src,
                                                           int64_t* __restrict__ l2g) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n) return;
    const int64_t din = rowptr[v + 1] - rowptr[v];
    const int64_t cend = v + 1 < n ? colptr[v + 1] : nnz;
    d_in[v] = (int32_t)din;
    d_out[v] = (int32_t)(cend - colptr[v]);
    d_global[v] = d_global_src ? d_global_src[v] : din;
    l2g[v] = l2g_src ? l2g_src[v] : v;
    if (v == n - 1) colptr[n] = nnz;
}

struct Owned {
    void* p = nullptr;
    ~Owned() { if (p) (void)hipFree(p); }
    grp_status alloc(size_t bytes) {
        if (hipMalloc(&p, bytes ? bytes : 4) != hipSuccess) {
            p = nullptr;
            (void)hipGetLastError();
            return fail(GRP_ENOMEM, "device allocation of %zu bytes failed", bytes);
        }
        return GRP_OK;
    }
};

static grp_status long_rows_of(const int64_t* ptr_dev, int64_t n, LongRows* out, int64_t cap_long, int64_t cap_chunks,
                               int64_t* scanned, void* tmp, size_t tmp_bytes, hipStream_t st) {
    out->n_long = out->n_chunks = 0;
    if (n == 0 || cap_long == 0) return GRP_OK;
    GRP_TRY(build_long_rows_device(ptr_dev, n, out, cap_long, cap_chunks, scanned, tmp, tmp_bytes, st));
    int64_t total = 0;
    GRP_HIP(hipMemcpyAsync(&total, scanned + n, sizeof total, hipMemcpyDeviceToHost, st));
    GRP_HIP(hipStreamSynchronize(st));
    out->n_long = (int32_t)(total >> 32);
    out->n_chunks = (int32_t)(total & 0xFFFFFFFFll);
    return GRP_OK;
}

static grp_status adopt_impl(grp_partition_t* h, const int64_t* rowptr, const int32_t* col, const int64_t* d_global_in,
                             const int64_t* l2g, int64_t slice_edges, hipStream_t st) {
    const int64_t n = h->n, nnz = h->nnz;
    const int64_t cap_long = nnz > SPMM_LONG_ROW ? nnz / SPMM_LONG_ROW + 1 : 0;
    const int64_t cap_chunks = cap_long ? nnz / SPMM_CHUNK + cap_long + 1 : 0;
    if (cap_chunks >= ((int64_t)1 << 31)) return fail(GRP_ERANGE, "more than 2^31 row chunks");
    // everything the handle owns, from one allocation
    auto carve = [&](void* base, size_t cap) {
        Bump b(base, cap);
        const size_t n1 = (size_t)(n > 0 ? n : 1), z1 = (size_t)(nnz > 0 ? nnz : 1);
        h->colptr = b.take<int64_t>(n1 + 1);
        h->row = b.take<int32_t>(z1);
        h->d_local_in = b.take<int32_t>(n1);
        h->d_local_out = b.take<int32_t>(n1);
        h->d_global_in = b.take<int64_t>(n1);
        h->l2g = b.take<int64_t>(n1);
        for (LongRows* lr : {&h->csr_long, &h->csc_long}) {
            if (cap_long == 0) continue;
            lr->long_row = b.take<int32_t>((size_t)cap_long);
            lr->long_first = b.take<int32_t>((size_t)cap_long + 1);
            lr->chunk_begin = b.take<int64_t>((size_t)cap_chunks);
            lr->chunk_end = b.take<int64_t>((size_t)cap_chunks);
        }
        return b.total();
    };
    h->slab_bytes = carve(nullptr, 0);
    if (hipMalloc(&h->slab, h->slab_bytes) != hipSuccess) {
        (void)hipGetLastError();
        h->slab = nullptr;
        return fail(GRP_ENOMEM, "device allocation of %zu bytes failed", h->slab_bytes);
    }
    (void)carve(h->slab, h->slab_bytes);
    h->rowptr = const_cast<int64_t*>(rowptr);
    h->col = const_cast<int32_t*>(col);
    h->borrowed_csr = true;

    // ---- checks and the histogram of the sources
    int shift = 0;
    while (n > 0 && ((n - 1) >> shift) >= AD_BINS) ++shift;
    Owned small;                                           // 4 counters, the emit cursor, the histogram
    GRP_TRY(small.alloc((8 + AD_BINS) * sizeof(unsigned long long)));
    unsigned long long* counters = (unsigned long long*)small.p;
    unsigned long long* cursor = counters + 4;
    unsigned long long* hist = counters + 8;
    GRP_TRY(launch_fill_zero(small.p, (8 + AD_BINS) * sizeof(unsigned long long), st));
    hipLaunchKernelGGL(adopt_check_ptr_kernel, dim3((unsigned)cdiv(n + 1, 256)), dim3(256), 0, st, rowptr, col, n, nnz, counters);
    GRP_LAUNCH_CHECK();
    unsigned long long host[8 + AD_BINS];
    GRP_HIP(hipMemcpyAsync(host, counters, 4 * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    GRP_HIP(hipStreamSynchronize(st));
    if (host[0]) return fail(GRP_EINVAL, "grp_partition_from_csr: %llu row pointers are not a non-decreasing sequence from 0 to nnz", host[0]);
    if (nnz > 0) {
        const int64_t runs = cdiv(nnz, (int64_t)1 << 20);
        hipLaunchKernelGGL(adopt_check_col_kernel, dim3((unsigned)(runs < 2048 ? runs : 2048)), dim3(256), 0, st, col, nnz, n,
                           shift, counters, hist);
        GRP_LAUNCH_CHECK();
    }
    GRP_HIP(hipMemcpyAsync(host, counters, sizeof host, hipMemcpyDeviceToHost, st));
    GRP_HIP(hipStreamSynchronize(st));
    if (host[1]) return fail(GRP_ERANGE, "grp_partition_from_csr: %llu column indices outside [0, %lld)", host[1], (long long)n);
    if (host[2] != host[3])
        return fail(GRP_EINVAL, "grp_partition_from_csr: the column indices of a row must be ascending (%llu descents inside rows)",
                    host[2] - host[3]);

    // ---- the transpose, one range of sources at a time
    if (nnz > 0) {
        const unsigned long long* hb = host + 8;
        const int64_t n_bins = ((n - 1) >> shift) + 1;
        unsigned long long biggest = 0;
        for (int64_t b = 0; b < n_bins; ++b) biggest = hb[b] > biggest ? hb[b] : biggest;
        int64_t cap = slice_edges > 0 ? slice_edges : ((int64_t)1 << 28);
        if (cap > nnz) cap = nnz;
        if ((unsigned long long)cap < biggest) cap = (int64_t)biggest;      // a bin is never cut
        const unsigned end_bit = 64;
        size_t sort_bytes = 0;
        GRP_HIP(rocprim::radix_sort_keys(nullptr, sort_bytes, (const uint64_t*)nullptr, (uint64_t*)nullptr, (size_t)cap, 0u, end_bit, st));
        Owned keys, sorted, tmp;
        GRP_TRY(keys.alloc((size_t)cap * sizeof(uint64_t)));
        GRP_TRY(sorted.alloc((size_t)cap * sizeof(uint64_t)));
        GRP_TRY(tmp.alloc(sort_bytes));
        const int64_t n_tiles = cdiv(nnz, AD_TILE);
        const unsigned emit_grid = (unsigned)(n_tiles < 4096 ? n_tiles : 4096);
        int64_t at = 0;
        for (int64_t b0 = 0; b0 < n_bins;) {
            int64_t b1 = b0;
            unsigned long long count = 0;
            while (b1 < n_bins && count + hb[b1] <= (unsigned long long)cap) count += hb[b1++];
            const int64_t lo = b0 << shift;
            const int64_t hi = b1 < n_bins ? (b1 << shift) : n;
            if (count > 0) {
                GRP_TRY(launch_fill_zero(cursor, 4 * sizeof(unsigned long long), st));
                hipLaunchKernelGGL(adopt_slice_keys_kernel, dim3(emit_grid), dim3(256), 0, st, rowptr, col, n, nnz, (int32_t)lo,
                                   (int32_t)hi, (uint64_t*)keys.p, (unsigned long long)cap, cursor);
                GRP_LAUNCH_CHECK();
                unsigned bits = 32 + (unsigned)(64 - __builtin_clzll((unsigned long long)(hi > 1 ? hi - 1 : 1)));
                if (bits > 64) bits = 64;
                size_t need = 0;                           // the algorithm, and with it the scratch, depends on the count
                GRP_HIP(rocprim::radix_sort_keys(nullptr, need, (const uint64_t*)keys.p, (uint64_t*)sorted.p, (size_t)count, 0u,
                                                 bits, st));
                if (need > sort_bytes) {
                    GRP_HIP(hipStreamSynchronize(st));
                    (void)hipFree(tmp.p);
                    tmp.p = nullptr;
                    GRP_TRY(tmp.alloc(need));
                    sort_bytes = need;
                }
                GRP_HIP(rocprim::radix_sort_keys(tmp.p, need, (const uint64_t*)keys.p, (uint64_t*)sorted.p, (size_t)count, 0u,
                                                 bits, st));
            }
            const int64_t work = (int64_t)count > hi - lo ? (int64_t)count : hi - lo;
            hipLaunchKernelGGL(adopt_slice_csc_kernel, dim3((unsigned)(cdiv(work, 256) < 16384 ? cdiv(work, 256) : 16384)),
                               dim3(256), 0, st, (const uint64_t*)sorted.p, (int64_t)count, at, (int32_t)lo, (int32_t)hi,
                               h->colptr, h->row);
            GRP_LAUNCH_CHECK();
            at += (int64_t)count;
            b0 = b1;
        }
        GRP_HIP(hipStreamSynchronize(st));                 // the temporaries are freed on return
        if (at != nnz) return fail(GRP_EHIP, "grp_partition_from_csr: transposed %lld of %lld edges", (long long)at, (long long)nnz);
    } else if (n > 0) {
        GRP_TRY(launch_fill_zero(h->colptr, (size_t)(n + 1) * sizeof(int64_t), st));
    }
    if (n > 0) {
        hipLaunchKernelGGL(adopt_finish_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, rowptr, h->colptr, n, nnz,
                           h->d_local_in, h->d_local_out, d_global_in, h->d_global_in, l2g, h->l2g);
        GRP_LAUNCH_CHECK();
    } else {
        GRP_TRY(launch_fill_zero(h->colptr, sizeof(int64_t), st));
    }
    if (cap_long) {
        const size_t scan_bytes = scan_temp_bytes(n + 1);
        const size_t scanned_bytes = (((size_t)n + 1) * sizeof(int64_t) + 255) & ~(size_t)255;
        Owned tmp;
        GRP_TRY(tmp.alloc(scanned_bytes + scan_bytes));
        int64_t* scanned = (int64_t*)tmp.p;
        void* scan_tmp = (char*)tmp.p + scanned_bytes;
        GRP_TRY(long_rows_of(h->rowptr, n, &h->csr_long, cap_long, cap_chunks, scanned, scan_tmp, scan_bytes, st));
        GRP_TRY(long_rows_of(h->colptr, n, &h->csc_long, cap_long, cap_chunks, scanned, scan_tmp, scan_bytes, st));
    }
    GRP_HIP(hipStreamSynchronize(st));
    GRP_TRY(build_slice_tasks(h->rowptr, h->col, n, nnz, &h->csr_long, st));
    GRP_TRY(build_slice_tasks(h->colptr, h->row, n, nnz, &h->csc_long, st));
    return GRP_OK;
}

}  // namespace grp

extern "C" grp_status grp_partition_from_csr(const int64_t* rowptr, const int32_t* col, int64_t n, int64_t nnz,
                                             const int64_t* d_global_in, const int64_t* l2g, int64_t slice_edges,
                                             void* stream, grp_partition_t** out) {
    using namespace grp;
    if (!out) return fail(GRP_EINVAL, "grp_partition_from_csr: out is null");
    *out = nullptr;
    if (n < 0 || nnz < 0 || slice_edges < 0) return fail(GRP_EINVAL, "grp_partition_from_csr: negative size");
    if (!rowptr || (nnz > 0 && !col)) return fail(GRP_EINVAL, "grp_partition_from_csr: null row pointers or column indices");
    if (n == 0 && nnz > 0) return fail(GRP_EINVAL, "grp_partition_from_csr: edges without nodes");
    if (n >= ((int64_t)1 << 31)) return fail(GRP_ERANGE, "n = %lld >= 2^31", (long long)n);
    grp_partition_t* h = new (std::nothrow) grp_partition_t();
    if (!h) return fail(GRP_ENOMEM, "host allocation failed");
    (void)hipGetDevice(&h->device);
    h->n = n;
    h->nnz = nnz;
    const grp_status s = adopt_impl(h, rowptr, col, d_global_in, l2g, slice_edges, (hipStream_t)stream);
    if (s != GRP_OK) {
        std::string keep = grp_last_error();
        grp_partition_destroy(h);
        set_error("%s", keep.c_str());
        return s;
    }
    *out = h;
    return GRP_OK;
}
