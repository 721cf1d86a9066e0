// Source-sliced schedule of the long rows of a CSR-like structure (built once with the partition).
//
// Why: a gather-bound aggregation over a graph without locality misses the L2 on almost every neighbour
// row (measured on a 2^24-node, 2^32-edge share: 0.82 line fills per edge), because the rows gathered
// at any one time are spread over all n sources.  The rows that hold most of the edges are long
// (96 % of the edges of a share with that mean degree sit in the fifth of the rows that are longer than 128 edges), and a row's sources are
// sorted, so a long row can be cut where its sources cross from one range of node ids into the next: the
// node ids are divided into SLICES = 64 equal ranges, every long row is cut at the boundaries between them
// (where the piece so far is long enough to be worth a task), and every piece into tasks of at most SLICE_TASK_MAX edges
// (a wavefront walks a task in passes of SLICE_PIECE edges).  The tasks are then processed slice by slice: at any one
// time the whole chip gathers from one 64th of the nodes, whose frequently used rows stay in the L2
// (measured with the sources restricted to one 64th: 0.14 fills per edge).  A task's result is a partial
// row; a long row's partial rows are added in task order (ascending source, the row's own edge order) by the
// combine pass, so the result does not depend on scheduling.
//
// Layout: tasks are numbered row-major (a long row's tasks are consecutive: row_task[j] .. row_task[j+1]),
// and the records are stored in processing order (a stable sort by slice, so that inside a slice they keep
// row order and neighbouring workgroups read neighbouring pieces of the index array).
#include "common.h"

#include <atomic>

#include <rocprim/rocprim.hpp>

namespace grp {

constexpr unsigned SLICE_KEY_BITS = SLICES <= 64 ? 6u : SLICES <= 128 ? 7u : 8u;
static_assert(SLICES <= 256 && (SLICES & (SLICES - 1)) == 0, "a slice key is one byte; the ranges are a power of two");
static std::atomic<int64_t> g_slice_min_nodes{(int64_t)1 << 19};
static std::atomic<int32_t> g_slice_min_percent{25};

static __device__ __forceinline__ int64_t lower_bound_idx(const int32_t* __restrict__ idx, int64_t b, int64_t e, int64_t want) {
    while (b < e) {
        const int64_t mid = (b + e) >> 1;
        if ((int64_t)idx[mid] < want) b = mid + 1; else e = mid;
    }
    return b;
}

// One wavefront per long row.  Lane s finds where the row's sources enter slice s; the row is then cut at such a
// boundary wherever the piece before it has reached SLICE_MIN_PIECE edges (a row of 600 edges is not worth 64
// pieces of 9: a piece costs a partial row and ~200 instructions; see the measurements beside the constant), and every piece into tasks of at most
// SLICE_TASK_MAX edges.  A task's key is the slice of its first edge.  EMIT = false: the row's number of tasks.
// EMIT = true: its task records (row-major numbering from row_task[j]) and their keys.
template <bool EMIT>
__global__ __launch_bounds__(256) void slice_rows_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ long_row, int64_t n_long, int shift,
                                                         int min_piece, int64_t* __restrict__ row_tasks,
                                                         SliceTask* __restrict__ recs, uint8_t* __restrict__ keys) {
    __shared__ int64_t cut_s[4][SLICES + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t j = (int64_t)blockIdx.x * 4 + wave;
    if (j >= n_long) return;                                   // uniform over the wavefront
    const int64_t r = long_row[j];
    if (r < 0) {                                               // an unused slot of a schedule built to its capacity
        if (!EMIT && lane == 0) row_tasks[j] = 0;
        return;
    }
    const int64_t b = ptr[r], e = ptr[r + 1];
    for (int sl = lane; sl < SLICES; sl += 64) cut_s[wave][sl] = sl == 0 ? b : lower_bound_idx(idx, b, e, (int64_t)sl << shift);
    if (lane == 0) cut_s[wave][SLICES] = e;
    __builtin_amdgcn_wave_barrier();                           // the wavefront's own LDS writes, read back below
    int64_t t = EMIT ? row_tasks[j] : 0;                       // (row_tasks holds the exclusive prefix sum when emitting)
    int64_t count = 0;
    int64_t from = b;                                          // start of the current piece
    int from_slice = 0;
    for (int s = 1; s <= SLICES; ++s) {                        // the same walk in every lane
        const int64_t at = cut_s[wave][s];
        const bool close = s == SLICES || at - from >= min_piece;
        if (!close) continue;
        const int64_t nt = (at - from + SLICE_TASK_MAX - 1) / SLICE_TASK_MAX;
        if (EMIT) {
            for (int64_t i = lane; i < nt; i += 64) {
                SliceTask rec;
                rec.begin = from + i * SLICE_TASK_MAX;
                rec.id = (uint32_t)(t + i);
                rec.len = (uint32_t)(at - rec.begin < SLICE_TASK_MAX ? at - rec.begin : SLICE_TASK_MAX);
                recs[t + i] = rec;
                keys[t + i] = (uint8_t)from_slice;
            }
        }
        t += nt;
        count += nt;
        from = at;
        from_slice = s;
    }
    if (!EMIT && lane == 0) row_tasks[j] = count;
}

// *total += the edges of the listed rows (one atomic per wavefront)
__global__ __launch_bounds__(256) void long_edges_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ long_row,
                                                         int64_t n_long, unsigned long long* __restrict__ total) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t len = 0;
    if (j < n_long) {
        const int64_t r = long_row[j];
        if (r >= 0) len = ptr[r + 1] - ptr[r];
    }
    for (int o = 32; o > 0; o >>= 1) len += __shfl_down(len, o, 64);
    if ((threadIdx.x & 63) == 0 && len > 0) atomicAdd(total, (unsigned long long)len);
}

// Builds lr->tasks / lr->row_task for the long rows already listed in lr (allocations owned by the caller's
// handle through these pointers).  Leaves lr untouched (n_tasks = 0) when the structure is too small to gain.
grp_status build_slice_tasks(const int64_t* ptr, const int32_t* idx, int64_t n, int64_t nnz, LongRows* lr, hipStream_t st) {
    lr->n_tasks = 0;
    lr->tasks = nullptr;
    lr->row_task = nullptr;
    if (n < g_slice_min_nodes.load() || lr->n_long <= 0) return GRP_OK;
    int shift = 0;
    while (((n - 1) >> shift) >= SLICES) ++shift;
    const int64_t n_long = lr->n_long;
    const int min_piece = SLICE_MIN_PIECE;
    int64_t* row_task = nullptr;
    GRP_HIP(hipMalloc((void**)&row_task, (size_t)(n_long + 1) * sizeof(int64_t)));
    auto fail_free = [&](grp_status s) { (void)hipFree(row_task); return s; };
    GRP_HIP(hipMemsetAsync(row_task + n_long, 0, sizeof(int64_t), st));
    {   // the long rows' share of the edges decides whether the schedule pays
        hipLaunchKernelGGL(long_edges_kernel, dim3((unsigned)cdiv(n_long, 256)), dim3(256), 0, st, ptr, lr->long_row, n_long,
                           (unsigned long long*)(row_task + n_long));
        int64_t long_edges = 0;
        if (hipMemcpyAsync(&long_edges, row_task + n_long, sizeof long_edges, hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return fail_free(fail(GRP_EHIP, "slice schedule: the long rows' edge count did not reach the host"));
        if (long_edges * 100 < nnz * (int64_t)g_slice_min_percent.load()) {
            (void)hipFree(row_task);
            return GRP_OK;
        }
        if (hipMemsetAsync(row_task + n_long, 0, sizeof(int64_t), st) != hipSuccess)
            return fail_free(fail(GRP_EHIP, "slice schedule: clearing the task total failed"));
    }
    const unsigned grid = (unsigned)cdiv(n_long, 4);
    hipLaunchKernelGGL(slice_rows_kernel<false>, dim3(grid), dim3(256), 0, st, ptr, idx, lr->long_row, n_long, shift, min_piece,
                       row_task, (SliceTask*)nullptr, (uint8_t*)nullptr);
    {
        size_t need = 0;
        if (rocprim::exclusive_scan(nullptr, need, row_task, row_task, (int64_t)0, (size_t)(n_long + 1), rocprim::plus<int64_t>(), st) != hipSuccess)
            return fail_free(fail(GRP_EHIP, "slice schedule: scan size query failed"));
        void* tmp = nullptr;
        if (hipMalloc(&tmp, need ? need : 4) != hipSuccess) { (void)hipGetLastError(); return fail_free(fail(GRP_ENOMEM, "slice schedule: scan scratch")); }
        const hipError_t e = rocprim::exclusive_scan(tmp, need, row_task, row_task, (int64_t)0, (size_t)(n_long + 1), rocprim::plus<int64_t>(), st);
        (void)hipStreamSynchronize(st);
        (void)hipFree(tmp);
        if (e != hipSuccess) return fail_free(fail(GRP_EHIP, "slice schedule: scan failed"));
    }
    int64_t n_tasks = 0;
    if (hipMemcpy(&n_tasks, row_task + n_long, sizeof n_tasks, hipMemcpyDeviceToHost) != hipSuccess)
        return fail_free(fail(GRP_EHIP, "slice schedule: task count did not reach the host"));
    if (n_tasks <= 0 || n_tasks >= ((int64_t)1 << 32)) {       // nothing to do, or more tasks than a 32-bit id holds
        (void)hipFree(row_task);
        return GRP_OK;
    }
    SliceTask *recs = nullptr, *sorted = nullptr;
    uint8_t *keys = nullptr, *keys_out = nullptr;
    void* tmp = nullptr;
    auto cleanup = [&]() { (void)hipFree(recs); (void)hipFree(keys); (void)hipFree(keys_out); (void)hipFree(tmp); };
    grp_status status = GRP_OK;
    do {
        if (hipMalloc((void**)&recs, (size_t)n_tasks * sizeof(SliceTask)) != hipSuccess ||
            hipMalloc((void**)&sorted, (size_t)n_tasks * sizeof(SliceTask)) != hipSuccess ||
            hipMalloc((void**)&keys, (size_t)n_tasks) != hipSuccess || hipMalloc((void**)&keys_out, (size_t)n_tasks) != hipSuccess) {
            (void)hipGetLastError();
            status = fail(GRP_ENOMEM, "slice schedule: %lld task records", (long long)n_tasks);
            break;
        }
        hipLaunchKernelGGL(slice_rows_kernel<true>, dim3(grid), dim3(256), 0, st, ptr, idx, lr->long_row, n_long, shift, min_piece,
                           row_task, recs, keys);
        size_t need = 0;
        if (rocprim::radix_sort_pairs(nullptr, need, keys, keys_out, recs, sorted, (size_t)n_tasks, 0u, SLICE_KEY_BITS, st) != hipSuccess ||
            hipMalloc(&tmp, need ? need : 4) != hipSuccess) {
            (void)hipGetLastError();
            status = fail(GRP_ENOMEM, "slice schedule: sort scratch");
            break;
        }
        if (rocprim::radix_sort_pairs(tmp, need, keys, keys_out, recs, sorted, (size_t)n_tasks, 0u, SLICE_KEY_BITS, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) {
            status = fail(GRP_EHIP, "slice schedule: sort failed");
            break;
        }
    } while (false);
    cleanup();
    if (status != GRP_OK) {
        (void)hipFree(sorted);
        (void)hipFree(row_task);
        return status;
    }
    lr->n_tasks = n_tasks;
    lr->tasks = sorted;
    lr->row_task = row_task;
    return GRP_OK;
}

}  // namespace grp

extern "C" grp_status grp_set_slice_policy(int64_t min_nodes, int32_t min_long_edge_percent) {
    if (min_nodes < 1 || min_long_edge_percent < 0 || min_long_edge_percent > 100)
        return grp::fail(GRP_EINVAL, "grp_set_slice_policy: %lld nodes, %d %%", (long long)min_nodes, min_long_edge_percent);
    grp::g_slice_min_nodes.store(min_nodes);
    grp::g_slice_min_percent.store(min_long_edge_percent);
    return GRP_OK;
}
