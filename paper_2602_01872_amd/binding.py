"""ctypes binding with the same names as the C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgrappa_hip.so")

GRP_MAX_LAYERS = 16
ARCH_SAGE_MEAN, ARCH_GCN, ARCH_GCN_RESIDUAL, ARCH_GAT = 0, 1, 2, 3
DTYPE_FP32, DTYPE_BF16 = 0, 1
EST_NONE, EST_NODE_LEVEL, EST_BATCH_MIN_DIST, EST_SHRINKAGE = 0, 1, 2, 3
OPT_SGD, OPT_ADAM = 0, 1
SCALE_NONE, SCALE_MEAN, SCALE_RSQRT = 0, 1, 2
OK, EINVAL, ERANGE, ENOMEM, EWORKSPACE, EHIP, EUNSUPPORTED = 0, -1, -2, -3, -4, -5, -6


class GrappaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"grappa status {status}: {message}")
        self.status = status


class PartitionView(C.Structure):
    _fields_ = [("n", C.c_int64), ("nnz", C.c_int64), ("l2g", C.c_void_p), ("rowptr", C.c_void_p),
                ("col", C.c_void_p), ("colptr", C.c_void_p), ("row", C.c_void_p),
                ("d_local_in", C.c_void_p), ("d_local_out", C.c_void_p), ("d_global_in", C.c_void_p)]


class ModelDesc(C.Structure):
    _fields_ = [("arch", C.c_int32), ("n_layers", C.c_int32), ("dims", C.c_int32 * (GRP_MAX_LAYERS + 1)),
                ("feat_dtype", C.c_int32), ("gcn_self_loops", C.c_int32)]


class OptimizerDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("reserved", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float)]


class PartitionWeights(C.Structure):
    _fields_ = [("csr_w", C.c_void_p), ("csc_w", C.c_void_p), ("w_local_in", C.c_void_p), ("w_global_in", C.c_void_p)]


class BlockView(C.Structure):
    _fields_ = [("n_dst", C.c_int64), ("n_src", C.c_int64), ("nnz", C.c_int64), ("rowptr", C.c_void_p), ("col", C.c_void_p),
                ("dst_nodes", C.c_void_p), ("src_nodes", C.c_void_p)]


class StepOpts(C.Structure):
    _fields_ = [("estimator", C.c_int32), ("full_graph", C.c_int32), ("n_seeds", C.c_int32),
                ("reserved", C.c_int32), ("seeds", C.c_void_p), ("fanouts", C.c_int32 * GRP_MAX_LAYERS),
                ("sampler_seed", C.c_uint64), ("batch_id", C.c_uint64), ("dropout_rate", C.c_float),
                ("flags", C.c_int32), ("dropout_seed", C.c_uint64), ("batch_id_dev", C.c_void_p)]


STEP_ONE_STREAM = 1
STATS_DTYPE = np.dtype([("loss", "<f8"), ("sum_ratio", "<f8"), ("R", "<f8"), ("S", "<i8"), ("nnz_used", "<i8")])
STATS_BYTES = STATS_DTYPE.itemsize

_lib = None


def load() -> C.CDLL:
    """Load the built library; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_size_t
    lib.grp_last_error.restype = C.c_char_p
    lib.grp_last_error.argtypes = []
    sigs = {
        "grp_partition": [vp, vp, i64, i64, i32, u64, i32, vp, C.POINTER(vp)],
        "grp_node_owners": [i64, i32, u64, vp, vp, vp],
        "grp_epoch_seeds": [vp, vp, u64, u64, vp, vp, C.POINTER(i64)],
        "grp_gather_rows": [vp, i64, i64, vp, i64, vp, vp, vp],
        "grp_partition_weighted": [vp, vp, vp, i64, i64, i32, u64, i32, vp, C.POINTER(vp)],
        "grp_partition_weights": [vp, C.POINTER(PartitionWeights)],
        "grp_partition_from_local_coo": [vp, vp, i64, i64, vp, vp, vp, C.POINTER(vp)],
        "grp_partition_from_csr": [vp, vp, i64, i64, vp, vp, i64, vp, C.POINTER(vp)],
        "grp_partition_halo": [vp, vp, i64, i64, i32, u64, i32, i32, vp, C.POINTER(vp)],
        "grp_partition_view": [vp, C.POINTER(PartitionView)],
        "grp_chunks_build": [vp, vp, i64, i64, i32, u64, vp, C.POINTER(vp)],
        "grp_chunks_build_assigned": [vp, vp, i64, i64, i32, vp, vp, C.POINTER(vp)],
        "grp_chunks_destroy": [vp],
        "grp_partition_from_chunks": [vp, i32, i32, vp, C.POINTER(vp)],
        "grp_partition_base_mask": [vp, C.POINTER(vp)],
        "grp_partition_destroy": [vp],
        "grp_step_workspace_bytes": [vp, C.POINTER(ModelDesc), C.POINTER(StepOpts), C.POINTER(sz)],
        "grp_step_activation": [vp, C.POINTER(ModelDesc), C.POINTER(StepOpts), vp, sz, i32, C.POINTER(vp), C.POINTER(i64)],
        "grp_step_block": [vp, C.POINTER(ModelDesc), C.POINTER(StepOpts), vp, sz, i32, C.POINTER(BlockView)],
        "grp_train_step": [vp, C.POINTER(ModelDesc), C.POINTER(StepOpts), vp, vp, vp, vp, vp, sz, vp, vp, vp],
        "grp_aggregate": [vp, i64, vp, i32, i64, i32, vp, vp, vp],
        "grp_aggregate_ptrs": [vp, i32, vp, i32, i64, i32, vp, vp, vp],
        "grp_optimizer_step": [C.POINTER(OptimizerDesc), i64, i64, vp, vp, vp, vp, vp],
        "grp_spmm_workspace_bytes": [vp, i32, i32, C.POINTER(sz)],
        "grp_spmm": [vp, i32, i32, i32, i32, vp, i64, i32, vp, i64, vp, sz, vp],
        "grp_spmm_static": [vp, i32, i32, i32, i32, vp, i64, i32, vp, i64, vp],
        "grp_gemm_nn": [i64, i32, i32, vp, i64, i32, vp, i64, vp, i64, vp],
        "grp_gemm_nt": [i64, i32, i32, vp, i64, i32, vp, i64, vp, i64, vp],
        "grp_gemm_tn": [i64, i32, i32, vp, i64, i32, vp, i64, vp, i64, vp, sz, vp],
        "grp_set_slice_policy": [i64, C.c_int32],
        "grp_controller_create": [i64, i32, C.c_double, i64, C.POINTER(vp)],
        "grp_controller_observe": [vp, vp, i32],
        "grp_controller_observe_stats": [vp, vp, i32],
        "grp_controller_end_epoch": [vp, C.POINTER(i32)],
        "grp_controller_state": [vp, C.POINTER(i64), C.POINTER(i64)],
        "grp_controller_destroy": [vp],
        "grp_profile_enable": [i32],
        "grp_profile_report": [C.c_char_p, sz],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = i32
    lib.grp_param_count.argtypes = [C.POINTER(ModelDesc)]
    lib.grp_param_count.restype = i64
    lib.grp_sweep_chunk.argtypes = [i32, i64, i32]
    lib.grp_sweep_chunk.restype = i32
    lib.grp_super_epoch_epochs.argtypes = [i64, i32]
    lib.grp_super_epoch_epochs.restype = i64
    lib.grp_gemm_tn_workspace_bytes.argtypes = [i64, i32, i32]
    lib.grp_gemm_tn_workspace_bytes.restype = sz
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise GrappaError(status, load().grp_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def model_desc(arch: int, dims, feat_dtype: int = DTYPE_FP32, gcn_self_loops: bool = True) -> ModelDesc:
    m = ModelDesc()
    m.arch = arch
    m.n_layers = len(dims) - 1
    for i, d in enumerate(dims[:GRP_MAX_LAYERS + 1]):
        m.dims[i] = int(d)
    m.feat_dtype = feat_dtype
    m.gcn_self_loops = 1 if gcn_self_loops else 0
    return m


def step_opts(estimator: int = EST_NONE, full_graph: bool = True, seeds=None, fanouts=(), sampler_seed: int = 0,
              batch_id: int = 0, dropout_rate: float = 0.0, dropout_seed: int = 0, batch_id_dev=None,
              flags: int = 0) -> StepOpts:
    """``batch_id_dev``: a one-element int64 device tensor holding the batch id (read when the step runs, see grappa.h)."""
    o = StepOpts()
    o.estimator = estimator
    o.full_graph = 1 if full_graph else 0
    o.n_seeds = 0 if seeds is None else int(seeds.numel())
    o.seeds = _ptr(seeds)
    for i, f in enumerate(fanouts):
        o.fanouts[i] = int(f)
    o.sampler_seed = sampler_seed
    o.batch_id = batch_id
    o.dropout_rate = dropout_rate
    o.dropout_seed = dropout_seed
    o.flags = flags
    if batch_id_dev is not None:
        assert batch_id_dev.is_cuda and batch_id_dev.dtype == torch.int64 and batch_id_dev.numel() == 1
    o.batch_id_dev = _ptr(batch_id_dev)
    o._keep = (seeds, batch_id_dev)
    return o


class Partition:
    """Owns a grp_partition_t handle; arrays are exposed as device tensors copied on request."""

    def __init__(self, handle: int):
        self.handle = handle
        v = PartitionView()
        _check(load().grp_partition_view(handle, C.byref(v)))
        self.view = v
        self.n, self.nnz = int(v.n), int(v.nnz)

    def array(self, name: str) -> np.ndarray:
        """Host copy of one of the handle's arrays (for tests)."""
        spec = {"l2g": (np.int64, self.n), "rowptr": (np.int64, self.n + 1), "col": (np.int32, self.nnz),
                "colptr": (np.int64, self.n + 1), "row": (np.int32, self.nnz), "d_local_in": (np.int32, self.n),
                "d_local_out": (np.int32, self.n), "d_global_in": (np.int64, self.n)}[name]
        dt, count = spec
        out = np.empty(count, dtype=dt)
        if count:
            torch.cuda.synchronize()
            _hip_memcpy_d2h(out, getattr(self.view, name))
        return out

    def device_array(self, name: str) -> torch.Tensor:
        """Device copy of one of the handle's arrays as a torch tensor (for checks at sizes where a host
        copy is too slow)."""
        dt, count = {"l2g": (torch.int64, self.n), "rowptr": (torch.int64, self.n + 1), "col": (torch.int32, self.nnz),
                     "colptr": (torch.int64, self.n + 1), "row": (torch.int32, self.nnz), "d_local_in": (torch.int32, self.n),
                     "d_local_out": (torch.int32, self.n), "d_global_in": (torch.int64, self.n)}[name]
        out = torch.empty(count, dtype=dt, device="cuda")
        if count:
            torch.cuda.synchronize()
            _hip_memcpy(out.data_ptr(), getattr(self.view, name), out.numel() * out.element_size(), 3)
            torch.cuda.synchronize()
        return out

    def weights(self):
        """Host copies of a weighted partition's arrays as a dict (None for an unweighted one)."""
        w = PartitionWeights()
        _check(load().grp_partition_weights(self.handle, C.byref(w)))
        if not w.csr_w and not w.w_local_in:
            return None
        out = {}
        torch.cuda.synchronize()
        for name, dt, count in (("csr_w", np.float32, self.nnz), ("csc_w", np.float32, self.nnz),
                                ("w_local_in", np.float64, self.n), ("w_global_in", np.float64, self.n)):
            a = np.empty(count, dtype=dt)
            if count:
                _hip_memcpy_d2h(a, getattr(w, name))
            out[name] = a
        return out

    def base_mask_ptr(self) -> int:
        """Device address of the uint8[n] base-chunk mask (0 for partitions not built from chunks)."""
        out = C.c_void_p()
        _check(load().grp_partition_base_mask(self.handle, C.byref(out)))
        return out.value or 0

    def base_mask(self) -> np.ndarray:
        """Host copy of the base-chunk mask (for tests)."""
        out = np.empty(self.n, dtype=np.uint8)
        p = self.base_mask_ptr()
        if not p:
            raise ValueError("this partition was not built from chunks")
        if self.n:
            torch.cuda.synchronize()
            _hip_memcpy_d2h(out, p)
        return out

    def destroy(self):
        if self.handle:
            _check(load().grp_partition_destroy(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


_hip = None


def _hip_memcpy(dst_ptr: int, src_ptr: int, nbytes: int, kind: int):
    global _hip
    if _hip is None:
        # the SONAME resolves to the HIP runtime torch already loaded (never a second copy)
        _hip = C.CDLL("libamdhip64.so.7")
        _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hip.hipMemcpy.restype = C.c_int
    rc = _hip.hipMemcpy(dst_ptr, src_ptr, nbytes, kind)
    if rc != 0:
        raise RuntimeError(f"hipMemcpy (kind {kind}) failed: {rc}")


def _hip_memcpy_d2h(dst: np.ndarray, src_ptr: int):
    _hip_memcpy(dst.ctypes.data, src_ptr, dst.nbytes, 2)


def grp_partition(src, dst, N: int, K: int, seed: int, part_id: int, stream=None) -> Partition:
    out = C.c_void_p()
    E = 0 if src is None else int(src.numel())
    _check(load().grp_partition(_ptr(src), _ptr(dst), E, N, K, seed, part_id, _stream(stream), C.byref(out)))
    return Partition(out.value)


def grp_node_owners(N: int, K: int, seed: int, owner_out, count_out=None, stream=None):
    """owner_out: int32 device tensor [N]; count_out: optional int64 device tensor [K]."""
    _check(load().grp_node_owners(N, K, seed, _ptr(owner_out), _ptr(count_out), _stream(stream)))


def grp_epoch_seeds(part: Partition, train_mask, sampler_seed: int, epoch: int, seeds_out, stream=None) -> int:
    """Fills ``seeds_out`` (int32 device tensor [n]) with the partition's training nodes in the order the
    epoch visits them and returns their number."""
    count = C.c_int64(0)
    _check(load().grp_epoch_seeds(part.handle, _ptr(train_mask), sampler_seed, epoch, _stream(stream), _ptr(seeds_out),
                                  C.byref(count)))
    return int(count.value)


def grp_gather_rows(src, idx, keep=None, stream=None):
    """Rows ``idx`` (int64 device tensor) of the dense tensor ``src`` ([n_src] or [n_src, F]) as a new tensor;
    rows whose ``keep`` byte (uint8 device tensor [n]) is 0 are zero-filled."""
    src = src.contiguous()
    n = int(idx.numel())
    out = torch.empty((n,) + tuple(src.shape[1:]), dtype=src.dtype, device=src.device)
    row_bytes = src.element_size() * (int(src[0].numel()) if src.dim() > 1 else 1) if src.shape[0] > 0 else src.element_size()
    _check(load().grp_gather_rows(_ptr(src), int(src.shape[0]), row_bytes, _ptr(idx), n, _ptr(keep), _ptr(out), _stream(stream)))
    return out


def grp_partition_weighted(src, dst, w, N: int, K: int, seed: int, part_id: int, stream=None) -> Partition:
    """``w``: float32 device tensor, one positive weight per edge."""
    out = C.c_void_p()
    E = 0 if src is None else int(src.numel())
    _check(load().grp_partition_weighted(_ptr(src), _ptr(dst), _ptr(w), E, N, K, seed, part_id, _stream(stream),
                                         C.byref(out)))
    return Partition(out.value)


def grp_partition_from_local_coo(src_local, dst_local, n: int, d_global_in=None, l2g=None, stream=None) -> Partition:
    out = C.c_void_p()
    E = 0 if src_local is None else int(src_local.numel())
    _check(load().grp_partition_from_local_coo(_ptr(src_local), _ptr(dst_local), E, n, _ptr(d_global_in), _ptr(l2g),
                                               _stream(stream), C.byref(out)))
    return Partition(out.value)


def grp_partition_from_csr(rowptr, col, n: int, d_global_in=None, l2g=None, slice_edges: int = 0, stream=None) -> Partition:
    """``rowptr`` int64 [n+1], ``col`` int32 [nnz] device tensors; the handle borrows them (kept alive by the
    returned object)."""
    out = C.c_void_p()
    nnz = 0 if col is None else int(col.numel())
    _check(load().grp_partition_from_csr(_ptr(rowptr), _ptr(col), n, nnz, _ptr(d_global_in), _ptr(l2g), slice_edges,
                                         _stream(stream), C.byref(out)))
    part = Partition(out.value)
    part._borrowed = (rowptr, col)
    return part


class Chunks:
    """Owns a grp_chunks_t handle (the graph split once into chunks)."""

    def __init__(self, handle: int, n_chunks: int):
        self.handle, self.n_chunks = handle, n_chunks

    def destroy(self):
        if self.handle:
            _check(load().grp_chunks_destroy(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def grp_chunks_build(src, dst, n_nodes: int, n_chunks: int, seed: int, stream=None) -> Chunks:
    out = C.c_void_p()
    E = 0 if src is None else int(src.numel())
    _check(load().grp_chunks_build(_ptr(src), _ptr(dst), E, n_nodes, n_chunks, seed, _stream(stream), C.byref(out)))
    return Chunks(out.value, n_chunks)


def grp_chunks_build_assigned(src, dst, n_nodes: int, n_chunks: int, chunk_of_node, stream=None) -> Chunks:
    """``chunk_of_node``: int32 device tensor [n_nodes] with values in [0, n_chunks)."""
    out = C.c_void_p()
    E = 0 if src is None else int(src.numel())
    _check(load().grp_chunks_build_assigned(_ptr(src), _ptr(dst), E, n_nodes, n_chunks, _ptr(chunk_of_node),
                                            _stream(stream), C.byref(out)))
    return Chunks(out.value, n_chunks)


def grp_partition_from_chunks(chunks: Chunks, base: int, swept: int, stream=None) -> Partition:
    out = C.c_void_p()
    _check(load().grp_partition_from_chunks(chunks.handle, base, swept, _stream(stream), C.byref(out)))
    return Partition(out.value)


def grp_partition_halo(src, dst, n_nodes: int, n_parts: int, seed: int, part_id: int, hops: int, stream=None) -> Partition:
    out = C.c_void_p()
    E = 0 if src is None else int(src.numel())
    _check(load().grp_partition_halo(_ptr(src), _ptr(dst), E, n_nodes, n_parts, seed, part_id, hops, _stream(stream),
                                     C.byref(out)))
    return Partition(out.value)


def grp_param_count(model: ModelDesc) -> int:
    return int(load().grp_param_count(C.byref(model)))


def grp_step_workspace_bytes(part: Partition, model: ModelDesc, opts: StepOpts) -> int:
    b = C.c_size_t()
    _check(load().grp_step_workspace_bytes(part.handle, C.byref(model), C.byref(opts), C.byref(b)))
    return int(b.value)


def grp_step_activation(part: Partition, model: ModelDesc, opts: StepOpts, workspace, layer: int):
    """(device pointer, pitch in floats) of layer ``layer``'s stored activation inside ``workspace``."""
    ptr, ld = C.c_void_p(), C.c_int64()
    _check(load().grp_step_activation(part.handle, C.byref(model), C.byref(opts), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), layer, C.byref(ptr), C.byref(ld)))
    return ptr.value, int(ld.value)


def grp_step_block(part: Partition, model: ModelDesc, opts: StepOpts, workspace, layer: int) -> BlockView:
    v = BlockView()
    _check(load().grp_step_block(part.handle, C.byref(model), C.byref(opts), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), layer, C.byref(v)))
    return v


def read_block(part: Partition, model: ModelDesc, opts: StepOpts, workspace, layer: int) -> dict:
    """Host copies of a sampled block's arrays (n_dst, n_src, nnz, rowptr, col, dst_nodes, src_nodes or None)."""
    v = grp_step_block(part, model, opts, workspace, layer)
    out = dict(n_dst=int(v.n_dst), n_src=int(v.n_src), nnz=int(v.nnz))
    for name, dt, count in (("rowptr", np.int64, out["n_dst"] + 1), ("col", np.int32, out["nnz"]),
                            ("dst_nodes", np.int32, out["n_dst"]), ("src_nodes", np.int32, out["n_src"])):
        ptr = getattr(v, name)
        if not ptr:
            out[name] = None
            continue
        a = np.empty(count, dtype=dt)
        if count:
            _hip_memcpy_d2h(a, ptr)
        out[name] = a
    return out


def read_activation(part: Partition, model: ModelDesc, opts: StepOpts, workspace, layer: int, rows, cols):
    """Host values of the stored activation at the (row, col) pairs given as equal-length int arrays."""
    ptr, ld = grp_step_activation(part, model, opts, workspace, layer)
    base = (ptr - workspace.data_ptr()) // 4
    flat = workspace.view(torch.float32)
    idx = torch.as_tensor(np.asarray(rows, dtype=np.int64) * ld + np.asarray(cols, dtype=np.int64), device=workspace.device) + base
    torch.cuda.synchronize()
    return flat[idx].cpu().numpy()


def grp_train_step(part: Partition, model: ModelDesc, opts: StepOpts, features, labels, train_mask, weights,
                   workspace, grad_out, stats_out, stream=None, workspace_bytes=None):
    wb = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(load().grp_train_step(part.handle, C.byref(model), C.byref(opts), _ptr(features), _ptr(labels),
                                 _ptr(train_mask), _ptr(weights), _ptr(workspace), wb, _stream(stream),
                                 _ptr(grad_out), _ptr(stats_out)))


def grp_aggregate(grads, ld_grads: int, stats, K: int, P: int, variant: int, update, c_out=None, stream=None):
    _check(load().grp_aggregate(_ptr(grads), ld_grads, _ptr(stats), K, P, variant, _stream(stream), _ptr(update),
                                _ptr(c_out)))


def grp_aggregate_ptrs(grad_tensors, stats, P: int, variant: int, update, c_out=None, stream=None):
    """``grad_tensors``: a list of K device tensors of at least P floats each (separately owned buffers)."""
    ptrs = torch.tensor([t.data_ptr() for t in grad_tensors], dtype=torch.int64, device=update.device)
    aligned = all(t.data_ptr() % 16 == 0 for t in grad_tensors)
    _check(load().grp_aggregate_ptrs(_ptr(ptrs), int(aligned), _ptr(stats), len(grad_tensors), P, variant, _stream(stream),
                                     _ptr(update), _ptr(c_out)))
    return ptrs          # keep alive until the stream has run the launch


def optimizer_desc(kind: int = OPT_ADAM, lr: float = 0.003, beta1: float = 0.9, beta2: float = 0.999,
                   eps: float = 1e-8) -> OptimizerDesc:
    o = OptimizerDesc()
    o.kind, o.lr, o.beta1, o.beta2, o.eps = kind, lr, beta1, beta2, eps
    return o


def grp_optimizer_step(opt: OptimizerDesc, P: int, step: int, theta, update, m=None, v=None, stream=None):
    _check(load().grp_optimizer_step(C.byref(opt), P, step, _ptr(theta), _ptr(update), _ptr(m), _ptr(v), _stream(stream)))


def grp_spmm_workspace_bytes(part: Partition, transposed: bool, F: int) -> int:
    b = C.c_size_t()
    _check(load().grp_spmm_workspace_bytes(part.handle, int(transposed), F, C.byref(b)))
    return int(b.value)


def grp_spmm(part: Partition, transposed: bool, scale: int, self_term: bool, F: int, X, ldx: int, x_dtype: int, Y,
             ldy: int, workspace=None, stream=None):
    """``workspace``: uint8 device tensor of at least grp_spmm_workspace_bytes; None: one is allocated here (torch) and
    kept with the Partition object for later calls."""
    if workspace is None:
        need = grp_spmm_workspace_bytes(part, transposed, F)
        workspace = getattr(part, "_spmm_ws", None)
        if need and (workspace is None or workspace.numel() < need):
            workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
            part._spmm_ws = workspace
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().grp_spmm(part.handle, int(transposed), scale, int(self_term), F, _ptr(X), ldx, x_dtype, _ptr(Y), ldy,
                           _ptr(workspace), wb, _stream(stream)))


def grp_spmm_static(part: Partition, transposed: bool, scale: int, self_term: bool, F: int, X, ldx: int, x_dtype: int, Y,
                    ldy: int, stream=None):
    _check(load().grp_spmm_static(part.handle, int(transposed), scale, int(self_term), F, _ptr(X), ldx, x_dtype, _ptr(Y), ldy,
                                  _stream(stream)))


def grp_gemm_nn(M, N, K, A, lda, a_dtype, B, ldb, Cm, ldc, stream=None):
    _check(load().grp_gemm_nn(M, N, K, _ptr(A), lda, a_dtype, _ptr(B), ldb, _ptr(Cm), ldc, _stream(stream)))


def grp_gemm_nt(M, N, K, A, lda, a_dtype, Bt, ldbt, Cm, ldc, stream=None):
    _check(load().grp_gemm_nt(M, N, K, _ptr(A), lda, a_dtype, _ptr(Bt), ldbt, _ptr(Cm), ldc, _stream(stream)))


def grp_gemm_tn_workspace_bytes(M, K, N) -> int:
    return int(load().grp_gemm_tn_workspace_bytes(M, K, N))


def grp_gemm_tn(M, K, N, A, lda, a_dtype, B, ldb, Cm, ldc, workspace, stream=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().grp_gemm_tn(M, K, N, _ptr(A), lda, a_dtype, _ptr(B), ldb, _ptr(Cm), ldc, _ptr(workspace), wb,
                              _stream(stream)))


def grp_set_slice_policy(min_nodes: int = 1 << 19, min_long_edge_percent: int = 25):
    _check(load().grp_set_slice_policy(min_nodes, min_long_edge_percent))


def grp_profile_enable(on):
    _check(load().grp_profile_enable(int(on)))


def grp_profile_report() -> dict:
    buf = C.create_string_buffer(1 << 16)
    _check(load().grp_profile_report(buf, len(buf)))
    out = {}
    for line in buf.value.decode().splitlines():
        name, cnt, ms, flops, nbytes = line.split()
        out[name] = dict(launches=int(cnt), ms=float(ms), flops=float(flops), bytes=float(nbytes))
    return out


def new_stats(K: int = 1, device="cuda") -> torch.Tensor:
    """Device buffer for K grp_step_stats records."""
    return torch.zeros(K * STATS_BYTES, dtype=torch.uint8, device=device)


def read_stats(stats: torch.Tensor) -> np.ndarray:
    """Host view of the records as a structured array (loss, sum_ratio, R, S, nnz_used)."""
    return np.frombuffer(stats.cpu().numpy().tobytes(), dtype=STATS_DTYPE)


def exported_symbols():
    return ["grp_last_error", "grp_partition", "grp_node_owners", "grp_epoch_seeds", "grp_gather_rows", "grp_partition_weighted", "grp_partition_weights", "grp_partition_from_local_coo", "grp_partition_from_csr", "grp_partition_view",
            "grp_partition_destroy", "grp_chunks_build", "grp_chunks_build_assigned", "grp_chunks_destroy", "grp_partition_from_chunks",
            "grp_partition_base_mask", "grp_partition_halo", "grp_param_count", "grp_step_workspace_bytes", "grp_step_activation", "grp_step_block", "grp_train_step",
            "grp_aggregate", "grp_aggregate_ptrs", "grp_optimizer_step", "grp_spmm", "grp_spmm_workspace_bytes", "grp_spmm_static", "grp_gemm_nn", "grp_gemm_nt", "grp_gemm_tn_workspace_bytes", "grp_gemm_tn",
            "grp_set_slice_policy", "grp_sweep_chunk", "grp_super_epoch_epochs", "grp_controller_create", "grp_controller_observe", "grp_controller_observe_stats", "grp_controller_end_epoch", "grp_controller_state", "grp_controller_destroy", "grp_profile_enable", "grp_profile_report"]
