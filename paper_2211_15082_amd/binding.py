"""Thin ctypes binding of libdgi.so.  Argument marshalling only: every step of the inference path runs in
the library's HIP kernels.  Function names mirror the C ABI in include/dgi.h.

Device buffers are torch tensors (torch is used for device memory and streams only); their data_ptr()
and the current stream's handle cross the boundary.  There is no CPU fallback: if the library is not
built, importing this module raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdgi.so")

OK, ERR_INVALID_ARG, ERR_BAD_GRAPH, ERR_UNSUPPORTED, ERR_OOM, ERR_DEVICE = range(6)
I32, I64 = 0, 1
HOST, DEVICE = 0, 1
F32, BF16 = 0, 1
AGG = {"sum": 0, "mean": 1, "gcn": 2, "gat": 3}
ACT = {"none": 0, "relu": 1, "elu": 2, "leaky_relu": 3}
ORDER = {"auto": 0, "agg_first": 1, "transform_first": 2, "agg_first_fused": 3, "agg_first_split": 4}
REORDER = {"none": 0, "degree": 1, "bfs_rcm": 2, "random": 3, "community": 4}
MAX_LAYERS = 16


class DgiError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("dgi status %d (%s): %s" % (status, _status_string(status), message))
        self.status = status


class LayerStruct(ctypes.Structure):
    _fields_ = [
        ("agg", ctypes.c_int32), ("act", ctypes.c_int32), ("act_slope", ctypes.c_float),
        ("in_dim", ctypes.c_int32), ("out_dim", ctypes.c_int32), ("heads", ctypes.c_int32),
        ("feat_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32), ("order", ctypes.c_int32),
        ("W_self", ctypes.c_void_p), ("W_neigh", ctypes.c_void_p), ("bias", ctypes.c_void_p),
        ("attn_src", ctypes.c_void_p), ("attn_dst", ctypes.c_void_p),
        ("attn_slope", ctypes.c_float), ("reserved", ctypes.c_int32),
    ]


class StatsStruct(ctypes.Structure):
    _fields_ = [
        ("num_layers", ctypes.c_int32), ("reserved", ctypes.c_int32), ("total_ms", ctypes.c_double),
        ("layer_ms", ctypes.c_double * MAX_LAYERS), ("agg_ms", ctypes.c_double * MAX_LAYERS),
        ("hub_ms", ctypes.c_double * MAX_LAYERS),
        ("gemm_ms", ctypes.c_double * MAX_LAYERS), ("agg_launches", ctypes.c_int64 * MAX_LAYERS),
        ("gemm_launches", ctypes.c_int64 * MAX_LAYERS), ("batches", ctypes.c_int64 * MAX_LAYERS),
        ("edges", ctypes.c_int64 * MAX_LAYERS), ("transform_first", ctypes.c_int32 * MAX_LAYERS),
        ("gather_width", ctypes.c_int32 * MAX_LAYERS), ("fused", ctypes.c_int32 * MAX_LAYERS),
        ("oom_retries", ctypes.c_int64),
        ("workspace_bytes", ctypes.c_int64),
    ]


class OptsStruct(ctypes.Structure):
    _fields_ = [
        ("batch_size", ctypes.c_int64), ("perm_new_of_old", ctypes.c_void_p), ("mem_budget_bytes", ctypes.c_uint64),
        ("stats", ctypes.POINTER(StatsStruct)), ("init_node_threshold", ctypes.c_int64),
        ("init_edge_threshold", ctypes.c_int64), ("jk_concat", ctypes.c_int32), ("host_stream_always", ctypes.c_int32),
    ]


class PartialStatsStruct(ctypes.Structure):
    _fields_ = [
        ("num_layers", ctypes.c_int32), ("all_nodes_from_layer", ctypes.c_int32),
        ("set_size", ctypes.c_int64 * (MAX_LAYERS + 1)), ("sub_nodes", ctypes.c_int64), ("sub_edges", ctypes.c_int64),
        ("rows_computed", ctypes.c_int64 * MAX_LAYERS),
    ]


class HostStatsStruct(ctypes.Structure):
    _fields_ = [
        ("num_layers", ctypes.c_int32), ("device_resident", ctypes.c_int32), ("total_ms", ctypes.c_double),
        ("load_ms", ctypes.c_double * MAX_LAYERS), ("compute_ms", ctypes.c_double * MAX_LAYERS), ("store_ms", ctypes.c_double * MAX_LAYERS),
        ("batches", ctypes.c_int64 * MAX_LAYERS), ("input_rows", ctypes.c_int64 * MAX_LAYERS), ("input_bytes", ctypes.c_int64 * MAX_LAYERS),
        ("output_bytes", ctypes.c_int64 * MAX_LAYERS), ("transform_bytes", ctypes.c_int64 * MAX_LAYERS), ("oom_retries", ctypes.c_int64), ("peak_batch_bytes", ctypes.c_int64),
        ("budget_bytes", ctypes.c_int64), ("slots", ctypes.c_int64),
    ]


class GraphInfoStruct(ctypes.Structure):
    _fields_ = [
        ("num_nodes", ctypes.c_int64), ("num_edges", ctypes.c_int64), ("max_in_degree", ctypes.c_int64),
        ("num_hub_rows", ctypes.c_int64), ("num_hub_edges", ctypes.c_int64), ("indptr_type", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("device_bytes", ctypes.c_uint64),
    ]


EXPORTS = [
    "dgi_graph_load", "dgi_graph_free", "dgi_graph_release_workspace", "dgi_graph_info", "dgi_graph_vector", "dgi_graph_csr", "dgi_graph_reorder",
    "dgi_layer_forward", "dgi_layer_forward_static", "dgi_layer_workspace_bytes", "dgi_infer", "dgi_infer_partial", "dgi_infer_host", "dgi_graph_sample", "dgi_infer_sampled", "dgi_plan_batch_end", "dgi_threshold_update",
    "dgi_threshold_halve", "dgi_batch_input_set_size", "dgi_reorder_permutation", "dgi_status_string",
    "dgi_last_error", "dgi_version", "dgi_host_alloc", "dgi_host_free",
]

if not os.path.exists(LIB_PATH):
    raise ImportError("libdgi.so is not built (%s): run `python -c 'import __graft_entry__ as g; g.build()'`" % LIB_PATH)
_lib = ctypes.CDLL(LIB_PATH)
for _name in EXPORTS:
    getattr(_lib, _name).restype = ctypes.c_int
_lib.dgi_status_string.restype = ctypes.c_char_p
_lib.dgi_last_error.restype = ctypes.c_char_p
_lib.dgi_version.restype = ctypes.c_int32


def _status_string(s):
    return _lib.dgi_status_string(ctypes.c_int(s)).decode()


def last_error():
    return _lib.dgi_last_error().decode()


def version():
    return int(_lib.dgi_version())


def _check(status):
    if status != OK:
        raise DgiError(status, last_error())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("unsupported tensor dtype %s" % t.dtype)


# ---------------------------------------------------------------------------------------------------
class Graph:
    """Owns a dgi_graph_t handle (and keeps borrowed device tensors alive)."""

    def __init__(self, handle, keep=()):
        self.handle = handle
        self._keep = keep

    def free(self):
        if self.handle:
            _lib.dgi_graph_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def release_workspace(self):
        _check(_lib.dgi_graph_release_workspace(self.handle))

    def info(self):
        s = GraphInfoStruct()
        _check(_lib.dgi_graph_info(self.handle, ctypes.byref(s)))
        return {k: getattr(s, k) for k, _ in GraphInfoStruct._fields_ if k != "reserved"}

    def vector(self, kind):
        n = self.info()["num_nodes"]
        out = np.empty(n, dtype=np.int32 if kind in (0, 1) else np.float32)
        _check(_lib.dgi_graph_vector(self.handle, ctypes.c_int32(kind), out.ctypes.data_as(ctypes.c_void_p)))
        return out

    def csr(self):
        i = self.info()
        ip = np.empty(i["num_nodes"] + 1, dtype=np.int64)
        ix = np.empty(i["num_edges"], dtype=np.int32)
        _check(_lib.dgi_graph_csr(self.handle, ip.ctypes.data_as(ctypes.c_void_p), ix.ctypes.data_as(ctypes.c_void_p)))
        return ip, ix


def graph_load(indptr, indices):
    """indptr / indices: numpy arrays (HOST, copied) or torch CUDA tensors (DEVICE, borrowed)."""
    handle = ctypes.c_void_p()
    if isinstance(indptr, np.ndarray):
        ip = np.ascontiguousarray(indptr)
        if ip.dtype not in (np.int32, np.int64):
            ip = ip.astype(np.int64)
        ix = np.ascontiguousarray(indices, dtype=np.int32)
        itype = I64 if ip.dtype == np.int64 else I32
        _check(_lib.dgi_graph_load(ctypes.c_int64(ip.size - 1), ctypes.c_int64(ix.size), ip.ctypes.data_as(ctypes.c_void_p),
                                   ctypes.c_int32(itype), ix.ctypes.data_as(ctypes.c_void_p), ctypes.c_int32(HOST), _stream(),
                                   ctypes.byref(handle)))
        return Graph(handle)
    import torch
    assert indptr.is_cuda and indices.is_cuda and indices.dtype == torch.int32
    ip, ix = indptr.contiguous(), indices.contiguous()
    itype = I64 if ip.dtype == torch.int64 else I32
    _check(_lib.dgi_graph_load(ctypes.c_int64(ip.numel() - 1), ctypes.c_int64(ix.numel()), _dptr(ip), ctypes.c_int32(itype),
                               _dptr(ix), ctypes.c_int32(DEVICE), _stream(), ctypes.byref(handle)))
    return Graph(handle, keep=(ip, ix))


def graph_reorder(graph, method, seed=0):
    """Returns (reordered Graph, perm_new_of_old as a torch int32 CUDA tensor)."""
    import torch
    n = graph.info()["num_nodes"]
    perm = torch.empty(max(n, 1), dtype=torch.int32, device="cuda")
    handle = ctypes.c_void_p()
    _check(_lib.dgi_graph_reorder(graph.handle, ctypes.c_int32(REORDER[method]), ctypes.c_uint64(seed), _stream(),
                                  ctypes.byref(handle), _dptr(perm), ctypes.c_int32(DEVICE)))
    return Graph(handle), perm[:n]


def make_layer(layer, device="cuda", feat_dtype=None):
    """dict (see oracle wrapper for the vocabulary) -> (LayerStruct, tensors kept alive).

    Weights are moved to `device` in the layer's feature dtype ('f32' default, or layer['feat_storage']
    == 'bf16'); bias and attention vectors stay fp32."""
    import torch
    storage = feat_dtype or layer.get("feat_storage", "f32")
    wdt = torch.bfloat16 if storage == "bf16" else torch.float32

    def dev(a, dt):
        if a is None:
            return None
        t = a if isinstance(a, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(a))
        return t.to(device=device, dtype=dt).contiguous()

    Wn, Ws = dev(layer["W_neigh"], wdt), dev(layer.get("W_self"), wdt)
    bias = dev(layer.get("bias"), torch.float32)
    a_s, a_d = dev(layer.get("attn_src"), torch.float32), dev(layer.get("attn_dst"), torch.float32)
    s = LayerStruct()
    s.agg = AGG[layer["agg"]]
    s.act = ACT[layer.get("act", "none")]
    s.act_slope = float(layer.get("act_slope", 0.01 if layer.get("act") == "leaky_relu" else 1.0))
    s.in_dim, s.out_dim = int(Wn.shape[0]), int(Wn.shape[1])
    s.heads = int(layer.get("heads", 1) or 1)
    s.feat_dtype = BF16 if storage == "bf16" else F32
    s.out_dtype = BF16 if layer.get("out_storage", "f32") == "bf16" else F32
    s.order = ORDER[layer.get("order", "auto")]
    s.W_self, s.W_neigh, s.bias = _dptr(Ws).value, _dptr(Wn).value, _dptr(bias).value
    s.attn_src, s.attn_dst = _dptr(a_s).value, _dptr(a_d).value
    s.attn_slope = float(layer.get("attn_slope", 0.2))
    return s, (Wn, Ws, bias, a_s, a_d)


def layer_workspace_bytes(graph, layer_struct, dst_begin, dst_end):
    b = ctypes.c_uint64()
    _check(_lib.dgi_layer_workspace_bytes(graph.handle, ctypes.byref(layer_struct), ctypes.c_int64(dst_begin),
                                          ctypes.c_int64(dst_end), ctypes.byref(b)))
    return int(b.value)


def layer_forward(graph, layer_struct, h_in, h_out, dst_begin, dst_end, workspace=None, ld_in=None, ld_out=None):
    """h_in / h_out: 2-D torch CUDA tensors (row stride = leading dimension)."""
    import torch
    ld_in = int(h_in.stride(0)) if ld_in is None else ld_in
    ld_out = int(h_out.stride(0)) if ld_out is None else ld_out
    if workspace is None:
        need = layer_workspace_bytes(graph, layer_struct, dst_begin, dst_end)
        workspace = torch.empty(need + 256, dtype=torch.uint8, device=h_in.device)
    off = (-workspace.data_ptr()) % 256
    _check(_lib.dgi_layer_forward(graph.handle, ctypes.byref(layer_struct), _dptr(h_in), ctypes.c_int64(ld_in), _dptr(h_out),
                                  ctypes.c_int64(ld_out), ctypes.c_int64(dst_begin), ctypes.c_int64(dst_end),
                                  ctypes.c_void_p(workspace.data_ptr() + off), ctypes.c_uint64(workspace.numel() - off), _stream()))
    return h_out


STATIC_WORKSPACE_BYTES = 32 << 20  # DGI_STATIC_WORKSPACE_BYTES


def layer_forward_static(graph, layer_struct, h_in, h_out, dst_begin, dst_end, ld_in=None, ld_out=None):
    """dgi_layer_forward_static: the same layer call on the library's static device workspace (nothing is allocated)."""
    ld_in = int(h_in.stride(0)) if ld_in is None else ld_in
    ld_out = int(h_out.stride(0)) if ld_out is None else ld_out
    _check(_lib.dgi_layer_forward_static(graph.handle, ctypes.byref(layer_struct), _dptr(h_in), ctypes.c_int64(ld_in), _dptr(h_out),
                                         ctypes.c_int64(ld_out), ctypes.c_int64(dst_begin), ctypes.c_int64(dst_end), _stream()))
    return h_out


def infer(graph, layer_structs, x, out, batch_size=0, perm_new_of_old=None, mem_budget_bytes=0, want_stats=False,
          init_node_threshold=0, init_edge_threshold=0, jk_concat=False):
    arr = (LayerStruct * len(layer_structs))(*layer_structs)
    opts = OptsStruct()
    opts.batch_size = int(batch_size)
    opts.perm_new_of_old = _dptr(perm_new_of_old).value
    opts.mem_budget_bytes = int(mem_budget_bytes)
    opts.init_node_threshold = int(init_node_threshold)
    opts.init_edge_threshold = int(init_edge_threshold)
    opts.jk_concat = 1 if jk_concat else 0
    stats = StatsStruct() if want_stats else None
    if stats is not None:
        opts.stats = ctypes.pointer(stats)
    _check(_lib.dgi_infer(graph.handle, arr, ctypes.c_int32(len(layer_structs)), _dptr(x), ctypes.c_int64(x.stride(0)),
                          _dptr(out), ctypes.c_int64(out.stride(0)), ctypes.byref(opts), _stream()))
    if stats is None:
        return None
    n = stats.num_layers
    d = {k: (list(getattr(stats, k))[:n] if hasattr(getattr(stats, k), "__len__") else getattr(stats, k))
         for k, _ in StatsStruct._fields_ if k != "reserved"}
    return d


def infer_partial(graph, layer_structs, x, targets, out, batch_size=0, mem_budget_bytes=0):
    """targets: torch int32 CUDA tensor; out: [len(targets), out_dim] CUDA tensor.  Returns the annotation stats."""
    arr = (LayerStruct * len(layer_structs))(*layer_structs)
    opts = OptsStruct()
    opts.batch_size = int(batch_size)
    opts.mem_budget_bytes = int(mem_budget_bytes)
    ps = PartialStatsStruct()
    _check(_lib.dgi_infer_partial(graph.handle, arr, ctypes.c_int32(len(layer_structs)), _dptr(x), ctypes.c_int64(x.stride(0)),
                                  _dptr(targets), ctypes.c_int64(targets.numel()), _dptr(out), ctypes.c_int64(out.stride(0)),
                                  ctypes.byref(opts), ctypes.byref(ps), _stream()))
    n = ps.num_layers
    return {"set_size": list(ps.set_size)[:n + 1], "all_nodes_from_layer": ps.all_nodes_from_layer,
            "sub_nodes": ps.sub_nodes, "sub_edges": ps.sub_edges, "rows_computed": list(ps.rows_computed)[:n]}


def graph_sample(graph, fanout, seed, layer):
    """The sampled graph of one layer (a new Graph handle)."""
    h = ctypes.c_void_p()
    _check(_lib.dgi_graph_sample(graph.handle, ctypes.c_int32(fanout), ctypes.c_uint64(seed), ctypes.c_int32(layer), _stream(), ctypes.byref(h)))
    return Graph(h)


def infer_sampled(graph, layer_structs, x, out, fanout, seed, batch_size=0, mem_budget_bytes=0):
    arr = (LayerStruct * len(layer_structs))(*layer_structs)
    opts = OptsStruct()
    opts.batch_size = int(batch_size)
    opts.mem_budget_bytes = int(mem_budget_bytes)
    _check(_lib.dgi_infer_sampled(graph.handle, arr, ctypes.c_int32(len(layer_structs)), _dptr(x), ctypes.c_int64(x.stride(0)),
                                  _dptr(out), ctypes.c_int64(out.stride(0)), ctypes.c_int32(fanout), ctypes.c_uint64(seed),
                                  ctypes.byref(opts), _stream()))


def infer_host(graph, layer_structs, x_host, out_host, batch_size=0, mem_budget_bytes=0, init_node_threshold=0,
               init_edge_threshold=0, stream_always=False):
    """x_host / out_host: pinned CPU tensors (torch `pin_memory=True`; the library refuses anything else).
    Returns the transfer statistics."""
    arr = (LayerStruct * len(layer_structs))(*layer_structs)
    opts = OptsStruct()
    opts.batch_size = int(batch_size)
    opts.mem_budget_bytes = int(mem_budget_bytes)
    opts.init_node_threshold = int(init_node_threshold)
    opts.init_edge_threshold = int(init_edge_threshold)
    opts.host_stream_always = 1 if stream_always else 0
    hs = HostStatsStruct()
    _check(_lib.dgi_infer_host(graph.handle, arr, ctypes.c_int32(len(layer_structs)), _dptr(x_host), ctypes.c_int64(x_host.stride(0)),
                               _dptr(out_host), ctypes.c_int64(out_host.stride(0)), ctypes.byref(opts), ctypes.byref(hs), _stream()))
    n = hs.num_layers
    return {k: (list(getattr(hs, k))[:n] if hasattr(getattr(hs, k), "__len__") else getattr(hs, k))
            for k, _ in HostStatsStruct._fields_ if k != "reserved"}


class _PinnedBlock:
    """Owner of one dgi_host_alloc block; frees it when the last tensor viewing it is gone."""

    def __init__(self, nbytes):
        p = ctypes.c_void_p()
        _check(_lib.dgi_host_alloc(ctypes.c_uint64(nbytes), ctypes.byref(p)))
        self.ptr, self.nbytes = p.value, nbytes

    def __del__(self):
        if getattr(self, "ptr", None):
            _lib.dgi_host_free(ctypes.c_void_p(self.ptr))
            self.ptr = None


def pinned_empty(shape, dtype):
    """A page-locked host tensor of exactly the requested size (torch's pinned allocator rounds sizes up to a power
    of two; at tens of gigabytes that is what runs the box out of lockable memory)."""
    import torch
    n = 1
    for d in shape:
        n *= int(d)
    block = _PinnedBlock(n * torch.empty((), dtype=dtype).element_size())
    buf = (ctypes.c_ubyte * max(block.nbytes, 1)).from_address(block.ptr)
    buf._dgi_block = block  # the tensor's storage holds `buf`, and `buf` holds the block: freed with the last view
    return torch.frombuffer(buf, dtype=dtype, count=n).reshape(*shape)


# ---- host-side planning helpers (no device access) ------------------------------------------------------
def plan_batch_end(indptr, row_limit, begin, n_t, n_i):
    ip = np.ascontiguousarray(indptr)
    itype = I64 if ip.dtype == np.int64 else I32
    assert ip.dtype in (np.int32, np.int64)
    end = ctypes.c_int64()
    _check(_lib.dgi_plan_batch_end(ip.ctypes.data_as(ctypes.c_void_p), ctypes.c_int32(itype), ctypes.c_int64(row_limit),
                                   ctypes.c_int64(begin), ctypes.c_int64(n_t), ctypes.c_int64(n_i), ctypes.byref(end)))
    return int(end.value)


def threshold_update(M_expected, M_k, n_t, n_i):
    a, b = ctypes.c_int64(n_t), ctypes.c_int64(n_i)
    _check(_lib.dgi_threshold_update(ctypes.c_double(M_expected), ctypes.c_double(M_k), ctypes.byref(a), ctypes.byref(b)))
    return int(a.value), int(b.value)


def threshold_halve(n_t, n_i):
    a, b = ctypes.c_int64(n_t), ctypes.c_int64(n_i)
    _check(_lib.dgi_threshold_halve(ctypes.byref(a), ctypes.byref(b)))
    return int(a.value), int(b.value)


def batch_input_set_size(indptr, indices, begin, end):
    ip = np.ascontiguousarray(indptr, dtype=np.int64)
    ix = np.ascontiguousarray(indices, dtype=np.int32)
    c = ctypes.c_int64()
    _check(_lib.dgi_batch_input_set_size(ctypes.c_int64(ip.size - 1), ip.ctypes.data_as(ctypes.c_void_p),
                                         ix.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(begin), ctypes.c_int64(end),
                                         ctypes.byref(c)))
    return int(c.value)


def reorder_permutation(indptr, indices, method, seed=0):
    ip = np.ascontiguousarray(indptr, dtype=np.int64)
    ix = np.ascontiguousarray(indices, dtype=np.int32)
    perm = np.empty(ip.size - 1, dtype=np.int32)
    _check(_lib.dgi_reorder_permutation(ctypes.c_int64(ip.size - 1), ip.ctypes.data_as(ctypes.c_void_p),
                                        ix.ctypes.data_as(ctypes.c_void_p), ctypes.c_int32(REORDER[method]),
                                        ctypes.c_uint64(seed), perm.ctypes.data_as(ctypes.c_void_p)))
    return perm
