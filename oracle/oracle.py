"""ctypes wrapper around the CPU oracle (dgi_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; the GPU
library never does.  All arithmetic lives in the C file; this module marshals numpy arrays.

Layer description used here (a plain dict, the same one the GPU binding accepts):
    agg: 'sum' | 'mean' | 'gcn' | 'gat';  act: 'none' | 'relu' | 'elu' | 'leaky_relu'
    W_self, W_neigh: float32 [in_dim, out_dim] (W_self may be None); bias: float32 [out_dim] or None
    heads, attn_src, attn_dst ([heads, head_dim]), attn_slope: GAT only
    act_slope: LeakyReLU slope / ELU alpha;  out_storage: 'f32' | 'bf16'
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dgi_oracle.c")
_LIB = os.path.join(_HERE, "libdgi_oracle.so")

AGG = {"sum": 0, "mean": 1, "gcn": 2, "gat": 3}
ACT = {"none": 0, "relu": 1, "elu": 2, "leaky_relu": 3}
STORAGE = {"f32": 0, "bf16": 1}


class _Layer(ctypes.Structure):
    _fields_ = [
        ("agg", ctypes.c_int), ("act", ctypes.c_int), ("act_slope", ctypes.c_double),
        ("in_dim", ctypes.c_int), ("out_dim", ctypes.c_int), ("heads", ctypes.c_int),
        ("W_self", ctypes.c_void_p), ("W_neigh", ctypes.c_void_p), ("bias", ctypes.c_void_p),
        ("attn_src", ctypes.c_void_p), ("attn_dst", ctypes.c_void_p), ("attn_slope", ctypes.c_double),
        ("out_storage", ctypes.c_int),
    ]


def build(force=False):
    """Compile the oracle with gcc (OpenMP over destination rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_layer_forward.restype = ctypes.c_int
        _lib.oracle_infer.restype = ctypes.c_int
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(lib().oracle_num_threads())


def set_threads(n):
    lib().oracle_set_threads(ctypes.c_int(int(n)))


def _f32(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _marshal_layer(layer, keep):
    W_neigh = _f32(layer["W_neigh"])
    W_self = _f32(layer.get("W_self"))
    bias = _f32(layer.get("bias"))
    a_src = _f32(layer.get("attn_src"))
    a_dst = _f32(layer.get("attn_dst"))
    keep.extend([W_neigh, W_self, bias, a_src, a_dst])
    in_dim, out_dim = W_neigh.shape
    if W_self is not None:
        assert W_self.shape == W_neigh.shape
    heads = int(layer.get("heads", 1) or 1)
    if layer["agg"] == "gat":
        assert a_src.size == out_dim and a_dst.size == out_dim and out_dim % heads == 0
    s = _Layer()
    s.agg = AGG[layer["agg"]]
    s.act = ACT[layer.get("act", "none")]
    s.act_slope = float(layer.get("act_slope", 0.01 if layer.get("act") == "leaky_relu" else 1.0))
    s.in_dim, s.out_dim, s.heads = int(in_dim), int(out_dim), heads
    s.W_self, s.W_neigh, s.bias = _ptr(W_self), _ptr(W_neigh), _ptr(bias)
    s.attn_src, s.attn_dst = _ptr(a_src), _ptr(a_dst)
    s.attn_slope = float(layer.get("attn_slope", 0.2))
    s.out_storage = STORAGE[layer.get("out_storage", "f32")]
    return s


def _csr(indptr, indices):
    ip = np.ascontiguousarray(np.asarray(indptr, dtype=np.int64))
    ix = np.ascontiguousarray(np.asarray(indices, dtype=np.int32))
    return ip, ix


def layer_forward(indptr, indices, layer, h_in, rows=None):
    """Rows `rows` (default: all) of one layer (Eq. 1), from the full input matrix h_in."""
    ip, ix = _csr(indptr, indices)
    n = ip.size - 1
    h = _f32(h_in)
    keep = []
    s = _marshal_layer(layer, keep)
    assert h.shape == (n, s.in_dim), (h.shape, n, s.in_dim)
    if rows is None:
        r, n_rows, rp = None, n, None
    else:
        r = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        assert r.size == 0 or (r.min() >= 0 and r.max() < n)
        n_rows, rp = r.size, r.ctypes.data_as(ctypes.c_void_p)
    out = np.empty((n_rows, s.out_dim), dtype=np.float32)
    rc = lib().oracle_layer_forward(ctypes.c_int64(n), _ptr(ip), _ptr(ix), ctypes.byref(s), _ptr(h), rp,
                                    ctypes.c_int64(n_rows), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle_layer_forward failed")
    return out


def infer(indptr, indices, layers, x):
    """Layer-wise inference of the whole model (Algorithm 2, one node per batch)."""
    ip, ix = _csr(indptr, indices)
    n = ip.size - 1
    h = _f32(x)
    keep = []
    arr = (_Layer * len(layers))(*[_marshal_layer(l, keep) for l in layers])
    assert h.shape == (n, arr[0].in_dim)
    out = np.empty((n, arr[len(layers) - 1].out_dim), dtype=np.float32)
    rc = lib().oracle_infer(ctypes.c_int64(n), _ptr(ip), _ptr(ix), arr, ctypes.c_int(len(layers)), _ptr(h), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle_infer failed")
    return out


def infer_jk(indptr, indices, layers, x):
    """Jumping-knowledge stack (the JKNet example of the paper's appendix): layers[:-1] form a chain, each output
    is kept, and the last layer is applied to their concatenation.  Plain composition of layer_forward."""
    hs = []
    h = _f32(x)
    for layer in layers[:-1]:
        h = layer_forward(indptr, indices, layer, h)
        hs.append(h)
    return layer_forward(indptr, indices, layers[-1], np.concatenate(hs, axis=1))


def infer_sampled(indptr, indices, layers, x, fanout, seed):
    """Sampling inference (Section 2): layer l runs on its own sampled graph (oracle/sampler.py); degrees in the
    mean and GCN normalisers are those of the sampled graph."""
    from . import sampler
    h = _f32(x)
    for l, layer in enumerate(layers):
        ip, ix = sampler.sample_csr(indptr, indices, fanout, seed, l)
        h = layer_forward(ip, ix, layer, h)
    return h
