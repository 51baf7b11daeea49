"""ctypes binding of libslonn.so: argument marshalling only.

Every step of the path (hash projection, selection, gathered-row forward, dense
baseline, table build) runs in the HIP library; PyTorch appears here only as the
owner of device memory and of the stream the kernels are enqueued on.  There is
no CPU fallback: if the library is missing, or a call fails, an exception is
raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslonn.so")

OK, EINVAL, ENOMEM, EHIP, EUNSUPPORTED, ECAP = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
ROWS_ARE_NODES, ROWS_ARE_INPUTS = 0, 1
ACT_NONE, ACT_RELU, ACT_SOFTMAX = 0, 1, 2
DENSE, ELL = 0, 1

EXPORTS = [
    "slonn_version", "slonn_model_create", "slonn_model_destroy", "slonn_build_tables",
    "slonn_tables_export", "slonn_tables_import", "slonn_tables_destroy", "slonn_workspace_bytes",
    "slonn_select", "slonn_sparse_forward", "slonn_dense_forward", "slonn_last_error",
    "slonn_profile_begin", "slonn_profile_end", "slonn_model_set_path",
    "slonn_model_set_hash_nodes_always_active",
    "slonn_policy_create", "slonn_policy_destroy", "slonn_policy_train_confidence",
    "slonn_policy_set_latency_profile", "slonn_policy_keep_aclo", "slonn_policy_keep_lcao",
    "slonn_sparse_forward_aclo",
    "slonn_forward_graph_create", "slonn_forward_graph_launch", "slonn_forward_graph_destroy",
    "slonn_activation_variance", "slonn_sample_hash_nodes", "slonn_model_set_hash_margin",
    "slonn_sparse_forward_static", "slonn_model_set_dense_arithmetic",
    "slonn_sample_hash_nodes_device", "slonn_model_set_tables_refreshable", "slonn_tables_refresh",
    "slonn_model_set_batches_in_flight", "slonn_probe_mfma_rate", "slonn_probe_l_two_read_rate",
]
STATIC_SCRATCH_BYTES = 64 << 20
PROF_KINDS = ("hash", "select", "gather", "dense", "ell", "finalize", "fused", "tiles")
PATH_AUTO, PATH_LAYERS, PATH_FUSED = 0, 1, 2


class SlonnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"slonn error {code}: {msg}")
        self.code = code


class LayerDesc(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("w_dtype", C.c_int32),
                ("w_layout", C.c_int32), ("act", C.c_int32), ("K", C.c_int32), ("L", C.c_int32),
                ("list_cap", C.c_int32), ("W", C.c_void_p), ("bias", C.c_void_p),
                ("hash_nodes", C.POINTER(C.c_int32))]


class Input(C.Structure):
    _fields_ = [("format", C.c_int32), ("x", C.c_void_p), ("idx", C.c_void_p), ("val", C.c_void_p),
                ("nnz", C.c_void_p), ("ell_stride", C.c_int32)]


class Output(C.Structure):
    _fields_ = [("dense", C.c_void_p), ("idx", C.c_void_p), ("val", C.c_void_p), ("cnt", C.c_void_p),
                ("stride", C.c_int32), ("argmax", C.c_void_p)]


class DebugTaps(C.Structure):
    _fields_ = [("codes", C.POINTER(C.c_void_p)), ("z", C.POINTER(C.c_void_p)),
                ("active_idx", C.POINTER(C.c_void_p)), ("active_cnt", C.POINTER(C.c_void_p)),
                ("layer_out", C.POINTER(C.c_void_p))]


_lib = None


def load() -> C.CDLL:
    """Load the library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2204_08400_amd.build`")
        lib = C.CDLL(LIB_PATH)
        lib.slonn_last_error.restype = C.c_char_p
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != OK:
        raise SlonnError(rc, load().slonn_last_error().decode(errors="replace"))


def _ptr(t) -> Optional[int]:
    """device pointer of a torch tensor (or None)"""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        if not torch.cuda.is_available():
            return None
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def slonn_version() -> str:
    buf = C.create_string_buffer(128)
    _check(load().slonn_version(buf, C.c_size_t(128)))
    return buf.value.decode()


def slonn_probe_mfma_rate(scratch, stream=None) -> float:
    """TFLOP/s of a register-only loop of the tile kernels' fp16 MFMAs (measurement aid, see slonn.h)."""
    out = C.c_double(0.0)
    _check(load().slonn_probe_mfma_rate(C.c_void_p(_ptr(scratch)), C.c_size_t(scratch.numel() * scratch.element_size()),
                                            C.c_void_p(_stream_ptr(stream)), C.byref(out)))
    return out.value


def slonn_probe_l_two_read_rate(scratch, stream=None):
    """(GB/s of all compute units together, GB/s of one unit alone) reading L2-resident rows (see slonn.h)."""
    a, b = C.c_double(0.0), C.c_double(0.0)
    _check(load().slonn_probe_l_two_read_rate(C.c_void_p(_ptr(scratch)), C.c_size_t(scratch.numel() * scratch.element_size()),
                                              C.c_void_p(_stream_ptr(stream)), C.byref(a), C.byref(b)))
    return a.value, b.value


class Model:
    """Owns a slonn_model handle; keeps the weight tensors it borrows alive."""

    def __init__(self, layers: Sequence[dict]):
        """layers: dicts with d_in, d_out, W (device tensor), bias (device tensor),
        act, w_dtype, w_layout, K, L, list_cap, hash_nodes (host int32 sequence)."""
        self._keep = []
        descs = (LayerDesc * len(layers))()
        for i, l in enumerate(layers):
            d = descs[i]
            d.d_in, d.d_out = int(l["d_in"]), int(l["d_out"])
            d.w_dtype = int(l.get("w_dtype", F32))
            d.w_layout = int(l.get("w_layout", ROWS_ARE_NODES))
            d.act = int(l.get("act", ACT_NONE))
            d.K, d.L = int(l.get("K", 0)), int(l.get("L", 0))
            d.list_cap = int(l.get("list_cap", 0))
            d.W = _ptr(l["W"]) if l.get("W") is not None else None
            d.bias = _ptr(l["bias"]) if l.get("bias") is not None else None
            hn = l.get("hash_nodes")
            if hn is not None:
                arr = (C.c_int32 * len(hn))(*[int(v) for v in hn])
                self._keep.append(arr)
                d.hash_nodes = C.cast(arr, C.POINTER(C.c_int32))
            self._keep += [l.get("W"), l.get("bias")]
        self.layers = [dict(l) for l in layers]
        self.n_layers = len(layers)
        h = C.c_void_p()
        _check(load().slonn_model_create(descs, len(layers), C.byref(h)))
        self.h = h

    def close(self):
        if getattr(self, "h", None) and load is not None:      # (module globals are gone at interpreter exit)
            load().slonn_model_destroy(self.h)
            self.h = None

    __del__ = close


class Tables:
    def __init__(self, model: Model, handle: C.c_void_p):
        self.model, self.h = model, handle

    def close(self):
        if getattr(self, "h", None) and load is not None:
            load().slonn_tables_destroy(self.h)
            self.h = None

    __del__ = close


def make_input(x=None, idx=None, val=None, nnz=None) -> Input:
    inp = Input()
    if x is not None:
        inp.format, inp.x = DENSE, _ptr(x)
    else:
        inp.format = ELL
        inp.idx, inp.val, inp.nnz = _ptr(idx), _ptr(val), _ptr(nnz)
        inp.ell_stride = int(idx.shape[1])
    inp._keep = (x, idx, val, nnz)
    return inp


def slonn_model_create(layers: Sequence[dict]) -> Model:
    return Model(layers)


def slonn_model_set_path(model: Model, path: int):
    _check(load().slonn_model_set_path(model.h, int(path)))


def slonn_model_set_batches_in_flight(model: Model, n: int):
    """Batches the caller keeps in flight on the device (a hint that sizes workgroups, see slonn.h)."""
    _check(load().slonn_model_set_batches_in_flight(model.h, int(n)))


def slonn_model_set_dense_arithmetic(model: Model, mode: int):
    """0: fp32 matrix cores (default); 1: two fp16 parts on the fp16 matrix cores (see slonn.h)."""
    _check(load().slonn_model_set_dense_arithmetic(model.h, int(mode)))


def slonn_model_set_hash_nodes_always_active(model: Model, on: bool):
    _check(load().slonn_model_set_hash_nodes_always_active(model.h, 1 if on else 0))


def slonn_build_tables(model: Model, X_build: Input, N: int, stream=None) -> Tables:
    h = C.c_void_p()
    _check(load().slonn_build_tables(model.h, C.byref(X_build), C.c_int64(N),
                                     C.c_void_p(_stream_ptr(stream)), C.byref(h)))
    return Tables(model, h)


def slonn_model_set_tables_refreshable(model: Model, on: bool):
    _check(load().slonn_model_set_tables_refreshable(model.h, int(bool(on))))


def slonn_tables_refresh(model: Model, tables: Tables, X_new: Input, N: int, stream=None):
    """Alg. 1 continued on N more training inputs (tables trained as refreshable)."""
    _check(load().slonn_tables_refresh(model.h, tables.h, C.byref(X_new), C.c_int64(N),
                                       C.c_void_p(_stream_ptr(stream))))


def slonn_tables_export_bytes(tables: Tables) -> int:
    """size of the blob slonn_tables_export would write"""
    n = C.c_size_t(0)
    _check(load().slonn_tables_export(tables.h, None, C.byref(n)))
    return n.value


def slonn_tables_export(tables: Tables) -> bytes:
    n = C.c_size_t(0)
    _check(load().slonn_tables_export(tables.h, None, C.byref(n)))
    buf = C.create_string_buffer(n.value)
    _check(load().slonn_tables_export(tables.h, buf, C.byref(n)))
    return buf.raw[:n.value]


def slonn_tables_import(model: Model, blob: bytes) -> Tables:
    h = C.c_void_p()
    _check(load().slonn_tables_import(model.h, blob, C.c_size_t(len(blob)), C.byref(h)))
    return Tables(model, h)


def slonn_workspace_bytes(model: Model, B_max: int) -> int:
    n = C.c_size_t(0)
    _check(load().slonn_workspace_bytes(model.h, int(B_max), C.byref(n)))
    return n.value


def slonn_select(model: Model, tables: Tables, layer: int, X_l, B: int, keep, keep_stride: int,
                 codes_out, z_out, active_idx, active_cnt, idx_stride: int, workspace, stream=None):
    _check(load().slonn_select(
        model.h, tables.h, int(layer), C.c_void_p(_ptr(X_l)), int(B), C.c_void_p(_ptr(keep)),
        int(keep_stride), C.c_void_p(_ptr(codes_out)), C.c_void_p(_ptr(z_out)),
        C.c_void_p(_ptr(active_idx)), C.c_void_p(_ptr(active_cnt)), int(idx_stride),
        C.c_void_p(_ptr(workspace)), C.c_size_t(workspace.numel() * workspace.element_size() if workspace is not None else 0),
        C.c_void_p(_stream_ptr(stream))))


def _ptr_array(tensors: Optional[Sequence], n: int):
    if tensors is None:
        return None
    arr = (C.c_void_p * n)()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t)
    return arr


def make_taps(n_layers: int, codes=None, z=None, active_idx=None, active_cnt=None, layer_out=None):
    taps = DebugTaps()
    keep = []
    for name, lst in (("codes", codes), ("z", z), ("active_idx", active_idx),
                      ("active_cnt", active_cnt), ("layer_out", layer_out)):
        arr = _ptr_array(lst, n_layers)
        keep.append((arr, lst))
        if arr is not None:
            setattr(taps, name, C.cast(arr, C.POINTER(C.c_void_p)))
    taps._keep = keep
    return taps


def make_output(dense=None, idx=None, val=None, cnt=None, stride=0, argmax=None) -> Output:
    out = Output()
    out.dense, out.idx, out.val, out.cnt = _ptr(dense), _ptr(idx), _ptr(val), _ptr(cnt)
    out.stride, out.argmax = int(stride), _ptr(argmax)
    out._keep = (dense, idx, val, cnt, argmax)
    return out


def slonn_sparse_forward(model: Model, tables: Optional[Tables], X: Input, B: int, keep,
                         keep_qstride: int, keep_lstride: int, Y: Output, taps: Optional[DebugTaps],
                         workspace, stream=None):
    _check(load().slonn_sparse_forward(
        model.h, tables.h if tables is not None else None, C.byref(X), int(B),
        C.c_void_p(_ptr(keep)), int(keep_qstride), int(keep_lstride), C.byref(Y),
        C.byref(taps) if taps is not None else None, C.c_void_p(_ptr(workspace)),
        C.c_size_t(workspace.numel() * workspace.element_size() if workspace is not None else 0),
        C.c_void_p(_stream_ptr(stream))))


def slonn_sparse_forward_static(model: Model, tables: Optional[Tables], X: Input, B: int, keep,
                                keep_qstride: int, keep_lstride: int, Y: Output, taps: Optional[DebugTaps],
                                stream=None):
    """slonn_sparse_forward on the library's static scratch array: the call allocates nothing."""
    _check(load().slonn_sparse_forward_static(
        model.h, tables.h if tables is not None else None, C.byref(X), int(B),
        C.c_void_p(_ptr(keep)), int(keep_qstride), int(keep_lstride), C.byref(Y),
        C.byref(taps) if taps is not None else None, C.c_void_p(_stream_ptr(stream))))


class Policy:
    """Owns a slonn_policy handle (k grid, Confidence LSH tables, latency profile)."""

    def __init__(self, K: int, L: int, k_grid: Sequence[float]):
        grid = (C.c_float * len(k_grid))(*[float(v) for v in k_grid])
        h = C.c_void_p()
        _check(load().slonn_policy_create(int(K), int(L), grid, len(k_grid), C.byref(h)))
        self.h, self.K, self.L, self.G = h, int(K), int(L), len(k_grid)

    def close(self):
        if getattr(self, "h", None) and load is not None:
            load().slonn_policy_destroy(self.h)
            self.h = None

    __del__ = close


def slonn_policy_create(K: int, L: int, k_grid: Sequence[float]) -> Policy:
    return Policy(K, L, k_grid)


def slonn_policy_train_confidence(policy: Policy, codes, conf, N: int, stream=None):
    _check(load().slonn_policy_train_confidence(policy.h, C.c_void_p(_ptr(codes)), C.c_void_p(_ptr(conf)),
                                                C.c_int64(int(N)), C.c_void_p(_stream_ptr(stream))))


def slonn_policy_set_latency_profile(policy: Policy, T: Sequence[Sequence[float]]):
    flat = [float(v) for row in T for v in row]
    arr = (C.c_float * len(flat))(*flat)
    _check(load().slonn_policy_set_latency_profile(policy.h, arr, len(T)))


def slonn_policy_keep_aclo(policy: Policy, codes, B: int, thr, thr_stride: int, keep_out, grid_idx_out=None,
                           c_hat_out=None, stream=None):
    _check(load().slonn_policy_keep_aclo(policy.h, C.c_void_p(_ptr(codes)), int(B), C.c_void_p(_ptr(thr)),
                                         int(thr_stride), C.c_void_p(_ptr(keep_out)),
                                         C.c_void_p(_ptr(grid_idx_out)), C.c_void_p(_ptr(c_hat_out)),
                                         C.c_void_p(_stream_ptr(stream))))


def slonn_policy_keep_lcao(policy: Policy, B: int, tau, tau_stride: int, t0, t0_stride: int, beta,
                           beta_stride: int, keep_out, grid_idx_out=None, violated_out=None, stream=None):
    _check(load().slonn_policy_keep_lcao(policy.h, int(B), C.c_void_p(_ptr(tau)), int(tau_stride),
                                         C.c_void_p(_ptr(t0)), int(t0_stride), C.c_void_p(_ptr(beta)),
                                         int(beta_stride), C.c_void_p(_ptr(keep_out)),
                                         C.c_void_p(_ptr(grid_idx_out)), C.c_void_p(_ptr(violated_out)),
                                         C.c_void_p(_stream_ptr(stream))))


def slonn_sparse_forward_aclo(model: Model, tables: Optional[Tables], policy: Policy, X: Input, B: int, thr,
                              thr_stride: int, keep_out, Y: Output, taps: Optional[DebugTaps], workspace,
                              stream=None):
    _check(load().slonn_sparse_forward_aclo(
        model.h, tables.h if tables is not None else None, policy.h, C.byref(X), int(B),
        C.c_void_p(_ptr(thr)), int(thr_stride), C.c_void_p(_ptr(keep_out)), C.byref(Y),
        C.byref(taps) if taps is not None else None, C.c_void_p(_ptr(workspace)),
        C.c_size_t(workspace.numel() * workspace.element_size() if workspace is not None else 0),
        C.c_void_p(_stream_ptr(stream))))


def slonn_model_set_hash_margin(model: Model, margin: float):
    _check(load().slonn_model_set_hash_margin(model.h, C.c_double(margin)))


def slonn_activation_variance(A, var_out, stream=None):
    """A: device float32 [N][n] (rows may be strided), var_out: device float64 [n]."""
    if A.dim() != 2 or A.stride(1) != 1:
        raise ValueError("A must be a 2-D tensor with unit column stride")
    _check(load().slonn_activation_variance(C.c_void_p(A.data_ptr()), C.c_int64(A.shape[0]), int(A.shape[1]),
                                            C.c_int64(A.stride(0)), C.c_void_p(_ptr(var_out)),
                                            C.c_void_p(_stream_ptr(stream))))


def slonn_sample_hash_nodes_device(variance, K: int, L: int, u, out, stream=None):
    """variance: device float64 [n]; u: device float64 [K*L]; out: device int32 [K*L]."""
    _check(load().slonn_sample_hash_nodes_device(C.c_void_p(_ptr(variance)), int(variance.numel()), int(K), int(L),
                                                 C.c_void_p(_ptr(u)), C.c_void_p(_ptr(out)),
                                                 C.c_void_p(_stream_ptr(stream))))


def slonn_sample_hash_nodes(variance: np.ndarray, K: int, L: int, u: np.ndarray) -> np.ndarray:
    """Host arrays: variance float64 [n], u float64 [K*L] in [0, 1); returns int32 [K*L]."""
    variance = np.ascontiguousarray(variance, dtype=np.float64)
    u = np.ascontiguousarray(u, dtype=np.float64)
    if u.shape[0] != K * L:
        raise ValueError("u must hold K*L draws")
    out = np.empty(K * L, dtype=np.int32)
    _check(load().slonn_sample_hash_nodes(variance.ctypes.data_as(C.c_void_p), int(variance.shape[0]), int(K),
                                          int(L), u.ctypes.data_as(C.c_void_p),
                                          out.ctypes.data_as(C.c_void_p)))
    return out


class ForwardGraph:
    """Owns a slonn_graph handle and keeps every baked-in buffer alive."""

    def __init__(self, handle, keep_alive):
        self.h, self._keep = handle, keep_alive

    def launch(self, stream=None):
        _check(load().slonn_forward_graph_launch(self.h, C.c_void_p(_stream_ptr(stream))))

    def close(self):
        if getattr(self, "h", None) and load is not None:
            load().slonn_forward_graph_destroy(self.h)
            self.h = None

    __del__ = close


def slonn_forward_graph_create(model: Model, tables: Optional[Tables], X: Input, B: int, keep, keep_qstride: int,
                               keep_lstride: int, Y: Output, workspace) -> ForwardGraph:
    h = C.c_void_p()
    _check(load().slonn_forward_graph_create(
        model.h, tables.h if tables is not None else None, C.byref(X), int(B), C.c_void_p(_ptr(keep)),
        int(keep_qstride), int(keep_lstride), C.byref(Y), C.c_void_p(_ptr(workspace)),
        C.c_size_t(workspace.numel() * workspace.element_size() if workspace is not None else 0), C.byref(h)))
    return ForwardGraph(h, (model, tables, X, keep, Y, workspace))


def slonn_dense_forward(model: Model, X: Input, B: int, Y, argmax, layer_out: Optional[Sequence],
                        workspace, stream=None):
    arr = _ptr_array(layer_out, model.n_layers)
    _check(load().slonn_dense_forward(
        model.h, C.byref(X), int(B), C.c_void_p(_ptr(Y)), C.c_void_p(_ptr(argmax)),
        C.cast(arr, C.POINTER(C.c_void_p)) if arr is not None else None,
        C.c_void_p(_ptr(workspace)),
        C.c_size_t(workspace.numel() * workspace.element_size() if workspace is not None else 0),
        C.c_void_p(_stream_ptr(stream))))


def slonn_profile_begin(max_launches: int):
    _check(load().slonn_profile_begin(int(max_launches)))


def slonn_profile_end() -> dict:
    """{kind: (total_ms, launches)} for the kernels launched since slonn_profile_begin."""
    ms = (C.c_double * len(PROF_KINDS))()
    cnt = (C.c_int64 * len(PROF_KINDS))()
    _check(load().slonn_profile_end(ms, cnt))
    return {k: (ms[i], cnt[i]) for i, k in enumerate(PROF_KINDS)}
