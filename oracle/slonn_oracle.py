"""Python face of the CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Thin ctypes marshalling around ``slonn_oracle.cpp`` plus the per-network loop
(for l in layers: select, sparse layer; commented "k% forward propagation"
procedure of Section 2.1).  Only tests, the smoke check and the CPU-baseline leg
of the benchmark may import this module; it never touches the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import struct
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slonn_oracle.cpp")
_LIB = os.path.join(_HERE, "libslonn_oracle.so")

TIE_EPS = 1e-6
BLOB_MAGIC = 0x544E4C53        # "SLNT"
BLOB_VERSION = 1


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (g++ -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread",
                               "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.so_tables_build.restype = C.c_void_p
        _lib.so_tables_from_lists.restype = C.c_void_p
        _lib.so_tables_bucket_count.restype = C.c_int64
        _lib.so_tables_csr.restype = C.c_int64
        _lib.so_conf_build.restype = C.c_void_p
        _lib.so_budget.restype = C.c_int32
        _lib.so_budget.argtypes = [C.c_float, C.c_int32]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def default_threads() -> int:
    return max(1, len(os.sched_getaffinity(0)))


def budget(keep: float, n: int) -> int:
    return int(lib().so_budget(C.c_float(float(keep)), n))


# --------------------------------------------------------------------------- #
# layer-level calls
# --------------------------------------------------------------------------- #
def dense_layer(layer, X, threads=1, want_pre=False):
    X = _f32(X)
    N = X.shape[0]
    out = np.empty((N, layer.d_out), np.float32)
    pre = np.empty((N, layer.d_out), np.float32) if want_pre else None
    W = np.ascontiguousarray(layer.W)
    lib().so_dense_layer(_p(W), layer.w_dtype, _p(layer.bias), layer.d_in, layer.d_out, layer.act,
                         _p(X), C.c_int64(N), _p(pre), _p(out), threads)
    return (out, pre) if want_pre else out


def dense_layer_ell(layer, idx, val, nnz, threads=1, rows_are_inputs=False):
    idx = np.ascontiguousarray(idx, np.int32)
    val = _f32(val)
    nnz = np.ascontiguousarray(nnz, np.int32)
    N = idx.shape[0]
    out = np.empty((N, layer.d_out), np.float32)
    W = np.ascontiguousarray(layer.W)
    lib().so_dense_layer_ell(_p(W), layer.w_dtype, int(rows_are_inputs), _p(layer.bias), layer.d_in,
                             layer.d_out, layer.act, _p(idx), _p(val), _p(nnz),
                             C.c_int64(idx.shape[1]), C.c_int64(N), _p(out), threads)
    return out


def hash_project(layer, X, threads=1):
    X = _f32(X)
    N = X.shape[0]
    hn = np.ascontiguousarray(layer.hash_nodes, np.int32)
    Z = np.empty((N, hn.size), np.float32)
    W = np.ascontiguousarray(layer.W)
    lib().so_hash_project(_p(W), layer.w_dtype, _p(layer.bias), layer.d_in, _p(hn), hn.size,
                          _p(X), C.c_int64(N), _p(Z), threads)
    return Z


def keys_from_z(Z, K, L, tie_eps=TIE_EPS):
    Z = _f32(Z)
    N = Z.shape[0]
    keys = np.empty((N, L), np.uint32)
    tie = np.empty(N, np.uint8)
    lib().so_keys(_p(Z), C.c_int64(N), K, L, _p(keys), _p(tie), C.c_float(tie_eps))
    return keys, tie.astype(bool)


class Tables:
    """Node Importance tables of one layer (owned handle)."""

    def __init__(self, handle, n, K, L, list_cap):
        self.h = C.c_void_p(handle)
        self.n, self.K, self.L, self.list_cap = n, K, L, list_cap

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:       # (module globals are gone at interpreter exit)
            lib().so_tables_free(self.h)
            self.h = None

    @classmethod
    def build(cls, n, K, L, list_cap, keys, act, keep_scores=False, threads=1):
        keys = np.ascontiguousarray(keys, np.uint32)
        act = _f32(act)
        h = lib().so_tables_build(n, K, L, list_cap, _p(keys), _p(act), C.c_int64(act.shape[0]),
                                  int(keep_scores), threads)
        return cls(h, n, K, L, list_cap)

    @classmethod
    def from_lists(cls, n, K, L, list_cap, dir_, ids, global_rank):
        dir_ = np.ascontiguousarray(dir_, np.uint32)
        ids = np.ascontiguousarray(ids, np.int32)
        gr = np.ascontiguousarray(global_rank, np.int32)
        h = lib().so_tables_from_lists(n, K, L, list_cap, _p(dir_), _p(ids), _p(gr))
        return cls(h, n, K, L, list_cap)

    def refresh(self, keys, act):
        """Alg. 1 continued on more training inputs (their keys [N][L], the layer's activations
        [N][n]); needs tables built with keep_scores."""
        keys = np.ascontiguousarray(keys, np.uint32)
        act = _f32(act)
        if lib().so_tables_refresh(self.h, _p(keys), _p(act), C.c_int64(act.shape[0])) != 0:
            raise ValueError("these tables did not keep their NodeScore sums")

    def bucket(self, b, key):
        buf = np.empty(self.n, np.int32)
        ln = lib().so_tables_bucket(self.h, b, C.c_uint32(int(key)), _p(buf), self.n)
        return buf[:ln].copy()

    def bucket_count(self, b, key):
        return int(lib().so_tables_bucket_count(self.h, b, C.c_uint32(int(key))))

    def bucket_scores(self, b, key):
        out = np.zeros(self.n, np.float64)
        ok = lib().so_tables_bucket_scores(self.h, b, C.c_uint32(int(key)), _p(out))
        return out if ok else None

    def global_rank(self):
        r = np.empty(self.n, np.int32)
        s = np.empty(self.n, np.float64)
        lib().so_tables_global(self.h, _p(r), _p(s))
        return r, s

    def select(self, keys, keep, stride=None, hash_first=None):
        """hash_first: the layer's hash node ids when they are always computed and never
        selected (active = hash nodes, then the others in merge order); None = plain."""
        keys = np.ascontiguousarray(keys, np.uint32)
        keep = _f32(keep).reshape(-1)
        N = keys.shape[0]
        stride = self.n if stride is None else stride
        active = np.full((N, stride), -1, np.int32)
        cnt = np.zeros(N, np.int32)
        if hash_first is not None:
            hn = np.ascontiguousarray(hash_first, np.int32)
            assert hn.size == self.K * self.L
            rc = lib().so_select_hash_first(self.h, _p(keys), _p(keep), C.c_int64(1 if keep.size > 1 else 0),
                                            C.c_int64(N), _p(hn), _p(active), _p(cnt), C.c_int64(stride))
        else:
            rc = lib().so_select(self.h, _p(keys), _p(keep), C.c_int64(1 if keep.size > 1 else 0),
                                 C.c_int64(N), _p(active), _p(cnt), C.c_int64(stride))
        if rc != 0:
            raise ValueError("budget exceeds the active-list stride")
        return active, cnt

    def csr(self):
        """(dir uint32 [L][2^K+1], ids int32) -- the flat form the table blob stores."""
        nb = 1 << self.K
        dir_ = np.zeros((self.L, nb + 1), np.uint32)
        total = int(lib().so_tables_csr(self.h, None, None))
        ids = np.zeros(total, np.int32)
        lib().so_tables_csr(self.h, _p(dir_), _p(ids))
        # offsets run on across tables: dir[b][2^K] == dir[b+1][0]
        return dir_, ids.astype(np.int32)


def sparse_layer(layer, X, active, cnt, threads=1, want_pre=False):
    X = _f32(X)
    N = X.shape[0]
    active = np.ascontiguousarray(active, np.int32)
    cnt = np.ascontiguousarray(cnt, np.int32)
    out = np.empty((N, layer.d_out), np.float32)
    pre = np.empty((N, layer.d_out), np.float32) if want_pre else None
    W = np.ascontiguousarray(layer.W)
    lib().so_sparse_layer(_p(W), layer.w_dtype, _p(layer.bias), layer.d_in, layer.d_out, layer.act,
                          _p(X), C.c_int64(N), _p(active), _p(cnt), C.c_int64(active.shape[1]),
                          _p(pre), _p(out), threads)
    return (out, pre) if want_pre else out


def argmax(out, active=None, cnt=None):
    out = _f32(out)
    N, n = out.shape
    pred = np.empty(N, np.int32)
    if active is not None:
        active = np.ascontiguousarray(active, np.int32)
        cnt = np.ascontiguousarray(cnt, np.int32)
        lib().so_argmax(_p(out), n, C.c_int64(N), _p(active), _p(cnt), C.c_int64(active.shape[1]),
                        _p(pred))
    else:
        lib().so_argmax(_p(out), n, C.c_int64(N), None, None, C.c_int64(0), _p(pred))
    return pred


# --------------------------------------------------------------------------- #
# choice of k per query (Section 2: ACLO / LCAO; Section 3.2: Confidence LSH tables)
# --------------------------------------------------------------------------- #
def activation_variance(A) -> np.ndarray:
    """Per-node variance of the activations A [N][n] over the N inputs, in float64
    (Section 3.4: the statistic the FreeHash nodes are sampled by); 1/N normalisation."""
    A = np.asarray(A, dtype=np.float64)
    mean = A.sum(axis=0) / A.shape[0]
    return ((A - mean) ** 2).sum(axis=0) / A.shape[0]


def sample_hash_nodes(variance, K: int, L: int, u) -> np.ndarray:
    """K*L distinct node ids drawn with probability proportional to ``variance``
    (Section 3.4), one uniform u[j] in [0, 1) per draw, sequentially and without
    replacement: draw j inverts the running sums of the remaining variances at
    u[j] times their total, then removes the drawn node.  Negative or non-finite
    variances count as zero; zero-variance nodes are only drawn (lowest id first)
    once no variance is left.  The j-th id serves table j // K, bit j % K.
    """
    v = np.asarray(variance, dtype=np.float64).copy()
    n, H = v.shape[0], K * L
    if H > n:
        raise ValueError("K*L exceeds the number of nodes in the layer")
    v[~np.isfinite(v)] = 0.0
    v = np.maximum(v, 0.0)
    out = np.empty(H, dtype=np.int32)
    taken = np.zeros(n, dtype=bool)
    for j in range(H):
        c = np.cumsum(v)                       # running sums, left to right
        total = c[-1]
        if total > 0.0:
            i = int(np.searchsorted(c, u[j] * total, side="right"))   # first running sum above the target
            i = min(i, n - 1)
            while v[i] <= 0.0:                 # landed on an exhausted id through rounding
                i = (i + 1) % n
        else:                                  # no variance left: lowest unused id
            i = int(np.argmin(taken))
        out[j] = i
        taken[i] = True
        v[i] = 0.0
    return out


class ConfidenceTables:
    """Per bucket, the sums and counts of the training inputs' confidences c(k_g, x')."""

    def __init__(self, K, L, k_grid, keys, conf):
        self.K, self.L = K, L
        self.k_grid = _f32(k_grid).reshape(-1)
        self.G = self.k_grid.size
        keys = np.ascontiguousarray(keys, np.uint32)
        conf = _f32(conf)
        assert keys.shape[1] == L and conf.shape == (keys.shape[0], self.G)
        self.h = C.c_void_p(lib().so_conf_build(K, L, self.G, _p(keys), _p(conf), C.c_int64(keys.shape[0])))

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib().so_conf_free(self.h)
            self.h = None

    def estimate(self, keys):
        """c_hat [Q][G] (float64) and the number of bucket-mates [Q]."""
        keys = np.ascontiguousarray(keys, np.uint32)
        Q = keys.shape[0]
        chat = np.empty((Q, self.G), np.float64)
        mates = np.empty(Q, np.int64)
        lib().so_conf_estimate(self.h, _p(keys), C.c_int64(Q), _p(chat), _p(mates))
        return chat, mates

    def choose_aclo(self, keys, thr):
        """ACLO: per query the smallest grid k whose estimated confidence reaches thr."""
        keys = np.ascontiguousarray(keys, np.uint32)
        Q = keys.shape[0]
        thr = _f32(thr).reshape(-1)
        keep = np.empty(Q, np.float32)
        g = np.empty(Q, np.int32)
        lib().so_choose_aclo(self.h, _p(keys), C.c_int64(Q), _p(self.k_grid), _p(thr),
                             C.c_int64(1 if thr.size > 1 else 0), _p(keep), _p(g))
        return keep, g


def choose_lcao(k_grid, T, tau, t0, beta):
    """LCAO: per query the largest grid k with t0 + T[beta][k] <= tau; (keep, grid index, violated)."""
    k_grid = _f32(k_grid).reshape(-1)
    T = _f32(T)
    assert T.ndim == 2 and T.shape[1] == k_grid.size
    tau, t0 = _f32(tau).reshape(-1), _f32(t0).reshape(-1)
    beta = np.ascontiguousarray(beta, np.int32).reshape(-1)
    Q = tau.size
    keep = np.empty(Q, np.float32)
    g = np.empty(Q, np.int32)
    bad = np.empty(Q, np.uint8)
    rc = lib().so_choose_lcao(_p(k_grid), k_grid.size, _p(T), T.shape[0], _p(tau), _p(t0), _p(beta),
                              C.c_int64(Q), _p(keep), _p(g), _p(bad))
    if rc != 0:
        raise ValueError("beta out of range")
    return keep, g, bad.astype(bool)


# --------------------------------------------------------------------------- #
# whole network
# --------------------------------------------------------------------------- #
class OracleNet:
    """The network loop: per layer, hash -> keys -> select -> sparse layer."""

    def __init__(self, layers: Sequence, threads: Optional[int] = None,
                 first_layer_rows_are_inputs: bool = False, hash_nodes_always_active: bool = False):
        self.layers = list(layers)
        # Section 3.4 variant: hash nodes are always computed and never selected
        self.hash_first = hash_nodes_always_active
        self.threads = default_threads() if threads is None else threads
        self.tables: List[Optional[Tables]] = [None] * len(self.layers)
        self.rows_are_inputs0 = first_layer_rows_are_inputs

    # -- first layer may take ELL input ------------------------------------- #
    def _first(self, X):
        if isinstance(X, tuple):
            idx, val, nnz = X
            return dense_layer_ell(self.layers[0], idx, val, nnz, self.threads, self.rows_are_inputs0)
        return None

    def dense_forward(self, X, upto: Optional[int] = None):
        """Full network (all nodes).  Returns the list of layer outputs."""
        outs = []
        cur = X
        for l, layer in enumerate(self.layers[:upto]):
            if l == 0 and isinstance(X, tuple):
                cur = self._first(X)
            else:
                cur = dense_layer(layer, cur, self.threads)
            outs.append(cur)
        return outs

    def build_tables(self, X_build, keep_scores=False):
        """Alg. 1 for every layer with a Node Activator; Input_l is the full
        network's (all nodes computed) input to layer l on the training set."""
        cur = X_build
        for l, layer in enumerate(self.layers):
            if layer.K > 0 and layer.L > 0:
                if isinstance(cur, tuple):
                    raise ValueError("a Node Activator on a sparse-input first layer is not supported")
                Z = hash_project(layer, cur, self.threads)
                keys, _ = keys_from_z(Z, layer.K, layer.L)
                act = dense_layer(layer, cur, self.threads)
                self.tables[l] = Tables.build(layer.d_out, layer.K, layer.L, layer.list_cap, keys, act,
                                              keep_scores, self.threads)
                cur = act
            elif l == 0 and isinstance(cur, tuple):
                cur = self._first(cur)
            else:
                cur = dense_layer(layer, cur, self.threads)
        return self.tables

    def refresh_tables(self, X_new):
        """Online refresh: every Node Activator continues Alg. 1 on the inputs X_new (Input_l is
        again the full network's input to layer l).  Tables must have been built with keep_scores."""
        cur = X_new
        for l, layer in enumerate(self.layers):
            if layer.K > 0 and layer.L > 0:
                Z = hash_project(layer, cur, self.threads)
                keys, _ = keys_from_z(Z, layer.K, layer.L)
                act = dense_layer(layer, cur, self.threads)
                self.tables[l].refresh(keys, act)
                cur = act
            elif l == 0 and isinstance(cur, tuple):
                cur = self._first(cur)
            else:
                cur = dense_layer(layer, cur, self.threads)
        return self.tables

    def sparse_forward(self, X, keep, taps=True):
        """keep: scalar, [N] (one k per query for all layers) or [N][n_layers]."""
        N = X[0].shape[0] if isinstance(X, tuple) else np.asarray(X).shape[0]
        keep = np.asarray(keep, np.float32)
        if keep.ndim == 0:
            keep = np.full((N,), keep, np.float32)
        res = {"layers": []}
        cur = X
        last_active = last_cnt = None
        for l, layer in enumerate(self.layers):
            k_l = keep if keep.ndim == 1 else np.ascontiguousarray(keep[:, l])
            tap = {}
            if layer.K > 0 and layer.L > 0:
                Z = hash_project(layer, cur, self.threads)
                keys, tie = keys_from_z(Z, layer.K, layer.L)
                active, cnt = self.tables[l].select(
                    keys, k_l, hash_first=layer.hash_nodes if self.hash_first else None)
                out = sparse_layer(layer, cur, active, cnt, self.threads)
                if taps:
                    tap = {"z": Z, "codes": keys, "tie": tie, "active": active, "cnt": cnt}
                last_active, last_cnt = active, cnt
            else:
                if l == 0 and isinstance(cur, tuple):
                    out = self._first(cur)
                else:
                    out = dense_layer(layer, cur, self.threads)
                last_active = last_cnt = None
            if taps:
                tap["out"] = out
            res["layers"].append(tap)
            cur = out
        res["out"] = cur
        res["argmax"] = argmax(cur, last_active, last_cnt)
        return res

    # -- k chosen per query from the first activated layer's codes ----------- #
    def first_activated(self) -> int:
        return next(l for l, lay in enumerate(self.layers) if lay.K > 0 and lay.L > 0)

    def first_codes(self, X):
        """Keys of the first activated layer (its input is exact: every earlier layer is
        computed in full).  Returns (keys, tie)."""
        l0 = self.first_activated()
        cur = X
        for l in range(l0):
            cur = self._first(cur) if (l == 0 and isinstance(cur, tuple)) else dense_layer(self.layers[l], cur, self.threads)
        Z = hash_project(self.layers[l0], cur, self.threads)
        return keys_from_z(Z, self.layers[l0].K, self.layers[l0].L)

    def sparse_forward_aclo(self, X, conf_tables: "ConfidenceTables", thr, taps=True):
        """Fig. 2 with step 2 under ACLO: the Confidence LSH tables are queried once per
        request with the first activated layer's keys, the chosen k serves every layer."""
        keys, _ = self.first_codes(X)
        keep, g = conf_tables.choose_aclo(keys, thr)
        res = self.sparse_forward(X, keep, taps=taps)
        res["keep"], res["grid_idx"] = keep, g
        return res

    # -- table blob ---------------------------------------------------------- #
    def export_tables(self) -> bytes:
        sets = [(l, t) for l, t in enumerate(self.tables) if t is not None]
        parts = [struct.pack("<4I", BLOB_MAGIC, BLOB_VERSION, len(sets), 0)]
        for l, t in sets:
            dir_, ids = t.csr()
            gr, _ = t.global_rank()
            hn = np.ascontiguousarray(self.layers[l].hash_nodes, np.int32)
            parts.append(struct.pack("<8I", l, t.K, t.L, t.n, t.list_cap, ids.size, 0, 0))
            parts += [hn.astype("<i4").tobytes(), dir_.astype("<u4").tobytes(),
                      ids.astype("<i4").tobytes(), gr.astype("<i4").tobytes()]
        return b"".join(parts)

    def import_tables(self, blob: bytes):
        magic, ver, nsets, _ = struct.unpack_from("<4I", blob, 0)
        if magic != BLOB_MAGIC or ver != BLOB_VERSION:
            raise ValueError("not a table blob")
        off = 16
        for _ in range(nsets):
            l, K, L, n, cap, tot, _, _ = struct.unpack_from("<8I", blob, off)
            off += 32
            hn = np.frombuffer(blob, "<i4", K * L, off); off += 4 * K * L
            nd = L * ((1 << K) + 1)
            dir_ = np.frombuffer(blob, "<u4", nd, off); off += 4 * nd
            ids = np.frombuffer(blob, "<i4", tot, off); off += 4 * tot
            gr = np.frombuffer(blob, "<i4", n, off); off += 4 * n
            if not np.array_equal(hn, np.asarray(self.layers[l].hash_nodes, np.int32)):
                raise ValueError("blob hash nodes differ from the model's")
            self.tables[l] = Tables.from_lists(n, K, L, cap, dir_, ids, gr)
        return self.tables
