"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "slonn.h")


@pytest.fixture(scope="module")
def slonn():
    from paper_2204_08400_amd import build, slonn as s
    if not os.path.exists(s.LIB_PATH):
        build.build_library()
    s.load()
    return s


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slonn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(slonn):
    names = _declared()
    assert len(names) >= 12
    lib = slonn.load()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in slonn.h but not exported"
    assert set(names) == set(slonn.EXPORTS)


def test_version_string(slonn):
    assert "gfx950" in slonn.slonn_version()


class _FakeTensor:
    """stands in for a device tensor: validation never dereferences it"""
    def __init__(self, addr=0x1000):
        self._a = addr
    def is_contiguous(self):
        return True
    def data_ptr(self):
        return self._a


def _layer(**kw):
    d = dict(d_in=8, d_out=16, W=_FakeTensor(), bias=_FakeTensor(), act=1, K=0, L=0)
    d.update(kw)
    return d


@pytest.mark.parametrize("layers, code", [
    ([], -1),
    ([_layer(d_in=0)], -1),
    ([_layer(W=None)], -1),
    ([_layer(), _layer(d_in=17)], -1),                                   # d_in mismatch
    ([_layer(act=2), _layer(d_in=16)], -1),                              # softmax before the last layer
    ([_layer(K=17, L=1, hash_nodes=list(range(17)), list_cap=4)], -1),   # K too large
    ([_layer(K=1, L=65, hash_nodes=list(range(65)), list_cap=4, d_out=128)], -1),
    ([_layer(K=3, L=6, hash_nodes=list(range(18)), list_cap=4)], -1),    # K*L > d_out
    ([_layer(K=2, L=2, hash_nodes=[0, 1, 2, 2], list_cap=4)], -1),       # duplicate hash node
    ([_layer(K=2, L=2, hash_nodes=[0, 1, 2, 16], list_cap=4)], -1),      # out of range
    ([_layer(K=2, L=2, hash_nodes=[0, 1, 2, 3], list_cap=0)], -1),
    ([_layer(K=2, L=0)], -1),
    ([_layer(w_dtype=7)], -1),
    ([_layer(), _layer(d_in=16, w_layout=1)], -4),                       # input-major beyond layer 0
    ([_layer(w_layout=1, K=2, L=2, hash_nodes=[0, 1, 2, 3], list_cap=4)], -4),
])
def test_model_create_rejects(slonn, layers, code):
    with pytest.raises(slonn.SlonnError) as e:
        slonn.slonn_model_create(layers)
    assert e.value.code == code
    assert str(e.value)


def test_null_handles_are_rejected(slonn):
    lib = slonn.load()
    n = C.c_size_t(0)
    assert lib.slonn_workspace_bytes(None, 4, C.byref(n)) == slonn.EINVAL
    assert lib.slonn_tables_export(None, None, C.byref(n)) == slonn.EINVAL
    h = C.c_void_p()
    assert lib.slonn_tables_import(None, b"x", C.c_size_t(1), C.byref(h)) == slonn.EINVAL
    assert lib.slonn_build_tables(None, None, C.c_int64(1), None, C.byref(h)) == slonn.EINVAL
    assert lib.slonn_sparse_forward(None, None, None, 1, None, 0, 0, None, None, None, C.c_size_t(0), None) == slonn.EINVAL
    assert lib.slonn_dense_forward(None, None, 1, None, None, None, None, C.c_size_t(0), None) == slonn.EINVAL
    assert lib.slonn_select(None, None, 0, None, 1, None, 0, None, None, None, None, 0, None, C.c_size_t(0), None) == slonn.EINVAL
    assert lib.slonn_model_set_path(None, 0) == slonn.EINVAL
    assert lib.slonn_model_set_hash_nodes_always_active(None, 1) == slonn.EINVAL
    assert lib.slonn_model_destroy(None) == 0 and lib.slonn_tables_destroy(None) == 0
    assert lib.slonn_policy_destroy(None) == 0
    assert lib.slonn_policy_train_confidence(None, None, None, C.c_int64(1), None) == slonn.EINVAL
    assert lib.slonn_policy_set_latency_profile(None, None, 1) == slonn.EINVAL
    assert lib.slonn_policy_keep_aclo(None, None, 1, None, 0, None, None, None, None) == slonn.EINVAL
    assert lib.slonn_policy_keep_lcao(None, 1, None, 0, None, 0, None, 0, None, None, None, None) == slonn.EINVAL
    assert lib.slonn_sparse_forward_aclo(None, None, None, None, 1, None, 0, None, None, None, None,
                                         C.c_size_t(0), None) == slonn.EINVAL
    assert lib.slonn_sparse_forward_static(None, None, None, 1, None, 0, 0, None, None, None) == slonn.EINVAL
    assert lib.slonn_model_set_dense_arithmetic(None, 1) == slonn.EINVAL
    assert lib.slonn_model_set_tables_refreshable(None, 1) == slonn.EINVAL
    assert lib.slonn_model_set_batches_in_flight(None, 2) == slonn.EINVAL
    assert lib.slonn_probe_mfma_rate(None, C.c_size_t(0), None, None) == slonn.EINVAL
    assert lib.slonn_probe_l_two_read_rate(None, C.c_size_t(0), None, None, None) == slonn.EINVAL
    assert lib.slonn_tables_refresh(None, None, None, C.c_int64(1), None) == slonn.EINVAL
    assert lib.slonn_sample_hash_nodes_device(None, 8, 1, 1, None, None, None) == slonn.EINVAL
    assert slonn.load().slonn_last_error()


def test_device_sampler_rejects_before_touching_the_device(slonn):
    """argument checks of slonn_sample_hash_nodes_device run on the host (pointers are never read)"""
    lib = slonn.load()
    p = C.c_void_p(0x1000)
    assert lib.slonn_sample_hash_nodes_device(p, 8, 3, 3, p, p, None) == slonn.EINVAL           # K*L > n
    assert lib.slonn_sample_hash_nodes_device(p, 0, 1, 1, p, p, None) == slonn.EINVAL
    assert lib.slonn_sample_hash_nodes_device(p, (1 << 20) + 1, 1, 1, p, p, None) == -4          # beyond 2^20 nodes


def test_binding_fails_loudly_without_library(slonn, monkeypatch, tmp_path):
    import importlib
    monkeypatch.setattr(slonn, "LIB_PATH", str(tmp_path / "nope.so"))
    monkeypatch.setattr(slonn, "_lib", None)
    with pytest.raises(FileNotFoundError):
        slonn.load()


@pytest.mark.parametrize("K,L,grid", [
    (0, 4, [0.5]), (17, 4, [0.5]), (4, 0, [0.5]), (4, 65, [0.5]),          # K, L out of range
    (4, 4, []), (4, 4, [0.1] * 17),                                         # grid size
    (4, 4, [0.0, 0.5]), (4, 4, [0.5, 1.5]), (4, 4, [0.5, 0.5]), (4, 4, [0.5, 0.25]),   # values, order
    (4, 4, [float("nan")]),
])
def test_policy_create_rejects(slonn, K, L, grid):
    """argument checks that come before any device memory is touched"""
    lib = slonn.load()
    arr = (C.c_float * max(len(grid), 1))(*grid)
    h = C.c_void_p()
    assert lib.slonn_policy_create(K, L, arr, len(grid), C.byref(h)) == slonn.EINVAL
    assert not h.value
    assert lib.slonn_policy_create(4, 4, None, 1, C.byref(h)) == slonn.EINVAL
    assert lib.slonn_policy_create(4, 4, arr, 1, None) == slonn.EINVAL


def test_sample_hash_nodes_matches_oracle(slonn):
    """The library's host-side sampler (Section 3.4) against the oracle's, id for id, on
    variances with zeros, negatives, NaN and infinities, including samples that exhaust the
    positive-variance nodes."""
    from oracle import slonn_oracle
    rng = np.random.default_rng(5)
    for n, K, L, zero_frac in [(7, 1, 7, 0.0), (64, 4, 6, 0.3), (500, 6, 10, 0.9), (300, 8, 16, 0.5),
                               (1000, 12, 50, 0.2), (33, 3, 11, 1.0)]:
        v = rng.random(n) * rng.choice([1e-6, 1.0, 1e6], size=n)
        v[rng.random(n) < zero_frac] = 0.0
        if n >= 64:
            v[3], v[10], v[20] = -1.0, np.nan, np.inf
        u = rng.random(K * L)
        got = slonn.slonn_sample_hash_nodes(v, K, L, u)
        want = slonn_oracle.sample_hash_nodes(v, K, L, u)
        assert got.tolist() == want.tolist(), (n, K, L)


def test_sample_hash_nodes_rejects(slonn):
    v = np.ones(8)
    with pytest.raises(slonn.SlonnError) as e:
        slonn.slonn_sample_hash_nodes(v, 3, 3, np.zeros(9))      # K*L > n
    assert e.value.code == -1
    lib = slonn.load()
    assert lib.slonn_sample_hash_nodes(None, 8, 1, 1, None, None) == -1
    assert lib.slonn_activation_variance(None, C.c_int64(4), 4, C.c_int64(4), None, None) == -1
    assert lib.slonn_model_set_hash_margin(None, C.c_double(2.0)) == -1
