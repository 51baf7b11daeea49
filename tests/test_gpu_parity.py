"""Parity of the HIP path (through the C ABI) with the CPU oracle, on the same seeded
inputs.  Integer results (codes, active lists, argmax) must match bit for bit once
queries whose hash projections are within 1e-6 of zero are set aside; fp32 outputs
must agree to a relative 1e-4."""
import json
import os

import numpy as np
import pytest

from paper_2204_08400_amd import workloads as wl

from helpers import (assert_close_rows, compare_sparse, make_case, make_queries, to_numpy_result)

pytestmark = pytest.mark.gpu

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")


@pytest.fixture(scope="module")
def rt():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X)")
    from paper_2204_08400_amd import runtime, slonn
    slonn.load()          # fails loudly when the HIP library is missing
    return runtime


def _say(msg):
    print(msg, flush=True)


def _gpu_net(rt, layers, net, rows_are_inputs=False, path="layers"):
    g = rt.Network(layers, first_layer_rows_are_inputs=rows_are_inputs)
    g.import_tables(net.export_tables())
    g.set_path(path)
    return g


def _fused_ok(case):
    """row lengths must be multiples of 16 bytes for the whole-network kernel"""
    mult = 8 if case.get("w_dtype", wl.W_F32) == wl.W_BF16 else 4
    dims = case["dims"]
    small = all(dims[i] * dims[i + 1] * (16 // mult) <= (8 << 20) for i in range(len(dims) - 1))
    return small and all(d % mult == 0 for d in dims[:-1])


def _keep_tensor(keep):
    import torch
    return torch.from_numpy(np.ascontiguousarray(keep, np.float32)).cuda()


def test_worked_example(rt, oracle):
    with open(GOLD) as f:
        gold = json.load(f)
    lay = wl.LayerData(2, 6, wl.ACT_RELU, wl.W_F32, np.asarray(gold["W"], np.float32),
                       np.asarray(gold["bias"], np.float32), 2, 2, 6, np.asarray(gold["hash_nodes"], np.int32))
    net = oracle.OracleNet([lay], threads=1)
    net.build_tables(np.asarray(gold["build"], np.float32))
    g = _gpu_net(rt, [lay], net)
    for q in gold["queries"]:
        x = np.asarray([q["x"]], np.float32)
        for m in range(1, 7):
            _say(f"worked example x={q['x']} m={m}")
            g.set_path("layers")     # d = 2: rows are not 16-byte multiples, per-layer path only
            r = to_numpy_result(g.sparse_forward(x, np.float32(m / 6), taps=True))
            assert r["taps"]["codes"][0][0].tolist() == q["keys"]
            assert r["taps"]["cnt"][0][0] == m
            want = q["order"][:m] if m < 6 else list(range(6))
            assert r["taps"]["active"][0][0, :m].tolist() == want
            if str(m) in q["outputs"]:
                assert r["out"][0].tolist() == q["outputs"][str(m)]


CASES = [
    # dims, K, L, kind, w_dtype, last_act, cap, B
    dict(dims=(100, 300, 260, 37), K=4, L=6, kind="u01", B=70),
    dict(dims=(130, 520, 19), K=5, L=3, kind="clip3", B=33, cap=200),
    dict(dims=(96, 1000, 640, 12), K=6, L=10, kind="u01", B=129, last_act=wl.ACT_SOFTMAX),
    dict(dims=(64, 384, 384, 10), K=4, L=8, kind="normal", B=65, w_dtype=wl.W_BF16),
    dict(dims=(75, 333, 21), K=3, L=64, kind="u01", B=5),                       # odd d: scalar path
    dict(dims=(256, 4096, 520, 10), K=6, L=12, kind="clip3", B=37, N_build=128),  # > 3 MiB matrices: row-block gather
    # hash-row counts that are no multiple of four / that leave few inputs per thread group in the
    # whole-network kernel's projection over non-zero inputs
    dict(dims=(128, 1200, 400, 16), K=3, L=7, kind="u01", B=21),
    dict(dims=(64, 1536, 1100, 10), K=10, L=60, kind="normal", B=9, N_build=128),
]


@pytest.mark.parametrize("path", ["layers", "fused"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c["dims"])))
def test_sparse_forward_matches_oracle(rt, oracle, case, path):
    import torch
    dims, B = case["dims"], case["B"]
    if path == "fused" and not _fused_ok(case):
        pytest.skip("model does not qualify for the whole-network kernel")
    layers, net, Xb = make_case(oracle, dims, case["K"], case["L"], seed=17, cap=case.get("cap"),
                                w_dtype=case.get("w_dtype", wl.W_F32), last_act=case.get("last_act", wl.ACT_NONE),
                                kind=case["kind"], N_build=case.get("N_build", 256))
    g = _gpu_net(rt, layers, net, path=path)
    X = make_queries(dims, B, seed=99, kind=case["kind"])
    for keep in (0.05, 0.3, 0.77, 1.0):
        _say(f"case {dims} path={path} keep={keep}")
        ref = net.sparse_forward(X, keep)
        got = to_numpy_result(g.sparse_forward(X, keep, taps=True))
        rep = compare_sparse(got, ref, layers, f"{dims} keep {keep}")
        _say(f"  report {rep}")
    # mixed per-query keep fractions (one k per query for all layers)
    keep = wl.keep_uniform(B, 0.02, 0.6, 5)
    _say(f"case {dims} per-query keep")
    ref = net.sparse_forward(X, keep)
    got = to_numpy_result(g.sparse_forward(X, _keep_tensor(keep), taps=True))
    compare_sparse(got, ref, layers, f"{dims} per-query keep")
    # per-layer keep fractions
    keep2 = np.stack([wl.keep_uniform(B, 0.05, 0.9, 6 + l) for l in range(len(layers))], axis=1)
    _say(f"case {dims} per-layer keep")
    ref = net.sparse_forward(X, keep2)
    got = to_numpy_result(g.sparse_forward(X, _keep_tensor(keep2), taps=True))
    compare_sparse(got, ref, layers, f"{dims} per-layer keep")


def test_dense_forward_matches_oracle(rt, oracle):
    for dims, w_dtype, B, kind in [((100, 300, 260, 37), wl.W_F32, 70, "u01"),
                                   ((257, 129, 65, 33), wl.W_F32, 131, "clip3"),
                                   ((75, 333, 21), wl.W_F32, 9, "u01"),
                                   ((64, 384, 384, 10), wl.W_BF16, 300, "normal")]:
        _say(f"dense {dims}")
        layers = wl.make_mlp(dims, seed=3, w_dtype=w_dtype, last_act=wl.ACT_SOFTMAX)
        net = oracle.OracleNet(layers)
        g = rt.Network(layers)
        X = make_queries(dims, B, seed=4, kind=kind)
        ref = net.dense_forward(X)
        got = g.dense_forward(X, layer_outs=True)
        for l in range(len(layers)):
            assert_close_rows(got["layers"][l].cpu().numpy(), ref[l], None, f"dense {dims} layer {l}")
        assert np.array_equal(got["argmax"].cpu().numpy(), oracle.argmax(ref[-1]))


@pytest.mark.parametrize("w_dtype", [wl.W_F32, wl.W_BF16], ids=["f32", "bf16"])
def test_dense_forward_in_f16_parts_matches_oracle(rt, oracle, w_dtype):
    """The full network in the sparse path's large-batch arithmetic (scaled operands as two fp16 parts
    on the fp16 matrix cores, slonn_model_set_dense_arithmetic) against the oracle's dense network, and
    that the unmasked tiles really ran for the large layers."""
    from paper_2204_08400_amd import slonn
    dims = (512, 2048, 2048, 16)
    layers, net, _ = make_case(oracle, dims, 4, 6, seed=41, kind="clip3", N_build=64, w_dtype=w_dtype)
    g = _gpu_net(rt, layers, net)
    X = make_queries(dims, 300, seed=42, kind="clip3")       # a ragged batch: 4 tiles of 64 and 44 queries
    ref = net.dense_forward(X)
    slonn.slonn_model_set_dense_arithmetic(g.model, 1)
    slonn.slonn_profile_begin(16)
    got = g.dense_forward(X, layer_outs=True)
    prof = slonn.slonn_profile_end()
    assert prof["dense"][1] == len(layers), prof
    for l in range(len(layers)):
        assert_close_rows(got["layers"][l].cpu().numpy(), ref[l], None, f"dense in f16 parts, layer {l}", depth=l + 1)
    assert np.array_equal(got["argmax"].cpu().numpy(), oracle.argmax(ref[-1]))
    # input rows that are not 16-byte aligned: the tile kernel cannot fetch them in 16-byte pieces, a
    # two-part copy is made first (split_rows_kernel) -- the same arithmetic, so the same bits
    import torch
    buf = torch.empty(X.size + 1, dtype=torch.float32, device="cuda:0")
    xm = buf[1:].view(X.shape[0], X.shape[1])
    xm.copy_(torch.from_numpy(np.ascontiguousarray(X, np.float32)))
    assert xm.data_ptr() % 16 == 4
    off = g.dense_forward(xm, layer_outs=True)
    for l in range(len(layers)):
        assert torch.equal(off["layers"][l], got["layers"][l]), f"layer {l}: misaligned input rows"
    # against the default arithmetic: the same results to fp32 rounding, not the same bits
    slonn.slonn_model_set_dense_arithmetic(g.model, 0)
    plain = g.dense_forward(X, layer_outs=True)
    assert_close_rows(got["layers"][1].cpu().numpy(), plain["layers"][1].cpu().numpy(), None, "f16 parts vs fp32 cores", depth=2)
    assert not np.array_equal(got["layers"][1].cpu().numpy(), plain["layers"][1].cpu().numpy())
    with pytest.raises(slonn.SlonnError):
        slonn.slonn_model_set_dense_arithmetic(g.model, 7)


@pytest.mark.parametrize("w_dtype", [wl.W_F32, wl.W_BF16], ids=["f32", "bf16"])
def test_tile_arithmetic_is_fp32_class_over_a_wide_dynamic_range(rt, oracle, w_dtype):
    """The tile kernel scales every row by a power of two and carries operands as two fp16 parts.
    Rows of the weights spread over 2^-25 .. 2^25 and the queries over 2^-30 .. 2^30, so that the
    second layer's inputs span 2^50 within one row; a row of zeros; a row with a single non-zero element.  Against
    the oracle's fp64 network the error must stay within the parity bound, and on the first layer
    within that of a plain fp32 evaluation of the same dot products (one fp32 multiply and one fp32
    add per element, in order)."""
    from paper_2204_08400_amd import slonn
    dims = (1024, 2048, 2048, 24)
    layers = wl.make_mlp(dims, seed=51, w_dtype=w_dtype)
    rng = np.random.default_rng(52)                     # (exponents only: no arithmetic of the method)
    for l, lay in enumerate(layers[:2]):
        k = rng.integers(-25, 26, size=lay.d_out).astype(np.float64)
        w = wl.bf16_bits_to_f32(lay.W) if w_dtype == wl.W_BF16 else lay.W
        w = (w.astype(np.float64) * np.exp2(k)[:, None]).astype(np.float32)      # exact: powers of two
        lay.W = wl.f32_to_bf16_bits(w) if w_dtype == wl.W_BF16 else w
        lay.bias = (lay.bias.astype(np.float64) * np.exp2(k)).astype(np.float32)
        if w_dtype == wl.W_F32:       # (fp32 layers get their tile weights when they are activated layers)
            lay.K, lay.L, lay.list_cap = 4, 6, lay.d_out
            lay.hash_nodes = np.arange(24, dtype=np.int32)
    X = make_queries(dims, 300, seed=53, kind="clip3")
    X = (X.astype(np.float64) * np.exp2(rng.integers(-30, 31, size=300).astype(np.float64))[:, None]).astype(np.float32)
    X[7] = 0.0
    X[11] = 0.0
    X[11, 333] = -1.5e-12
    net = oracle.OracleNet(layers)
    g = rt.Network(layers)
    ref = net.dense_forward(X)
    slonn.slonn_model_set_dense_arithmetic(g.model, 1)
    slonn.slonn_profile_begin(16)
    got = g.dense_forward(X, layer_outs=True)
    prof = slonn.slonn_profile_end()
    assert prof["dense"][1] == len(layers), prof         # every layer through the tiles
    worst = [assert_close_rows(got["layers"][l].cpu().numpy(), ref[l], None, f"wide range, layer {l}", depth=l + 1)
             for l in range(len(layers))]
    assert np.array_equal(got["argmax"].cpu().numpy(), oracle.argmax(ref[-1]))
    lay = layers[0]
    w32 = wl.bf16_bits_to_f32(lay.W) if w_dtype == wl.W_BF16 else lay.W
    plain = np.zeros((X.shape[0], lay.d_out), np.float32)
    wt = np.ascontiguousarray(w32.T)
    for k in range(lay.d_in):                                            # fp32 products, fp32 sums, in order
        plain += X[:, k:k + 1] * wt[k][None, :]
    plain = np.maximum(plain + lay.bias, np.float32(0.0))
    scale = np.maximum(np.abs(ref[0]).max(axis=1, keepdims=True), 1e-300)
    err_plain = float((np.abs(plain.astype(np.float64) - ref[0]) / scale).max())
    _say(f"  wide range {('f32', 'bf16')[w_dtype == wl.W_BF16]}: tiles {worst} of the row maximum, plain fp32 {err_plain:.3e}")
    assert worst[0] <= err_plain, (worst[0], err_plain)


def test_keep_one_equals_dense_path(rt, oracle):
    dims = (100, 300, 260, 37)
    layers, net, _ = make_case(oracle, dims, 4, 6, seed=17)
    g = _gpu_net(rt, layers, net)
    X = make_queries(dims, 70, seed=5)
    s = g.sparse_forward(X, 1.0)
    d = g.dense_forward(X)
    assert_close_rows(s["out"].cpu().numpy(), d["out"].cpu().numpy(), None, "keep 1.0 vs dense kernel")
    assert np.array_equal(s["argmax"].cpu().numpy(), d["argmax"].cpu().numpy())


def test_select_teacher_forced(rt, oracle):
    """GPU select fed the oracle's own layer inputs: codes and lists bit-exact per layer."""
    dims = (96, 1000, 640, 12)
    layers, net, _ = make_case(oracle, dims, 6, 10, seed=23)
    g = _gpu_net(rt, layers, net)
    X = make_queries(dims, 77, seed=6)
    keep = wl.keep_uniform(77, 0.01, 0.5, 8)
    ref = net.sparse_forward(X, keep)
    cur = X
    for l in (0, 1):
        _say(f"teacher-forced select layer {l}")
        r = g.select(l, cur, _keep_tensor(keep))
        tap = ref["layers"][l]
        ok = ~tap["tie"]
        assert np.array_equal(r["codes"].cpu().numpy().view(np.uint32)[ok], tap["codes"][ok])
        act = r["active"].cpu().numpy()
        assert np.array_equal(r["cnt"].cpu().numpy()[ok], tap["cnt"][ok])
        for q in np.nonzero(ok)[0]:
            assert np.array_equal(act[q, :tap["cnt"][q]], tap["active"][q, :tap["cnt"][q]])
        cur = tap["out"]


@pytest.mark.parametrize("path", ["auto", "layers"])
@pytest.mark.parametrize("n_out", [3000, 50000], ids=["block-select", "wide-select"])
def test_ell_input_and_activated_softmax_output(rt, oracle, n_out, path):
    """Wide sparse-input model with the Node Activator on the output layer only.  The
    50 000-node output is too wide for a 4-byte-per-node map in LDS and takes the select
    kernel that keeps one bit per node."""
    dims = (5000, 128, n_out)
    from paper_2204_08400_amd import slonn
    _say(slonn.slonn_version())
    layers, net, _ = make_case(oracle, dims, 8, 12, seed=31, hashed=[1], cap=400, last_act=wl.ACT_SOFTMAX,
                               ell_nnz=40, N_build=300)
    # the GPU stores the first layer input-major
    import copy
    glayers = [copy.copy(l) for l in layers]
    glayers[0].W = np.ascontiguousarray(layers[0].W.T)
    g = rt.Network(glayers, first_layer_rows_are_inputs=True)
    g.import_tables(net.export_tables())
    g.set_path(path)
    X = make_queries(dims, 50, seed=7, ell_nnz=40)
    for keep in (0.005, 0.05, 0.2, wl.keep_uniform(50, 0.0001, 1.0, 3)):
        keep = _keep_tensor(keep) if np.ndim(keep) else keep
        _say(f"ELL case path={path} keep={'mixed' if not np.isscalar(keep) else keep}")
        ref = net.sparse_forward(X, keep.cpu().numpy() if not np.isscalar(keep) else keep)
        res = g.sparse_forward(X, keep, taps=True, compact=True)
        got = to_numpy_result(res)
        compare_sparse(got, ref, layers, f"ELL {path}")
        ok = ~ref["layers"][1]["tie"]
        for q in np.nonzero(ok)[0]:
            c = ref["layers"][1]["cnt"][q]
            assert got["cnt"][q] == c
            assert np.array_equal(got["idx"][q, :c], ref["layers"][1]["active"][q, :c])
            np.testing.assert_allclose(got["val"][q, :c], ref["out"][q, got["idx"][q, :c]], rtol=1e-4, atol=1e-9)
            assert abs(got["val"][q, :c].sum() - 1.0) < 1e-4


def test_batches_in_flight_hint_changes_workgroups_not_results(rt, oracle):
    """slonn_model_set_batches_in_flight sizes the workgroups of the whole-network kernels (1024
    threads per query, or 512 / 256 so that several queries share a compute unit).  Every size must
    match the oracle, for the dense-input kernel and for the wide sparse-input one."""
    import copy
    from paper_2204_08400_amd import slonn
    dims = (96, 1000, 640, 12)
    layers, net, _ = make_case(oracle, dims, 6, 10, seed=23, last_act=wl.ACT_SOFTMAX)
    g = _gpu_net(rt, layers, net, path="fused")
    X = make_queries(dims, 40, seed=6)
    keep = wl.keep_uniform(40, 0.01, 0.9, 8)
    ref = net.sparse_forward(X, keep)
    for n in (1, 8, 64):      # 40 queries a batch: 1024, 512 and 256 threads per query
        _say(f"dense-input whole-network kernel, {n} batches in flight")
        g.set_batches_in_flight(n)
        compare_sparse(to_numpy_result(g.sparse_forward(X, _keep_tensor(keep), taps=True)), ref, layers, f"in flight {n}")
    with pytest.raises(slonn.SlonnError):
        g.set_batches_in_flight(0)
    dims = (5000, 128, 50000)
    layers, net, _ = make_case(oracle, dims, 8, 12, seed=31, hashed=[1], cap=400, last_act=wl.ACT_SOFTMAX,
                               ell_nnz=40, N_build=300)
    glayers = [copy.copy(l) for l in layers]
    glayers[0].W = np.ascontiguousarray(layers[0].W.T)
    g = rt.Network(glayers, first_layer_rows_are_inputs=True)
    g.import_tables(net.export_tables())
    g.set_path("fused")
    X = make_queries(dims, 50, seed=7, ell_nnz=40)
    keep = wl.keep_uniform(50, 0.0001, 0.3, 3)
    ref = net.sparse_forward(X, keep)
    for n in (1, 64):
        _say(f"wide sparse-input whole-network kernel, {n} batches in flight")
        g.set_batches_in_flight(n)
        got = to_numpy_result(g.sparse_forward(X, _keep_tensor(keep), taps=True, compact=True))
        compare_sparse(got, ref, layers, f"ELL in flight {n}")
        ok = ~ref["layers"][1]["tie"]
        for q in np.nonzero(ok)[0]:
            c = ref["layers"][1]["cnt"][q]
            assert got["cnt"][q] == c
            assert np.array_equal(got["idx"][q, :c], ref["layers"][1]["active"][q, :c])


@pytest.mark.parametrize("path", ["layers", "fused"])
def test_edge_cases(rt, oracle, path):
    import torch
    dims = (40, 64, 64, 8)
    layers, net, _ = make_case(oracle, dims, 3, 2, seed=41, cap=5)   # short lists: fallback dominates
    g = _gpu_net(rt, layers, net, path=path)
    # single query, smallest budget, tiny keep
    X = make_queries(dims, 1, seed=8)
    for keep in (1e-6, 1.0 / 64, 0.999):
        ref = net.sparse_forward(X, keep)
        got = to_numpy_result(g.sparse_forward(X, keep, taps=True))
        compare_sparse(got, ref, layers, f"edge keep {keep}")
    # keep fractions outside (0, 1] are clamped the same way on both sides
    Xo = make_queries(dims, 6, seed=9)
    odd_keep = np.asarray([0.0, -1.0, np.nan, 1.5, np.inf, 0.3], np.float32)
    ref = net.sparse_forward(Xo, odd_keep)
    got = to_numpy_result(g.sparse_forward(Xo, _keep_tensor(odd_keep), taps=True))
    compare_sparse(got, ref, layers, "clamped keep")
    assert got["taps"]["cnt"][0].tolist() == [1, 1, 1, 64, 64, 19]
    # an all-zero query (every projection equals the bias)
    Xz = np.zeros((3, 40), np.float32)
    ref = net.sparse_forward(Xz, 0.25)
    got = to_numpy_result(g.sparse_forward(Xz, 0.25, taps=True))
    compare_sparse(got, ref, layers, "zero input")
    # argument errors come back as exceptions, not faults
    from paper_2204_08400_amd import slonn
    with pytest.raises(slonn.SlonnError):
        g.select(2, X, 0.5)              # output layer has no Node Activator
    odd = rt.Network(wl.make_mlp((75, 33, 5), seed=1))
    with pytest.raises(slonn.SlonnError):
        odd.set_path("fused")            # 75 floats per row is not a multiple of 16 bytes
    with pytest.raises(slonn.SlonnError):
        slonn.slonn_sparse_forward(g.model, g.tables, g.to_input(X), 0, torch.ones(1, device="cuda"), 0, 0,
                                   slonn.make_output(), None, g.workspace(1))


@pytest.mark.parametrize("w_dtype", [wl.W_F32, wl.W_BF16], ids=["f32", "bf16"])
def test_few_queries_take_a_workgroup_per_row(rt, oracle, w_dtype):
    """Up to six queries every selected row of 4 KB or more is fetched by a workgroup of its own
    (no staging in LDS, 4 partial sums per row added in a fixed order); batches 1, 3 and 6, an
    activated layer with rows of 2048 elements and the 40-node output layer with the identity
    list, against the oracle; batch 7 takes the other kernels and must agree as well."""
    from paper_2204_08400_amd import slonn
    dims = (2048, 2304, 40)
    layers, net, _ = make_case(oracle, dims, 5, 6, seed=91, hashed=[0], N_build=96, w_dtype=w_dtype,
                               kind="clip3")
    g = _gpu_net(rt, layers, net)
    Xq = make_queries(dims, 7, seed=92, kind="clip3")
    keep = np.asarray([0.3, 0.0005, 1.0, 0.11, 0.5, 0.25, 0.2], np.float32)
    for B in (1, 3, 6, 7):
        ref = net.sparse_forward(Xq[:B], keep[:B])
        slonn.slonn_profile_begin(16)
        got = to_numpy_result(g.sparse_forward(Xq[:B], _keep_tensor(keep[:B]), taps=True))
        prof = slonn.slonn_profile_end()
        assert prof["gather"][1] == 2 and prof["tiles"][1] == 0 and prof["dense"][1] == 0, prof
        _say(f"  batch {B}: {compare_sparse(got, ref, layers, f'row kernel batch {B}')}")


def test_few_queries_on_layers_with_many_tables(rt, oracle):
    """Up to four queries on layers with 48 tables or more take rounds of 12 288 slots in the select
    kernel (a thread takes twelve consecutive slots); budgets from one node to the whole layer and
    lists that run out (cap 50); five queries take the usual rounds and must agree as well."""
    dims = (64, 1536, 1100, 10)
    for cap in (None, 50):
        layers, net, _ = make_case(oracle, dims, 6, 64, seed=61, cap=cap, N_build=192, kind="normal")
        g = _gpu_net(rt, layers, net, path="layers")
        Xq = make_queries(dims, 5, seed=62, kind="normal")
        keep = np.asarray([[0.3, 0.2, 1], [0.0005, 0.6, 1], [1.0, 0.1, 1], [0.9, 0.05, 1], [0.5, 0.25, 1]], np.float32)
        for B in (1, 3, 4, 5):
            ref = net.sparse_forward(Xq[:B], keep[:B])
            got = to_numpy_result(g.sparse_forward(Xq[:B], _keep_tensor(keep[:B]), taps=True))
            _say(f"  cap {cap} batch {B}: {compare_sparse(got, ref, layers, f'many tables, cap {cap}, batch {B}')}")


@pytest.mark.gpu
def test_hash_node_choice_matches_oracle(rt, oracle):
    """Section 3.4: per-node activation variance on the device against the oracle's float64
    variance (same activation matrix; ragged sizes, a strided view, a single row), then the
    variance-proportional draws, id for id."""
    import torch
    from paper_2204_08400_amd import slonn
    rng = np.random.default_rng(21)
    for N, n, pad in [(1003, 130, 0), (257, 64, 5), (1, 70, 0), (4099, 1000, 24), (3, 1, 0)]:
        _say(f"activation variance N={N} n={n} pad={pad}")
        A = np.maximum(rng.normal(size=(N, n + pad)) * rng.random(n + pad) * 3 + 0.2, 0).astype(np.float32)
        A[:, ::7] = 0.0                                   # dead nodes: variance exactly 0
        dev = torch.from_numpy(A).cuda()
        view = dev[:, :n]                                 # row stride n + pad
        var = torch.empty(n, dtype=torch.float64, device="cuda")
        slonn.slonn_activation_variance(view, var)
        got = var.cpu().numpy()
        want = oracle.activation_variance(A[:, :n])
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=0)
        assert (got[::7] == 0).all()
        if n >= 64:
            K, L = 4, 8
            u = wl.hash_node_draws(K, L, seed=N)
            assert rt.hash_nodes_by_variance(view, K, L, u).tolist() == oracle.sample_hash_nodes(want, K, L, u).tolist()


def test_device_hash_node_draws_match_oracle(rt, oracle):
    """The variance-proportional draws on the device (one wavefront, running sums in node order)
    against the oracle's, id for id, on the same variances: ragged layer widths, more draws than
    nodes with variance (the rest come lowest id first), negative / infinite / NaN entries (count
    as zero), a draw target in the last chunk, and the library's host sampler beside both."""
    import torch
    from paper_2204_08400_amd import slonn
    rng = np.random.default_rng(5)
    cases = []
    for n, K, L in [(70, 4, 8), (64, 2, 3), (1000, 6, 10), (129, 8, 16), (8192, 12, 64), (5, 1, 5), (100003, 4, 6)]:
        v = rng.random(n) ** 3
        v[::5] = 0.0
        cases.append((v, K, L, f"n={n}"))
    v = np.zeros(90); v[[3, 17, 80]] = [2.0, 1.0, 0.5]
    cases.append((v, 3, 4, "three nodes with variance, twelve draws"))
    v = rng.random(200); v[5] = np.nan; v[6] = np.inf; v[7] = -np.inf; v[8] = -3.0
    cases.append((v, 5, 6, "non-finite and negative entries"))
    v = np.zeros(300); v[299] = 1.0
    cases.append((v, 2, 2, "all variance on the last node"))
    cases.append((np.zeros(77), 3, 5, "no variance at all"))
    for v, K, L, what in cases:
        _say(f"device hash-node draws: {what} K={K} L={L}")
        u = wl.hash_node_draws(K, L, seed=len(v))
        want = oracle.sample_hash_nodes(v, K, L, u)
        vd = torch.from_numpy(v).cuda()
        ud = torch.from_numpy(u).cuda()
        out = torch.full((K * L,), -1, dtype=torch.int32, device="cuda")
        slonn.slonn_sample_hash_nodes_device(vd, K, L, ud, out)
        got = out.cpu().numpy()
        assert got.tolist() == want.tolist(), what
        assert slonn.slonn_sample_hash_nodes(v, K, L, u).tolist() == want.tolist(), what
        assert len(set(got.tolist())) == K * L


BUILD_CASES = [
    dict(dims=(100, 300, 260, 37), K=4, L=6, cap=200, N=500, hashed=None, last_act=wl.ACT_NONE),
    dict(dims=(48, 10000, 16), K=5, L=4, cap=400, N=300, hashed=[0], last_act=wl.ACT_NONE),       # wide ReLU layer
    dict(dims=(48, 128, 12000), K=6, L=5, cap=300, N=300, hashed=[1], last_act=wl.ACT_SOFTMAX),   # wide softmax layer
    # the width of the extreme-classification output layers (Table 1): 100 000 softmax nodes, few inputs
    dict(dims=(64, 128, 100000), K=5, L=3, cap=600, N=96, hashed=[1], last_act=wl.ACT_SOFTMAX),
    # lists longer than the LDS sort holds on a layer wider than it: whole buckets are radix-sorted
    dict(dims=(48, 128, 12000), K=4, L=3, cap=10000, N=200, hashed=[1], last_act=wl.ACT_SOFTMAX),
    # masses of exactly equal sums (the layer's rows repeat with period 2): no threshold isolates the
    # head of a list, every bucket falls back to the full sort; equal sums rank by ascending id
    dict(dims=(32, 20000, 8), K=3, L=2, cap=500, N=120, hashed=[0], last_act=wl.ACT_NONE, repeat_rows=2),
]


@pytest.mark.parametrize("case", BUILD_CASES, ids=lambda c: "x".join(map(str, c["dims"])))
def test_build_tables_matches_oracle(rt, oracle, case):
    """Alg. 1 on the device against the oracle's: lists equal up to swaps of nodes whose sums
    agree to 1e-5 relative (the device sums fp32 activations of its own dense pass); tables
    built on either side give the same selection when both sides load the same blob."""
    dims = case["dims"]
    layers, net, Xb = make_case(oracle, dims, case["K"], case["L"], seed=17, cap=case["cap"], N_build=case["N"],
                                hashed=case["hashed"], last_act=case["last_act"], repeat_rows=case.get("repeat_rows", 0))
    hashed = [l for l, lay in enumerate(layers) if lay.K > 0]
    g = rt.Network(layers)
    _say(f"device build {dims}")
    g.build_tables(Xb)
    blob = g.export_tables()
    net_g = oracle.OracleNet(layers)
    net_g.import_tables(blob)            # oracle consumes the device-built tables
    net_s = oracle.OracleNet(layers)
    net_s.build_tables(Xb, keep_scores=True)
    for l in hashed:
        tg, ts = net_g.tables[l], net_s.tables[l]
        swaps = mism = 0
        for b in range(layers[l].L):
            for key in range(1 << layers[l].K):
                lg, ls = tg.bucket(b, key), ts.bucket(b, key)
                if ls.size == 0 and lg.size == 0:
                    continue
                sc = ts.bucket_scores(b, key)
                if sc is None or lg.size != ls.size:
                    mism += 1              # a training input hashed differently (projection within rounding of 0)
                    continue
                for a, c in zip(lg, ls):
                    if a != c:
                        swaps += 1
                        assert abs(sc[a] - sc[c]) <= 1e-5 * max(abs(sc[a]), abs(sc[c])), (l, b, key, a, c)
        _say(f"layer {l}: {swaps} rank swaps among near-equal sums, {mism} buckets with different membership")
        assert mism <= (2 if l > hashed[0] else 0)
        gg, _ = tg.global_rank()
        gs, ss = ts.global_rank()
        for a, c in zip(gg, gs):
            if a != c:
                assert abs(ss[a] - ss[c]) <= 1e-5 * max(abs(ss[a]), abs(ss[c]), 1e-30)
    # same blob on both sides: selection and outputs agree
    X = make_queries(dims, 64, seed=9)
    ref = net_g.sparse_forward(X, 0.02)
    got = to_numpy_result(g.sparse_forward(X, 0.02, taps=True))
    compare_sparse(got, ref, layers, "device-built tables")
    # the device build is reproducible bit for bit
    g2 = rt.Network(layers)
    g2.build_tables(Xb)
    assert g2.export_tables() == blob


@pytest.mark.parametrize("case", [
    dict(dims=(60, 200, 150, 9), K=4, L=5, cap=None, hashed=None, last_act=wl.ACT_NONE),
    dict(dims=(40, 96, 9000), K=3, L=3, cap=300, hashed=[1], last_act=wl.ACT_SOFTMAX),       # wide layer
], ids=["two-hidden", "wide-softmax"])
def test_tables_refresh_matches_oracle_and_full_build(rt, oracle, case):
    """Online refresh (Alg. 1 continued): tables trained on A on the device and refreshed with B,
    then C, must be bit for bit the tables the device trains on A + B + C at once, and match the
    oracle's refreshed tables under the same rules as a build (swaps only among sums equal to 1e-5);
    the forward pass on the refreshed tables agrees with the oracle on the same blob."""
    from paper_2204_08400_amd import slonn
    dims = case["dims"]
    layers, net, Xa = make_case(oracle, dims, case["K"], case["L"], seed=29, cap=case["cap"], N_build=150,
                                hashed=case["hashed"], last_act=case["last_act"], keep_scores=True)
    hashed = [l for l, lay in enumerate(layers) if lay.K > 0]
    Xb = make_queries(dims, 90, seed=301)
    Xc = make_queries(dims, 7, seed=302)
    g = rt.Network(layers)
    g.set_tables_refreshable(True)
    _say(f"refresh {dims}: device build on A, refresh with B and C")
    g.build_tables(Xa)
    only_a = g.export_tables()
    g.refresh_tables(Xb)
    g.refresh_tables(Xc)
    blob = g.export_tables()
    assert blob != only_a
    g_full = rt.Network(layers)
    g_full.set_tables_refreshable(True)
    g_full.build_tables(np.concatenate([Xa, Xb, Xc]))
    assert g_full.export_tables() == blob, "refreshed tables differ from a build on all inputs"
    # the oracle's refresh
    net.refresh_tables(Xb)
    net.refresh_tables(Xc)
    net_g = oracle.OracleNet(layers)
    net_g.import_tables(blob)
    for l in hashed:
        tg, ts = net_g.tables[l], net.tables[l]
        swaps = mism = 0
        for b in range(layers[l].L):
            for key in range(1 << layers[l].K):
                lg, ls = tg.bucket(b, key), ts.bucket(b, key)
                if ls.size == 0 and lg.size == 0:
                    continue
                sc = ts.bucket_scores(b, key)
                if sc is None or lg.size != ls.size:
                    mism += 1
                    continue
                for a, c in zip(lg, ls):
                    if a != c:
                        swaps += 1
                        assert abs(sc[a] - sc[c]) <= 1e-5 * max(abs(sc[a]), abs(sc[c])), (l, b, key, a, c)
        _say(f"layer {l}: {swaps} rank swaps among near-equal sums, {mism} buckets with different membership")
        assert mism <= (2 if l > hashed[0] else 0)
        gg, _ = tg.global_rank()
        gs, ss = ts.global_rank()
        for a, c in zip(gg, gs):
            if a != c:
                assert abs(ss[a] - ss[c]) <= 1e-5 * max(abs(ss[a]), abs(ss[c]), 1e-30)
    X = make_queries(dims, 48, seed=9)
    ref = net_g.sparse_forward(X, 0.05)
    got = to_numpy_result(g.sparse_forward(X, 0.05, taps=True))
    compare_sparse(got, ref, layers, "refreshed tables")
    # tables that kept no sums refuse
    g2 = rt.Network(layers)
    g2.build_tables(Xa)
    with pytest.raises(slonn.SlonnError) as e:
        g2.refresh_tables(Xb)
    assert e.value.code == -4


# --------------------------------------------------------------------------- #
# the benchmark configurations at their real shapes
# --------------------------------------------------------------------------- #
def _config_case(rt, cfg_name, n_build, n_query, seed_w=0, list_cap=None):
    """The network of a benchmark configuration exactly as bench.py sets it up: hash nodes
    from the device's dense pass, tables built on the device; the oracle loads the same
    table blob (the build itself is compared with the oracle's in its own test)."""
    import torch
    from oracle import slonn_oracle
    cfg = wl.CONFIGS[cfg_name]
    layers = wl.make_mlp(cfg.dims, seed=seed_w, w_dtype=cfg.w_dtype, last_act=cfg.last_act)
    Xb = wl.make_inputs(cfg, n_build, seed=1)
    plain = rt.Network(layers)
    xb = torch.from_numpy(Xb).cuda()
    dn = plain.dense_forward(xb, layer_outs=True)
    for l in cfg.hashed_layers:
        layers[l].K, layers[l].L = cfg.K, cfg.L
        layers[l].list_cap = layers[l].d_out if list_cap is None else list_cap
        layers[l].hash_nodes = rt.hash_nodes_by_variance(dn["layers"][l], cfg.K, cfg.L,
                                                         wl.hash_node_draws(cfg.K, cfg.L, seed=3 + l))
    del plain, dn
    g = rt.Network(layers)
    g.build_tables(xb)
    net = slonn_oracle.OracleNet(layers)
    net.import_tables(g.export_tables())
    Xq = wl.make_inputs(cfg, n_query, seed=2)
    return cfg, layers, g, net, Xq


def test_config_c1_fmnist_shape(rt, oracle):
    """784-112-10, K=6 L=10, keep 0.25, batches of 1 and 64 (full 1000-input sets)."""
    cfg, layers, g, net, Xq = _config_case(rt, "C1", 1000, 1000)
    ref = net.sparse_forward(Xq, 0.25)
    for path in ("fused", "layers"):
        g.set_path(path)
        for B in (1, 64):
            _say(f"C1 path={path} batch={B}")
            n = 8 if B == 1 else 1000
            outs = []
            for s in range(0, n, B):
                outs.append(to_numpy_result(g.sparse_forward(Xq[s:s + B], 0.25, taps=True)))
            got = {"out": np.concatenate([o["out"] for o in outs]),
                   "argmax": np.concatenate([o["argmax"] for o in outs]),
                   "taps": {k: [None if outs[0]["taps"][k][l] is None else
                                np.concatenate([o["taps"][k][l] for o in outs]) for l in range(2)]
                            for k in outs[0]["taps"]}}
            sub = {"out": ref["out"][:n], "argmax": ref["argmax"][:n],
                   "layers": [{k: v[:n] for k, v in lay.items()} for lay in ref["layers"]]}
            _say(f"  {compare_sparse(got, sub, layers, f'C1 {path} B={B}')}")


def test_config_c2_bench_shape(rt, oracle):
    """The workload bench.py times (784-1024-1024-10, K=8 L=16, batch 256, path auto):
    full 10 000-input build set, the first 1024 queries in batches of 256, checked with
    taps; then the same batches without taps, as timed, must give the same bits."""
    import torch
    cfg, layers, g, net, Xq = _config_case(rt, "C2", 10000, 1024)
    g.set_path("auto")
    for keep in (0.05, 0.25, 1.0):
        _say(f"C2 keep={keep}")
        ref = net.sparse_forward(Xq, keep)
        for s in range(0, 1024, 256):
            xb = Xq[s:s + 256]
            got = to_numpy_result(g.sparse_forward(xb, keep, taps=True))
            sub = {"out": ref["out"][s:s + 256], "argmax": ref["argmax"][s:s + 256],
                   "layers": [{k: v[s:s + 256] for k, v in lay.items()} for lay in ref["layers"]]}
            rep = compare_sparse(got, sub, layers, f"C2 keep {keep} batch {s // 256}")
            plain = to_numpy_result(g.sparse_forward(xb, keep))
            assert np.array_equal(plain["out"], got["out"]) and np.array_equal(plain["argmax"], got["argmax"])
        _say(f"  last batch report {rep}")


def test_config_c3_shape_sampled(rt, oracle):
    """3072-4096-4096-4096-100, K=10 L=32 (per-layer path): tables from a 4096-input build
    set, 48 queries checked in full against the oracle, batch 32 and a ragged batch of 16."""
    cfg, layers, g, net, Xq = _config_case(rt, "C3", 4096, 48)
    for keep in (0.05, 0.5):
        _say(f"C3 keep={keep}")
        ref = net.sparse_forward(Xq, keep)
        outs = [to_numpy_result(g.sparse_forward(Xq[s:e], keep, taps=True)) for s, e in ((0, 32), (32, 48))]
        got = {"out": np.concatenate([o["out"] for o in outs]),
               "argmax": np.concatenate([o["argmax"] for o in outs]),
               "taps": {k: [None if outs[0]["taps"][k][l] is None else
                            np.concatenate([o["taps"][k][l] for o in outs]) for l in range(4)]
                        for k in outs[0]["taps"]}}
        _say(f"  {compare_sparse(got, ref, layers, f'C3 keep {keep}')}")


@pytest.mark.timeout(600)
def test_config_c3_timed_batch_sampled(rt, oracle):
    """C3 at the batch bench.py times (1024 queries, path auto: integer hash, select, then per 128
    queries either the masked tiles on the fp16 matrix cores - keep 0.1 and above - or the row-block
    gather), over the keep sweep; the oracle computes the first and the last query of every group
    of 16 (128 queries: both sides of every 16- and 128-query boundary of the tiles and unions)."""
    from paper_2204_08400_amd import slonn
    B = 1024
    cfg, layers, g, net, Xq = _config_case(rt, "C3", 4096, B, list_cap=2049)
    sample = np.asarray([q for q in range(B) if q % 16 in (0, 15)])
    for keep in (0.05, 0.1, 0.25, 0.5):
        _say(f"C3 batch 1024 keep={keep}: GPU pass")
        slonn.slonn_profile_begin(64)
        res = g.sparse_forward(Xq, keep, taps=True)
        prof = slonn.slonn_profile_end()
        # per hidden layer the masked tiles and the per-query pass for what they leave
        assert prof["tiles"][1] == len(cfg.hashed_layers) and prof["gather"][1] == len(cfg.hashed_layers), prof
        assert prof["dense"][1] == 1, prof
        got = to_numpy_result(res)
        _say(f"C3 batch 1024 keep={keep}: oracle on {len(sample)} sampled queries")
        ref = net.sparse_forward(Xq[sample], keep)
        sub = {"out": got["out"][sample], "argmax": got["argmax"][sample],
               "taps": {k: [None if t is None else t[sample] for t in v] for k, v in got["taps"].items()}}
        _say(f"  {compare_sparse(sub, ref, layers, 'C3 batch 1024')}")


def test_config_c5_shape_sampled(rt, oracle):
    """Deep bf16 MLP with mixed per-query keep fractions, at reduced depth/width so the
    oracle finishes in seconds: 1024-[2048]x3-1000, K=12 L=64, keep ~ U[0.02, 0.3]."""
    import dataclasses
    base = wl.CONFIGS["C5"]
    cfg = dataclasses.replace(base, dims=(1024, 2048, 2048, 2048, 1000), hashed_layers=(0, 1, 2))
    wl.CONFIGS["C5small"] = cfg
    try:
        cfg, layers, g, net, Xq = _config_case(rt, "C5small", 3000, 96)
    finally:
        del wl.CONFIGS["C5small"]
    keep = wl.keep_uniform(96, 0.02, 0.3, 7)
    ref = net.sparse_forward(Xq, keep)
    for path in ("layers", "fused"):
        g.set_path(path)
        _say(f"C5-shaped path={path}")
        got = to_numpy_result(g.sparse_forward(Xq, _keep_tensor(keep), taps=True))
        _say(f"  {compare_sparse(got, ref, layers, f'C5-shaped {path}')}")


@pytest.mark.timeout(900)
def test_config_c5_full_width_sampled(rt, oracle):
    """C5 at its real shape (1024-[8192]x6-1000, bf16 weights, K=12 L=64, batch 2048, per-query
    keep ~ U[0.02, 0.3]) in the launch configuration bench.py times (path auto: per-layer path,
    masked tiles on the fp16 matrix cores for the 128-query tiles with large budgets, unions of
    16 queries for the others).  Tables are built on the
    device from 256 inputs to keep the blob the oracle loads near 1 GB; the oracle then computes
    a sample of queries one by one."""
    from paper_2204_08400_amd import slonn
    B = 2048
    cfg, layers, g, net, Xq = _config_case(rt, "C5", 256, B, list_cap=2459)
    keep = wl.keep_uniform(B, cfg.keep_range[0], cfg.keep_range[1], 6)
    # the timed batch, and a medium one that takes the same kernels in their other shapes: tiles of
    # 64 x 128, 1024-thread select workgroups, the integer hash below batch 256 (large projections)
    # (sampled: the first and the last query of every group of 16, i.e. both sides of every 16- and
    # 128-query boundary of the unions and tiles)
    for b in (2048, 192):
        sample = np.asarray([q for q in range(b) if q % 16 in (0, 15)])
        _say(f"C5 full width, batch {b}: GPU pass")
        slonn.slonn_profile_begin(64)
        res = g.sparse_forward(Xq[:b], _keep_tensor(keep[:b]), taps=True)
        prof = slonn.slonn_profile_end()
        # tiles + unions per hidden layer
        assert prof["tiles"][1] == len(cfg.hashed_layers) and prof["gather"][1] == len(cfg.hashed_layers), prof
        # per hidden layer the select kernel (which also writes the tiles' pair masks) and the unions;
        # 2048 select workgroups do not fit the device at once: one more launch orders them by budget
        assert prof["select"][1] == 2 * len(cfg.hashed_layers) + (1 if b == 2048 else 0), prof
        got = to_numpy_result(res)
        _say(f"C5 full width, batch {b}: oracle on the sampled queries")
        ref = net.sparse_forward(Xq[sample], keep[sample])
        sub = {"out": got["out"][sample], "argmax": got["argmax"][sample],
               "taps": {k: [None if t is None else t[sample] for t in v] for k, v in got["taps"].items()}}
        # six sparse layers deep the projections are of order 1e-3 (every layer keeps 2-30 % of its
        # nodes), so the absolute 1e-6 tie zone catches a few per cent of the queries here
        rep = compare_sparse(sub, ref, layers, f"C5 full width batch {b}", max_tainted=len(sample) // 10)
        _say(f"  {rep}")


@pytest.mark.parametrize("path", ["auto", "layers"])
def test_config_c4_shape(rt, oracle, path):
    """Wiki10/Delicious-shaped model at its real width: 100 000 sparse features (100
    non-zeros) -> 128 -> 100 000 softmax outputs, K=12 L=50 on the output layer, keep
    0.005 (500 nodes), batch 128.  Tables come from the oracle on a 256-input build set (the
    device build of a layer this wide is compared with the oracle's in test_build_tables_matches_oracle)."""
    import copy
    cfg = wl.CONFIGS["C4"]
    layers, net, _ = make_case(oracle, cfg.dims, cfg.K, cfg.L, seed=0, hashed=[1], cap=600,
                               last_act=wl.ACT_SOFTMAX, ell_nnz=cfg.ell_nnz, N_build=256)
    glayers = [copy.copy(l) for l in layers]
    glayers[0].W = np.ascontiguousarray(layers[0].W.T)        # input-major first layer on the device
    g = rt.Network(glayers, first_layer_rows_are_inputs=True)
    g.import_tables(net.export_tables())
    g.set_path(path)      # auto: the whole-network kernel for wide sparse-input models
    X = make_queries(cfg.dims, 128, seed=2, ell_nnz=cfg.ell_nnz)
    from paper_2204_08400_amd import slonn
    slonn.slonn_profile_begin(32)
    g.sparse_forward(X, 0.005, compact=True, dense=False)
    prof = slonn.slonn_profile_end()
    assert (prof["fused"][1] == 1) == (path == "auto"), prof
    _say(f"C4 sparse forward path={path}")
    ref = net.sparse_forward(X, 0.005)
    got = to_numpy_result(g.sparse_forward(X, 0.005, taps=True, compact=True))
    # 600 projections per query on logits of order 0.1: the absolute 1e-6 tie zone takes a few queries
    rep = compare_sparse(got, ref, layers, "C4", max_tainted=6)
    _say(f"  {rep}")
    ok = ~ref["layers"][1]["tie"]
    assert (got["cnt"][ok] == 500).all()
    for q in np.nonzero(ok)[0]:
        assert np.array_equal(got["idx"][q, :500], ref["layers"][1]["active"][q, :500])
        np.testing.assert_allclose(got["val"][q, :500], ref["out"][q, got["idx"][q, :500]], rtol=1e-4, atol=1e-9)
    # compact-only output (no dense [B][100000] row is ever written): same ids, values, argmax
    lean = to_numpy_result(g.sparse_forward(X, 0.005, compact=True, dense=False))
    assert np.array_equal(lean["cnt"], got["cnt"]) and np.array_equal(lean["argmax"], got["argmax"])
    assert np.array_equal(lean["idx"][:, :500], got["idx"][:, :500])
    assert np.array_equal(lean["val"][:, :500], got["val"][:, :500])


def test_runs_are_bit_reproducible(rt, oracle):
    """No float atomics or order-dependent reductions on the path: two runs of the same
    batch give identical bits on both paths (a cheap race detector)."""
    dims = (96, 1000, 640, 12)
    layers, net, _ = make_case(oracle, dims, 6, 10, seed=23)
    X = make_queries(dims, 200, seed=6)
    keep = _keep_tensor(wl.keep_uniform(200, 0.01, 0.9, 8))
    for path in ("layers", "fused"):
        g = _gpu_net(rt, layers, net, path=path)
        a = to_numpy_result(g.sparse_forward(X, keep, taps=True))
        for _ in range(3):
            b = to_numpy_result(g.sparse_forward(X, keep, taps=True))
            assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["argmax"], b["argmax"])
            for l in (0, 1):
                assert np.array_equal(a["taps"]["active"][l], b["taps"]["active"][l])
                assert np.array_equal(a["taps"]["z"][l], b["taps"]["z"][l])


def test_workspace_for_a_large_batch_serves_smaller_ones(rt, oracle):
    """A workspace sized for the largest batch must serve every smaller one: the size never
    shrinks as the batch grows (also where a small batch uses scratch a large one does not: the
    split reduction of a skinny output layer), and a pass in the larger workspace gives the
    bits of a pass in its own."""
    import torch
    from paper_2204_08400_amd import slonn
    dims = (48, 2048, 128)
    layers, net, _ = make_case(oracle, dims, 4, 3, seed=77, hashed=[0], N_build=64)
    g = _gpu_net(rt, layers, net)
    g.set_path("layers")
    sizes = [slonn.slonn_workspace_bytes(g.model, b) for b in (1, 2, 7, 32, 64, 65, 256, 1024, 4096)]
    assert sizes == sorted(sizes), sizes
    X = torch.from_numpy(make_queries(dims, 512, seed=9)).cuda()
    slonn.slonn_profile_begin(16)
    own = to_numpy_result(g.sparse_forward(X, 0.5))           # 64 tiles of 32 x 32: the output layer splits its reduction
    assert slonn.slonn_profile_end()["dense"][1] == 1
    g.workspace(4096)
    big = to_numpy_result(g.sparse_forward(X, 0.5))
    assert np.array_equal(own["out"], big["out"]) and np.array_equal(own["argmax"], big["argmax"])
    ref = net.sparse_forward(X.cpu().numpy(), 0.5)
    assert_close_rows(own["out"], ref["out"], None, "skinny output layer with split reduction")


def test_argument_errors_on_device(rt, oracle):
    import torch
    from paper_2204_08400_amd import slonn
    dims = (40, 64, 64, 8)
    layers, net, _ = make_case(oracle, dims, 3, 2, seed=41)
    g = _gpu_net(rt, layers, net)
    X = torch.from_numpy(make_queries(dims, 4, seed=8)).cuda()
    keep = torch.full((1,), 0.5, device="cuda")
    ws = g.workspace(4)
    out = slonn.make_output(dense=torch.empty((4, 8), device="cuda"))
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(slonn.SlonnError) as e:       # workspace too small
        g.set_path("layers")
        slonn.slonn_sparse_forward(g.model, g.tables, g.to_input(X), 4, keep, 0, 0, out, None, small)
    assert e.value.code == slonn.ENOMEM
    with pytest.raises(slonn.SlonnError) as e:       # active-list stride below the layer width
        slonn.slonn_select(g.model, g.tables, 0, X, 4, keep, 0, None, None,
                           torch.empty((4, 10), dtype=torch.int32, device="cuda"),
                           torch.empty(4, dtype=torch.int32, device="cuda"), 10, ws)
    assert e.value.code == slonn.ECAP
    with pytest.raises(slonn.SlonnError) as e:       # tables of another model
        other = _gpu_net(rt, layers, net)
        slonn.slonn_sparse_forward(g.model, other.tables, g.to_input(X), 4, keep, 0, 0, out, None, ws)
    assert e.value.code == slonn.EINVAL
    with pytest.raises(slonn.SlonnError):            # a corrupted blob is refused
        blob = bytearray(net.export_tables())
        blob[60] ^= 0xFF
        g.import_tables(bytes(blob))
    with pytest.raises(slonn.SlonnError):            # batch beyond the documented maximum
        slonn.slonn_workspace_bytes(g.model, (1 << 20) + 1)


@pytest.mark.parametrize("w_dtype,d,n,B", [(wl.W_F32, 512, 4096, 519), (wl.W_F32, 544, 4040, 519),
                                           (wl.W_F32, 520, 4096, 519), (wl.W_BF16, 1024, 4096, 519),
                                           (wl.W_BF16, 1032, 4096, 519), (wl.W_BF16, 1024, 4096, 1031),
                                           (wl.W_F32, 512, 4096, 200)],
                         ids=["f32-tiles", "f32-tiles-ragged", "f32-rows-not-32", "bf16", "bf16-ragged-rows",
                              "bf16-128x128-tiles", "f32-batch-200"])
def test_grouped_evaluation_matches_oracle(rt, oracle, w_dtype, d, n, B):
    """Large batch on the per-layer path, evaluation across queries on the matrix cores.
    fp32 rows of a multiple of 32 elements: masked 128 x 128 tiles on the fp16 cores (two
    fp16 parts per operand), decided per 128 queries by their mean budget; other fp32 rows:
    groups of 16 queries whose lists overlap, union of rows on the fp32 cores; bf16 weights:
    every group of 16 on the bf16 cores.  The rest stays on the per-query gather.  Same results
    either way."""
    from paper_2204_08400_amd import slonn
    dims = (d, n, 24)
    layers, net, _ = make_case(oracle, dims, 6, 8, seed=61, hashed=[0], cap=1500, N_build=192, kind="clip3",
                               w_dtype=w_dtype)
    g = _gpu_net(rt, layers, net, path="layers")
    # (B = 512 + 7 and 1024 + 7: ragged last group; 200: a last tile of 72 queries)
    X = make_queries(dims, B, seed=62, kind="clip3")
    # third case: the first 128 queries with small budgets (their tile stays on the per-query
    # gather), the others large
    split = np.where(np.arange(B) < 128, 0.02, 0.35).astype(np.float32)
    for keep in (0.3, wl.keep_uniform(B, 0.0001, 0.3, 9), split):
        _say(f"grouped evaluation {'f32' if w_dtype == wl.W_F32 else 'bf16'} keep={'mixed' if np.ndim(keep) else keep}")
        ref = net.sparse_forward(X, keep)
        kt = _keep_tensor(keep) if np.ndim(keep) else keep
        slonn.slonn_profile_begin(64)
        got = to_numpy_result(g.sparse_forward(X, kt, taps=True))
        prof = slonn.slonn_profile_end()
        # layer 0: tiles (or unions on the fp32 cores) + per-query pass for fp32; tiles + unions of
        # 16 for bf16 (unions only when the rows are not a multiple of 32 elements); the output
        # layer (17 tiles of 32x32) is too small for the matrix-core kernel and takes one more
        # gather launch with the identity list
        assert prof["tiles"][1] == (0 if d % 32 else 1), prof
        assert prof["tiles"][1] + prof["gather"][1] == (2 if (w_dtype == wl.W_BF16 and d % 32) else 3), prof
        assert prof["dense"][1] == 0, prof
        _say(f"  {compare_sparse(got, ref, layers, 'grouped')}")
    # the same launch configuration with the hash nodes at the head of every list (Section 3.4
    # variant): their outputs come from the projections, the tiles and unions leave them out
    ref_net = oracle.OracleNet(layers, hash_nodes_always_active=True)
    ref_net.tables = net.tables
    g.set_hash_nodes_always_active(True)
    _say("grouped evaluation, hash nodes always active")
    ref = ref_net.sparse_forward(X, split)
    got = to_numpy_result(g.sparse_forward(X, _keep_tensor(split), taps=True))
    _say(f"  {compare_sparse(got, ref, layers, 'grouped hash-first')}")


@pytest.mark.parametrize("w_dtype", [wl.W_F32, wl.W_BF16], ids=["f32", "bf16"])
def test_integer_hash_projection_matches_oracle(rt, oracle, w_dtype):
    """Large batches take their hash projections from the int8 matrix cores (fixed-point digits,
    exact integer sums, every sign certified against a rigorous bound, uncertain projections
    recomputed in fp64).  Codes and active sets match the oracle bit for bit as everywhere;
    with a margin that sends EVERY projection through the fp64 recomputation the codes and
    active sets stay the same and the outputs agree to the usual tolerance; rows of zeros, tiny
    and huge magnitudes go through the same path."""
    dims = (192, 640, 2048, 16)           # d = 192 and 640: multiples of 64, several chunks, ragged tiles
    layers, net, _ = make_case(oracle, dims, 5, 9, seed=131, cap=700, N_build=160, kind="clip3", w_dtype=w_dtype)
    g = _gpu_net(rt, layers, net, path="layers")
    B = 600                               # ragged: four full 128-query tiles and a tail of 88
    X = make_queries(dims, B, seed=132, kind="clip3")
    X[5] = 0.0                            # a row of zeros: projections are the biases
    X[6] *= 1e-20                         # tiny inputs
    X[7] *= 1e15                          # huge inputs
    X[8, 1:] = 0.0                        # a single non-zero
    X[9] *= 1e-38                         # subnormal inputs
    keep = wl.keep_uniform(B, 0.02, 0.5, 3)
    _say("integer hash: oracle")
    ref = net.sparse_forward(X, keep)
    _say("integer hash: default margin")
    got = to_numpy_result(g.sparse_forward(X, _keep_tensor(keep), taps=True))
    _say(f"  {compare_sparse(got, ref, layers, 'integer hash')}")
    g.set_hash_margin(1e300)
    _say("integer hash: every projection recomputed")
    got2 = to_numpy_result(g.sparse_forward(X, _keep_tensor(keep), taps=True))
    _say(f"  {compare_sparse(got2, ref, layers, 'integer hash, all recomputed')}")
    ok = np.ones(B, bool)
    for l in range(len(layers) - 1):
        ok &= ~ref["layers"][l]["tie"]
    for l in range(len(layers) - 1):
        assert np.array_equal(got["taps"]["codes"][l][ok], got2["taps"]["codes"][l][ok])
    g.set_hash_margin(2.0)


@pytest.mark.parametrize("path", ["layers", "fused"])
def test_selected_hash_nodes_reuse_their_projection(rt, oracle, path):
    """Section 3.4: a hash projection is the node's own pre-activation.  Where a hash node is
    selected, the whole-network kernel and the row-block path take its output from the
    projection (bit for bit act(z_h)) instead of fetching the row again; the oracle computes
    every active node from its row, and both must agree to the usual tolerance."""
    dims = (640, 1536, 40)           # 1536 x 640 fp32 = 3.75 MiB with 2560-byte rows: row-block path
    layers, net, _ = make_case(oracle, dims, 5, 8, seed=71, hashed=[0], cap=800, N_build=160, kind="u01")
    g = _gpu_net(rt, layers, net, path=path)
    B = 48
    X = make_queries(dims, B, seed=72, kind="u01")
    hn = layers[0].hash_nodes
    for keep in (0.2, 1.0):
        _say(f"hash reuse path={path} keep={keep}")
        ref = net.sparse_forward(X, keep)
        got = to_numpy_result(g.sparse_forward(X, keep, taps=True))
        _say(f"  {compare_sparse(got, ref, layers, 'reuse ' + path)}")
        z = got["taps"]["z"][0]
        out = got["taps"]["out"][0]
        reused = 0
        for q in range(B):
            act = set(got["taps"]["active"][0][q, :got["taps"]["cnt"][0][q]].tolist())
            for h, node in enumerate(hn):
                if int(node) in act:
                    assert out[q, node] == max(z[q, h], np.float32(0)), (q, h, node)
                    reused += 1
        assert reused > 0


def test_masked_tiles_behind_the_wide_select_kernel(rt, oracle):
    """A bf16 layer too wide for the select kernel's per-node LDS map (50 000 nodes: the bitmap
    variant runs) at a batch that takes the masked tiles: the bitmap kernel writes the tiles' pair
    masks from its finished lists.  Keep 0.15 serves every tile, keep 0.03 none (unions of 16)."""
    from paper_2204_08400_amd import slonn
    dims = (256, 50000, 16)
    layers, net, _ = make_case(oracle, dims, 8, 10, seed=91, hashed=[0], cap=8000, N_build=96, kind="clip3",
                               w_dtype=wl.W_BF16)
    g = _gpu_net(rt, layers, net, path="layers")
    B = 256
    X = make_queries(dims, B, seed=92, kind="clip3")
    for keep, tiles in ((0.15, 1), (0.03, 0)):
        _say(f"wide select + masked tiles, keep {keep}")
        ref = net.sparse_forward(X, keep)
        slonn.slonn_profile_begin(16)
        res = g.sparse_forward(X, keep, taps=True)
        prof = slonn.slonn_profile_end()
        got = to_numpy_result(res)
        _say(f"  {compare_sparse(got, ref, layers, 'wide select + tiles')}")
        # the tile kernel is launched either way (unserved tiles leave at once) and the unions follow;
        # the output layer's 50 000-element rows do not fit the LDS staging of the gather kernels: it
        # takes the kernel that reads the activations from global memory
        assert prof["tiles"][1] == 1 and prof["gather"][1] == 2, prof


HASH_FIRST_CASES = [
    # small layers (fused eligible), a row-block layer, a bf16 net, a wide activated output layer
    dict(dims=(96, 1000, 640, 12), K=6, L=10, kind="u01", B=67, last_act=wl.ACT_SOFTMAX),
    dict(dims=(640, 1536, 40), K=5, L=8, kind="u01", B=48, hashed=[0], cap=800),
    dict(dims=(128, 768, 512, 10), K=4, L=16, kind="clip3", B=130, w_dtype=wl.W_BF16),
    # a batch and a layer that take the masked tiles: the hash nodes at the head of the lists get
    # their bits in the pair masks of the served tiles
    dict(dims=(640, 4096, 40), K=5, L=8, kind="u01", B=192, hashed=[0], cap=1400),
]


@pytest.mark.parametrize("path", ["layers", "fused"])
@pytest.mark.parametrize("case", HASH_FIRST_CASES, ids=lambda c: "x".join(map(str, c["dims"])))
def test_hash_nodes_always_active_matches_oracle(rt, oracle, case, path):
    """Section 3.4 variant: hash nodes head every active list and are never selected;
    budgets below K*L give exactly the hash nodes."""
    dims = case["dims"]
    if path == "fused" and not _fused_ok(case):
        pytest.skip("model does not qualify for the whole-network kernel")
    layers, net, _ = make_case(oracle, dims, case["K"], case["L"], seed=81, hashed=case.get("hashed"),
                               cap=case.get("cap"), N_build=200, kind=case["kind"],
                               w_dtype=case.get("w_dtype", wl.W_F32), last_act=case.get("last_act", wl.ACT_NONE))
    ref_net = oracle.OracleNet(layers, hash_nodes_always_active=True)
    ref_net.tables = net.tables
    g = _gpu_net(rt, layers, net, path=path)
    g.set_hash_nodes_always_active(True)
    B = case["B"]
    X = make_queries(dims, B, seed=82, kind=case["kind"])
    H = case["K"] * case["L"]
    for keep in (0.01, 0.3, wl.keep_uniform(B, 0.0001, 1.0, 5), 1.0):
        _say(f"hash-first {dims} path={path} keep={'mixed' if np.ndim(keep) else keep}")
        ref = ref_net.sparse_forward(X, keep)
        kt = _keep_tensor(keep) if np.ndim(keep) else keep
        got = to_numpy_result(g.sparse_forward(X, kt, taps=True))
        _say(f"  {compare_sparse(got, ref, layers, 'hash-first ' + path)}")
        for l, lay in enumerate(layers):
            if lay.K > 0:
                c = got["taps"]["cnt"][l]
                assert (c >= min(H, lay.d_out)).all()
    # the stand-alone selection entry point follows the same setting
    import torch
    l0 = 0
    ref = ref_net.sparse_forward(X, 0.3)["layers"][l0]
    sel = g.select(l0, X, 0.3)
    ok = ~ref["tie"]
    cnt = sel["cnt"].cpu().numpy()
    act = sel["active"].cpu().numpy()
    assert np.array_equal(cnt[ok], ref["cnt"][ok])
    for q in np.nonzero(ok)[0]:
        assert np.array_equal(act[q, :cnt[q]], ref["active"][q, :cnt[q]])
    g.set_hash_nodes_always_active(False)
    plain = net.sparse_forward(X, 0.3)
    got = to_numpy_result(g.sparse_forward(X, 0.3, taps=True))
    compare_sparse(got, plain, layers, "back to plain " + path)


@pytest.mark.parametrize("path", ["auto", "layers"])
def test_hash_nodes_always_active_wide_output_layer(rt, oracle, path):
    """The variant on a wide activated softmax output layer (bitmap select kernel), compact output."""
    d0, n_out = 4000, 50000
    dims = (d0, 64, n_out)
    layers, net, _ = make_case(oracle, dims, 6, 12, seed=91, hashed=[1], cap=600, N_build=96,
                               last_act=wl.ACT_SOFTMAX, ell_nnz=30)
    ref_net = oracle.OracleNet(layers, hash_nodes_always_active=True)
    ref_net.tables = net.tables
    import copy
    glayers = [copy.copy(l) for l in layers]
    glayers[0].W = np.ascontiguousarray(layers[0].W.T)      # the GPU stores the first layer input-major
    g = rt.Network(glayers, first_layer_rows_are_inputs=True)
    g.import_tables(net.export_tables())
    g.set_path(path)
    g.set_hash_nodes_always_active(True)
    X = make_queries(dims, 40, seed=92, ell_nnz=30)
    for keep in (0.0005, 0.004):
        _say(f"hash-first wide output keep={keep}")
        ref = ref_net.sparse_forward(X, keep)
        got = to_numpy_result(g.sparse_forward(X, keep, taps=True, compact=True))
        _say(f"  {compare_sparse(got, ref, layers, 'hash-first wide')}")
        ok = ~ref["layers"][1]["tie"]
        for q in np.nonzero(ok)[0]:
            c = ref["layers"][1]["cnt"][q]
            assert got["cnt"][q] == c
            assert np.array_equal(got["idx"][q, :c], ref["layers"][1]["active"][q, :c])
            np.testing.assert_allclose(got["val"][q, :c], ref["out"][q, ref["layers"][1]["active"][q, :c]],
                                       rtol=1e-4, atol=1e-6 * float(ref["out"][q].max()))


# --------------------------------------------------------------------------- #
# choice of k per query (ACLO / LCAO)
# --------------------------------------------------------------------------- #
def _dyadic_conf(rng, shape):
    """confidences -k/64 in [-10, 0], last grid point (the full network) exactly 0"""
    c = (-rng.integers(0, 640, size=shape) / 64.0).astype(np.float32)
    c[:, -1] = 0.0
    return c


def test_worked_k_selection_example(rt, oracle):
    import torch
    from paper_2204_08400_amd import slonn
    with open(os.path.join(os.path.dirname(__file__), "golden", "k_selection_example.json")) as f:
        gold = json.load(f)
    dev = "cuda:0"
    p = slonn.slonn_policy_create(gold["K"], gold["L"], gold["k_grid"])
    codes = torch.tensor(gold["train_keys"], dtype=torch.int32, device=dev)
    conf = torch.tensor(gold["train_conf"], dtype=torch.float32, device=dev)
    slonn.slonn_policy_train_confidence(p, codes, conf, codes.shape[0])
    for a in gold["aclo"]:
        _say(f"worked ACLO example {a}")
        kq = torch.tensor([a["keys"]], dtype=torch.int32, device=dev)
        thr = torch.tensor([a["thr"]], dtype=torch.float32, device=dev)
        keep = torch.zeros(1, dtype=torch.float32, device=dev)
        chat = torch.zeros((1, 2), dtype=torch.float64, device=dev)
        slonn.slonn_policy_keep_aclo(p, kq, 1, thr, 0, keep, None, chat)
        assert keep.item() == np.float32(a["keep"])
        want = next(q["c_hat"] for q in gold["queries"] if q["keys"] == a["keys"])
        assert chat.cpu().numpy()[0].tolist() == want
    lc = gold["lcao"]
    p2 = slonn.slonn_policy_create(1, 1, lc["k_grid"])
    slonn.slonn_policy_set_latency_profile(p2, lc["T"])
    for c in lc["cases"] + [{"tau": 100.0, "t0": 0.0, "beta": 7, "keep": 0.1, "violated": True}]:
        _say(f"worked LCAO example {c}")
        tau = torch.tensor([c["tau"]], dtype=torch.float32, device=dev)
        t0 = torch.tensor([c["t0"]], dtype=torch.float32, device=dev)
        beta = torch.tensor([c["beta"]], dtype=torch.int32, device=dev)
        keep = torch.zeros(1, dtype=torch.float32, device=dev)
        bad = torch.zeros(1, dtype=torch.int32, device=dev)
        slonn.slonn_policy_keep_lcao(p2, 1, tau, 0, t0, 0, beta, 0, keep, None, bad)
        assert keep.item() == np.float32(c["keep"]) and bool(bad.item()) == c["violated"]


def test_policy_tables_and_decisions_match_oracle(rt, oracle):
    """Confidence tables trained on the device from random keys: estimates bit for bit equal
    to the oracle's (double sums in the same order), same ACLO and LCAO decisions; sizes span
    many 64-input chunks with a ragged tail, empty buckets and heavily loaded ones."""
    import torch
    from paper_2204_08400_amd import slonn
    dev = "cuda:0"
    rng = np.random.default_rng(21)
    for K, L, G, N, B in [(8, 16, 5, 10000, 777), (3, 2, 1, 70, 5), (10, 32, 16, 4133, 300), (12, 5, 7, 999, 64)]:
        _say(f"policy K={K} L={L} G={G} N={N} B={B}")
        grid = np.sort(rng.choice(np.arange(1, 200), size=G, replace=False)).astype(np.float32) / 200.0
        # skewed keys: a few heavy buckets and many empty ones
        keys = (rng.integers(0, 1 << K, size=(N, L)) * rng.integers(0, 2, size=(N, L))).astype(np.uint32)
        conf = rng.normal(-2.0, 1.0, size=(N, G)).astype(np.float32)
        ot = oracle.ConfidenceTables(K, L, grid, keys, conf)
        p = slonn.slonn_policy_create(K, L, grid.tolist())
        slonn.slonn_policy_train_confidence(p, torch.from_numpy(keys.view(np.int32)).to(dev),
                                            torch.from_numpy(conf).to(dev), N)
        Q = rng.integers(0, 1 << K, size=(B, L)).astype(np.uint32)
        Q[: B // 2] = keys[rng.integers(0, N, B // 2)]         # half the queries land in trained buckets
        chat_ref, _ = ot.estimate(Q)
        thr = rng.normal(-2.0, 0.5, B).astype(np.float32)
        thr[:3] = chat_ref[:3, 0].astype(np.float32)            # thresholds right at an estimate
        keep_ref, g_ref = ot.choose_aclo(Q, thr)
        keep = torch.zeros(B, dtype=torch.float32, device=dev)
        gi = torch.zeros(B, dtype=torch.int32, device=dev)
        chat = torch.zeros((B, G), dtype=torch.float64, device=dev)
        slonn.slonn_policy_keep_aclo(p, torch.from_numpy(Q.view(np.int32)).to(dev), B,
                                     torch.from_numpy(thr).to(dev), 1, keep, gi, chat)
        assert np.array_equal(chat.cpu().numpy(), chat_ref)
        assert np.array_equal(gi.cpu().numpy(), g_ref)
        assert np.array_equal(keep.cpu().numpy(), keep_ref)
        # LCAO on the same grid
        nbeta = 4
        T = np.sort(rng.uniform(0.05, 3.0, size=(nbeta, G)).astype(np.float32), axis=1)
        slonn.slonn_policy_set_latency_profile(p, T.tolist())
        tau = rng.uniform(0.0, 4.0, B).astype(np.float32)
        t0 = rng.uniform(0.0, 0.5, B).astype(np.float32)
        beta = rng.integers(0, nbeta, B).astype(np.int32)
        k_ref, g2_ref, bad_ref = oracle.choose_lcao(grid, T, tau, t0, beta)
        bad = torch.zeros(B, dtype=torch.int32, device=dev)
        slonn.slonn_policy_keep_lcao(p, B, torch.from_numpy(tau).to(dev), 1, torch.from_numpy(t0).to(dev), 1,
                                     torch.from_numpy(beta).to(dev), 1, keep, gi, bad)
        assert np.array_equal(keep.cpu().numpy(), k_ref)
        assert np.array_equal(gi.cpu().numpy(), g2_ref)
        assert np.array_equal(bad.cpu().numpy().astype(bool), bad_ref)


@pytest.mark.parametrize("path", ["layers", "fused"])
def test_forward_under_aclo_matches_oracle(rt, oracle, path):
    """Fig. 2 with the choice of k inside the pass: the first activated layer's keys pick k
    from the Confidence LSH tables, the pass continues with that k on every layer."""
    import torch
    from paper_2204_08400_amd import slonn
    dims = (96, 1000, 640, 12)
    K, L = 6, 10
    layers, net, Xb = make_case(oracle, dims, K, L, seed=101, N_build=300, kind="u01", last_act=wl.ACT_SOFTMAX)
    g = _gpu_net(rt, layers, net, path=path)
    rng = np.random.default_rng(22)
    grid = np.asarray([0.03, 0.1, 0.25, 0.5, 1.0], np.float32)
    # training keys from the device (slonn_select's codes), confidences synthetic
    sel = g.select(0, Xb, 0.5)
    tkeys_gpu = sel["codes"].cpu().numpy().view(np.uint32)
    tkeys, ttie = net.first_codes(Xb)
    assert np.array_equal(tkeys_gpu[~ttie], tkeys[~ttie])
    conf = _dyadic_conf(rng, (Xb.shape[0], grid.size))
    ot = oracle.ConfidenceTables(K, L, grid, tkeys, conf)
    p = slonn.slonn_policy_create(K, L, grid.tolist())
    slonn.slonn_policy_train_confidence(p, torch.from_numpy(tkeys.view(np.int32)).cuda(),
                                        torch.from_numpy(conf).cuda(), Xb.shape[0])
    B = 150
    X = make_queries(dims, B, seed=102, kind="u01")
    for thr in (-4.0, rng.uniform(-7.0, -1.0, B).astype(np.float32)):
        _say(f"ACLO forward path={path} thr={'per query' if np.ndim(thr) else thr}")
        ref = net.sparse_forward_aclo(X, ot, thr)
        tt = _keep_tensor(thr) if np.ndim(thr) else thr
        got = to_numpy_result(g.sparse_forward(X, None, taps=True, policy=p, thr=tt))
        keep = g.sparse_forward(X, None, policy=p, thr=tt)["keep"].cpu().numpy()
        ok = ~ref["layers"][0]["tie"]
        assert np.array_equal(keep[ok], ref["keep"][ok])
        assert len(set(ref["keep"].tolist())) > 1
        _say(f"  {compare_sparse(got, ref, layers, 'aclo ' + path)}")


@pytest.mark.parametrize("path,B", [("layers", 1), ("layers", 5), ("fused", 3)])
def test_recorded_forward_replays_like_eager(rt, oracle, path, B):
    """A forward pass recorded into a HIP graph: several replays with fresh inputs and keep
    fractions written into the baked-in buffers, eager work and synchronisations in between,
    every replay compared with the eager call bit for bit (and the first with the oracle)."""
    import torch
    from paper_2204_08400_amd import slonn
    dims = (640, 1536, 520, 10)
    layers, net, _ = make_case(oracle, dims, 5, 8, seed=111, cap=800, N_build=160, kind="u01")
    g = _gpu_net(rt, layers, net, path=path)
    dev = "cuda:0"
    x_static = torch.zeros((B, dims[0]), dtype=torch.float32, device=dev)
    keep_static = torch.zeros(B, dtype=torch.float32, device=dev)
    y_static = torch.zeros((B, dims[-1]), dtype=torch.float32, device=dev)
    a_static = torch.zeros(B, dtype=torch.int32, device=dev)
    inp = slonn.make_input(x=x_static)
    out = slonn.make_output(dense=y_static, argmax=a_static)
    ws = g.workspace(B)
    Xall = make_queries(dims, 6 * B, seed=112, kind="u01")
    keeps = wl.keep_uniform(6 * B, 0.02, 0.6, 7)
    x_static.copy_(torch.from_numpy(Xall[:B]))
    keep_static.copy_(torch.from_numpy(keeps[:B]))
    torch.cuda.synchronize()
    graph = slonn.slonn_forward_graph_create(g.model, g.tables, inp, B, keep_static, 1, 0, out, ws)
    stream = torch.cuda.current_stream()
    for r in range(6):
        _say(f"recorded forward path={path} B={B} replay {r}")
        xs, ks = Xall[r * B:(r + 1) * B], keeps[r * B:(r + 1) * B]
        x_static.copy_(torch.from_numpy(xs))
        keep_static.copy_(torch.from_numpy(ks))
        y_static.fill_(-1.0)
        graph.launch(stream)
        torch.cuda.synchronize()
        got_y, got_a = y_static.cpu().numpy().copy(), a_static.cpu().numpy().copy()
        # the program's own eager work between replays
        eager = to_numpy_result(g.sparse_forward(xs, _keep_tensor(ks)))
        assert np.array_equal(got_y, eager["out"]) and np.array_equal(got_a, eager["argmax"])
        if r == 0:
            ref = net.sparse_forward(xs, ks)
            ok = np.ones(B, bool)
            for l in (0, 1):
                ok &= ~ref["layers"][l]["tie"]
            assert_close_rows(got_y, ref["out"], ok, "recorded forward")
    graph.close()


@pytest.mark.parametrize("path", ["layers", "fused"])
def test_maximum_batch(rt, oracle, path):
    """The documented maximum of 2^20 queries in one call (tiny layers so that the oracle
    finishes in seconds): codes, active lists and outputs of every query."""
    dims = (16, 32, 8)
    layers, net, _ = make_case(oracle, dims, 2, 2, seed=121, hashed=[0])
    g = _gpu_net(rt, layers, net, path=path)
    B = 1 << 20
    X = make_queries(dims, B, seed=122)
    _say(f"maximum batch path={path}")
    ref = net.sparse_forward(X, 0.25)
    got = to_numpy_result(g.sparse_forward(X, 0.25, taps=True))
    tap = ref["layers"][0]
    ok = ~tap["tie"]
    m = int(tap["cnt"][0])
    assert (got["taps"]["cnt"][0] == m).all()
    assert np.array_equal(got["taps"]["codes"][0].view(np.uint32)[ok], tap["codes"][ok])
    assert np.array_equal(got["taps"]["active"][0][ok, :m], tap["active"][ok, :m])
    assert np.array_equal(got["argmax"][ok], ref["argmax"][ok])
    assert_close_rows(got["out"], ref["out"], ok, "maximum batch")
    assert ok.sum() > 0.9 * B
    if path == "layers":
        # compact output of a last layer without a Node Activator: every node, ascending, for all 2^20
        # queries (the batch runs along the grid's x dimension there)
        _say("maximum batch: compact output")
        r = to_numpy_result(g.sparse_forward(X, 0.25, compact=True))
        assert (r["cnt"] == dims[-1]).all()
        assert (r["idx"] == np.arange(dims[-1], dtype=np.int32)[None, :]).all()
        assert_close_rows(r["out"], ref["out"], ok, "maximum batch, compact call")


def test_maximum_batch_wide_hash(rt, oracle):
    """2^20 queries against 128 hash rows: every tile shape of the batch-wide projection kernels puts
    more than 65 535 tiles of queries along the batch, which the launcher cuts into chunks."""
    dims = (16, 160, 4)
    layers, net, _ = make_case(oracle, dims, 4, 32, seed=123, hashed=[0], N_build=64)
    g = _gpu_net(rt, layers, net, path="layers")
    B = 1 << 20
    X = make_queries(dims, B, seed=124)
    _say("maximum batch, 128 hash rows: select on the device")
    sel = g.select(0, X, 0.05)
    codes = sel["codes"].cpu().numpy().view(np.uint32)
    z = sel["z"].cpu().numpy()
    # the oracle on a sample of the queries spread over the whole batch, both chunks included
    pick = np.concatenate([np.arange(0, B, 4099), np.arange(B - 64, B), np.arange((1 << 19) - 32, (1 << 19) + 32)])
    Z = oracle.hash_project(layers[0], X[pick])
    keys, tie = oracle.keys_from_z(Z, 4, 32)
    okq = ~tie
    assert np.array_equal(codes[pick][okq], keys[okq])
    np.testing.assert_allclose(z[pick], Z, rtol=1e-6, atol=1e-6 * float(np.abs(Z).max()))
    active, cnt = net.tables[0].select(keys, np.float32(0.05))
    got_a = sel["active"].cpu().numpy()[pick]
    got_c = sel["cnt"].cpu().numpy()[pick]
    assert np.array_equal(got_c[okq], cnt[okq])
    m = int(cnt[0])
    assert np.array_equal(got_a[okq, :m], active[okq, :m])


def test_two_streams_with_their_own_workspaces_do_not_interfere(rt, oracle):
    """bench.py deals the batches of a step to two HIP streams, each with its own workspace and output
    buffers.  Calls in flight on both streams at once must give, bit for bit, what the same calls
    give one after the other (the library keeps no per-call state outside the workspace), on the
    per-layer path (workspace in use) and on the whole-network kernel."""
    import torch
    from paper_2204_08400_amd import slonn
    B, rounds = 96, 6
    keep = torch.full((1,), 0.2, dtype=torch.float32, device="cuda")
    for path, dims in (("layers", (512, 4096, 520, 10)), ("fused", (256, 1024, 512, 10))):
        layers, net, _ = make_case(oracle, dims, 6, 12, seed=31, kind="clip3", N_build=128)
        Xs = [torch.from_numpy(make_queries(dims, B, seed=700 + i, kind="clip3")).cuda() for i in range(2 * rounds)]
        g = _gpu_net(rt, layers, net, path=path)
        nbytes = slonn.slonn_workspace_bytes(g.model, B)
        lanes = []
        for s in (torch.cuda.current_stream(), torch.cuda.Stream()):
            lanes.append(dict(stream=s, ws=torch.empty(nbytes, dtype=torch.uint8, device="cuda")))
        # one after the other on one stream
        want = []
        for x in Xs:
            y = torch.empty((B, dims[-1]), dtype=torch.float32, device="cuda")
            a = torch.empty(B, dtype=torch.int32, device="cuda")
            slonn.slonn_sparse_forward(g.model, g.tables, slonn.make_input(x=x), B, keep, 0, 0,
                                       slonn.make_output(dense=y, argmax=a), None, lanes[0]["ws"], lanes[0]["stream"])
            want.append((y, a))
        torch.cuda.synchronize()
        # the same calls dealt to the two streams in turn, nothing waited for in between
        _say(f"two streams, path={path}")
        got = []
        lanes[1]["stream"].wait_stream(lanes[0]["stream"])
        for i, x in enumerate(Xs):
            ln = lanes[i % 2]
            y = torch.empty((B, dims[-1]), dtype=torch.float32, device="cuda")
            a = torch.empty(B, dtype=torch.int32, device="cuda")
            slonn.slonn_sparse_forward(g.model, g.tables, slonn.make_input(x=x), B, keep, 0, 0,
                                       slonn.make_output(dense=y, argmax=a), None, ln["ws"], ln["stream"])
            got.append((y, a))
        torch.cuda.synchronize()
        for i, ((y, a), (yw, aw)) in enumerate(zip(got, want)):
            assert torch.equal(y, yw) and torch.equal(a, aw), f"path {path}: call {i} differs when two streams overlap"
        # and the oracle agrees with one of them
        ref = net.sparse_forward(Xs[3].cpu().numpy(), 0.2)
        assert_close_rows(got[3][0].cpu().numpy(), ref["out"], None, "two streams vs oracle",
                          depth=len(layers))
