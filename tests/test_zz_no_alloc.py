"""The entry point that allocates nothing (slonn_sparse_forward_static: the per-batch workspace is a
static device array inside the library) against slonn_sparse_forward with a caller-provided
workspace: same kernels, so every integer result must be identical and the fp32 outputs equal to
the parity bar (they are bit-identical here: the launch sequence does not depend on where the
workspace lies).  Two calls in a row, the second with a smaller batch, so that whatever the first
call left in the shared array is what the second one finds there."""
import numpy as np
import pytest

from paper_2204_08400_amd import workloads as wl

from helpers import assert_close_rows, compare_sparse, make_case, make_queries, to_numpy_result

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _static_forward(g, slonn, torch, X, keep):
    """Network.sparse_forward(taps=True), but through slonn_sparse_forward_static."""
    inp = g.to_input(X)
    B = g.batch_of(inp)
    dev = g.device
    keep_t = torch.full((1,), float(keep), dtype=torch.float32, device=dev)
    n_last = g.dims_out[-1]
    dense = torch.full((B, n_last), -7.0, dtype=torch.float32, device=dev)
    argmax = torch.full((B,), -1, dtype=torch.int32, device=dev)
    out = slonn.make_output(dense=dense, argmax=argmax)
    codes, z, aidx, acnt, lout = [], [], [], [], []
    for l in g.host_layers:
        act = l.K > 0 and l.L > 0
        codes.append(torch.zeros((B, l.L), dtype=torch.int32, device=dev) if act else None)
        z.append(torch.zeros((B, l.K * l.L), dtype=torch.float32, device=dev) if act else None)
        aidx.append(torch.full((B, l.d_out), -1, dtype=torch.int32, device=dev) if act else None)
        acnt.append(torch.zeros(B, dtype=torch.int32, device=dev) if act else None)
        lout.append(torch.empty((B, l.d_out), dtype=torch.float32, device=dev))
    tp = slonn.make_taps(g.n_layers, codes, z, aidx, acnt, lout)
    slonn.slonn_sparse_forward_static(g.model, g.tables, inp, B, keep_t, 0, 0, out, tp)
    torch.cuda.synchronize()
    return {"out": dense, "argmax": argmax, "taps": dict(codes=codes, z=z, active=aidx, cnt=acnt, out=lout)}


def test_static_scratch_forward_matches_workspace_forward(oracle):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("this test needs a GPU (run with -m gpu on an MI355X)")
    from paper_2204_08400_amd import runtime, slonn
    slonn.load()
    dims = (512, 4096, 520, 10)          # 8 MiB of 2 KiB rows: select regroups the lists by row block
    layers, net, _ = make_case(oracle, dims, 6, 12, seed=23, kind="clip3", N_build=128)
    g = runtime.Network(layers)
    g.import_tables(net.export_tables())
    g.set_path("layers")                 # the per-layer path is the one that uses the workspace
    need = slonn.slonn_workspace_bytes(g.model, 70)
    assert need <= slonn.STATIC_SCRATCH_BYTES, need
    for B, keep in ((70, 0.3), (33, 0.1)):      # the second call is the smaller one
        _say(f"static scratch: dims {dims} B={B} keep={keep}")
        X = make_queries(dims, B, seed=41 + B, kind="clip3")
        want = to_numpy_result(g.sparse_forward(X, keep, taps=True))
        got = to_numpy_result(_static_forward(g, slonn, torch, X, keep))
        for l, lay in enumerate(layers):
            if lay.K > 0:
                assert np.array_equal(got["taps"]["codes"][l], want["taps"]["codes"][l]), f"layer {l}: codes"
                assert np.array_equal(got["taps"]["cnt"][l], want["taps"]["cnt"][l]), f"layer {l}: budgets"
                for q in range(B):
                    c = want["taps"]["cnt"][l][q]
                    assert np.array_equal(got["taps"]["active"][l][q, :c], want["taps"]["active"][l][q, :c]), \
                        f"layer {l} query {q}: active list"
            assert_close_rows(got["taps"]["out"][l], want["taps"]["out"][l], what=f"layer {l} output")
        assert np.array_equal(got["argmax"], want["argmax"])
        assert_close_rows(got["out"], want["out"], what="final output")
        # and against the oracle itself, to the same bar as every other parity test
        ref = net.sparse_forward(X, keep)
        rep = compare_sparse(got, ref, layers, f"static scratch B={B}")
        _say(f"  report {rep}")


def test_static_scratch_rejects_a_batch_beyond_the_array(oracle):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("this test needs a GPU (run with -m gpu on an MI355X)")
    from paper_2204_08400_amd import runtime, slonn
    dims = (64, 2048, 10)
    layers, net, _ = make_case(oracle, dims, 4, 8, seed=5, N_build=64)
    g = runtime.Network(layers)
    g.import_tables(net.export_tables())
    B = 8192
    assert slonn.slonn_workspace_bytes(g.model, B) > slonn.STATIC_SCRATCH_BYTES
    x = torch.zeros((B, dims[0]), dtype=torch.float32, device="cuda")
    keep_t = torch.full((1,), 0.5, dtype=torch.float32, device="cuda")
    out = slonn.make_output(dense=torch.empty((B, dims[-1]), dtype=torch.float32, device="cuda"),
                            argmax=torch.empty(B, dtype=torch.int32, device="cuda"))
    _say("static scratch: oversized batch must be refused on the host")
    with pytest.raises(slonn.SlonnError) as e:
        slonn.slonn_sparse_forward_static(g.model, g.tables, slonn.make_input(x=x), B, keep_t, 0, 0, out, None)
    assert e.value.code == -5          # SLONN_ECAP
    assert "static array" in str(e.value)
