"""Shared set-up for the parity tests: seeded synthetic cases and the comparison
rules (bit-exact integers with rounding ties set aside, relative 1e-4 on fp32)."""
from __future__ import annotations

import numpy as np

from paper_2204_08400_amd import workloads as wl

REL_TOL = 1e-4          # fp32 outputs, relative to the largest output of the query-layer


def make_case(oracle, dims, K, L, seed, hashed=None, cap=None, N_build=256, w_dtype=wl.W_F32,
              last_act=wl.ACT_NONE, kind="u01", ell_nnz=0, threads=None, repeat_rows=0, keep_scores=False):
    """Layers with variance-sampled hash nodes, the oracle net with tables built.  repeat_rows = p > 0:
    the rows (and biases) of every activated layer repeat with period p, so that masses of nodes have
    exactly equal activations."""
    layers = wl.make_mlp(dims, seed=seed, w_dtype=w_dtype, last_act=last_act)
    if repeat_rows:
        for l in (range(len(layers) - 1) if hashed is None else hashed):
            lay = layers[l]
            src = np.arange(lay.d_out) % repeat_rows
            lay.W = np.ascontiguousarray(lay.W[src])
            lay.bias = np.ascontiguousarray(lay.bias[src])
    hashed = list(range(len(layers) - 1)) if hashed is None else list(hashed)
    if ell_nnz:
        Xb = wl.inputs_ell(N_build, dims[0], ell_nnz, seed + 1)
    elif kind == "u01":
        Xb = wl.inputs_uniform_half_zero(N_build, dims[0], seed + 1)
    else:
        Xb = wl.inputs_normal_clipped(N_build, dims[0], seed + 1, 3.0 if kind == "clip3" else None)
    net = oracle.OracleNet(layers, threads=threads)
    dense = net.dense_forward(Xb, upto=(max(hashed) + 1) if hashed else 0)
    for l in hashed:
        lay = layers[l]
        lay.K, lay.L = K, L
        lay.list_cap = lay.d_out if cap is None else cap
        lay.hash_nodes = oracle.sample_hash_nodes(oracle.activation_variance(dense[l]), K, L,
                                                  wl.hash_node_draws(K, L, seed + 3 + l))
    net.build_tables(Xb, keep_scores=keep_scores)
    return layers, net, Xb


def make_queries(dims, N, seed, kind="u01", ell_nnz=0):
    if ell_nnz:
        return wl.inputs_ell(N, dims[0], ell_nnz, seed)
    if kind == "u01":
        return wl.inputs_uniform_half_zero(N, dims[0], seed)
    return wl.inputs_normal_clipped(N, dims[0], seed, 3.0 if kind == "clip3" else None)


def assert_close_rows(got: np.ndarray, ref: np.ndarray, rows=None, what="", depth=1):
    """Per query: max|g-o| <= tol*max|o| and element-wise |g-o| <= tol*|o| + depth*1e-6*max|o|.
    depth = number of layers whose fp32 rounding the values carry (1 for a first layer): an output
    near zero is a cancellation of terms of the size of max|o|, so its error does not shrink with
    it, and a layer's inputs carry the rounding of every layer before it."""
    if rows is not None:
        got, ref = got[rows], ref[rows]
    if ref.size == 0:
        return 0.0
    scale = np.maximum(np.abs(ref).max(axis=1, keepdims=True), 1e-30)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    worst = float((err / scale).max())
    assert worst <= REL_TOL, f"{what}: max error {worst:.3e} of the row maximum"
    bound = REL_TOL * np.abs(ref) + depth * 1e-6 * scale
    bad = err > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements beyond the element-wise bound "
                           f"(worst error / bound {float((err / bound).max()):.2f})")
    return worst


def compare_sparse(res_gpu: dict, res_ref: dict, layers, what="", max_tainted=None):
    """Compare a GPU sparse forward (with taps, as numpy) with the oracle's.

    A query is *tainted* from the first layer on where one of its hash projections
    lies within 1e-6 of zero (its key then depends on summation order); tainted
    queries are set aside and counted, everything else must agree: codes and active
    lists bit for bit, outputs to REL_TOL, argmax exactly.  At most max_tainted queries may be
    set aside (default: 2, or 1 % of the queries if that is more; a test that plants ties says
    how many it expects).  Returns a report dict.
    """
    N = res_ref["out"].shape[0]
    tainted = np.zeros(N, bool)
    rep = {"queries": N, "code_mismatch_in_tie_zone": 0, "max_rel_err": 0.0}
    for l, lay in enumerate(layers):
        ref = res_ref["layers"][l]
        g = res_gpu["taps"]
        if lay.K > 0 and lay.L > 0:
            tainted |= ref["tie"]
            ok = ~tainted
            codes_g = g["codes"][l].view(np.uint32) if g["codes"][l].dtype != np.uint32 else g["codes"][l]
            mism = (codes_g != ref["codes"]).any(axis=1)
            rep["code_mismatch_in_tie_zone"] += int((mism & tainted).sum())
            assert not (mism & ok).any(), f"{what} layer {l}: {int((mism & ok).sum())} code mismatches outside the tie zone"
            # a tainted query whose codes nevertheless agree is still comparable at this layer
            assert np.array_equal(g["cnt"][l][ok], ref["cnt"][ok]), f"{what} layer {l}: budgets differ"
            for q in np.nonzero(ok)[0]:
                c = ref["cnt"][q]
                assert np.array_equal(g["active"][l][q, :c], ref["active"][q, :c]), \
                    f"{what} layer {l} query {q}: active list differs"
            # projections of layer l > 0 inherit the fp32 rounding of the previous layer's output
            zs = max(float(np.abs(ref["z"]).max()), 1e-30)
            np.testing.assert_allclose(g["z"][l][ok], ref["z"][ok], rtol=REL_TOL, atol=1e-6 * zs,
                                       err_msg=f"{what} layer {l}: hash projections")
        ok = ~tainted
        rep["max_rel_err"] = max(rep["max_rel_err"],
                                 assert_close_rows(g["out"][l], ref["out"], ok, f"{what} layer {l} output",
                                                   depth=l + 1))
        # dropped nodes are exactly +0 on both sides
        if lay.act == wl.ACT_RELU:
            assert not np.signbit(g["out"][l]).any(), f"{what} layer {l}: negative zero or value after ReLU"
        if lay.K > 0:
            for q in np.nonzero(ok)[0][:64]:
                mask = np.ones(lay.d_out, bool)
                mask[ref["active"][q, :ref["cnt"][q]]] = False
                assert not g["out"][l][q, mask].any(), f"{what} layer {l} query {q}: dropped node not zero"
    ok = ~tainted
    assert np.array_equal(res_gpu["argmax"][ok], res_ref["argmax"][ok]), f"{what}: argmax differs"
    assert_close_rows(res_gpu["out"], res_ref["out"], ok, f"{what} final output", depth=len(layers))
    rep["tainted"] = int(tainted.sum())
    limit = max(2, -(-N // 100)) if max_tainted is None else max_tainted
    assert rep["tainted"] <= limit, f"{what}: {rep['tainted']} of {N} queries set aside as ties (limit {limit})"
    return rep


def to_numpy_result(res: dict) -> dict:
    """GPU result (torch tensors) -> numpy, same structure."""
    def cv(t):
        return None if t is None else t.detach().cpu().numpy()
    out = {"out": cv(res.get("out")), "argmax": cv(res["argmax"])}
    if "taps" in res:
        out["taps"] = {k: [cv(t) for t in v] for k, v in res["taps"].items()}
    for k in ("idx", "val", "cnt"):
        if k in res:
            out[k] = cv(res[k])
    return out
