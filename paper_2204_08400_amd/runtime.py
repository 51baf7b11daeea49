"""Convenience holder around the C-ABI binding: uploads a synthetic network's
arrays with PyTorch (device memory only), keeps the handles and the workspace,
and returns outputs as tensors.  No arithmetic happens here."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import slonn


def _dev(a: np.ndarray, device):
    if a.dtype == np.uint16:          # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16).copy()).to(device)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32).copy()).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def hash_nodes_by_variance(acts: torch.Tensor, K: int, L: int, u: np.ndarray) -> np.ndarray:
    """K*L hash nodes of a layer from its activations [N][n] over the tables' training set
    (device tensor): variance on the device, the draws u consumed by the library's sampler."""
    var = torch.empty(acts.shape[1], dtype=torch.float64, device=acts.device)
    slonn.slonn_activation_variance(acts, var)
    ud = torch.from_numpy(np.ascontiguousarray(u, np.float64)).to(acts.device)
    out = torch.empty(K * L, dtype=torch.int32, device=acts.device)
    slonn.slonn_sample_hash_nodes_device(var, K, L, ud, out)
    return out.cpu().numpy()          # model creation takes the ids from the host


class Network:
    def __init__(self, layers: Sequence, device="cuda:0", first_layer_rows_are_inputs=False):
        """layers: workloads.LayerData-like objects (host numpy arrays)."""
        self.device = torch.device(device)
        self.host_layers = list(layers)
        descs = []
        for i, l in enumerate(layers):
            descs.append(dict(
                d_in=l.d_in, d_out=l.d_out, w_dtype=l.w_dtype, act=l.act, K=l.K, L=l.L,
                list_cap=l.list_cap,
                w_layout=slonn.ROWS_ARE_INPUTS if (i == 0 and first_layer_rows_are_inputs) else slonn.ROWS_ARE_NODES,
                W=_dev(np.ascontiguousarray(l.W), self.device), bias=_dev(l.bias, self.device),
                hash_nodes=None if l.hash_nodes is None else [int(v) for v in l.hash_nodes]))
        self.model = slonn.slonn_model_create(descs)
        self.n_layers = len(descs)
        self.dims_out = [l.d_out for l in layers]
        self.tables: Optional[slonn.Tables] = None
        self._ws = None
        self._ws_B = 0

    def set_path(self, path: str):
        """'auto' | 'layers' | 'fused' (raises if the model does not qualify)."""
        slonn.slonn_model_set_path(self.model, {"auto": 0, "layers": 1, "fused": 2}[path])

    def set_hash_nodes_always_active(self, on: bool):
        """Hash nodes always computed and never selected (see slonn.h)."""
        slonn.slonn_model_set_hash_nodes_always_active(self.model, on)

    def set_batches_in_flight(self, n: int):
        """Batches kept in flight on separate streams (a hint, see slonn.h)."""
        slonn.slonn_model_set_batches_in_flight(self.model, n)

    def set_hash_margin(self, margin: float):
        """Certification margin of the integer hash projections (diagnostic, see slonn.h)."""
        slonn.slonn_model_set_hash_margin(self.model, margin)

    # -- helpers -------------------------------------------------------------- #
    def workspace(self, B: int):
        if self._ws is None or B > self._ws_B:
            nbytes = slonn.slonn_workspace_bytes(self.model, B)
            self._ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self._ws_B = B
        return self._ws

    def to_input(self, X) -> slonn.Input:
        if isinstance(X, slonn.Input):
            return X
        if isinstance(X, tuple):
            idx, val, nnz = (t if torch.is_tensor(t) else _dev(np.ascontiguousarray(t), self.device) for t in X)
            return slonn.make_input(idx=idx, val=val, nnz=nnz)
        x = X if torch.is_tensor(X) else _dev(np.ascontiguousarray(X, np.float32), self.device)
        return slonn.make_input(x=x)

    @staticmethod
    def batch_of(inp: slonn.Input) -> int:
        x, idx, _, _ = inp._keep
        return int(x.shape[0] if x is not None else idx.shape[0])

    # -- tables --------------------------------------------------------------- #
    def build_tables(self, X_build):
        inp = self.to_input(X_build)
        self.tables = slonn.slonn_build_tables(self.model, inp, self.batch_of(inp))
        return self.tables

    def set_tables_refreshable(self, on: bool):
        """Before build_tables: keep the NodeScore sums so that refresh_tables can continue Alg. 1."""
        slonn.slonn_model_set_tables_refreshable(self.model, on)

    def refresh_tables(self, X_new):
        inp = self.to_input(X_new)
        slonn.slonn_tables_refresh(self.model, self.tables, inp, self.batch_of(inp))
        return self.tables

    def import_tables(self, blob: bytes):
        self.tables = slonn.slonn_tables_import(self.model, blob)
        return self.tables

    def export_tables(self) -> bytes:
        return slonn.slonn_tables_export(self.tables)

    # -- forward -------------------------------------------------------------- #
    def sparse_forward(self, X, keep, taps: bool = False, compact: bool = False, dense: bool = True,
                       policy=None, thr=None):
        """keep: device float tensor [B] or [B][n_layers], or a python float.  With a policy
        (slonn.Policy) and thr (device float tensor [B] or a python float) k is chosen inside the
        pass under ACLO, keep is ignored and the chosen fractions come back as res["keep"]."""
        inp = self.to_input(X)
        B = self.batch_of(inp)
        dev = self.device
        if policy is not None:
            if not torch.is_tensor(thr):
                thr = torch.full((1,), float(thr), dtype=torch.float32, device=dev)
            keep = torch.zeros(B, dtype=torch.float32, device=dev)
            qs, ls = 1, 0
        elif not torch.is_tensor(keep):
            keep = torch.full((1,), float(keep), dtype=torch.float32, device=dev)
            qs, ls = 0, 0
        elif keep.dim() == 1:
            qs, ls = (1 if keep.numel() > 1 else 0), 0
        else:
            qs, ls = keep.shape[1], 1
        n_last = self.dims_out[-1]
        res = {}
        dense = torch.empty((B, n_last), dtype=torch.float32, device=dev) if dense else None
        argmax = torch.empty(B, dtype=torch.int32, device=dev)
        kw = dict(dense=dense, argmax=argmax)
        if compact:
            res["idx"] = torch.full((B, n_last), -1, dtype=torch.int32, device=dev)
            res["val"] = torch.zeros((B, n_last), dtype=torch.float32, device=dev)
            res["cnt"] = torch.zeros(B, dtype=torch.int32, device=dev)
            kw.update(idx=res["idx"], val=res["val"], cnt=res["cnt"], stride=n_last)
        out = slonn.make_output(**kw)
        tp = None
        if taps:
            codes, z, aidx, acnt, lout = [], [], [], [], []
            for l in self.host_layers:
                act = l.K > 0 and l.L > 0
                codes.append(torch.zeros((B, l.L), dtype=torch.int32, device=dev) if act else None)
                z.append(torch.zeros((B, l.K * l.L), dtype=torch.float32, device=dev) if act else None)
                aidx.append(torch.full((B, l.d_out), -1, dtype=torch.int32, device=dev) if act else None)
                acnt.append(torch.zeros(B, dtype=torch.int32, device=dev) if act else None)
                lout.append(torch.empty((B, l.d_out), dtype=torch.float32, device=dev))
            tp = slonn.make_taps(self.n_layers, codes, z, aidx, acnt, lout)
            res["taps"] = dict(codes=codes, z=z, active=aidx, cnt=acnt, out=lout)
        if policy is not None:
            slonn.slonn_sparse_forward_aclo(self.model, self.tables, policy, inp, B, thr,
                                            1 if thr.numel() > 1 else 0, keep, out, tp, self.workspace(B))
            res["keep"] = keep
        else:
            slonn.slonn_sparse_forward(self.model, self.tables, inp, B, keep, qs, ls, out, tp, self.workspace(B))
        res["out"], res["argmax"] = dense, argmax
        return res

    def dense_forward(self, X, layer_outs: bool = False):
        inp = self.to_input(X)
        B = self.batch_of(inp)
        dev = self.device
        Y = torch.empty((B, self.dims_out[-1]), dtype=torch.float32, device=dev)
        argmax = torch.empty(B, dtype=torch.int32, device=dev)
        louts = None
        if layer_outs:
            louts = [torch.empty((B, n), dtype=torch.float32, device=dev) for n in self.dims_out]
        slonn.slonn_dense_forward(self.model, inp, B, Y, argmax, louts, self.workspace(B))
        return {"out": Y, "argmax": argmax, "layers": louts}

    def select(self, layer: int, X_l, keep):
        l = self.host_layers[layer]
        x = X_l if torch.is_tensor(X_l) else _dev(np.ascontiguousarray(X_l, np.float32), self.device)
        B = x.shape[0]
        dev = self.device
        if not torch.is_tensor(keep):
            keep = torch.full((1,), float(keep), dtype=torch.float32, device=dev)
        ks = 1 if keep.numel() > 1 else 0
        codes = torch.zeros((B, l.L), dtype=torch.int32, device=dev)
        z = torch.zeros((B, l.K * l.L), dtype=torch.float32, device=dev)
        aidx = torch.full((B, l.d_out), -1, dtype=torch.int32, device=dev)
        acnt = torch.zeros(B, dtype=torch.int32, device=dev)
        slonn.slonn_select(self.model, self.tables, layer, x, B, keep, ks, codes, z, aidx, acnt, l.d_out,
                           self.workspace(B))
        return {"codes": codes, "z": z, "active": aidx, "cnt": acnt}
