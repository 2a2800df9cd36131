"""ctypes front end of the CPU oracle interpreter (`interp.c`).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the CPU
baseline leg of the benchmark; never by the product path.

`Oracle(graph, params, real="f64")` evaluates the graph one node at a time in
id order (Section 3.3) and differentiates it in reverse id order; values and
gradients come back as flat arrays in node-id order with `v_off` offsets.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_LIBS = {}


def lib_path(real: str) -> Path:
    return _HERE / f"_interp_{real}.so"


def build(force: bool = False) -> None:
    """Compile interp.c twice with gcc: fp64 (reference) and fp32 (timed baseline)."""
    src = _HERE / "interp.c"
    for real, ctype in (("f64", "double"), ("f32", "float")):
        out = lib_path(real)
        if not force and out.exists() and out.stat().st_mtime >= src.stat().st_mtime:
            continue
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", f"-DREAL={ctype}",
               str(src), "-o", str(out), "-lm"]
        subprocess.run(cmd, check=True)


class _GraphT(ctypes.Structure):
    _fields_ = [
        ("n", ctypes.c_int64),
        ("op", ctypes.c_void_p), ("out_dim", ctypes.c_void_p),
        ("in_off", ctypes.c_void_p), ("in_idx", ctypes.c_void_p),
        ("param", ctypes.c_void_p), ("bias", ctypes.c_void_p),
        ("aux0", ctypes.c_void_p), ("aux1", ctypes.c_void_p),
        ("payload", ctypes.c_void_p),
        ("n_params", ctypes.c_int64),
        ("p_rows", ctypes.c_void_p), ("p_cols", ctypes.c_void_p),
        ("p_off", ctypes.c_void_p), ("v_off", ctypes.c_void_p),
    ]


def _load(real: str):
    if real not in _LIBS:
        build()
        lib = ctypes.CDLL(str(lib_path(real)))
        lib.oracle_forward.restype = ctypes.c_int
        lib.oracle_forward.argtypes = [ctypes.POINTER(_GraphT), ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_backward.restype = ctypes.c_int
        lib.oracle_backward.argtypes = [ctypes.POINTER(_GraphT), ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_real_bytes.restype = ctypes.c_int
        assert lib.oracle_real_bytes() == (8 if real == "f64" else 4)
        _LIBS[real] = lib
    return _LIBS[real]


class Oracle:
    def __init__(self, graph, params, real: str = "f64", n_nodes: int | None = None):
        self.real = real
        self.dtype = np.float64 if real == "f64" else np.float32
        self.lib = _load(real)
        g = graph
        n = g.n if n_nodes is None else int(n_nodes)
        self.n = n
        c = np.ascontiguousarray
        self._keep = dict(
            op=c(g.op, np.uint8), out_dim=c(g.out_dim, np.uint32), in_off=c(g.in_off, np.uint32),
            in_idx=c(g.in_idx, np.uint32) if g.in_idx.size else np.zeros(1, np.uint32),
            param=c(g.param, np.int32), bias=c(g.bias, np.int32),
            aux0=c(g.aux0, np.int32), aux1=c(g.aux1, np.int32),
            payload=c(g.payload, np.float32) if g.payload.size else np.zeros(1, np.float32))
        mats = params.mats
        self.p_rows = np.asarray([m.shape[0] for m in mats], np.int64)
        self.p_cols = np.asarray([m.shape[1] for m in mats], np.int64)
        sizes = self.p_rows * self.p_cols
        self.p_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        self.pdata = (np.concatenate([m.reshape(-1) for m in mats]).astype(self.dtype)
                      if mats else np.zeros(1, self.dtype))
        self.v_off = np.concatenate([[0], np.cumsum(g.out_dim[:n].astype(np.int64))]).astype(np.int64)
        k = self._keep
        self.gt = _GraphT(
            n, k["op"].ctypes.data, k["out_dim"].ctypes.data, k["in_off"].ctypes.data,
            k["in_idx"].ctypes.data, k["param"].ctypes.data, k["bias"].ctypes.data,
            k["aux0"].ctypes.data, k["aux1"].ctypes.data, k["payload"].ctypes.data,
            len(mats), self.p_rows.ctypes.data, self.p_cols.ctypes.data,
            self.p_off.ctypes.data, self.v_off.ctypes.data)
        self.val = None
        self.grad = None
        self.pgrad = None

    def set_params(self, flat: np.ndarray) -> None:
        self.pdata = np.ascontiguousarray(flat, self.dtype)

    def forward(self) -> np.ndarray:
        self.val = np.empty(max(1, int(self.v_off[-1])), self.dtype)
        rc = self.lib.oracle_forward(ctypes.byref(self.gt), self.pdata.ctypes.data,
                                     self.val.ctypes.data)
        if rc != 0:
            raise RuntimeError(f"oracle_forward failed: {rc}")
        return self.val

    def backward(self, root: int) -> None:
        assert self.val is not None
        self.grad = np.empty_like(self.val)
        self.pgrad = np.empty(max(1, int(self.p_off[-1])), self.dtype)
        rc = self.lib.oracle_backward(ctypes.byref(self.gt), self.pdata.ctypes.data,
                                      self.val.ctypes.data, int(root),
                                      self.grad.ctypes.data, self.pgrad.ctypes.data)
        if rc != 0:
            raise RuntimeError(f"oracle_backward failed: {rc}")

    def value(self, v: int) -> np.ndarray:
        return self.val[self.v_off[v]:self.v_off[v + 1]]

    def node_grad(self, v: int) -> np.ndarray:
        return self.grad[self.v_off[v]:self.v_off[v + 1]]

    def param_grad(self, p: int) -> np.ndarray:
        return self.pgrad[self.p_off[p]:self.p_off[p + 1]].reshape(self.p_rows[p], self.p_cols[p])

    def sgd_params(self, lr: float) -> list:
        """Parameters after one plain gradient-descent update (Section 2, the update that closes
        each training step): theta - lr * dL/dtheta, per parameter, in the oracle's precision."""
        assert self.pgrad is not None
        out = []
        for p in range(len(self.p_rows)):
            theta = self.pdata[self.p_off[p]:self.p_off[p + 1]].reshape(self.p_rows[p], self.p_cols[p])
            out.append(theta - lr * self.param_grad(p))
        return out
