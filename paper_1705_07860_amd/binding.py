"""Thin ctypes binding over libob.so: argument marshalling only.

Every step of the path (scheduling, batched forward, batched backward) runs in the HIP
library; this module allocates the device arena through PyTorch (`torch.empty` on cuda) and
hands raw pointers across the C ABI.  Function names mirror include/ob.h.

If the library has not been built, or there is no GPU when a device call is made, this fails
loudly; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
from ctypes import POINTER, byref, c_float, c_int, c_int32, c_size_t, c_uint8, c_uint32, c_uint64, c_void_p
from pathlib import Path

import numpy as np

HERE = Path(__file__).resolve().parent
LIB_PATH = HERE / "libob.so"

OB_NOBATCH, OB_BYDEPTH, OB_BYAGENDA, OB_MANUAL = 0, 1, 2, 3
OB_LAUNCH_STREAM, OB_LAUNCH_GRAPH, OB_LAUNCH_PERSISTENT = 0, 1, 2
OB_DBG_DEPTH, OB_DBG_SIG, OB_DBG_SUCC_OFF, OB_DBG_SUCC_EDGE, OB_DBG_ORDER, OB_DBG_VAL_OFF = range(6)
OB_DBG_TILES_FWD, OB_DBG_TILES_PULL, OB_DBG_CHAINS, OB_DBG_LORDER = 6, 7, 8, 9
OB_DBG_SET_DEPTH_SPIN = 0
OB_DBG_SET_CONCAT_COPY = 1

ERRORS = {0: "OB_OK", -1: "OB_E_BADID", -2: "OB_E_DIM", -3: "OB_E_RANGE", -4: "OB_E_NOTSCALAR",
          -5: "OB_E_OOM", -6: "OB_E_STATE", -7: "OB_E_HIP", -8: "OB_E_ARG"}


class ObError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{ERRORS.get(code, code)}: {msg}")
        self.code = code


class ObStats(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in (
        "n_nodes", "n_edges", "n_steps", "n_batches", "n_tiles_fwd", "n_tiles_bwd_pull", "n_tiles_bwd_dx",
        "n_param_uses", "n_launch_fwd", "n_launch_bwd", "n_launch_sched", "n_slots")] + \
        [(n, c_uint64) for n in ("value_floats", "grad_floats", "arena_used_bytes", "upload_bytes")] + \
        [(n, c_float) for n in ("ms_upload", "ms_schedule", "ms_forward", "ms_backward", "ms_param_grads",
                                "ms_graph_build")] + \
        [(n, c_int32) for n in ("n_stages", "n_proxies", "n_depth_retries", "n_launch_bwd_steps",
                                "n_view_batches", "n_uncopied_batches")] + \
        [(n, c_uint64) for n in ("view_floats", "uncopied_floats")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_ if not n.startswith("reserved")}


_lib = None


def lib():
    """Loads libob.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_1705_07860_amd.build` "
                               "(there is no fallback path)")
        # PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  It must be in the process
        # before libob.so so that the loader binds the library to that same runtime instance;
        # two runtimes in one process cannot share device pointers or streams.
        import torch  # noqa: F401
        hip_rt = Path(torch.__file__).resolve().parent / "lib" / "libamdhip64.so"
        if hip_rt.exists():
            ctypes.CDLL(str(hip_rt), mode=ctypes.RTLD_GLOBAL)
        L = ctypes.CDLL(str(LIB_PATH))
        vp, i, sz = c_void_p, c_int, c_size_t
        pf, pi = POINTER(c_float), POINTER(c_int)
        sigs = {
            "ob_ctx_create": (i, [vp, sz, vp, POINTER(vp)]),
            "ob_ctx_destroy": (i, [vp]),
            "ob_ctx_fork": (i, [vp, vp, sz, vp, POINTER(vp)]),
            "ob_ctx_set_schedule_stream": (i, [vp, vp]),
            "ob_schedule": (i, [vp, i]),
            "ob_schedule_async": (i, [vp, i]),
            "ob_ctx_set_mode": (i, [vp, i]),
            "ob_ctx_set_launch": (i, [vp, i]),
            "ob_ctx_set_fusion": (i, [vp, i]),
            "ob_last_error": (ctypes.c_char_p, [vp]),
            "ob_param_create": (i, [vp, i, i, vp, pi]),
            "ob_param_write": (i, [vp, i, vp]),
            "ob_param_read": (i, [vp, i, vp, sz]),
            "ob_param_grad_zero": (i, [vp]),
            "ob_param_grad_read": (i, [vp, i, vp, sz]),
            "ob_graph_new": (i, [vp]),
            "ob_graph_size": (i, [vp, pi, pi]),
            "ob_add_input": (i, [vp, i, vp]),
            "ob_add_lookup": (i, [vp, i, i]),
            "ob_add_matvec": (i, [vp, i, i, i]),
            "ob_add_unary": (i, [vp, i, i]),
            "ob_add_nary": (i, [vp, i, i, vp]),
            "ob_add_slice": (i, [vp, i, i, i]),
            "ob_add_pick_nls": (i, [vp, i, i]),
            "ob_add_sqnorm": (i, [vp, i]),
            "ob_add_bulk": (i, [vp, i, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz]),
            "ob_set_manual_batches": (i, [vp, vp, sz]),
            "ob_upload": (i, [vp]),
            "ob_forward": (i, [vp, i]),
            "ob_backward": (i, [vp, i]),
            "ob_sync": (i, [vp]),
            "ob_reset": (i, [vp]),
            "ob_value_read": (i, [vp, i, vp, sz]),
            "ob_grad_read": (i, [vp, i, vp, sz]),
            "ob_all_read": (i, [vp, i, vp, sz]),
            "ob_schedule_read": (i, [vp, pi, vp, vp, vp, vp, sz, sz]),
            "ob_stats_read": (i, [vp, POINTER(ObStats)]),
            "ob_debug_read": (i, [vp, i, vp, sz, POINTER(sz)]),
            "ob_debug_set": (i, [vp, i, c_uint64]),
            "ob_param_sgd_step": (i, [vp, c_float, i]),
            "ob_test_sort": (i, [vp, sz, vp, vp, i, i, vp, vp]),
            "ob_sort_pairs_noalloc": (i, [vp, sz, vp, vp, i, i]),
            "ob_stream_create_on_cus": (i, [i, i, POINTER(vp)]),
            "ob_stream_destroy": (i, [vp]),
            "ob_test_scan": (i, [vp, sz, vp, vp, vp]),
            "ob_test_gemm": (i, [vp, i, i, i, vp, vp, vp]),
            "ob_test_launch_cost": (i, [vp, i, i, POINTER(c_float)]),
        }
        for name, (res, args) in sigs.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        L._ob_names = list(sigs)
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(c_void_p)


OB_NOALLOC_MAX_PAIRS = 262144


def sort_pairs_noalloc(stream_ptr, n: int, keys_ptr: int, vals_ptr: int, lo_bit: int, n_bits: int):
    """ob_sort_pairs_noalloc on raw device pointers (allocates nothing); raises ObError on failure."""
    L = lib()
    rc = L.ob_sort_pairs_noalloc(c_void_p(stream_ptr), n, c_void_p(keys_ptr), c_void_p(vals_ptr), lo_bit, n_bits)
    if rc < 0:
        raise ObError(rc, (L.ob_last_error(None) or b"").decode())


def stream_create_on_cus(first_cu: int, n_cus: int) -> int:
    """ob_stream_create_on_cus: the raw hipStream_t (wrap it with torch.cuda.ExternalStream to record events on it)."""
    L = lib()
    h = c_void_p()
    rc = L.ob_stream_create_on_cus(first_cu, n_cus, ctypes.byref(h))
    if rc < 0:
        raise ObError(rc, (L.ob_last_error(None) or b"").decode())
    return h.value


def stream_destroy(stream_ptr: int):
    L = lib()
    rc = L.ob_stream_destroy(c_void_p(stream_ptr))
    if rc < 0:
        raise ObError(rc, (L.ob_last_error(None) or b"").decode())


class Context:
    """One library context over a caller-owned device arena (a torch uint8 CUDA tensor) and
    stream.  `arena_bytes=0` builds a host-only context (graph definition and validation work,
    device calls fail)."""

    def __init__(self, arena_bytes: int = 1 << 30, stream=None, mode: int = OB_BYDEPTH,
                 launch: int = OB_LAUNCH_STREAM, parent: "Context | None" = None, sched_stream=None):
        self.L = lib()
        self._arena = None
        self._parent = parent
        ptr, stream_ptr = None, None
        if arena_bytes:
            import torch
            if not torch.cuda.is_available():
                raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
            self._arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
            ptr = self._arena.data_ptr()
            # a stream of its own (default priority): the legacy default stream cannot be captured
            s = stream if stream is not None else torch.cuda.Stream()
            self._stream = s
            stream_ptr = s.cuda_stream
        self.h = c_void_p()
        if parent is not None:
            rc = self.L.ob_ctx_fork(parent.h, c_void_p(ptr), arena_bytes, c_void_p(stream_ptr), byref(self.h))
            if rc:
                raise ObError(rc, (self.L.ob_last_error(parent.h) or b"").decode())
        else:
            rc = self.L.ob_ctx_create(c_void_p(ptr), arena_bytes, c_void_p(stream_ptr), byref(self.h))
            if rc:
                raise ObError(rc, (self.L.ob_last_error(None) or b"").decode())
            self.set_mode(mode)
            self.set_launch(launch)
        if sched_stream is not None:
            self._sched_stream = sched_stream
            self._ck(self.L.ob_ctx_set_schedule_stream(self.h, c_void_p(sched_stream.cuda_stream)))

    # -- plumbing
    def _ck(self, rc: int) -> int:
        if rc < 0:
            raise ObError(rc, (self.L.ob_last_error(self.h) or b"").decode())
        return rc

    def close(self):
        if self.h:
            self.L.ob_ctx_destroy(self.h)
            self.h = c_void_p()
        self._arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_schedule_stream(self, stream):
        """Upload and scheduling go to `stream` (a torch stream) from the next upload on; only while no graph is on the device."""
        self._sched_stream = stream
        self._ck(self.L.ob_ctx_set_schedule_stream(self.h, c_void_p(stream.cuda_stream)))

    def set_mode(self, mode: int):
        self._ck(self.L.ob_ctx_set_mode(self.h, mode))

    def set_launch(self, launch: int):
        self._ck(self.L.ob_ctx_set_launch(self.h, launch))

    def sgd_step(self, lr: float, zero_grad: bool = True):
        self._ck(self.L.ob_param_sgd_step(self.h, float(lr), 1 if zero_grad else 0))

    def set_fusion(self, on):
        """0 / False: one launch per depth level; 1 / True: fused, early placement; 2: fused, late placement."""
        self._ck(self.L.ob_ctx_set_fusion(self.h, int(on)))

    # -- parameters
    def param_create(self, mat: np.ndarray) -> int:
        m = np.ascontiguousarray(mat, np.float32)
        assert m.ndim == 2
        out = c_int()
        self._ck(self.L.ob_param_create(self.h, m.shape[0], m.shape[1], _ptr(m), byref(out)))
        return out.value

    def params_create(self, params) -> list:
        return [self.param_create(m) for m in params.mats]

    def param_write(self, pid: int, mat: np.ndarray):
        m = np.ascontiguousarray(mat, np.float32)
        self._ck(self.L.ob_param_write(self.h, pid, _ptr(m)))

    def param_read(self, pid: int, shape) -> np.ndarray:
        out = np.empty(shape, np.float32)
        self._ck(self.L.ob_param_read(self.h, pid, _ptr(out), out.size))
        return out

    def param_grad_zero(self):
        self._ck(self.L.ob_param_grad_zero(self.h))

    def param_grad_read(self, pid: int, shape) -> np.ndarray:
        out = np.empty(shape, np.float32)
        self._ck(self.L.ob_param_grad_read(self.h, pid, _ptr(out), out.size))
        return out

    # -- graph definition
    def graph_new(self):
        self._ck(self.L.ob_graph_new(self.h))

    def graph_size(self):
        n, e = c_int(), c_int()
        self._ck(self.L.ob_graph_size(self.h, byref(n), byref(e)))
        return n.value, e.value

    def add_input(self, vec) -> int:
        v = np.ascontiguousarray(vec, np.float32).reshape(-1)
        return self._ck(self.L.ob_add_input(self.h, v.shape[0], _ptr(v)))

    def add_lookup(self, table: int, row: int) -> int:
        return self._ck(self.L.ob_add_lookup(self.h, table, row))

    def add_matvec(self, w: int, b: int, x: int) -> int:
        return self._ck(self.L.ob_add_matvec(self.h, w, b, x))

    def add_unary(self, op: int, x: int) -> int:
        return self._ck(self.L.ob_add_unary(self.h, op, x))

    def add_nary(self, op: int, xs) -> int:
        a = np.ascontiguousarray(xs, np.int32)
        return self._ck(self.L.ob_add_nary(self.h, op, a.shape[0], _ptr(a)))

    def add_slice(self, x: int, lo: int, hi: int) -> int:
        return self._ck(self.L.ob_add_slice(self.h, x, lo, hi))

    def add_pick_nls(self, x: int, label: int) -> int:
        return self._ck(self.L.ob_add_pick_nls(self.h, x, label))

    def add_sqnorm(self, x: int) -> int:
        return self._ck(self.L.ob_add_sqnorm(self.h, x))

    def add_bulk(self, g) -> int:
        """Appends a whole workloads.Graph (flat arrays) in one call."""
        c = np.ascontiguousarray
        arrs = [c(g.op, np.uint8), c(g.out_dim, np.uint32), c(g.in_off, np.uint32),
                c(g.in_idx, np.uint32) if g.in_idx.size else np.zeros(1, np.uint32),
                c(g.param, np.int32), c(g.bias, np.int32), c(g.aux0, np.int32), c(g.aux1, np.int32),
                c(g.payload, np.float32) if g.payload.size else np.zeros(1, np.float32)]
        return self._ck(self.L.ob_add_bulk(self.h, int(g.op.shape[0]), *[_ptr(a) for a in arrs],
                                           int(g.payload.size)))

    def set_manual_batches(self, batch_of_node):
        """Manual batching: one batch label per node of the current graph (see OB_MANUAL)."""
        a = np.ascontiguousarray(batch_of_node, np.int32)
        self._ck(self.L.ob_set_manual_batches(self.h, _ptr(a), int(a.shape[0])))

    # -- execution
    def upload(self):
        self._ck(self.L.ob_upload(self.h))

    def fork(self, arena_bytes: int = 1 << 30, stream=None, sched_stream=None) -> "Context":
        """A context with its own graph, arena and stream that shares this one's parameters."""
        return Context(arena_bytes=arena_bytes, stream=stream, parent=self, sched_stream=sched_stream)

    def schedule(self, node: int):
        self._ck(self.L.ob_schedule(self.h, node))

    def schedule_async(self, node: int):
        self._ck(self.L.ob_schedule_async(self.h, node))

    def forward(self, node: int):
        self._ck(self.L.ob_forward(self.h, node))

    def backward(self, node: int):
        self._ck(self.L.ob_backward(self.h, node))

    def sync(self):
        self._ck(self.L.ob_sync(self.h))

    def reset(self):
        self._ck(self.L.ob_reset(self.h))

    # -- reads
    def value_read(self, node: int, dim: int) -> np.ndarray:
        out = np.empty(dim, np.float32)
        self._ck(self.L.ob_value_read(self.h, node, _ptr(out), dim))
        return out

    def grad_read(self, node: int, dim: int) -> np.ndarray:
        out = np.empty(dim, np.float32)
        self._ck(self.L.ob_grad_read(self.h, node, _ptr(out), dim))
        return out

    def all_read(self, which: int, total: int) -> np.ndarray:
        out = np.empty(max(total, 1), np.float32)
        self._ck(self.L.ob_all_read(self.h, which, _ptr(out), total))
        return out[:total]

    def schedule_read(self):
        nb = c_int()
        self._ck(self.L.ob_schedule_read(self.h, byref(nb), None, None, None, None, 0, 0))
        n, _ = self.graph_size()
        st = self.stats()
        n = st["n_nodes"]
        depth = np.empty(nb.value, np.int32)
        sig = np.empty(nb.value, np.uint64)
        off = np.empty(nb.value + 1, np.int32)
        ids = np.empty(max(n, 1), np.int32)
        self._ck(self.L.ob_schedule_read(self.h, byref(nb), _ptr(depth), _ptr(sig), _ptr(off), _ptr(ids),
                                         nb.value, n))
        return off.astype(np.int64), ids[:n].astype(np.int64), depth.astype(np.int64), sig

    def stats(self) -> dict:
        s = ObStats()
        self._ck(self.L.ob_stats_read(self.h, byref(s)))
        return s.as_dict()

    def debug_read(self, which: int) -> np.ndarray:
        nw = c_size_t()
        self._ck(self.L.ob_debug_read(self.h, which, None, 0, byref(nw)))
        out = np.empty(max(nw.value, 1), np.uint32)
        self._ck(self.L.ob_debug_read(self.h, which, _ptr(out), nw.value, byref(nw)))
        out = out[:nw.value]
        return out.view(np.uint64) if which == OB_DBG_SIG else out

    def debug_set(self, which: int, value: int):
        self._ck(self.L.ob_debug_set(self.h, which, int(value)))

    # -- stand-alone primitives (tests)
    def test_sort(self, keys, vals, lo_bit, n_bits):
        k = np.ascontiguousarray(keys, np.uint64)
        v = np.ascontiguousarray(vals, np.uint32)
        ko, vo = np.empty_like(k), np.empty_like(v)
        self._ck(self.L.ob_test_sort(self.h, k.shape[0], _ptr(k), _ptr(v), lo_bit, n_bits, _ptr(ko), _ptr(vo)))
        return ko, vo

    def test_scan(self, a):
        a = np.ascontiguousarray(a, np.uint32)
        out = np.empty(max(a.shape[0], 1), np.uint32)
        tot = np.zeros(1, np.uint32)
        self._ck(self.L.ob_test_scan(self.h, a.shape[0], _ptr(a), _ptr(out), _ptr(tot)))
        return out[:a.shape[0]], int(tot[0])

    def test_launch_cost(self, n: int = 2000, touch: int = 0) -> float:
        out = c_float()
        self._ck(self.L.ob_test_launch_cost(self.h, n, touch, byref(out)))
        return float(out.value)

    def test_gemm(self, A, B):
        A = np.ascontiguousarray(A, np.float32)
        B = np.ascontiguousarray(B, np.float32)
        C = np.empty((A.shape[0], B.shape[0]), np.float32)
        self._ck(self.L.ob_test_gemm(self.h, A.shape[0], B.shape[0], A.shape[1], _ptr(A), _ptr(B), _ptr(C)))
        return C
