"""Thin ctypes binding of libdsq (argument marshalling only).

Function names mirror include/dsq.h.  Every step of the path runs in the library's HIP kernels;
there is no Python or CPU fallback: if libdsq.so is missing or fails to load, importing a symbol
from here raises.  torch is imported first on purpose, so that the library binds to the same HIP
runtime as the tensors whose device pointers are passed in.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch  # noqa: F401  (must be loaded before libdsq.so: one HIP runtime per process)

from .workloads import (KIND_IDENTITY, KIND_QUANT_MAXABS, KIND_SIGN_MEANABS, KIND_TOPK, KIND_QUANT_L2NORM, KIND_RAND_SPARSE, KIND_GSPAR,  # noqa: F401
                        TOPO_CSR, TOPO_RING, TOPO_TORUS2D, Config)

DS_OK, DS_EINVAL, DS_ENOMEM, DS_EHIP, DS_ESTATE = range(5)
_STATUS = {0: "DS_OK", 1: "DS_EINVAL", 2: "DS_ENOMEM", 3: "DS_EHIP", 4: "DS_ESTATE"}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdsq.so")

EXPORTS = ["ds_validate_config", "ds_build_topology", "ds_message_bytes", "ds_init", "ds_step",
           "ds_read_state", "ds_write_state", "ds_read_messages", "ds_state_ptrs", "ds_message_ptr",
           "ds_step_count", "ds_plan_name", "ds_last_error", "ds_destroy", "ds_bench_copy",
           "ds_topk_candidate_rows", "ds_set_mixing", "ds_diagnostics", "ds_set_rates", "ds_workload_gradient", "ds_bench_stream", "ds_build_id", "ds_step_static", "ds_init_ex"]


class ds_comp(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("bits", ctypes.c_int32), ("block", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("k", ctypes.c_uint64)]


class ds_workload(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("kind", ctypes.c_int32), ("N", ctypes.c_uint64), ("scale", ctypes.c_float),
                ("reserved", ctypes.c_float), ("seed", ctypes.c_uint64)]


class ds_plan_request(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("tile_plan", ctypes.c_int32), ("pitch_skew", ctypes.c_int64),
                ("autotune", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class ds_config(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("topo", ctypes.c_int32), ("N", ctypes.c_uint64),
                ("torus_rows", ctypes.c_int32), ("torus_cols", ctypes.c_int32),
                ("W_rowptr", ctypes.c_void_p), ("W_col", ctypes.c_void_p), ("W_val", ctypes.c_void_p),
                ("comp", ds_comp), ("gamma", ctypes.c_float), ("eta", ctypes.c_float),
                ("seed", ctypes.c_uint64), ("algo", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class DsqError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: {_STATUS.get(status, status)}{(': ' + detail) if detail else ''}")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libdsq.so (built by paper_1907_07346_amd/build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_1907_07346_amd.build` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, u64, i32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int
        cfgp, u64p = ctypes.POINTER(ds_config), ctypes.POINTER(ctypes.c_uint64)
        L.ds_validate_config.argtypes, L.ds_validate_config.restype = [cfgp, ctypes.c_char_p, u64], i32
        L.ds_build_topology.argtypes, L.ds_build_topology.restype = [cfgp, vp, vp, vp, u64, u64p], i32
        L.ds_message_bytes.argtypes, L.ds_message_bytes.restype = [cfgp], u64
        L.ds_build_id.argtypes, L.ds_build_id.restype = [], ctypes.c_char_p
        L.ds_step_static.argtypes = [cfgp, vp, vp, u64, vp, u64, vp, u64, vp, ctypes.c_char_p, u64]
        L.ds_step_static.restype = i32
        L.ds_init.argtypes, L.ds_init.restype = [cfgp, ctypes.POINTER(vp)], i32
        L.ds_init_ex.argtypes = [cfgp, ctypes.POINTER(ds_plan_request), ctypes.c_char_p, u64, ctypes.POINTER(vp)]
        L.ds_init_ex.restype = i32
        L.ds_step.argtypes, L.ds_step.restype = [vp, vp, u64, vp], i32
        L.ds_read_state.argtypes, L.ds_read_state.restype = [vp, vp, vp], i32
        L.ds_set_mixing.argtypes, L.ds_set_mixing.restype = [vp, vp, vp, vp], i32
        L.ds_set_rates.argtypes, L.ds_set_rates.restype = [vp, ctypes.c_float, ctypes.c_float], i32
        L.ds_workload_gradient.argtypes = [ctypes.POINTER(ds_workload), u64, vp, u64, vp, u64, vp]
        L.ds_workload_gradient.restype = i32
        L.ds_diagnostics.argtypes, L.ds_diagnostics.restype = [vp, ctypes.POINTER(ctypes.c_double)], i32
        L.ds_write_state.argtypes, L.ds_write_state.restype = [vp, vp, vp, u64], i32
        L.ds_read_messages.argtypes, L.ds_read_messages.restype = [vp, vp, u64, u64p], i32
        L.ds_state_ptrs.argtypes, L.ds_state_ptrs.restype = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), u64p], i32
        L.ds_message_ptr.argtypes, L.ds_message_ptr.restype = [vp, ctypes.POINTER(vp), u64p], i32
        L.ds_step_count.argtypes, L.ds_step_count.restype = [vp], u64
        L.ds_topk_candidate_rows.argtypes, L.ds_topk_candidate_rows.restype = [vp, ctypes.POINTER(ctypes.c_uint32)], i32
        L.ds_plan_name.argtypes, L.ds_plan_name.restype = [vp], ctypes.c_char_p
        L.ds_last_error.argtypes, L.ds_last_error.restype = [vp], ctypes.c_char_p
        L.ds_destroy.argtypes, L.ds_destroy.restype = [vp], None
        L.ds_bench_copy.argtypes, L.ds_bench_copy.restype = [vp, vp, u64, vp], i32
        L.ds_bench_stream.argtypes, L.ds_bench_stream.restype = [vp, vp, vp, u64, vp], i32
        _lib = L
    return _lib


def make_config(n: int, N: int, topo: int, kind: int, gamma: float, eta: float, *, bits: int = 0,
                block: int = 0, k: int = 0, torus=(0, 0), seed: int = 0, W_csr=None, algo: int = 0):
    """Fills a ds_config. W_csr = (rowptr int32, col int32, val float32) numpy arrays for TOPO_CSR.

    Returns (config, keepalive): keepalive holds the arrays the config points to.
    """
    c = ds_config()
    c.n, c.topo, c.N = n, topo, N
    c.torus_rows, c.torus_cols = torus
    keep = None
    if W_csr is not None:
        rp = np.ascontiguousarray(W_csr[0], dtype=np.int32)
        co = np.ascontiguousarray(W_csr[1], dtype=np.int32)
        va = np.ascontiguousarray(W_csr[2], dtype=np.float32)
        keep = (rp, co, va)
        c.W_rowptr, c.W_col, c.W_val = rp.ctypes.data, co.ctypes.data, va.ctypes.data
    c.comp.kind, c.comp.bits, c.comp.block, c.comp.k = kind, bits, block, k
    c.gamma, c.eta, c.seed = gamma, eta, seed
    c.algo = algo
    return c, keep


def ds_workload_gradient(kind: str, n: int, N: int, scale: float, seed: int, t: int, g: "torch.Tensor", x_ptr: int = 0,
                         x_ld: int = 0, stream: Optional["torch.cuda.Stream"] = None):
    """Fills the CUDA float32 tensor g (n, >= N) with the deterministic gradients of step t (see detgen.py)."""
    from .detgen import GRAD_KINDS
    assert g.is_cuda and g.dtype == torch.float32 and g.dim() == 2 and g.shape[0] == n and g.stride(1) == 1
    w = ds_workload(n, GRAD_KINDS[kind], N, scale, 0.0, seed)
    s = stream if stream is not None else torch.cuda.current_stream()
    st = lib().ds_workload_gradient(ctypes.byref(w), t, x_ptr, x_ld, g.data_ptr(), g.stride(0), s.cuda_stream)
    if st != DS_OK:
        raise RuntimeError(f"ds_workload_gradient failed with status {st}")


def config_from_workload(w: Config):
    return make_config(w.n, w.N, w.topo, w.kind, w.gamma, w.eta, bits=w.bits, block=w.block, k=w.k,
                       torus=w.torus, seed=w.seed, algo=w.algo)


def ds_validate_config(cfg: ds_config):
    buf = ctypes.create_string_buffer(256)
    st = lib().ds_validate_config(ctypes.byref(cfg), buf, 256)
    return st, buf.value.decode()


def ds_build_topology(cfg: ds_config):
    cap = max(1, cfg.n) * max(1, cfg.n)
    cap = min(cap, 16 * max(1, cfg.n) + 16)
    rowptr = np.zeros(max(1, cfg.n) + 1, np.int32)
    col = np.zeros(cap, np.int32)
    val = np.zeros(cap, np.float32)
    nnz = ctypes.c_uint64(0)
    st = lib().ds_build_topology(ctypes.byref(cfg), rowptr.ctypes.data, col.ctypes.data, val.ctypes.data,
                                 cap, ctypes.byref(nnz))
    if st != DS_OK:
        raise DsqError(st, "ds_build_topology")
    return rowptr, col[:nnz.value].copy(), val[:nnz.value].copy()


def ds_message_bytes(cfg: ds_config) -> int:
    return int(lib().ds_message_bytes(ctypes.byref(cfg)))


def ds_bench_copy(dst: "torch.Tensor", src: "torch.Tensor", stream=None):
    """Plain device copy of src into dst (same byte size, multiple of 16) with the library's copy kernel."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and dst.is_cuda and src.is_cuda
    s = stream if stream is not None else torch.cuda.current_stream()
    st = lib().ds_bench_copy(dst.data_ptr(), src.data_ptr(), nbytes, s.cuda_stream)
    if st != DS_OK:
        raise DsqError(st, "ds_bench_copy")


def ds_bench_stream(x: "torch.Tensor", d: "Optional[torch.Tensor]", g: "torch.Tensor", stream=None):
    """x += g, d += g with the library's 3-loads / 2-stores streaming kernel (the access mix of ds_step); d = None:
    x += g alone, 2 loads / 1 store (the mix of the DCD-PSGD step)."""
    nbytes = x.numel() * x.element_size()
    assert (d is None or d.numel() * d.element_size() == nbytes) and g.numel() * g.element_size() == nbytes
    assert x.is_cuda and (d is None or d.is_cuda) and g.is_cuda
    s = stream if stream is not None else torch.cuda.current_stream()
    st = lib().ds_bench_stream(x.data_ptr(), d.data_ptr() if d is not None else None, g.data_ptr(), nbytes, s.cuda_stream)
    if st != DS_OK:
        raise DsqError(st, "ds_bench_stream")


def ds_step_static(cfg: ds_config, x: "torch.Tensor", delta: "torch.Tensor", g: "torch.Tensor", msg: "torch.Tensor", t: int,
                   stream: Optional["torch.cuda.Stream"] = None):
    """One step on caller-owned CUDA tensors (x, delta: float32 (n, ld); g: float32 (n, >= N); msg: uint8), nothing allocated."""
    for a in (x, delta, g):
        assert a.is_cuda and a.dtype == torch.float32 and a.dim() == 2 and a.stride(1) == 1
    assert msg.is_cuda and msg.dtype == torch.uint8 and msg.is_contiguous() and msg.numel() >= ds_message_bytes(cfg)
    assert x.stride(0) == delta.stride(0)
    s = stream if stream is not None else torch.cuda.current_stream()
    buf = ctypes.create_string_buffer(256)
    st = lib().ds_step_static(ctypes.byref(cfg), x.data_ptr(), delta.data_ptr(), x.stride(0), g.data_ptr(), g.stride(0),
                              msg.data_ptr(), t, s.cuda_stream, buf, 256)
    if st != DS_OK:
        raise DsqError(st, "ds_step_static", buf.value.decode())


class DeepSqueeze:
    """Owner of one ds_handle. Methods are the C calls with the same names."""

    def __init__(self, cfg: ds_config, keepalive=None, plan: Optional[dict] = None):
        """plan: None (ds_init) or a dict with any of variant, tile_plan, pitch_skew, autotune (ds_init_ex)."""
        self._h = ctypes.c_void_p()
        self.cfg = cfg
        self._keep = keepalive
        buf = ctypes.create_string_buffer(256)
        if plan is None:
            st = lib().ds_init_ex(ctypes.byref(cfg), None, buf, 256, ctypes.byref(self._h))
        else:
            req = ds_plan_request(plan.get("variant", 0), plan.get("tile_plan", -1), plan.get("pitch_skew", -1),
                                  plan.get("autotune", 1), 0)
            st = lib().ds_init_ex(ctypes.byref(cfg), ctypes.byref(req), buf, 256, ctypes.byref(self._h))
        if st != DS_OK:
            raise DsqError(st, "ds_init", buf.value.decode())
        self.n, self.N = int(cfg.n), int(cfg.N)

    @classmethod
    def from_workload(cls, w: Config, plan: Optional[dict] = None) -> "DeepSqueeze":
        cfg, keep = config_from_workload(w)
        return cls(cfg, keep, plan)

    def _check(self, st: int, where: str):
        if st != DS_OK:
            raise DsqError(st, where, self.ds_last_error())

    def ds_step(self, g: "torch.Tensor", stream: Optional["torch.cuda.Stream"] = None):
        """g: CUDA float32 tensor (n, >=N) with unit column stride; runs on `stream` (default: current)."""
        assert g.is_cuda and g.dtype == torch.float32 and g.dim() == 2 and g.shape[0] == self.n
        assert g.stride(1) == 1 and g.shape[1] >= self.N
        s = stream if stream is not None else torch.cuda.current_stream()
        self._check(lib().ds_step(self._h, g.data_ptr(), g.stride(0) if self.n > 1 else max(g.stride(0), g.shape[1]),
                                  s.cuda_stream), "ds_step")

    def ds_step_raw(self, g_ptr: int, g_ld: int, stream_ptr: int = 0) -> int:
        return lib().ds_step(self._h, g_ptr, g_ld, stream_ptr)

    def ds_set_mixing(self, W_csr):
        """W_csr = (rowptr int32, col int32, val float32): the mixing matrix for the following steps."""
        rp = np.ascontiguousarray(W_csr[0], dtype=np.int32)
        co = np.ascontiguousarray(W_csr[1], dtype=np.int32)
        va = np.ascontiguousarray(W_csr[2], dtype=np.float32)
        self._check(lib().ds_set_mixing(self._h, rp.ctypes.data, co.ctypes.data, va.ctypes.data), "ds_set_mixing")

    def ds_set_rates(self, gamma: float, eta: float):
        self._check(lib().ds_set_rates(self._h, gamma, eta), "ds_set_rates")

    def ds_read_state(self, want_delta: bool = True):
        x = np.empty((self.n, self.N), np.float32)
        d = np.empty((self.n, self.N), np.float32) if want_delta else None
        self._check(lib().ds_read_state(self._h, x.ctypes.data, d.ctypes.data if want_delta else None), "ds_read_state")
        return x, d

    def ds_write_state(self, x: Optional[np.ndarray], delta: Optional[np.ndarray], t: int):
        if x is not None:
            x = np.ascontiguousarray(x, np.float32)
            assert x.shape == (self.n, self.N)
        if delta is not None:
            delta = np.ascontiguousarray(delta, np.float32)
            assert delta.shape == (self.n, self.N)
        self._check(lib().ds_write_state(self._h, x.ctypes.data if x is not None else None,
                                         delta.ctypes.data if delta is not None else None, t), "ds_write_state")

    def ds_read_messages(self) -> np.ndarray:
        total = ds_message_bytes(self.cfg)
        buf = np.empty(total, np.uint8)
        got = ctypes.c_uint64(0)
        self._check(lib().ds_read_messages(self._h, buf.ctypes.data, total, ctypes.byref(got)), "ds_read_messages")
        assert got.value == total
        return buf

    def ds_state_ptrs(self):
        x, d, ld = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_uint64()
        self._check(lib().ds_state_ptrs(self._h, ctypes.byref(x), ctypes.byref(d), ctypes.byref(ld)), "ds_state_ptrs")
        return x.value, d.value, ld.value

    def ds_message_ptr(self):
        p, b = ctypes.c_void_p(), ctypes.c_uint64()
        self._check(lib().ds_message_ptr(self._h, ctypes.byref(p), ctypes.byref(b)), "ds_message_ptr")
        return p.value, b.value

    def ds_diagnostics(self) -> dict:
        out = (ctypes.c_double * 4)()
        self._check(lib().ds_diagnostics(self._h, out), "ds_diagnostics")
        return {"consensus_sq": out[0], "delta_sq": out[1], "delta_mixed_sq": out[2], "message_bytes": int(out[3])}

    def ds_topk_candidate_rows(self) -> int:
        c = ctypes.c_uint32(0)
        self._check(lib().ds_topk_candidate_rows(self._h, ctypes.byref(c)), "ds_topk_candidate_rows")
        return int(c.value)

    def ds_step_count(self) -> int:
        return int(lib().ds_step_count(self._h))

    def ds_plan_name(self) -> str:
        return lib().ds_plan_name(self._h).decode()

    def ds_last_error(self) -> str:
        return lib().ds_last_error(self._h).decode()

    def ds_destroy(self):
        if self._h:
            lib().ds_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.ds_destroy()
        except Exception:
            pass
