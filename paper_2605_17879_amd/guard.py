"""ctypes binding of the C ABI in ``include/guard.h`` -- argument marshalling only.

Every function of the header is reachable as ``Detector.<name without gd_>``
taking torch CUDA tensors; PyTorch supplies device memory and streams, nothing
else.  No step of the detector is computed here.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libguard_hip.so")
_lib = None

GD_OK = 0
_STATUS = {0: "GD_OK", 1: "GD_ERR_INVALID_ARG", 2: "GD_ERR_BAD_CONFIG",
           3: "GD_ERR_BUFFER_TOO_SMALL", 4: "GD_ERR_UNSUPPORTED", 5: "GD_ERR_HIP"}
NODE_SUM_SCALED = 0
NODE_MAX = 1

EXPORTS = ("gd_default_config", "gd_create", "gd_destroy", "gd_state_bytes", "gd_bind_state",
           "gd_set_streaming_steps", "gd_score_batch", "gd_update_window", "gd_flags",
           "gd_topk_nodes", "gd_severity", "gd_sweep_score", "gd_probe_read", "gd_last_error",
           "gd_default_ledger_config", "gd_ledger_bytes", "gd_bind_ledger", "gd_update_ledger",
           "gd_ledger_flags", "gd_topk_nodes_mean", "gd_set_streaming_hints", "gd_apply_membership",
           "gd_update_ledger_static", "gd_ledger_static_scratch_bytes")


class GuardError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{_STATUS.get(status, status)}: {msg}")
        self.status = status


class _CConfig(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("n_ranks", ctypes.c_uint32),
                ("gpus_per_node", ctypes.c_uint32), ("n_metrics", ctypes.c_uint32),
                ("primary_metric", ctypes.c_uint32), ("min_signals", ctypes.c_uint32),
                ("window", ctypes.c_uint32), ("persist_k", ctypes.c_uint32),
                ("topk", ctypes.c_uint32), ("node_agg", ctypes.c_uint32),
                ("z_threshold", ctypes.c_float), ("node_scale", ctypes.c_float),
                ("rel_floor", ctypes.c_float), ("abs_floor", ctypes.c_float),
                ("direction", ctypes.c_int8 * 8)]


class _CLedgerConfig(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("score_quant", ctypes.c_float),
                ("recur_limit", ctypes.c_uint32), ("reserved", ctypes.c_uint32),
                ("recur_horizon", ctypes.c_uint64)]


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libguard_hip.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2605_17879_amd.build` "
            "(or __graft_entry__.build()); there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
    lib.gd_default_config.argtypes = [ctypes.POINTER(_CConfig), u32, u32, u32, u32]
    lib.gd_default_config.restype = None
    lib.gd_create.argtypes = [ctypes.POINTER(_CConfig), ctypes.POINTER(vp)]
    lib.gd_create.restype = ctypes.c_int
    lib.gd_destroy.argtypes = [vp]
    lib.gd_destroy.restype = ctypes.c_int
    lib.gd_state_bytes.argtypes = [vp]
    lib.gd_state_bytes.restype = ctypes.c_size_t
    lib.gd_bind_state.argtypes = [vp, vp, ctypes.c_size_t]
    lib.gd_bind_state.restype = ctypes.c_int
    lib.gd_set_streaming_steps.argtypes = [vp, u32]
    lib.gd_set_streaming_steps.restype = ctypes.c_int
    lib.gd_set_streaming_hints.argtypes = [vp, vp, vp]
    lib.gd_set_streaming_hints.restype = ctypes.c_int
    lib.gd_score_batch.argtypes = [vp, vp, u32] + [vp] * 9
    lib.gd_score_batch.restype = ctypes.c_int
    lib.gd_update_window.argtypes = [vp, vp, vp, vp, u32, u64, vp]
    lib.gd_update_window.restype = ctypes.c_int
    lib.gd_flags.argtypes = [vp] * 8
    lib.gd_flags.restype = ctypes.c_int
    lib.gd_topk_nodes.argtypes = [vp, u32, vp, vp, vp]
    lib.gd_topk_nodes.restype = ctypes.c_int
    lib.gd_severity.argtypes = [vp, vp, u32, vp, ctypes.c_float, ctypes.c_float, vp, vp, vp]
    lib.gd_severity.restype = ctypes.c_int
    f32 = ctypes.c_float
    lib.gd_sweep_score.argtypes = [vp, vp, vp, u32, f32, f32, f32, vp, vp, vp, vp, vp]
    lib.gd_sweep_score.restype = ctypes.c_int
    lib.gd_probe_read.argtypes = [vp, vp, u64, vp, vp]
    lib.gd_probe_read.restype = ctypes.c_int
    lib.gd_default_ledger_config.argtypes = [ctypes.POINTER(_CLedgerConfig)]
    lib.gd_default_ledger_config.restype = None
    lib.gd_ledger_bytes.argtypes = [vp, u32]
    lib.gd_ledger_bytes.restype = ctypes.c_size_t
    lib.gd_bind_ledger.argtypes = [vp, ctypes.POINTER(_CLedgerConfig), vp, ctypes.c_size_t, u32]
    lib.gd_bind_ledger.restype = ctypes.c_int
    lib.gd_update_ledger.argtypes = [vp, vp, vp, vp, u32, u64, vp]
    lib.gd_update_ledger.restype = ctypes.c_int
    lib.gd_update_ledger_static.argtypes = [vp, vp, vp, vp, u32, u64, vp]
    lib.gd_update_ledger_static.restype = ctypes.c_int
    lib.gd_ledger_static_scratch_bytes.argtypes = []
    lib.gd_ledger_static_scratch_bytes.restype = ctypes.c_size_t
    lib.gd_ledger_flags.argtypes = [vp] * 11
    lib.gd_ledger_flags.restype = ctypes.c_int
    lib.gd_topk_nodes_mean.argtypes = [vp, u32, vp, vp, vp]
    lib.gd_topk_nodes_mean.restype = ctypes.c_int
    lib.gd_apply_membership.argtypes = [vp, vp, u32, vp, vp]
    lib.gd_apply_membership.restype = ctypes.c_int
    lib.gd_last_error.argtypes = [vp]
    lib.gd_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


@dataclass
class Config:
    """Mirror of ``gd_config``; ``None`` fields take the library's defaults."""

    n_ranks: int
    n_metrics: int
    window: int
    persist_k: int
    gpus_per_node: int = 8
    primary_metric: int = 0
    min_signals: Optional[int] = None
    topk: Optional[int] = None
    node_agg: int = NODE_SUM_SCALED
    z_threshold: Optional[float] = None
    node_scale: Optional[float] = None
    rel_floor: Optional[float] = None
    abs_floor: Optional[float] = None
    direction: Sequence[int] = field(default_factory=tuple)

    def to_c(self) -> _CConfig:
        c = _CConfig()
        load_library().gd_default_config(ctypes.byref(c), self.n_ranks, self.n_metrics,
                                         self.window, self.persist_k)
        c.gpus_per_node = self.gpus_per_node
        c.primary_metric = self.primary_metric
        c.node_agg = self.node_agg
        for name in ("min_signals", "topk", "z_threshold", "node_scale", "rel_floor", "abs_floor"):
            v = getattr(self, name)
            if v is not None:
                setattr(c, name, v)
        for i, d in enumerate(self.direction):
            c.direction[i] = int(d)
        return c


def _p(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Detector:
    """One ``gd_handle`` plus its (torch-allocated) window state."""

    def __init__(self, cfg: Config, device="cuda:0"):
        import torch
        self._torch = torch
        self.lib = load_library()
        self.cfg = cfg
        self.ccfg = cfg.to_c()
        h = ctypes.c_void_p()
        st = self.lib.gd_create(ctypes.byref(self.ccfg), ctypes.byref(h))
        if st != GD_OK:
            raise GuardError(st, (self.lib.gd_last_error(None) or b"").decode())
        self.h = h
        self.device = torch.device(device)
        self.R, self.M = cfg.n_ranks, cfg.n_metrics
        self.N = self.R // cfg.gpus_per_node
        self.RW, self.NW = (self.R + 63) // 64, (self.N + 63) // 64
        self.state = torch.zeros(self.state_bytes(), dtype=torch.uint8, device=self.device)
        self.bind_state(self.state)
        self.steps_seen = 0

    def close(self):
        if getattr(self, "h", None):
            self.lib.gd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != GD_OK:
            raise GuardError(st, (self.lib.gd_last_error(self.h) or b"").decode())

    def _stream(self, stream) -> int:
        s = stream if stream is not None else self._torch.cuda.current_stream(self.device)
        return s.cuda_stream

    # ---- the C ABI, one method per entry point --------------------------------
    def state_bytes(self) -> int:
        return int(self.lib.gd_state_bytes(self.h))

    def bind_state(self, state):
        self._check(self.lib.gd_bind_state(self.h, state.data_ptr(), state.numel() * state.element_size()))
        self.state = state

    def set_streaming_steps(self, max_steps: int):
        """Batches of at most max_steps steps are scored one workgroup per column (0: never)."""
        self._check(self.lib.gd_set_streaming_steps(self.h, max_steps))

    def set_streaming_hints(self, med=None, mad=None):
        """One-step calls start their selection from these [M] medians and MADs (device
        tensors, typically the previous call's outputs; kept alive here)."""
        self._hints = (med, mad)
        self._check(self.lib.gd_set_streaming_hints(self.h, _p(med), _p(mad)))

    def apply_membership(self, x, active, stream=None):
        """NaN (missing) in place wherever active[T][ceil(R/64)] (int64 bit words) has a clear bit."""
        T = x.shape[0]
        assert x.is_cuda and x.is_contiguous() and tuple(x.shape) == (T, self.M, self.R)
        assert active.is_cuda and active.is_contiguous() and tuple(active.shape) == (T, self.RW)
        self._check(self.lib.gd_apply_membership(self.h, x.data_ptr(), T, active.data_ptr(), self._stream(stream)))

    def alloc_outputs(self, T: int, want_z: bool = False) -> dict:
        """Output tensors of gd_score_batch for T steps (plain allocation)."""
        torch, d = self._torch, self.device
        o = dict(
            med=torch.empty((T, self.M), dtype=torch.float32, device=d),
            mad=torch.empty((T, self.M), dtype=torch.float32, device=d),
            z=torch.empty((T, self.M, self.R), dtype=torch.float32, device=d) if want_z else None,
            exceed_mask=torch.empty((T, self.R), dtype=torch.uint8, device=d),
            rank_anom=torch.empty((T, self.RW), dtype=torch.int64, device=d),
            node_z=torch.empty((T, self.N), dtype=torch.float32, device=d),
            node_mask=torch.empty((T, self.N), dtype=torch.uint8, device=d),
            node_anom=torch.empty((T, self.NW), dtype=torch.int64, device=d))
        return o

    def score_batch(self, x, out: dict, stream=None):
        T = x.shape[0]
        assert x.is_cuda and x.is_contiguous() and x.dtype == self._torch.float32
        assert tuple(x.shape) == (T, self.M, self.R)
        self._check(self.lib.gd_score_batch(
            self.h, x.data_ptr(), T, _p(out["med"]), _p(out["mad"]), _p(out.get("z")),
            _p(out["exceed_mask"]), _p(out["rank_anom"]), _p(out["node_z"]), _p(out["node_mask"]),
            _p(out["node_anom"]), self._stream(stream)))

    def update_window(self, out: dict, T: int, first_step_index: Optional[int] = None, stream=None):
        first = self.steps_seen if first_step_index is None else first_step_index
        self._check(self.lib.gd_update_window(self.h, _p(out["rank_anom"]), _p(out["node_anom"]),
                                              _p(out["node_z"]), T, first, self._stream(stream)))
        self.steps_seen = first + T

    def alloc_flags(self) -> dict:
        torch, d = self._torch, self.device
        return dict(rank_flag=torch.empty(self.R, dtype=torch.uint8, device=d),
                    rank_count=torch.empty(self.R, dtype=torch.int16, device=d),
                    rank_first=torch.empty(self.R, dtype=torch.int32, device=d),
                    node_flag=torch.empty(self.N, dtype=torch.uint8, device=d),
                    node_count=torch.empty(self.N, dtype=torch.int16, device=d),
                    node_first=torch.empty(self.N, dtype=torch.int32, device=d))

    def flags(self, f: dict, stream=None):
        self._check(self.lib.gd_flags(self.h, _p(f.get("rank_flag")), _p(f.get("rank_count")),
                                      _p(f.get("rank_first")), _p(f.get("node_flag")),
                                      _p(f.get("node_count")), _p(f.get("node_first")),
                                      self._stream(stream)))

    def alloc_severity(self) -> dict:
        torch, d = self._torch, self.device
        return dict(slowdown=torch.empty(self.N, dtype=torch.float32, device=d),
                    tier=torch.empty(self.N, dtype=torch.uint8, device=d))

    def severity(self, x, out: dict, sev: dict, moderate: float = 0.10, severe: float = 0.20,
                 stream=None):
        """Tiers of the flagged nodes from the batch x that `out` was scored from."""
        T = x.shape[0]
        assert x.is_cuda and x.is_contiguous() and tuple(x.shape) == (T, self.M, self.R)
        self._check(self.lib.gd_severity(self.h, x.data_ptr(), T, _p(out["med"]), moderate, severe,
                                         _p(sev["slowdown"]), _p(sev["tier"]), self._stream(stream)))

    def sweep_score(self, flops, bw, tol_compute: float = 0.05, tol_sym: float = 0.10,
                    tol_bw: float = 0.15, stream=None) -> dict:
        """Single-node sweep scoring of flops[B][8], bw[B][8][8] (device tensors)."""
        torch, d = self._torch, self.device
        B = flops.shape[0]
        assert flops.is_cuda and flops.is_contiguous() and tuple(flops.shape) == (B, 8)
        assert bw.is_cuda and bw.is_contiguous() and tuple(bw.shape) == (B, 8, 8)
        out = dict(shortfall=torch.empty((B, 8), dtype=torch.float32, device=d),
                   gpu_mask=torch.empty(B, dtype=torch.uint8, device=d),
                   link_mask=torch.empty(B, dtype=torch.int32, device=d),
                   verdict=torch.empty(B, dtype=torch.uint8, device=d))
        self._check(self.lib.gd_sweep_score(self.h, flops.data_ptr(), bw.data_ptr(), B, tol_compute,
                                            tol_sym, tol_bw, _p(out["shortfall"]), _p(out["gpu_mask"]),
                                            _p(out["link_mask"]), _p(out["verdict"]),
                                            self._stream(stream)))
        return out

    def probe_read(self, x, sink, stream=None):
        """Stream x through the chip with the scoring kernel's load pattern (a diagnostic)."""
        self._check(self.lib.gd_probe_read(self.h, x.data_ptr(), x.numel() * x.element_size(),
                                           sink.data_ptr(), self._stream(stream)))

    def alloc_topk(self, k: int) -> dict:
        torch, d = self._torch, self.device
        return dict(idx=torch.empty(k, dtype=torch.int32, device=d),
                    key=torch.empty(k, dtype=torch.int64, device=d))

    def topk_nodes(self, k: int, tk: dict, stream=None):
        self._check(self.lib.gd_topk_nodes(self.h, k, _p(tk["idx"]), _p(tk.get("key")),
                                           self._stream(stream)))

    # ---- the ledger ---------------------------------------------------------------
    def ledger_bytes(self, max_T: int) -> int:
        return int(self.lib.gd_ledger_bytes(self.h, max_T))

    def bind_ledger(self, ledger, max_T: int, score_quant: Optional[float] = None,
                    recur_limit: Optional[int] = None, recur_horizon: Optional[int] = None):
        c = _CLedgerConfig()
        self.lib.gd_default_ledger_config(ctypes.byref(c))
        if score_quant is not None:
            c.score_quant = score_quant
        if recur_limit is not None:
            c.recur_limit = recur_limit
        if recur_horizon is not None:
            c.recur_horizon = recur_horizon
        self._check(self.lib.gd_bind_ledger(self.h, ctypes.byref(c), ledger.data_ptr(),
                                            ledger.numel() * ledger.element_size(), max_T))
        self.ledger = ledger
        self.ledger_steps_seen = 0

    def alloc_ledger(self, max_T: int, **cfg):
        """A fresh (zeroed) ledger for batches of up to max_T steps, bound to the handle."""
        led = self._torch.zeros(self.ledger_bytes(max_T), dtype=self._torch.uint8, device=self.device)
        self.bind_ledger(led, max_T, **cfg)
        return led

    def update_ledger(self, out: dict, T: int, first_step_index: Optional[int] = None, stream=None):
        first = self.ledger_steps_seen if first_step_index is None else first_step_index
        self._check(self.lib.gd_update_ledger(self.h, _p(out["exceed_mask"]), _p(out["node_mask"]),
                                              _p(out["node_z"]), T, first, self._stream(stream)))
        self.ledger_steps_seen = first + T

    def update_ledger_static(self, out: dict, T: int, first_step_index: Optional[int] = None, stream=None):
        """gd_update_ledger with the library's static work area (the call allocates nothing)."""
        first = self.ledger_steps_seen if first_step_index is None else first_step_index
        self._check(self.lib.gd_update_ledger_static(self.h, _p(out["exceed_mask"]), _p(out["node_mask"]),
                                                     _p(out["node_z"]), T, first, self._stream(stream)))
        self.ledger_steps_seen = first + T

    def ledger_static_scratch_bytes(self) -> int:
        return int(self.lib.gd_ledger_static_scratch_bytes())

    def alloc_ledger_flags(self) -> dict:
        torch, d = self._torch, self.device
        e = lambda n, t: torch.empty(n, dtype=t, device=d)
        return dict(rank_pmask=e(self.R, torch.uint8), rank_pflag=e(self.R, torch.uint8),
                    rank_pfirst=e(self.R, torch.int32), node_pmask=e(self.N, torch.uint8),
                    node_pflag=e(self.N, torch.uint8), node_pfirst=e(self.N, torch.int32),
                    node_score_sum=e(self.N, torch.int32), node_episodes=e(self.N, torch.uint8),
                    node_terminal_first=e(self.N, torch.int32))

    def ledger_flags(self, f: dict, stream=None):
        self._check(self.lib.gd_ledger_flags(
            self.h, _p(f.get("rank_pmask")), _p(f.get("rank_pflag")), _p(f.get("rank_pfirst")),
            _p(f.get("node_pmask")), _p(f.get("node_pflag")), _p(f.get("node_pfirst")),
            _p(f.get("node_score_sum")), _p(f.get("node_episodes")),
            _p(f.get("node_terminal_first")), self._stream(stream)))

    def topk_nodes_mean(self, k: int, tk: dict, stream=None):
        self._check(self.lib.gd_topk_nodes_mean(self.h, k, _p(tk["idx"]), _p(tk.get("key")),
                                                self._stream(stream)))
