"""Thin ctypes binding of libindexmem (see include/indexmem.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch
supplies device memory and the stream.  There is no CPU fallback: if the library cannot be
loaded or built, importing a function from here and calling it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

from . import build as _build

IM_OK, IM_ERR_INVALID_ARG, IM_ERR_UNSUPPORTED, IM_ERR_LAUNCH = 0, -1, -2, -3
IM_STATUS_APPEND_OVERFLOW, IM_STATUS_LIVE_EXCEEDED, IM_STATUS_OVER_BUDGET = 1, 2, 8
IM_STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = [
    "im_workspace_bytes", "im_create", "im_destroy", "im_last_error", "im_set_max_live",
    "im_query_status", "im_append_kv", "im_append_kv_hidden", "im_index_score", "im_topb_select", "im_memory_update",
    "im_compact_kv", "im_gather_kept", "im_decode_attn_with_readout", "im_decode_attn_with_readout_static", "im_decode_step", "im_attend_step", "im_attend_step_hidden", "im_decode_step_shared", "im_decode_step_shared_hidden", "im_stream_read", "im_profile_start",
    "im_profile_stop",
]


class ImConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "capacity", "n_idx_heads", "idx_dim",
        "mem_dim", "gate_in_dim", "n_sink", "n_recent", "fold_block", "max_queries", "head_shared")] + [
        ("rms_eps", C.c_float), ("mem_eps", C.c_float), ("softmax_scale", C.c_float)]


class ImParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("Uq", "G", "Uk", "norm_q_w", "norm_k_w", "Wtheta", "wg")] + [
        ("cg", C.c_float)]


class ImState(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("K", "V", "Kidx", "pos", "len", "n_projected", "M", "b")]


class IndexMemError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libindexmem error {code}: {msg}")
        self.code = code


_lib: Optional[C.CDLL] = None


def load_library(build_if_missing: bool = True) -> C.CDLL:
    """Load libindexmem.so from the package directory (building it with hipcc if absent)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB_PATH
    if not os.path.exists(path):
        if not build_if_missing:
            raise FileNotFoundError(f"{path} is not built; run __graft_entry__.build()")
        _build.build_library()
    lib = C.CDLL(path)
    vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    lib.im_workspace_bytes.restype = C.c_size_t
    lib.im_workspace_bytes.argtypes = [C.POINTER(ImConfig)]
    lib.im_create.restype = i32
    lib.im_create.argtypes = [C.POINTER(ImConfig), vp, C.c_size_t, C.POINTER(vp)]
    lib.im_destroy.restype = None
    lib.im_destroy.argtypes = [vp]
    lib.im_last_error.restype = C.c_char_p
    lib.im_last_error.argtypes = [vp]
    lib.im_set_max_live.restype = i32
    lib.im_set_max_live.argtypes = [vp, i32]
    lib.im_query_status.restype = i32
    lib.im_query_status.argtypes = [vp, C.POINTER(i32), vp]
    lib.im_append_kv.restype = i32
    lib.im_append_kv.argtypes = [vp, C.POINTER(ImState), vp, vp, vp, i32, vp]
    lib.im_append_kv_hidden.restype = i32
    lib.im_append_kv_hidden.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, vp, vp, i32, vp]
    lib.im_index_score.restype = i32
    lib.im_index_score.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, vp, i32, vp, vp]
    lib.im_topb_select.restype = i32
    lib.im_topb_select.argtypes = [vp, vp, C.POINTER(ImState), i32, vp, vp, vp, vp, vp]
    lib.im_memory_update.restype = i32
    lib.im_memory_update.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, f32, f32, vp]
    lib.im_compact_kv.restype = i32
    lib.im_compact_kv.argtypes = [vp, C.POINTER(ImState), vp, vp, vp, vp, vp]
    lib.im_gather_kept.restype = i32
    lib.im_gather_kept.argtypes = [vp, C.POINTER(ImState), C.POINTER(ImState), i32, vp, vp, vp, vp, vp]
    lib.im_decode_attn_with_readout.restype = i32
    lib.im_decode_attn_with_readout.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, vp, vp]
    lib.im_decode_attn_with_readout_static.restype = i32
    lib.im_decode_attn_with_readout_static.argtypes = [C.POINTER(ImConfig), i32, C.POINTER(ImParams), C.POINTER(ImState),
                                                       vp, vp, vp, vp, vp]
    lib.im_decode_step.restype = i32
    lib.im_decode_step.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, vp, vp, vp, vp, i32,
                                   f32, f32, vp, vp, vp, vp, vp]
    lib.im_attend_step.restype = i32
    lib.im_attend_step.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, vp, vp, vp, vp, vp]
    lib.im_attend_step_hidden.restype = i32
    lib.im_attend_step_hidden.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, vp, vp, vp, vp, vp, vp]
    lib.im_decode_step_shared.restype = i32
    lib.im_decode_step_shared.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, vp, vp, vp,
                                          f32, f32, vp, vp, vp]
    lib.im_decode_step_shared_hidden.restype = i32
    lib.im_decode_step_shared_hidden.argtypes = [vp, C.POINTER(ImParams), C.POINTER(ImState), vp, vp, vp, vp, vp, vp,
                                                 f32, f32, vp, vp, vp]
    lib.im_stream_read.restype = i32
    lib.im_stream_read.argtypes = [vp, C.c_size_t, C.c_uint32, vp, vp]
    lib.im_profile_start.restype = i32
    lib.im_profile_start.argtypes = [vp, i32, i32]
    lib.im_profile_stop.restype = i32
    lib.im_profile_stop.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(i32), vp]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to libindexmem must be contiguous"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


@dataclass
class Config:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    capacity: int
    n_idx_heads: int
    head_dim: int = 128
    idx_dim: int = 64
    mem_dim: int = 128
    gate_in_dim: int = 0          # 0: n_q_heads * head_dim
    n_sink: int = 4
    n_recent: int = 0
    fold_block: int = 64
    max_queries: int = 1
    rms_eps: float = 1e-6
    mem_eps: float = 1e-6
    softmax_scale: float = 0.0    # 0: 1 / sqrt(head_dim)
    head_shared: int = 0          # 1: one indexer key / eviction set / memory per sequence (idx_dim 16)

    def c_struct(self) -> ImConfig:
        gate = self.gate_in_dim or self.n_q_heads * self.head_dim
        scale = self.softmax_scale or self.head_dim ** -0.5
        return ImConfig(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.capacity,
                        self.n_idx_heads, self.idx_dim, self.mem_dim, gate, self.n_sink,
                        self.n_recent, self.fold_block, self.max_queries, self.head_shared, self.rms_eps,
                        self.mem_eps, scale)

    def set_shape(self):
        """Leading axes of everything kept per set: (B, H_kv), or (B,) in the head-shared layout."""
        return (self.batch,) if self.head_shared else (self.batch, self.n_kv_heads)


class Params:
    """Slow weights of one layer as device tensors (bf16)."""

    def __init__(self, Uq, G, Uk, Wtheta, wg, cg=0.0, norm_q_w=None, norm_k_w=None):
        self.Uq, self.G, self.Uk, self.Wtheta, self.wg = Uq, G, Uk, Wtheta, wg
        self.norm_q_w, self.norm_k_w, self.cg = norm_q_w, norm_k_w, float(cg)
        self.c = ImParams(_ptr(Uq), _ptr(G), _ptr(Uk), _ptr(norm_q_w), _ptr(norm_k_w), _ptr(Wtheta),
                          _ptr(wg), self.cg)


class State:
    """State of one layer: slot arrays, lengths and the memory state, all device tensors."""

    def __init__(self, cfg: Config, device="cuda"):
        B, Hk, Cc, D = cfg.batch, cfg.n_kv_heads, cfg.capacity, cfg.head_dim
        S = cfg.set_shape()
        z = dict(device=device)
        self.K = torch.zeros((B, Hk, Cc, D), dtype=torch.bfloat16, **z)
        self.V = torch.zeros((B, Hk, Cc, D), dtype=torch.bfloat16, **z)
        self.Kidx = torch.zeros(S + (Cc, cfg.idx_dim), dtype=torch.bfloat16, **z)
        self.pos = torch.zeros(S + (Cc,), dtype=torch.int32, **z)
        self.len = torch.zeros(S, dtype=torch.int32, **z)
        self.n_projected = torch.zeros(S, dtype=torch.int32, **z)
        self.M = torch.zeros(S + (cfg.mem_dim, D), dtype=torch.float32, **z)
        self.b = torch.zeros(S + (cfg.mem_dim,), dtype=torch.float32, **z)
        self.c = ImState(*(_ptr(t) for t in (self.K, self.V, self.Kidx, self.pos, self.len,
                                             self.n_projected, self.M, self.b)))


class Handle:
    """Owns the workspace tensor and the library handle of one configuration."""

    def __init__(self, cfg: Config, device="cuda"):
        self.lib = load_library()
        self.cfg = cfg
        self._c_cfg = cfg.c_struct()
        nbytes = self.lib.im_workspace_bytes(C.byref(self._c_cfg))
        if nbytes == 0:
            # let im_create report which field is wrong
            h = C.c_void_p()
            rc = self.lib.im_create(C.byref(self._c_cfg), None, 0, C.byref(h))
            raise IndexMemError(rc, "invalid configuration")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        base = (self.workspace.data_ptr() + 255) & ~255
        h = C.c_void_p()
        rc = self.lib.im_create(C.byref(self._c_cfg), base, nbytes, C.byref(h))
        if rc != IM_OK:
            raise IndexMemError(rc, "im_create failed")
        self.h = h

    def check(self, rc: int) -> None:
        if rc != IM_OK:
            raise IndexMemError(rc, self.lib.im_last_error(self.h).decode())

    def __del__(self):
        try:
            if getattr(self, "h", None):
                self.lib.im_destroy(self.h)
                self.h = None
        except Exception:
            pass


# ---- the library's calls, same names, tensors in place of pointers -------------------------
def im_set_max_live(h: Handle, max_live: int) -> None:
    h.check(h.lib.im_set_max_live(h.h, max_live))


def im_query_status(h: Handle) -> int:
    out = C.c_int32(0)
    h.check(h.lib.im_query_status(h.h, C.byref(out), _stream()))
    return out.value


def im_append_kv(h: Handle, st: State, k_new, v_new, pos_new) -> None:
    n_new = pos_new.shape[1]   # (k_new = v_new = None: the rows are already in place)
    h.check(h.lib.im_append_kv(h.h, C.byref(st.c), _ptr(k_new), _ptr(v_new), _ptr(pos_new), n_new,
                               _stream()))


def im_append_kv_hidden(h: Handle, p: Params, st: State, k_new, v_new, x_new, pos_new) -> None:
    n_new = pos_new.shape[1]
    h.check(h.lib.im_append_kv_hidden(h.h, C.byref(p.c), C.byref(st.c), _ptr(k_new), _ptr(v_new), _ptr(x_new),
                                      _ptr(pos_new), n_new, _stream()))


def im_index_score(h: Handle, p: Params, st: State, q_new, x_gate, q_pos, scores_out) -> None:
    n_q = q_new.shape[1]
    h.check(h.lib.im_index_score(h.h, C.byref(p.c), C.byref(st.c), _ptr(q_new), _ptr(x_gate),
                                 _ptr(q_pos), n_q, _ptr(scores_out), _stream()))


def im_topb_select(h: Handle, scores, st: State, budget: int, keep_idx, evict_idx, n_keep, n_evict) -> None:
    h.check(h.lib.im_topb_select(h.h, _ptr(scores), C.byref(st.c), budget, _ptr(keep_idx),
                                 _ptr(evict_idx), _ptr(n_keep), _ptr(n_evict), _stream()))


def im_memory_update(h: Handle, p: Params, st: State, evict_idx, n_evict, lam: float, eta: float) -> None:
    h.check(h.lib.im_memory_update(h.h, C.byref(p.c), C.byref(st.c), _ptr(evict_idx), _ptr(n_evict),
                                   lam, eta, _stream()))


def im_compact_kv(h: Handle, st: State, keep_idx, n_keep, evict_idx, n_evict) -> None:
    h.check(h.lib.im_compact_kv(h.h, C.byref(st.c), _ptr(keep_idx), _ptr(n_keep), _ptr(evict_idx),
                                _ptr(n_evict), _stream()))


def im_gather_kept(h: Handle, src: State, dst: State, dst_capacity: int, keep_idx, n_keep, evict_idx, n_evict) -> None:
    h.check(h.lib.im_gather_kept(h.h, C.byref(src.c), C.byref(dst.c), dst_capacity, _ptr(keep_idx), _ptr(n_keep),
                                 _ptr(evict_idx), _ptr(n_evict), _stream()))


def im_decode_attn_with_readout(h: Handle, p: Params, st: State, q, out, readout_dbg=None) -> None:
    h.check(h.lib.im_decode_attn_with_readout(h.h, C.byref(p.c), C.byref(st.c), _ptr(q), _ptr(out),
                                              _ptr(readout_dbg), _stream()))


def im_decode_attn_with_readout_static(cfg: Config, max_live: int, p: Params, st: State, q, out,
                                       readout_dbg=None, status_dev=None) -> None:
    """The same without a handle or a workspace (the library's built-in scratch buffer)."""
    lib = load_library()
    c = cfg.c_struct()
    rc = lib.im_decode_attn_with_readout_static(C.byref(c), max_live, C.byref(p.c), C.byref(st.c), _ptr(q), _ptr(out),
                                                _ptr(readout_dbg), _ptr(status_dev), _stream())
    if rc != IM_OK:
        raise IndexMemError(rc, lib.im_last_error(None).decode())


def im_decode_step(h: Handle, p: Params, st: State, q, x_gate, q_pos, k_new, v_new, pos_new, budget: int,
                   lam: float, eta: float, out, readout_dbg=None, evicted_slot=None, scores_dbg=None) -> None:
    h.check(h.lib.im_decode_step(h.h, C.byref(p.c), C.byref(st.c), _ptr(q), _ptr(x_gate), _ptr(q_pos),
                                 _ptr(k_new), _ptr(v_new), _ptr(pos_new), budget, lam, eta, _ptr(out),
                                 _ptr(readout_dbg), _ptr(evicted_slot), _ptr(scores_dbg), _stream()))


def im_attend_step(h: Handle, p: Params, st: State, q, k_new, v_new, pos_new, out, readout_dbg=None) -> None:
    h.check(h.lib.im_attend_step(h.h, C.byref(p.c), C.byref(st.c), _ptr(q), _ptr(k_new), _ptr(v_new),
                                 _ptr(pos_new), _ptr(out), _ptr(readout_dbg), _stream()))


def im_attend_step_hidden(h: Handle, p: Params, st: State, q, x_new, k_new, v_new, pos_new, out,
                          readout_dbg=None) -> None:
    h.check(h.lib.im_attend_step_hidden(h.h, C.byref(p.c), C.byref(st.c), _ptr(q), _ptr(x_new), _ptr(k_new),
                                        _ptr(v_new), _ptr(pos_new), _ptr(out), _ptr(readout_dbg), _stream()))


def im_decode_step_shared(h: Handle, p: Params, st: State, q, k_new, v_new, pos_new, evict_slot, lam: float,
                          eta: float, out, readout_dbg=None) -> None:
    h.check(h.lib.im_decode_step_shared(h.h, C.byref(p.c), C.byref(st.c), _ptr(q), _ptr(k_new), _ptr(v_new),
                                        _ptr(pos_new), _ptr(evict_slot), lam, eta, _ptr(out),
                                        _ptr(readout_dbg), _stream()))


def im_decode_step_shared_hidden(h: Handle, p: Params, st: State, q, x_new, k_new, v_new, pos_new, evict_slot,
                                 lam: float, eta: float, out, readout_dbg=None) -> None:
    h.check(h.lib.im_decode_step_shared_hidden(h.h, C.byref(p.c), C.byref(st.c), _ptr(q), _ptr(x_new), _ptr(k_new),
                                               _ptr(v_new), _ptr(pos_new), _ptr(evict_slot), lam, eta, _ptr(out),
                                               _ptr(readout_dbg), _stream()))


def im_stream_read(src: torch.Tensor, nbytes: int, never: int, sink: torch.Tensor) -> None:
    """One plain streaming read of the first nbytes of src (measurement only; see indexmem.h)."""
    lib = load_library()
    rc = lib.im_stream_read(_ptr(src), nbytes, never, _ptr(sink), _stream())
    if rc != IM_OK:
        raise IndexMemError(rc, lib.im_last_error(None).decode())


IM_PROFILE_MAIN, IM_PROFILE_PREP, IM_PROFILE_PREP_AND_MAIN = 0, 1, 2


def im_profile_start(h: Handle, max_records: int, span: int = IM_PROFILE_MAIN) -> None:
    """Bracket part of every following im_decode_step's launches with HIP events (see indexmem.h)."""
    h._prof_max = max_records
    h.check(h.lib.im_profile_start(h.h, max_records, span))


def im_profile_stop(h: Handle):
    """Returns the list of span durations (ms) recorded since im_profile_start."""
    buf = (C.c_float * h._prof_max)()
    n = C.c_int32(0)
    h.check(h.lib.im_profile_stop(h.h, buf, C.byref(n), _stream()))
    return [buf[i] for i in range(n.value)]
