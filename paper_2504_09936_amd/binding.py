"""ctypes binding of libkeepkv.so: argument marshalling only.

Every function has the name and meaning of the C entry point declared in include/keepkv.h;
tensors are torch tensors on the GPU (used here purely as device memory), passed down as raw
pointers together with the current torch stream.  There is no fallback: if the HIP library has
not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("KEEPKV_LIB") or os.path.join(_HERE, "libkeepkv.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} not found: build the HIP library first (python -m paper_2504_09936_amd.build)")

_lib = C.CDLL(LIB_PATH)

F32, BF16 = 0, 1
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_DEVICE = range(5)


class _Layout(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float)]


class _Cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("votes", C.c_void_p), ("log_s", C.c_void_p),
                ("born", C.c_void_p), ("t_obs", C.c_void_p), ("len", C.c_void_p), ("capacity", C.c_int32), ("len_hint", C.c_int32),
                ("plan_slots_per_split", C.c_int32), ("plan_wavefronts", C.c_int32)]


_P = C.c_void_p
_lib.keepkv_strerror.restype = C.c_char_p
_lib.keepkv_strerror.argtypes = [C.c_int]
_lib.keepkv_version.restype = C.c_int32
_lib.keepkv_workspace_bytes.restype = C.c_size_t
_lib.keepkv_workspace_bytes.argtypes = [C.POINTER(_Layout), C.c_int32, C.c_int32]
_lib.keepkv_append.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, _P, _P, _P]
_lib.keepkv_decode_attn.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, _P, _P, _P, _P, C.c_size_t, _P]
_lib.keepkv_workspace_init.argtypes = [_P, C.c_size_t, _P]
_lib.keepkv_decode_step.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, _P, _P, _P, _P, C.c_float, _P, _P,
                                    C.c_size_t, _P]
_lib.keepkv_decode_step_static.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, _P, _P, _P, _P, C.c_float, _P, _P]
_lib.keepkv_score.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, C.c_float, _P]
_lib.keepkv_score_window.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, C.c_int32, C.c_float, C.c_int32, _P]
_lib.keepkv_select.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), C.c_int32, C.c_int32, C.c_int32,
                               C.c_float, _P, _P, _P, _P, C.c_size_t, _P]
_lib.keepkv_select_by_key.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, C.c_int32, C.c_int32, C.c_int32,
                                      _P, _P, _P, _P, C.c_size_t, _P]
_lib.keepkv_match.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), C.c_int32, _P, _P, _P, C.c_float,
                              _P, _P, _P, C.c_size_t, _P]
_lib.keepkv_merge.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), C.POINTER(_Cache), C.c_int32, _P, _P, _P,
                              _P, C.c_float, _P, _P, C.c_size_t, _P]
_lib.keepkv_select_aged.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                    _P, _P, _P, _P, C.c_size_t, _P]
_lib.keepkv_merge_inplace.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), _P, C.c_int32, _P, _P, _P, _P, C.c_float,
                                      _P, _P]
_lib.keepkv_prefill_match.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), C.c_float, _P, _P, _P, C.c_size_t, _P]
_lib.keepkv_prefill_merge.argtypes = [C.POINTER(_Layout), C.POINTER(_Cache), C.POINTER(_Cache), _P, C.c_float, _P,
                                      C.c_size_t, _P]
_lib.keepkv_probe_read.argtypes = [_P, C.c_size_t, C.c_int32, _P, _P]
_lib.keepkv_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_int32, _P, C.POINTER(C.c_double), _P]
_lib.keepkv_decode_plan.argtypes = [C.POINTER(_Layout), C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                    C.POINTER(C.c_int32)]
for _f in ("select_aged", "merge_inplace", "prefill_match", "prefill_merge", "decode_step_static", "decode_plan", "probe_read", "probe_mfma", "append", "decode_attn", "decode_step", "workspace_init", "score", "score_window", "select",
           "select_by_key", "match",
           "merge"):
    getattr(_lib, "keepkv_" + _f).restype = C.c_int

EXPORTS = ["keepkv_strerror", "keepkv_version", "keepkv_workspace_bytes", "keepkv_workspace_init", "keepkv_decode_plan",
           "keepkv_append", "keepkv_decode_attn", "keepkv_decode_step", "keepkv_decode_step_static", "keepkv_score", "keepkv_score_window", "keepkv_select",
           "keepkv_select_by_key", "keepkv_select_aged", "keepkv_match", "keepkv_merge", "keepkv_merge_inplace", "keepkv_prefill_match", "keepkv_prefill_merge",
           "keepkv_probe_read", "keepkv_probe_mfma"]


class KeepKVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_lib.keepkv_strerror(status).decode()} (status {status})")


def _check(st: int, where: str) -> None:
    if st != OK:
        raise KeepKVError(st, where)


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


@dataclass
class Layout:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: int
    scale: float

    def c(self) -> _Layout:
        return _Layout(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.dtype, self.scale)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == BF16 else torch.float32


class Cache:
    """One layer's cache as device tensors (plain storage; no arithmetic happens here)."""

    def __init__(self, layout: Layout, capacity: int, device="cuda"):
        B, H, D = layout.batch, layout.n_kv_heads, layout.head_dim
        self.layout, self.capacity = layout, capacity
        self.len_hint = 0     # host-side upper bound on len (0 = unknown); see keepkv_cache.len_hint
        self.plan_slots_per_split = 0   # decode launch overrides (0 = automatic); see keepkv_cache
        self.plan_wavefronts = 0
        self.k = torch.zeros(B, H, capacity, D, dtype=layout.torch_dtype, device=device)
        self.v = torch.zeros(B, H, capacity, D, dtype=layout.torch_dtype, device=device)
        self.votes = torch.zeros(B, H, capacity, dtype=torch.int32, device=device)
        self.log_s = torch.full((B, H, capacity), float("-inf"), dtype=torch.float32, device=device)
        self.born = torch.zeros(B, H, capacity, dtype=torch.int32, device=device)
        self.t_obs = torch.zeros(B, H, dtype=torch.int32, device=device)
        self.len = torch.zeros(B, H, dtype=torch.int32, device=device)

    FIELDS = ("k", "v", "votes", "log_s", "born", "t_obs", "len")

    def state(self) -> dict:
        """Host copies of every array of the cache (for dumps and replays of a failing step; plain copies)."""
        torch.cuda.synchronize()
        d = {f: getattr(self, f).detach().cpu().clone() for f in self.FIELDS}
        d["capacity"] = torch.tensor(self.capacity)
        return d

    def load_state(self, d: dict) -> None:
        if int(d["capacity"]) != self.capacity:
            raise ValueError("cache state of another capacity")
        for f in self.FIELDS:
            t = getattr(self, f)
            if tuple(d[f].shape) != tuple(t.shape) or d[f].dtype != t.dtype:
                raise ValueError(f"cache state field {f} does not fit this cache")
            t.copy_(d[f])

    def save(self, path: str) -> None:
        torch.save(self.state(), path)

    def load(self, path: str) -> None:
        self.load_state(torch.load(path, map_location="cpu", weights_only=True))

    def c(self) -> _Cache:
        return _Cache(self.k.data_ptr(), self.v.data_ptr(), self.votes.data_ptr(), self.log_s.data_ptr(),
                      self.born.data_ptr(), self.t_obs.data_ptr(), self.len.data_ptr(), self.capacity, int(self.len_hint),
                      int(self.plan_slots_per_split), int(self.plan_wavefronts))


def version() -> int:
    return int(_lib.keepkv_version())


def workspace_bytes(layout: Layout, capacity: int, budget: int) -> int:
    return int(_lib.keepkv_workspace_bytes(C.byref(layout.c()), capacity, budget))


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def new_workspace(layout: Layout, capacity: int, budget: int, device="cuda"):
    """Allocate a workspace tensor of the required size and clear its control words."""
    ws = torch.empty(workspace_bytes(layout, capacity, budget), dtype=torch.uint8, device=device)
    workspace_init(ws)
    return ws


def workspace_init(workspace) -> None:
    _check(_lib.keepkv_workspace_init(_ptr(workspace), _nbytes(workspace), _stream()), "keepkv_workspace_init")


def decode_step(layout: Layout, cache: Cache, q, k_t, v_t, out, logits_out, alpha: float, overflow, workspace) -> None:
    _check(_lib.keepkv_decode_step(C.byref(layout.c()), C.byref(cache.c()), _ptr(q), _ptr(k_t), _ptr(v_t), _ptr(out),
                                   _ptr(logits_out), alpha, _ptr(overflow), _ptr(workspace), _nbytes(workspace),
                                   _stream()), "keepkv_decode_step")


def decode_step_static(layout: Layout, cache: Cache, q, k_t, v_t, out, logits_out, alpha: float, overflow) -> None:
    _check(_lib.keepkv_decode_step_static(C.byref(layout.c()), C.byref(cache.c()), _ptr(q), _ptr(k_t), _ptr(v_t),
                                          _ptr(out), _ptr(logits_out), alpha, _ptr(overflow), _stream()),
           "keepkv_decode_step_static")


def append(layout: Layout, cache: Cache, k_t, v_t, overflow=None) -> None:
    _check(_lib.keepkv_append(C.byref(layout.c()), C.byref(cache.c()), _ptr(k_t), _ptr(v_t), _ptr(overflow),
                              _stream()), "keepkv_append")


def decode_attn(layout: Layout, cache: Cache, q, out, logits_out, lse_out, workspace) -> None:
    _check(_lib.keepkv_decode_attn(C.byref(layout.c()), C.byref(cache.c()), _ptr(q), _ptr(out), _ptr(logits_out),
                                   _ptr(lse_out), _ptr(workspace),
                                   0 if workspace is None else workspace.numel() * workspace.element_size(),
                                   _stream()), "keepkv_decode_attn")


def score(layout: Layout, cache: Cache, logits, alpha: float) -> None:
    _check(_lib.keepkv_score(C.byref(layout.c()), C.byref(cache.c()), _ptr(logits), alpha, _stream()),
           "keepkv_score")


def score_window(layout: Layout, cache: Cache, q_win, window: int, alpha: float, first_pos: int = -1) -> None:
    _check(_lib.keepkv_score_window(C.byref(layout.c()), C.byref(cache.c()), _ptr(q_win), window, alpha, first_pos,
                                    _stream()), "keepkv_score_window")


def select(layout: Layout, cache: Cache, budget: int, n_sink: int, n_recent: int, alpha: float,
           keep_idx, evict_idx, n_evict, workspace) -> None:
    _check(_lib.keepkv_select(C.byref(layout.c()), C.byref(cache.c()), budget, n_sink, n_recent, alpha,
                              _ptr(keep_idx), _ptr(evict_idx), _ptr(n_evict), _ptr(workspace),
                              0 if workspace is None else workspace.numel() * workspace.element_size(),
                              _stream()), "keepkv_select")


def decode_plan(layout: Layout, capacity: int):
    """(n_split, slots_per_split, wavefronts) of a decode call on this layout and capacity."""
    ns, per, wv = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(_lib.keepkv_decode_plan(C.byref(layout.c()), capacity, C.byref(ns), C.byref(per), C.byref(wv)),
           "keepkv_decode_plan")
    return ns.value, per.value, wv.value


def select_by_key(layout: Layout, cache: Cache, rank, budget: int, n_sink: int, n_recent: int,
                  keep_idx, evict_idx, n_evict, workspace) -> None:
    _check(_lib.keepkv_select_by_key(C.byref(layout.c()), C.byref(cache.c()), _ptr(rank), budget, n_sink, n_recent,
                                     _ptr(keep_idx), _ptr(evict_idx), _ptr(n_evict), _ptr(workspace),
                                     _nbytes(workspace), _stream()), "keepkv_select_by_key")


def probe_read(src, n_workgroups: int, sink) -> None:
    _check(_lib.keepkv_probe_read(_ptr(src), _nbytes(src), n_workgroups, _ptr(sink), _stream()), "keepkv_probe_read")


def probe_mfma(n_workgroups: int, iters: int, sink, random_operands: bool = False) -> float:
    flops = C.c_double(0.0)
    _check(_lib.keepkv_probe_mfma(n_workgroups, iters, 1 if random_operands else 0, _ptr(sink), C.byref(flops), _stream()),
           "keepkv_probe_mfma")
    return flops.value


def match(layout: Layout, cache: Cache, budget: int, keep_idx, evict_idx, n_evict, threshold: float,
          match_out, sim_out, workspace) -> None:
    _check(_lib.keepkv_match(C.byref(layout.c()), C.byref(cache.c()), budget, _ptr(keep_idx), _ptr(evict_idx),
                             _ptr(n_evict), threshold, _ptr(match_out), _ptr(sim_out), _ptr(workspace),
                             0 if workspace is None else workspace.numel() * workspace.element_size(),
                             _stream()), "keepkv_match")


def select_aged(layout: Layout, cache: Cache, order, budget: int, n_sink: int, n_recent: int, alpha: float,
                keep_idx, evict_idx, n_evict, workspace) -> None:
    _check(_lib.keepkv_select_aged(C.byref(layout.c()), C.byref(cache.c()), _ptr(order), budget, n_sink, n_recent, alpha,
                                   _ptr(keep_idx), _ptr(evict_idx), _ptr(n_evict), _ptr(workspace), _nbytes(workspace),
                                   _stream()), "keepkv_select_aged")


def merge_inplace(layout: Layout, cache: Cache, order, budget: int, keep_idx, evict_idx, n_evict, match_in,
                  alpha: float, dropped_votes) -> None:
    _check(_lib.keepkv_merge_inplace(C.byref(layout.c()), C.byref(cache.c()), _ptr(order), budget, _ptr(keep_idx),
                                     _ptr(evict_idx), _ptr(n_evict), _ptr(match_in), alpha, _ptr(dropped_votes), _stream()),
           "keepkv_merge_inplace")


def prefill_match(layout: Layout, cache: Cache, threshold: float, near, sim_out, workspace) -> None:
    _check(_lib.keepkv_prefill_match(C.byref(layout.c()), C.byref(cache.c()), threshold, _ptr(near), _ptr(sim_out),
                                     _ptr(workspace), _nbytes(workspace), _stream()), "keepkv_prefill_match")


def prefill_merge(layout: Layout, src: Cache, dst: Cache, near, alpha: float, workspace) -> None:
    _check(_lib.keepkv_prefill_merge(C.byref(layout.c()), C.byref(src.c()), C.byref(dst.c()), _ptr(near), alpha,
                                     _ptr(workspace), _nbytes(workspace), _stream()), "keepkv_prefill_merge")


def merge(layout: Layout, src: Cache, dst: Cache, budget: int, keep_idx, evict_idx, n_evict, match_in,
          alpha: float, dropped_votes, workspace) -> None:
    _check(_lib.keepkv_merge(C.byref(layout.c()), C.byref(src.c()), C.byref(dst.c()), budget, _ptr(keep_idx),
                             _ptr(evict_idx), _ptr(n_evict), _ptr(match_in), alpha, _ptr(dropped_votes),
                             _ptr(workspace),
                             0 if workspace is None else workspace.numel() * workspace.element_size(),
                             _stream()), "keepkv_merge")
