"""ctypes binding of librevive.so: argument marshalling only.

Function names and argument order follow include/revive.h.  torch is used for device memory
(tensors whose data_ptr() is handed to the library) and for the stream handle; no step of the
layer is computed here.  There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "librevive.so"
_lib = None

SCORE_FN = {"softmax": 0, "sigmoid": 1}
DTYPE = {"fp32": 0, "bf16": 1}
TORCH_DTYPE = {"fp32": torch.float32, "bf16": torch.bfloat16}

KERNEL_NAMES = ["router_gemm", "route_topk", "dispatch_index",
                "dispatch_permute", "ffn_tiles", "ffn_gate_up", "ffn_down", "ffn_shared_gate_up",
                "ffn_shared_down", "combine", "expert_counts"]


class ReviveError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_status_name(status)} ({status}): {message}")
        self.status = status


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("T_max", "H", "E", "k", "I", "I_shared", "n_ranks", "slots_per_rank", "max_replicas",
                 "score_fn", "n_group", "topk_group", "dtype")] + [("route_scale", C.c_float)]


class MapStats(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_live_slots", "n_live_experts", "n_lost_experts", "n_degraded_experts")]

    def as_dict(self) -> Dict[str, int]:
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


def lib_path() -> str:
    return os.path.join(_PKG_DIR, _LIB_NAME)


def lib() -> C.CDLL:
    """Load librevive.so (once) and declare its prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -m paper_2602_21140_amd.build); "
                          "there is no fallback path")
    L = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    P = C.POINTER
    protos = {
        "revive_create": (C.c_int, [P(Config), P(vp)]),
        "revive_destroy": (C.c_int, [vp]),
        "revive_workspace_bytes": (C.c_int, [vp, P(sz)]),
        "revive_bind_workspace": (C.c_int, [vp, vp, sz]),
        "revive_set_placement": (C.c_int, [vp, vp]),
        "revive_update_map": (C.c_int, [vp, vp, vp, P(MapStats)]),
        "revive_update_map_experts": (C.c_int, [vp, vp, vp, vp, P(MapStats)]),
        "revive_get_map": (C.c_int, [vp, vp, vp, vp]),
        "revive_build_map_experts": (C.c_int, [P(Config), vp, vp, vp, vp, vp, vp, P(MapStats)]),
        "revive_compact_ranks": (C.c_int, [vp, i32, i32, i32]),
        "revive_mask_every_nth": (C.c_int, [i32, i32, vp]),
        "revive_mask_most_activated": (C.c_int, [vp, i32, i32, vp]),
        "revive_expert_counts": (C.c_int, [vp, vp, i32, vp, vp]),
        "revive_build_map": (C.c_int, [P(Config), vp, vp, vp, vp, vp, P(MapStats)]),
        "revive_route": (C.c_int, [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]),
        "revive_dispatch": (C.c_int, [vp, vp, vp, i32, vp, vp, vp, vp, vp]),
        "revive_set_token_offset": (C.c_int, [vp, C.c_int64]),
        "revive_get_rank_map": (C.c_int, [vp, vp, vp]),
        "revive_rank_offsets": (C.c_int, [vp, vp, vp, vp]),
        "revive_dispatch_static": (C.c_int, [vp, vp, vp, i32, vp, vp, vp, vp, vp]),
        "revive_expert_ffn": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]),
        "revive_shared_ffn": (C.c_int, [vp, vp, vp, vp, vp, i32, vp]),
        "revive_combine": (C.c_int, [vp, vp, vp, vp, vp, i32, vp, vp]),
        "revive_graph_begin": (C.c_int, [vp, vp]),
        "revive_graph_end": (C.c_int, [vp, vp, P(vp)]),
        "revive_graph_launch": (C.c_int, [vp, vp]),
        "revive_graph_exec_id": (C.c_size_t, [vp]),
        "revive_graph_destroy": (C.c_int, [vp]),
        "revive_set_kernel_timing": (C.c_int, [vp, i32]),
        "revive_kernel_time": (C.c_int, [vp, i32, P(C.c_double), P(C.c_int64)]),
        "revive_reset_kernel_times": (C.c_int, [vp]),
        "revive_kernel_name": (C.c_char_p, [i32]),
        "revive_last_error": (C.c_char_p, [vp]),
        "revive_status_name": (C.c_char_p, [C.c_int]),
    }
    for name, (res, args) in protos.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


EXPORTS = ["revive_create", "revive_destroy", "revive_workspace_bytes", "revive_bind_workspace",
           "revive_set_placement", "revive_update_map", "revive_update_map_experts", "revive_get_map", "revive_build_map",
           "revive_build_map_experts", "revive_compact_ranks", "revive_mask_every_nth", "revive_mask_most_activated", "revive_expert_counts",
           "revive_get_rank_map", "revive_rank_offsets", "revive_set_token_offset",
           "revive_route", "revive_dispatch", "revive_dispatch_static", "revive_expert_ffn", "revive_shared_ffn", "revive_combine",
           "revive_graph_begin", "revive_graph_end", "revive_graph_launch", "revive_graph_exec_id",
           "revive_graph_destroy", "revive_set_kernel_timing", "revive_kernel_time",
           "revive_reset_kernel_times", "revive_kernel_name", "revive_last_error", "revive_status_name"]


def _status_name(status: int) -> str:
    return lib().revive_status_name(status).decode()


def make_config(cfg, T_max: Optional[int] = None, route_scale: float = 1.0) -> Config:
    """C config from a synth.LayerConfig-like object (any object with the same field names)."""
    return Config(T_max=cfg.T if T_max is None else T_max, H=cfg.H, E=cfg.E, k=cfg.k, I=cfg.I,
                  I_shared=cfg.I_shared, n_ranks=cfg.n_ranks, slots_per_rank=cfg.slots_per_rank,
                  max_replicas=cfg.max_replicas, score_fn=SCORE_FN[cfg.score_fn], n_group=cfg.n_group,
                  topk_group=cfg.topk_group, dtype=DTYPE[cfg.dtype], route_scale=route_scale)


def compact_ranks(logical_rank, failed_device: int, switched_device: int = -1) -> np.ndarray:
    """revive_compact_ranks on a copy of logical_rank (int32[n]); raises on bad input."""
    r = np.array(logical_rank, dtype=np.int32)
    rc = lib().revive_compact_ranks(r.ctypes.data, r.shape[0], failed_device, switched_device)
    if rc != 0:
        raise ReviveError(rc, lib().revive_last_error(None).decode())
    return r


def mask_every_nth(E: int, n: int) -> np.ndarray:
    """revive_mask_every_nth: uint8[E], 1 for the experts whose index is a multiple of n."""
    m = np.zeros(E, dtype=np.uint8)
    rc = lib().revive_mask_every_nth(E, n, m.ctypes.data)
    if rc != 0:
        raise ReviveError(rc, lib().revive_last_error(None).decode())
    return m


def mask_most_activated(counts: np.ndarray, n_fail: int) -> np.ndarray:
    """revive_mask_most_activated: uint8[E], 1 for the n_fail most frequently activated experts."""
    c = np.ascontiguousarray(counts, dtype=np.int64)
    m = np.zeros(c.shape[0], dtype=np.uint8)
    rc = lib().revive_mask_most_activated(c.ctypes.data, c.shape[0], n_fail, m.ctypes.data)
    if rc != 0:
        raise ReviveError(rc, lib().revive_last_error(None).decode())
    return m


def build_map_host(cfg, phys_to_logical: np.ndarray, rank_failed: np.ndarray, route_scale: float = 1.0,
                   expert_failed: Optional[np.ndarray] = None):
    """revive_build_map(_experts): the library's host-side map construction, no GPU needed.

    Returns (status, l2p_table [E, max_replicas], l2p_count [E], slot_alive [P], stats dict)."""
    c = make_config(cfg, route_scale=route_scale)
    p2l = np.ascontiguousarray(phys_to_logical, dtype=np.int32)
    failed = np.ascontiguousarray(rank_failed, dtype=np.uint8)
    assert p2l.shape[0] == cfg.n_ranks * cfg.slots_per_rank and failed.shape[0] == cfg.n_ranks
    table = np.zeros((cfg.E, cfg.max_replicas), dtype=np.int32)
    count = np.zeros(cfg.E, dtype=np.int32)
    alive = np.zeros(p2l.shape[0], dtype=np.uint8)
    stats = MapStats()
    ef = None if expert_failed is None else np.ascontiguousarray(expert_failed, dtype=np.uint8)
    rc = lib().revive_build_map_experts(C.byref(c), p2l.ctypes.data, failed.ctypes.data,
                                        None if ef is None else ef.ctypes.data, table.ctypes.data,
                                        count.ctypes.data, alive.ctypes.data, C.byref(stats))
    return rc, table, count, alive, stats.as_dict()


def pack_router(w_router: torch.Tensor) -> torch.Tensor:
    """[H, E] router matrix -> the library's output-major [E, H] layout."""
    return w_router.t().contiguous()


TILE_ROWS, TILE_K = 128, 32   # tiled weight layout of bf16 layers (include/revive.h)


def _tile(w: torch.Tensor) -> torch.Tensor:
    """[rows, K] -> the tiled layout [ceil(rows/128)*128, K] (same storage order as
    [rows/128][K/32][128][32]); rows zero-padded to a multiple of 128."""
    rows, K = w.shape
    assert K % TILE_K == 0
    pad = -rows % TILE_ROWS
    if pad:
        w = torch.cat([w, w.new_zeros(pad, K)], dim=0)
    rp = rows + pad
    return w.reshape(rp // TILE_ROWS, TILE_ROWS, K // TILE_K, TILE_K).permute(0, 2, 1, 3).contiguous().reshape(rp, K)


def _untile(t: torch.Tensor, rows: int) -> torch.Tensor:
    rp, K = t.shape
    w = t.reshape(rp // TILE_ROWS, K // TILE_K, TILE_ROWS, TILE_K).permute(0, 2, 1, 3).reshape(rp, K)
    return w[:rows]


def padded_rows(rows: int) -> int:
    return rows + (-rows % TILE_ROWS)


def pack_expert(gate: torch.Tensor, up: torch.Tensor, down: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """Math-layout expert matrices (gate/up [H, I], down [I, H]) -> the library's layouts.

    fp32: w_gate_up = [gate^T; up^T] as [2I, H], w_down = down^T as [H, I].
    bf16: the same matrices in the tiled layout (each of gate^T, up^T, down^T tiled separately)."""
    if gate.dtype == torch.bfloat16:
        return torch.cat([_tile(gate.t()), _tile(up.t())], dim=0).contiguous(), _tile(down.t())
    return torch.cat([gate.t(), up.t()], dim=0).contiguous(), down.t().contiguous()


def unpack_expert(w_gate_up: torch.Tensor, w_down: torch.Tensor, H: int, I: int):
    """Inverse of pack_expert: (gate [H, I], up [H, I], down [I, H])."""
    if w_gate_up.dtype == torch.bfloat16:
        ip = padded_rows(I)
        return (_untile(w_gate_up[:ip], I).t(), _untile(w_gate_up[ip:], I).t(), _untile(w_down, H).t())
    return w_gate_up[:I].t(), w_gate_up[I:].t(), w_down.t()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


class ReviveLayer:
    """One MoE layer context.  Methods mirror the C calls one to one; tensors are allocated here
    (torch owns the memory) and handed to the library by pointer."""

    def __init__(self, cfg, device="cuda:0", T_max: Optional[int] = None, route_scale: float = 1.0):
        self.L = lib()
        self.cfg = cfg
        self.device = torch.device(device)
        self.dtype = TORCH_DTYPE[cfg.dtype]
        self.T_max = cfg.T if T_max is None else T_max
        self.P = cfg.n_ranks * cfg.slots_per_rank
        self._ctx = C.c_void_p()
        self._cfg_c = make_config(cfg, self.T_max, route_scale)
        with torch.cuda.device(self.device):
            rc = self.L.revive_create(C.byref(self._cfg_c), C.byref(self._ctx))
            if rc != 0:
                raise ReviveError(rc, self.L.revive_last_error(None).decode())
            nbytes = C.c_size_t()
            self._check(self.L.revive_workspace_bytes(self._ctx, C.byref(nbytes)))
            self.workspace = torch.empty(max(256, nbytes.value), dtype=torch.uint8, device=self.device)
            self._check(self.L.revive_bind_workspace(self._ctx, self.workspace.data_ptr(), self.workspace.numel()))
        self._w_tabs = None
        self._graphs: List[C.c_void_p] = []

    # -- plumbing --------------------------------------------------------------------------
    def _check(self, rc: int):
        if rc != 0:
            raise ReviveError(rc, self.L.revive_last_error(self._ctx).decode())

    @staticmethod
    def _stream(stream: Optional[torch.cuda.Stream]) -> int:
        s = torch.cuda.current_stream() if stream is None else stream
        return s.cuda_stream

    def close(self):
        if self._ctx:
            for g in self._graphs:
                self.L.revive_graph_destroy(g)
            self._graphs = []
            self.L.revive_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def empty(self, *shape, dtype=None) -> torch.Tensor:
        return torch.empty(*shape, dtype=self.dtype if dtype is None else dtype, device=self.device)

    # -- map -------------------------------------------------------------------------------
    def set_placement(self, phys_to_logical: np.ndarray):
        p2l = np.ascontiguousarray(phys_to_logical, dtype=np.int32)
        assert p2l.shape == (self.P,)
        self.phys_to_logical = p2l
        self._check(self.L.revive_set_placement(self._ctx, p2l.ctypes.data))

    def update_map(self, rank_failed: np.ndarray, stream=None, expert_failed: Optional[np.ndarray] = None) -> Dict[str, int]:
        failed = np.ascontiguousarray(rank_failed, dtype=np.uint8)
        assert failed.shape == (self.cfg.n_ranks,)
        stats = MapStats()
        if expert_failed is None:
            self._check(self.L.revive_update_map(self._ctx, failed.ctypes.data, self._stream(stream), C.byref(stats)))
        else:
            ef = np.ascontiguousarray(expert_failed, dtype=np.uint8)
            assert ef.shape == (self.cfg.E,)
            self._check(self.L.revive_update_map_experts(self._ctx, failed.ctypes.data, ef.ctypes.data,
                                                         self._stream(stream), C.byref(stats)))
        return stats.as_dict()

    def expert_counts(self, topk_logical, T: int, counts=None, stream=None):
        """counts[e] += activations of e in topk_logical [T, k]; counts: int64 [E] on the device."""
        if counts is None:
            counts = torch.zeros(self.cfg.E, dtype=torch.int64, device=self.device)
        self._check(self.L.revive_expert_counts(self._ctx, _ptr(topk_logical), T, _ptr(counts), self._stream(stream)))
        return counts

    def update_map_status(self, rank_failed: np.ndarray, stream=None) -> int:
        """As update_map but returns the status code instead of raising."""
        failed = np.ascontiguousarray(rank_failed, dtype=np.uint8)
        return self.L.revive_update_map(self._ctx, failed.ctypes.data, self._stream(stream), None)

    def get_map(self):
        table = np.zeros((self.cfg.E, self.cfg.max_replicas), dtype=np.int32)
        count = np.zeros(self.cfg.E, dtype=np.int32)
        alive = np.zeros(self.P, dtype=np.uint8)
        self._check(self.L.revive_get_map(self._ctx, table.ctypes.data, count.ctypes.data, alive.ctypes.data))
        return table, count, alive

    def set_token_offset(self, first_token: int):
        """revive_set_token_offset: x is rows [first_token, first_token + T) of a larger batch."""
        self._check(self.L.revive_set_token_offset(self._ctx, int(first_token)))

    def get_rank_map(self):
        """(logical_rank int32[R], n_live_ranks) of the map in force (host copies)."""
        lr = np.zeros(self.cfg.n_ranks, dtype=np.int32)
        n = C.c_int32()
        self._check(self.L.revive_get_rank_map(self._ctx, lr.ctypes.data, C.byref(n)))
        return lr, int(n.value)

    def rank_offsets(self, slot_offsets, out=None, stream=None):
        """revive_rank_offsets: int32[R+1] compacted rank segment boundaries of a dispatched buffer."""
        if out is None:
            out = self.empty(self.cfg.n_ranks + 1, dtype=torch.int32)
        self._check(self.L.revive_rank_offsets(self._ctx, _ptr(slot_offsets), _ptr(out), self._stream(stream)))
        return out

    # -- weights ---------------------------------------------------------------------------
    def set_expert_weights(self, w_gate_up: Sequence[Optional[torch.Tensor]], w_down: Sequence[Optional[torch.Tensor]]):
        """Per-slot packed weights (lists of P tensors, None for empty slots) -> device pointer tables."""
        assert len(w_gate_up) == self.P and len(w_down) == self.P
        for gu, dn in zip(w_gate_up, w_down):
            if gu is not None:
                tiled = self.dtype == torch.bfloat16
                gu_rows = 2 * (padded_rows(self.cfg.I) if tiled else self.cfg.I)
                dn_rows = padded_rows(self.cfg.H) if tiled else self.cfg.H
                assert gu.shape == (gu_rows, self.cfg.H) and gu.dtype == self.dtype and gu.is_contiguous()
                assert dn.shape == (dn_rows, self.cfg.I) and dn.dtype == self.dtype and dn.is_contiguous()
        self._w_keep = (list(w_gate_up), list(w_down))
        gu_tab = torch.tensor([0 if t is None else t.data_ptr() for t in w_gate_up], dtype=torch.int64)
        dn_tab = torch.tensor([0 if t is None else t.data_ptr() for t in w_down], dtype=torch.int64)
        self._w_tabs = (gu_tab.to(self.device), dn_tab.to(self.device))

    # -- data path -------------------------------------------------------------------------
    def route(self, x, w_router, T: int, logits=None, logits_given=False, out=None, stream=None):
        k = self.cfg.k
        if logits is None:
            logits = self.empty(T, self.cfg.E, dtype=torch.float32)
        if out is None:
            out = (self.empty(T, k, dtype=torch.int32), self.empty(T, k, dtype=torch.float32),
                   self.empty(T, k, dtype=torch.int32))
        top_l, top_w, top_p = out
        self._check(self.L.revive_route(self._ctx, _ptr(x), _ptr(w_router), _ptr(logits), int(bool(logits_given)), T,
                                        _ptr(top_l), _ptr(top_w), _ptr(top_p), self._stream(stream)))
        return logits, top_l, top_w, top_p

    def dispatch(self, x, topk_phys, T: int, out=None, stream=None, static_scratch=False):
        """revive_dispatch, or with static_scratch revive_dispatch_static (which needs `out`: it is
        for callers that allocate nothing)."""
        N = T * self.cfg.k
        if out is None:
            assert not static_scratch, "the allocation-free entry point takes caller-owned outputs"
            out = (self.empty(N, self.cfg.H), self.empty(self.P + 1, dtype=torch.int32),
                   self.empty(N, dtype=torch.int32), self.empty(N, dtype=torch.int32))
        x_perm, slot_offsets, dst_row, src_of = out
        fn = self.L.revive_dispatch_static if static_scratch else self.L.revive_dispatch
        self._check(fn(self._ctx, _ptr(x), _ptr(topk_phys), T, _ptr(x_perm), _ptr(slot_offsets),
                                           _ptr(dst_row), _ptr(src_of), self._stream(stream)))
        return x_perm, slot_offsets, dst_row, src_of

    def expert_ffn(self, x_perm, slot_offsets, T: int, x=None, w_sh_gate_up=None, w_sh_down=None, out=None,
                   shared=True, stream=None):
        assert self._w_tabs is not None, "set_expert_weights first"
        N = T * self.cfg.k
        use_shared = shared and w_sh_gate_up is not None
        if out is None:
            out = (self.empty(N, self.cfg.H), self.empty(T, self.cfg.H) if use_shared else None)
        y_perm, y_shared = out
        self._check(self.L.revive_expert_ffn(self._ctx, _ptr(x_perm), _ptr(slot_offsets), _ptr(self._w_tabs[0]),
                                             _ptr(self._w_tabs[1]), _ptr(y_perm), _ptr(x) if use_shared else None,
                                             _ptr(w_sh_gate_up) if use_shared else None,
                                             _ptr(w_sh_down) if use_shared else None,
                                             _ptr(y_shared) if use_shared else None, T, self._stream(stream)))
        return y_perm, y_shared

    def shared_ffn(self, x, w_sh_gate_up, w_sh_down, T: int, out=None, stream=None):
        if out is None:
            out = self.empty(T, self.cfg.H)
        self._check(self.L.revive_shared_ffn(self._ctx, _ptr(x), _ptr(w_sh_gate_up), _ptr(w_sh_down), _ptr(out), T,
                                             self._stream(stream)))
        return out

    def combine(self, y_perm, dst_row, topk_weight, y_shared, T: int, out=None, stream=None):
        if out is None:
            out = self.empty(T, self.cfg.H)
        self._check(self.L.revive_combine(self._ctx, _ptr(y_perm), _ptr(dst_row), _ptr(topk_weight), _ptr(y_shared), T,
                                          _ptr(out), self._stream(stream)))
        return out

    # -- graph replay ----------------------------------------------------------------------
    def graph_begin(self, stream: torch.cuda.Stream):
        self._check(self.L.revive_graph_begin(self._ctx, stream.cuda_stream))

    def graph_end(self, stream: torch.cuda.Stream) -> C.c_void_p:
        g = C.c_void_p()
        self._check(self.L.revive_graph_end(self._ctx, stream.cuda_stream, C.byref(g)))
        self._graphs.append(g)
        return g

    def graph_launch(self, g, stream: torch.cuda.Stream):
        rc = self.L.revive_graph_launch(g, stream.cuda_stream)
        if rc != 0:
            raise ReviveError(rc, self.L.revive_last_error(None).decode())

    def graph_exec_id(self, g) -> int:
        return int(self.L.revive_graph_exec_id(g))

    # -- timing ----------------------------------------------------------------------------
    def set_kernel_timing(self, enabled: bool):
        self._check(self.L.revive_set_kernel_timing(self._ctx, int(enabled)))

    def reset_kernel_times(self):
        self._check(self.L.revive_reset_kernel_times(self._ctx))

    def kernel_times(self) -> Dict[str, Tuple[float, int]]:
        """{kernel name: (total ms, launches)} since the last reset."""
        out = {}
        for i, name in enumerate(KERNEL_NAMES):
            ms, n = C.c_double(), C.c_int64()
            self._check(self.L.revive_kernel_time(self._ctx, i, C.byref(ms), C.byref(n)))
            out[name] = (ms.value, n.value)
        return out
