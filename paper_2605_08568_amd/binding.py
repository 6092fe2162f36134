"""ctypes binding of include/parse.h.  Argument marshalling only: names and meaning follow the header."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

PARSE_F32, PARSE_BF16 = 0, 1
PARSE_ROWMAJOR, PARSE_MFMA16 = 0, 1
PARSE_PREFILL, PARSE_DECODE = 0, 1
PARSE_SCHED_AUTO, PARSE_SCHED_FUSED, PARSE_SCHED_TILES, PARSE_SCHED_PLANNED = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libparse.so")


class ParseError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = f"{where}: {status_string(status)} ({status})"
        if status == -6:
            msg += ": " + lib().parse_last_hip_error().decode()
        super().__init__(msg)


class _Layer(C.Structure):
    _fields_ = [("n", C.c_int32), ("m", C.c_int32), ("R", C.c_int32), ("G", C.c_int32),
                ("dtype", C.c_int32), ("layout", C.c_int32), ("Vt", C.c_void_p), ("Ut", C.c_void_p)]


class _Patterns(C.Structure):
    _fields_ = [("Vt_S", C.c_void_p), ("Ut_S", C.c_void_p), ("subsets", C.c_void_p),
                ("subset_stride", C.c_int32), ("n_patterns", C.c_int32), ("k", C.c_int32),
                ("Vt_shared", C.c_void_p), ("Ut_shared", C.c_void_p), ("n_shared", C.c_int32),
                ("schedule", C.c_int32)]


_lib = None


def lib():
    """The loaded C-ABI library; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2605_08568_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(_LIB_PATH)
    vp, i32, sz, f32 = C.c_void_p, C.c_int32, C.c_size_t, C.c_float
    L.parse_status_string.restype = C.c_char_p; L.parse_status_string.argtypes = [C.c_int]
    L.parse_last_hip_error.restype = C.c_char_p; L.parse_last_hip_error.argtypes = []
    L.parse_version.restype = C.c_int; L.parse_version.argtypes = []
    L.parse_check_offsets.restype = C.c_int; L.parse_check_offsets.argtypes = [vp, i32, i32]
    L.parse_check_subset.restype = C.c_int; L.parse_check_subset.argtypes = [vp, i32, i32]
    L.parse_layer_to_mfma16.restype = C.c_int
    L.parse_layer_to_mfma16.argtypes = [C.POINTER(_Layer), vp, vp, vp]
    L.parse_route_workspace_bytes.restype = sz; L.parse_route_workspace_bytes.argtypes = [i32, i32, i32]
    L.parse_pool.restype = C.c_int
    L.parse_pool.argtypes = [vp, i32, i32, vp, i32, i32, vp, vp, sz, vp]
    L.parse_route.restype = C.c_int
    L.parse_route.argtypes = [vp, i32, i32, vp, i32, i32, vp, i32, i32, vp, i32, vp, vp, vp, sz, vp]
    L.parse_route_shared.restype = C.c_int
    L.parse_route_shared.argtypes = [vp, i32, i32, vp, i32, i32, vp, i32, i32, i32, vp, i32, vp, vp, vp, sz, vp]
    L.parse_cache_set_shared.restype = C.c_int; L.parse_cache_set_shared.argtypes = [vp, i32]
    L.parse_route_ranks_workspace_bytes.restype = sz
    L.parse_route_ranks_workspace_bytes.argtypes = [i32, i32, i32, i32]
    L.parse_route_ranks.restype = C.c_int
    L.parse_route_ranks.argtypes = [vp, i32, i32, vp, i32, i32, vp, i32, i32, vp, i32, vp, vp, vp, sz, vp]
    L.parse_pack_ranks.restype = C.c_int
    L.parse_pack_ranks.argtypes = [C.POINTER(_Layer), vp, i32, i32, i32, vp, vp, vp]
    L.parse_router_grad_workspace_bytes.restype = sz
    L.parse_router_grad_workspace_bytes.argtypes = [C.POINTER(_Layer), i32, i32]
    L.parse_router_grad.restype = C.c_int
    L.parse_router_grad.argtypes = [C.POINTER(_Layer), vp, vp, i32, vp, i32, vp, vp, vp, vp, i32, i32, f32, f32, vp, vp,
                                    vp, sz, vp]
    L.parse_cache_create.restype = C.c_int
    L.parse_cache_create.argtypes = [C.POINTER(vp), i32, i32, i32, i32, i32]
    L.parse_cache_destroy.restype = C.c_int; L.parse_cache_destroy.argtypes = [vp]
    L.parse_cache_clear.restype = C.c_int; L.parse_cache_clear.argtypes = [vp, vp]
    L.parse_cache_count.restype = C.c_int; L.parse_cache_count.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), vp]
    L.parse_cache_insert.restype = C.c_int; L.parse_cache_insert.argtypes = [vp, vp, vp, vp]
    L.parse_cache_lookup.restype = C.c_int
    L.parse_cache_lookup.argtypes = [vp, vp, i32, f32, vp, vp, vp, vp]
    L.parse_cache_lookup_or_route.restype = C.c_int
    L.parse_cache_lookup_or_route.argtypes = [vp, vp, i32, f32, vp, i32, vp, vp, vp, vp, vp]
    L.parse_bucket_patterns.restype = C.c_int
    L.parse_bucket_patterns.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    L.parse_pack_experts.restype = C.c_int
    L.parse_pack_experts.argtypes = [C.POINTER(_Layer), vp, i32, vp, vp, vp]
    L.parse_pack_patterns.restype = C.c_int
    L.parse_pack_patterns.argtypes = [C.POINTER(_Layer), vp, i32, i32, vp, vp, i32, vp, vp, vp]
    L.parse_pack_new_entries.restype = C.c_int
    L.parse_pack_new_entries.argtypes = [C.POINTER(_Layer), vp, i32, i32, i32, vp, vp, i32, vp, vp, vp]
    L.parse_lowrank_workspace_bytes.restype = sz
    L.parse_lowrank_workspace_bytes.argtypes = [i32, C.POINTER(_Layer), i32, i32, i32, i32]
    L.parse_prefill_plan_bytes.restype = sz; L.parse_prefill_plan_bytes.argtypes = [i32, i32, i32]
    L.parse_prefill_plan.restype = C.c_int; L.parse_prefill_plan.argtypes = [vp, vp, i32, i32, i32, vp, sz, vp]
    L.parse_bucket_and_plan.restype = C.c_int
    L.parse_bucket_and_plan.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, sz, vp]
    L.parse_lowrank_prefill_planned_workspace_bytes.restype = sz
    L.parse_lowrank_prefill_planned_workspace_bytes.argtypes = [C.POINTER(_Layer), i32, i32, i32, i32]
    L.parse_lowrank_prefill_planned.restype = C.c_int
    L.parse_lowrank_prefill_planned.argtypes = [C.POINTER(_Layer), C.POINTER(_Patterns), vp, i32, vp, vp, i32, vp, vp, vp,
                                                sz, vp]
    L.parse_lowrank_decode_multi_workspace_bytes.restype = sz
    L.parse_lowrank_decode_multi_workspace_bytes.argtypes = [C.POINTER(_Layer), i32]
    L.parse_lowrank_decode_multi.restype = C.c_int
    L.parse_lowrank_decode_multi.argtypes = [C.POINTER(_Layer), C.POINTER(_Patterns), i32, vp, i32, vp,
                                             C.POINTER(C.c_void_p), vp, sz, vp]
    L.parse_lowrank_prefill_multi_workspace_bytes.restype = sz
    L.parse_lowrank_prefill_multi_workspace_bytes.argtypes = [C.POINTER(_Layer), C.POINTER(_Patterns), i32, i32]
    L.parse_lowrank_prefill_multi.restype = C.c_int
    L.parse_lowrank_prefill_multi.argtypes = [C.POINTER(_Layer), C.POINTER(_Patterns), i32, vp, i32, vp, vp, i32,
                                              C.POINTER(C.c_void_p), vp, sz, vp]
    L.parse_lowrank_forward.restype = C.c_int
    L.parse_lowrank_forward.argtypes = [i32, C.POINTER(_Layer), C.POINTER(_Patterns), vp, i32, vp, vp, i32, vp, vp,
                                        sz, vp]
    L.parse_probe_mfma_bf16.restype = C.c_int; L.parse_probe_mfma_bf16.argtypes = [vp, i32, i32, vp, vp]
    L.parse_probe_read.restype = C.c_int; L.parse_probe_read.argtypes = [vp, sz, i32, vp, vp]
    L.parse_probe_copy.restype = C.c_int; L.parse_probe_copy.argtypes = [vp, vp, sz, vp]
    L.parse_decode_plan_bytes.restype = sz; L.parse_decode_plan_bytes.argtypes = [i32]
    L.parse_decode_plan.restype = C.c_int
    L.parse_decode_plan.argtypes = [C.POINTER(_Layer), C.POINTER(_Patterns), i32, vp, i32, vp, sz, vp]
    L.parse_lowrank_decode_planned_workspace_bytes.restype = sz
    L.parse_lowrank_decode_planned_workspace_bytes.argtypes = [C.POINTER(_Layer), i32]
    L.parse_lowrank_decode_planned.restype = C.c_int
    L.parse_lowrank_decode_planned.argtypes = [C.POINTER(_Layer), i32, vp, i32, vp, C.POINTER(C.c_void_p), vp, sz, vp]
    L.parse_lowrank_decode_static_capacity.restype = sz; L.parse_lowrank_decode_static_capacity.argtypes = []
    L.parse_lowrank_decode_static.restype = C.c_int
    L.parse_lowrank_decode_static.argtypes = [C.POINTER(_Layer), C.POINTER(_Patterns), vp, i32, vp, vp, vp]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().parse_status_string(status).decode()


def version() -> int:
    return lib().parse_version()


def _check(status: int, where: str):
    if status != 0:
        raise ParseError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def bf16_from_bits(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy uint16 bfloat16 bit patterns -> torch.bfloat16 tensor on `device` (no value conversion)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PARSE_F32
    if t.dtype == torch.bfloat16:
        return PARSE_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


class Layer:
    """parse_layer: device tensors Vt [R][n] and Ut [R][m] (row-major view; in PARSE_MFMA16 the same
    number of elements in operand order)."""

    def __init__(self, Vt: torch.Tensor, Ut: torch.Tensor, n: int, m: int, R: int, G: int,
                 layout: int = PARSE_ROWMAJOR):
        self.Vt, self.Ut, self.n, self.m, self.R, self.G, self.layout = Vt, Ut, n, m, R, G, layout
        self.dtype = _dtype_code(Vt)

    @property
    def gs(self) -> int:
        return self.R // self.G

    def c(self) -> _Layer:
        return _Layer(self.n, self.m, self.R, self.G, self.dtype, self.layout, self.Vt.data_ptr(), self.Ut.data_ptr())


class Patterns:
    """parse_patterns."""

    def __init__(self, k: int, n_patterns: int, Vt_S=None, Ut_S=None, subsets=None, subset_stride=None,
                 Vt_shared=None, Ut_shared=None, n_shared: int = 0, schedule: int = PARSE_SCHED_AUTO):
        self.k, self.n_patterns, self.Vt_S, self.Ut_S, self.subsets = k, n_patterns, Vt_S, Ut_S, subsets
        self.subset_stride = k if subset_stride is None else subset_stride
        self.Vt_shared, self.Ut_shared, self.n_shared = Vt_shared, Ut_shared, n_shared
        self.schedule = schedule

    def with_schedule(self, schedule: int) -> "Patterns":
        """The same patterns with another prefill schedule (parse_prefill_schedule)."""
        return Patterns(self.k, self.n_patterns, self.Vt_S, self.Ut_S, self.subsets, self.subset_stride,
                        self.Vt_shared, self.Ut_shared, self.n_shared, schedule)

    def c(self) -> _Patterns:
        return _Patterns(None if self.Vt_S is None else self.Vt_S.data_ptr(),
                         None if self.Ut_S is None else self.Ut_S.data_ptr(),
                         None if self.subsets is None else self.subsets.data_ptr(),
                         self.subset_stride, self.n_patterns, self.k,
                         None if self.Vt_shared is None else self.Vt_shared.data_ptr(),
                         None if self.Ut_shared is None else self.Ut_shared.data_ptr(), self.n_shared,
                         self.schedule)


def check_offsets(tok_offsets_host: np.ndarray, rows: int) -> int:
    a = np.ascontiguousarray(tok_offsets_host, dtype=np.int32)
    return lib().parse_check_offsets(a.ctypes.data_as(C.c_void_p), len(a) - 1, rows)


def check_subset(subset_host: np.ndarray, G: int) -> int:
    a = np.ascontiguousarray(subset_host, dtype=np.int32)
    return lib().parse_check_subset(a.ctypes.data_as(C.c_void_p), len(a), G)


def layer_to_mfma16(layer: Layer) -> Layer:
    Vt = torch.empty_like(layer.Vt); Ut = torch.empty_like(layer.Ut)
    cl = layer.c()
    _check(lib().parse_layer_to_mfma16(C.byref(cl), _ptr(Vt), _ptr(Ut), _stream()), "parse_layer_to_mfma16")
    return Layer(Vt, Ut, layer.n, layer.m, layer.R, layer.G, PARSE_MFMA16)


def route_workspace_bytes(rows: int, P: int, d: int) -> int:
    return lib().parse_route_workspace_bytes(rows, P, d)


def route(X, tok_offsets, Wr, k, subset_out=None, subset_stride=None, scores_out=None, emb_out=None,
          workspace=None, n_shared=None):
    """parse_route (parse_route_shared when n_shared is given).  X [rows][d], tok_offsets int32 device [P+1],
    Wr float device [G][d]."""
    rows, d = X.shape
    P = tok_offsets.numel() - 1
    G = Wr.shape[0]
    stride = k if subset_stride is None else subset_stride
    if subset_out is None:
        subset_out = torch.empty((P, stride), dtype=torch.int32, device=X.device)
    if workspace is None:
        workspace = torch.empty(max(route_workspace_bytes(rows, P, d), 256), dtype=torch.uint8, device=X.device)
    if n_shared is None:
        _check(lib().parse_route(_ptr(X), _dtype_code(X), rows, _ptr(tok_offsets), P, d, _ptr(Wr), G, k,
                                 _ptr(subset_out), stride, _ptr(scores_out), _ptr(emb_out), _ptr(workspace),
                                 workspace.numel(), _stream()), "parse_route")
    else:
        _check(lib().parse_route_shared(_ptr(X), _dtype_code(X), rows, _ptr(tok_offsets), P, d, _ptr(Wr), G, k, n_shared,
                                        _ptr(subset_out), stride, _ptr(scores_out), _ptr(emb_out), _ptr(workspace),
                                        workspace.numel(), _stream()), "parse_route_shared")
    return subset_out


def pool(X, tok_offsets, emb_out=None, workspace=None):
    """parse_pool: the prompt embeddings [P][d] (float32) alone."""
    rows, d = X.shape
    P = tok_offsets.numel() - 1
    if emb_out is None:
        emb_out = torch.empty((P, d), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = torch.empty(max(route_workspace_bytes(rows, P, d), 256), dtype=torch.uint8, device=X.device)
    _check(lib().parse_pool(_ptr(X), _dtype_code(X), rows, _ptr(tok_offsets), P, d, _ptr(emb_out), _ptr(workspace),
                            workspace.numel(), _stream()), "parse_pool")
    return emb_out


class Cache:
    """parse_cache handle."""

    def __init__(self, capacity: int, d: int, L: int, k: int, max_batch: int):
        self.capacity, self.d, self.L, self.k, self.max_batch = capacity, d, L, k, max_batch
        h = C.c_void_p()
        _check(lib().parse_cache_create(C.byref(h), capacity, d, L, k, max_batch), "parse_cache_create")
        self._h = h

    def close(self):
        if self._h:
            lib().parse_cache_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def clear(self):
        _check(lib().parse_cache_clear(self._h, _stream()), "parse_cache_clear")

    def set_shared(self, n_shared: int):
        _check(lib().parse_cache_set_shared(self._h, n_shared), "parse_cache_set_shared")

    def count(self) -> int:
        n, dropped = C.c_int32(0), C.c_int32(0)
        _check(lib().parse_cache_count(self._h, C.byref(n), C.byref(dropped), _stream()), "parse_cache_count")
        return n.value

    def dropped(self) -> int:
        """Explicit inserts dropped (cache full) since create / clear."""
        n, dropped = C.c_int32(0), C.c_int32(0)
        _check(lib().parse_cache_count(self._h, C.byref(n), C.byref(dropped), _stream()), "parse_cache_count")
        return dropped.value

    def insert(self, emb, subsets):
        _check(lib().parse_cache_insert(self._h, _ptr(emb), _ptr(subsets), _stream()), "parse_cache_insert")

    def lookup(self, emb, tau, entry_out=None, sim_out=None, subset_out=None):
        P = emb.shape[0]
        dev = emb.device
        entry_out = torch.empty(P, dtype=torch.int32, device=dev) if entry_out is None else entry_out
        sim_out = torch.empty(P, dtype=torch.float32, device=dev) if sim_out is None else sim_out
        if subset_out is None:
            subset_out = torch.full((P, self.L, self.k), -1, dtype=torch.int32, device=dev)
        _check(lib().parse_cache_lookup(self._h, _ptr(emb), P, tau, _ptr(entry_out), _ptr(sim_out), _ptr(subset_out),
                                        _stream()), "parse_cache_lookup")
        return entry_out, sim_out, subset_out

    def lookup_or_route(self, emb, tau, Wr, entry_out=None, hit_out=None, sim_out=None, subset_out=None):
        P = emb.shape[0]
        dev = emb.device
        G = Wr.shape[-2]
        entry_out = torch.empty(P, dtype=torch.int32, device=dev) if entry_out is None else entry_out
        hit_out = torch.empty(P, dtype=torch.uint8, device=dev) if hit_out is None else hit_out
        sim_out = torch.empty(P, dtype=torch.float32, device=dev) if sim_out is None else sim_out
        if subset_out is None:
            subset_out = torch.empty((P, self.L, self.k), dtype=torch.int32, device=dev)
        _check(lib().parse_cache_lookup_or_route(self._h, _ptr(emb), P, tau, _ptr(Wr), G, _ptr(entry_out),
                                                 _ptr(hit_out), _ptr(sim_out), _ptr(subset_out), _stream()),
               "parse_cache_lookup_or_route")
        return entry_out, hit_out, sim_out, subset_out


def bucket_patterns(subset, k, subset_stride=None, out=None):
    """parse_bucket_patterns -> (pattern_id[P], perm[P], bucket_off[P+1], n_patterns[1], rep[P]) device int32."""
    P = subset.shape[0]
    stride = (subset.numel() // P) if subset_stride is None else subset_stride
    dev = subset.device
    if out is None:
        out = (torch.empty(P, dtype=torch.int32, device=dev), torch.empty(P, dtype=torch.int32, device=dev),
               torch.empty(P + 1, dtype=torch.int32, device=dev), torch.empty(1, dtype=torch.int32, device=dev),
               torch.empty(P, dtype=torch.int32, device=dev))
    pid, perm, off, npat, rep = out
    _check(lib().parse_bucket_patterns(_ptr(subset), P, k, stride, _ptr(pid), _ptr(perm), _ptr(off), _ptr(npat),
                                       _ptr(rep), _stream()), "parse_bucket_patterns")
    return out


def pack_experts(layer: Layer, subset, Vt_S=None, Ut_S=None):
    """parse_pack_experts: subset int32 device [k] -> (Vt_S [k*gs][n], Ut_S [k*gs][m])."""
    k = subset.numel()
    if Vt_S is None:
        Vt_S = torch.empty((k * layer.gs, layer.n), dtype=layer.Vt.dtype, device=layer.Vt.device)
    if Ut_S is None:
        Ut_S = torch.empty((k * layer.gs, layer.m), dtype=layer.Ut.dtype, device=layer.Ut.device)
    cl = layer.c()
    _check(lib().parse_pack_experts(C.byref(cl), _ptr(subset), k, _ptr(Vt_S), _ptr(Ut_S), _stream()),
           "parse_pack_experts")
    return Vt_S, Ut_S


def pack_patterns(layer: Layer, subset, subset_stride, k, rep, n_patterns, max_patterns, Vt_S=None, Ut_S=None):
    """parse_pack_patterns -> (Vt_S [max_patterns][k*gs][n], Ut_S [max_patterns][k*gs][m])."""
    if Vt_S is None:
        Vt_S = torch.empty((max_patterns, k * layer.gs, layer.n), dtype=layer.Vt.dtype, device=layer.Vt.device)
    if Ut_S is None:
        Ut_S = torch.empty((max_patterns, k * layer.gs, layer.m), dtype=layer.Ut.dtype, device=layer.Ut.device)
    cl = layer.c()
    _check(lib().parse_pack_patterns(C.byref(cl), _ptr(subset), subset_stride, k, _ptr(rep), _ptr(n_patterns),
                                     max_patterns, _ptr(Vt_S), _ptr(Ut_S), _stream()), "parse_pack_patterns")
    return Vt_S, Ut_S


def pack_new_entries(layer: Layer, subset, subset_stride, k, entry, hit, Vt_S, Ut_S):
    """parse_pack_new_entries: packs the subsets of this batch's new cache entries into their slots of
    Vt_S [n_slots][k*gs][n] / Ut_S [n_slots][k*gs][m]."""
    cl = layer.c()
    _check(lib().parse_pack_new_entries(C.byref(cl), _ptr(subset), subset_stride, k, entry.numel(), _ptr(entry),
                                        _ptr(hit), Vt_S.shape[0], _ptr(Vt_S), _ptr(Ut_S), _stream()),
           "parse_pack_new_entries")
    return Vt_S, Ut_S


def lowrank_workspace_bytes(mode: int, layer: Layer, rows: int, k: int, P: int = 0, n_patterns: int = 0) -> int:
    """parse_lowrank_workspace_bytes; P and n_patterns size the planned prefill schedule (0: the other schedules only)."""
    cl = layer.c()
    return lib().parse_lowrank_workspace_bytes(mode, C.byref(cl), rows, k, P, n_patterns)


def prefill_plan_bytes(rows: int, P: int, n_patterns: int) -> int:
    return int(lib().parse_prefill_plan_bytes(rows, P, n_patterns))


def prefill_plan(tok_offsets, pattern_id, rows: int, n_patterns: int, plan=None):
    """parse_prefill_plan -> the plan buffer (uint8 device tensor)."""
    P = pattern_id.numel()
    if plan is None:
        plan = torch.empty(prefill_plan_bytes(rows, P, n_patterns), dtype=torch.uint8, device=pattern_id.device)
    _check(lib().parse_prefill_plan(_ptr(tok_offsets), _ptr(pattern_id), P, rows, n_patterns, _ptr(plan), plan.numel(),
                                    _stream()), "parse_prefill_plan")
    return plan


def bucket_and_plan(subset, k, subset_stride, tok_offsets, plan_pattern_id, rows: int, n_patterns: int, out=None, plan=None):
    """parse_bucket_and_plan -> (bucket outputs as bucket_patterns, plan as prefill_plan)."""
    P = plan_pattern_id.numel()
    stride = (subset.numel() // P) if subset_stride is None else subset_stride
    dev = subset.device
    if out is None:
        out = (torch.empty(P, dtype=torch.int32, device=dev), torch.empty(P, dtype=torch.int32, device=dev),
               torch.empty(P + 1, dtype=torch.int32, device=dev), torch.empty(1, dtype=torch.int32, device=dev),
               torch.empty(P, dtype=torch.int32, device=dev))
    if plan is None:
        plan = torch.empty(prefill_plan_bytes(rows, P, n_patterns), dtype=torch.uint8, device=dev)
    pid, perm, off, npat, rep = out
    _check(lib().parse_bucket_and_plan(_ptr(subset), P, k, stride, _ptr(pid), _ptr(perm), _ptr(off), _ptr(npat), _ptr(rep),
                                       _ptr(tok_offsets), _ptr(plan_pattern_id), rows, n_patterns, _ptr(plan), plan.numel(),
                                       _stream()), "parse_bucket_and_plan")
    return out, plan


def lowrank_prefill_planned_workspace_bytes(layer: Layer, rows: int, P: int, k: int, n_patterns: int) -> int:
    cl = layer.c()
    return int(lib().parse_lowrank_prefill_planned_workspace_bytes(C.byref(cl), rows, P, k, n_patterns))


def lowrank_prefill_planned(layer: Layer, patterns: Patterns, X, tok_offsets, pattern_id, plan, Y=None, workspace=None):
    """parse_lowrank_prefill_planned.  Returns Y [rows][m]."""
    rows, P = X.shape[0], pattern_id.numel()
    if Y is None:
        Y = torch.empty((rows, layer.m), dtype=X.dtype, device=X.device)
    if workspace is None:
        need = lowrank_prefill_planned_workspace_bytes(layer, rows, P, patterns.k, patterns.n_patterns)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    cl, cp = layer.c(), patterns.c()
    _check(lib().parse_lowrank_prefill_planned(C.byref(cl), C.byref(cp), _ptr(X), rows, _ptr(tok_offsets), _ptr(pattern_id), P,
                                               _ptr(plan), _ptr(Y),
                                               _ptr(workspace), workspace.numel(), _stream()),
           "parse_lowrank_prefill_planned")
    return Y


def lowrank_forward(mode: int, layer: Layer, patterns: Patterns, X, tok_offsets, pattern_id, Y=None,
                    workspace=None, no_workspace=False):
    """parse_lowrank_forward.  Returns Y [rows][m].  no_workspace=True passes NULL (bf16 prefill: fused kernel)."""
    rows = X.shape[0]
    P = pattern_id.numel()
    if Y is None:
        Y = torch.empty((rows, layer.m), dtype=X.dtype, device=X.device)
    need = lowrank_workspace_bytes(mode, layer, rows, patterns.k, P, patterns.n_patterns)
    if workspace is None and need > 0 and not no_workspace:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    cl, cp = layer.c(), patterns.c()
    _check(lib().parse_lowrank_forward(mode, C.byref(cl), C.byref(cp), _ptr(X), rows, _ptr(tok_offsets),
                                       _ptr(pattern_id), P, _ptr(Y), _ptr(workspace),
                                       0 if workspace is None else workspace.numel(), _stream()),
           "parse_lowrank_forward")
    return Y


def lowrank_decode_static(layer: Layer, patterns: Patterns, X, pattern_id, Y):
    """parse_lowrank_decode_static: the decode step on the library's fixed scratch array; Y is the caller's."""
    cl, cp = layer.c(), patterns.c()
    _check(lib().parse_lowrank_decode_static(C.byref(cl), C.byref(cp), _ptr(X), X.shape[0], _ptr(pattern_id), _ptr(Y),
                                             _stream()), "parse_lowrank_decode_static")
    return Y


def probe_mfma_bf16(data, workgroups: int, iters: int, out):
    _check(lib().parse_probe_mfma_bf16(_ptr(data), workgroups, iters, _ptr(out), _stream()), "parse_probe_mfma_bf16")


def probe_read(src, nbytes: int, workgroups: int, sink=None):
    _check(lib().parse_probe_read(_ptr(src), nbytes, workgroups, _ptr(sink), _stream()), "parse_probe_read")


def probe_copy(src, dst, nbytes: int):
    _check(lib().parse_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream()), "parse_probe_copy")


def decode_plan(layers, patterns, pattern_id, plan=None):
    """parse_decode_plan -> the plan buffer (uint8 device tensor) for these layers and this batch."""
    nl = len(layers)
    if plan is None:
        plan = torch.empty(int(lib().parse_decode_plan_bytes(nl)), dtype=torch.uint8, device=pattern_id.device)
    larr = (_Layer * nl)(*[l.c() for l in layers])
    parr = (_Patterns * nl)(*[p.c() for p in patterns])
    _check(lib().parse_decode_plan(larr, parr, nl, _ptr(pattern_id), pattern_id.numel(), _ptr(plan), plan.numel(),
                                   _stream()), "parse_decode_plan")
    return plan


def lowrank_decode_planned_workspace_bytes(layers) -> int:
    arr = (_Layer * len(layers))(*[l.c() for l in layers])
    return int(lib().parse_lowrank_decode_planned_workspace_bytes(arr, len(layers)))


def lowrank_decode_planned(layers, X, plan, Ys=None, workspace=None):
    """parse_lowrank_decode_planned: one decode step of several layers that share X over a ready plan."""
    rows, nl = X.shape[0], len(layers)
    if Ys is None:
        Ys = [torch.empty((rows, l.m), dtype=X.dtype, device=X.device) for l in layers]
    if workspace is None:
        workspace = torch.empty(max(lowrank_decode_planned_workspace_bytes(layers), 256), dtype=torch.uint8, device=X.device)
    larr = (_Layer * nl)(*[l.c() for l in layers])
    yarr = (C.c_void_p * nl)(*[y.data_ptr() for y in Ys])
    _check(lib().parse_lowrank_decode_planned(larr, nl, _ptr(X), rows, _ptr(plan), yarr, _ptr(workspace),
                                              workspace.numel(), _stream()), "parse_lowrank_decode_planned")
    return Ys


def lowrank_decode_multi_workspace_bytes(layers) -> int:
    arr = (_Layer * len(layers))(*[l.c() for l in layers])
    return int(lib().parse_lowrank_decode_multi_workspace_bytes(arr, len(layers)))


def lowrank_decode_multi(layers, patterns, X, pattern_id, Ys=None, workspace=None):
    """parse_lowrank_decode_multi: one decode step of several layers that share X.  Returns the list of Y."""
    rows = X.shape[0]
    nl = len(layers)
    if Ys is None:
        Ys = [torch.empty((rows, l.m), dtype=X.dtype, device=X.device) for l in layers]
    if workspace is None:
        workspace = torch.empty(max(lowrank_decode_multi_workspace_bytes(layers), 256), dtype=torch.uint8, device=X.device)
    larr = (_Layer * nl)(*[l.c() for l in layers])
    parr = (_Patterns * nl)(*[p.c() for p in patterns])
    yarr = (C.c_void_p * nl)(*[y.data_ptr() for y in Ys])
    _check(lib().parse_lowrank_decode_multi(larr, parr, nl, _ptr(X), rows, _ptr(pattern_id), yarr, _ptr(workspace),
                                            workspace.numel(), _stream()), "parse_lowrank_decode_multi")
    return Ys


def lowrank_prefill_multi_workspace_bytes(layers, patterns, rows: int) -> int:
    nl = len(layers)
    larr = (_Layer * nl)(*[l.c() for l in layers])
    parr = (_Patterns * nl)(*[p.c() for p in patterns])
    return int(lib().parse_lowrank_prefill_multi_workspace_bytes(larr, parr, nl, rows))


def lowrank_prefill_multi(layers, patterns, X, tok_offsets, pattern_id, Ys=None, workspace=None):
    """parse_lowrank_prefill_multi: prefill of several layers that share X in two launches.  Returns the list of Y."""
    rows, nl = X.shape[0], len(layers)
    P = pattern_id.numel()
    if Ys is None:
        Ys = [torch.empty((rows, l.m), dtype=X.dtype, device=X.device) for l in layers]
    larr = (_Layer * nl)(*[l.c() for l in layers])
    parr = (_Patterns * nl)(*[p.c() for p in patterns])
    if workspace is None:
        need = int(lib().parse_lowrank_prefill_multi_workspace_bytes(larr, parr, nl, rows))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    yarr = (C.c_void_p * nl)(*[y.data_ptr() for y in Ys])
    _check(lib().parse_lowrank_prefill_multi(larr, parr, nl, _ptr(X), rows, _ptr(tok_offsets), _ptr(pattern_id), P, yarr,
                                             _ptr(workspace), workspace.numel(), _stream()), "parse_lowrank_prefill_multi")
    return Ys


def route_ranks(X, tok_offsets, Wr, K, subset_out=None, subset_stride=None, scores_out=None, emb_out=None,
                workspace=None):
    """parse_route_ranks: rank-granular routing.  Wr float device [G][d] -> subset int32 [P][K] ascending."""
    rows, d = X.shape
    P = tok_offsets.numel() - 1
    G = Wr.shape[0]
    stride = K if subset_stride is None else subset_stride
    if subset_out is None:
        subset_out = torch.empty((P, stride), dtype=torch.int32, device=X.device)
    if workspace is None:
        need = int(lib().parse_route_ranks_workspace_bytes(rows, P, d, G))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    _check(lib().parse_route_ranks(_ptr(X), _dtype_code(X), rows, _ptr(tok_offsets), P, d, _ptr(Wr), G, K,
                                   _ptr(subset_out), stride, _ptr(scores_out), _ptr(emb_out), _ptr(workspace),
                                   workspace.numel(), _stream()), "parse_route_ranks")
    return subset_out


def pack_ranks(layer: Layer, subset, K, n_patterns, subset_stride=None, Vt_S=None, Ut_S=None):
    """parse_pack_ranks: gathers K rank rows per pattern of a row-major bf16 layer into operand-order blocks."""
    stride = K if subset_stride is None else subset_stride
    if Vt_S is None:
        Vt_S = torch.empty((n_patterns, K, layer.n), dtype=layer.Vt.dtype, device=layer.Vt.device)
    if Ut_S is None:
        Ut_S = torch.empty((n_patterns, K, layer.m), dtype=layer.Ut.dtype, device=layer.Ut.device)
    cl = layer.c()
    _check(lib().parse_pack_ranks(C.byref(cl), _ptr(subset), stride, K, n_patterns, _ptr(Vt_S), _ptr(Ut_S), _stream()),
           "parse_pack_ranks")
    return Vt_S, Ut_S


def rankmajor_left_factor(layer_rowmajor: Layer):
    """Ut ([R][m] row-major bf16) reordered like a right factor (what parse_router_grad takes as Ut_rankmajor)."""
    tmp = Layer(layer_rowmajor.Ut, layer_rowmajor.Ut, layer_rowmajor.m, layer_rowmajor.m, layer_rowmajor.R,
                layer_rowmajor.G, PARSE_ROWMAJOR)
    return layer_to_mfma16(tmp).Vt


def router_grad(layer: Layer, Ut_rankmajor, X, tok_offsets, Y_hat, Y_dense, emb, scores, k, temperature, eps,
                workspace=None):
    """parse_router_grad -> (loss [P], grad_Wr [G][d])."""
    rows, P, d = X.shape[0], tok_offsets.numel() - 1, emb.shape[1]
    cl = layer.c()
    if workspace is None:
        need = int(lib().parse_router_grad_workspace_bytes(C.byref(cl), rows, P))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    loss = torch.empty(P, dtype=torch.float32, device=X.device)
    grad = torch.empty((layer.G, d), dtype=torch.float32, device=X.device)
    _check(lib().parse_router_grad(C.byref(cl), _ptr(Ut_rankmajor), _ptr(X), rows, _ptr(tok_offsets), P, _ptr(Y_hat),
                                   _ptr(Y_dense), _ptr(emb), _ptr(scores), d, k, temperature, eps, _ptr(loss), _ptr(grad),
                                   _ptr(workspace), workspace.numel(), _stream()), "parse_router_grad")
    return loss, grad
