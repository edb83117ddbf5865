"""Thin ctypes binding of the C ABI declared in include/freeze.h.

Argument marshalling only: every step of a look-up runs in the HIP kernels of
libfreeze_hip.so.  PyTorch supplies device memory (tensors) and the stream.
There is no fallback: if the library is not built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "_lib", "libfreeze_hip.so")

FREEZE_OK, FREEZE_EINVAL, FREEZE_ELAYER, FREEZE_ENOTBUILT, FREEZE_EWORKSPACE, FREEZE_EHIP = 0, -1, -2, -3, -4, -5
FREEZE_ESCRATCH = -6
FREEZE_STATIC_SCRATCH_BYTES = 32 << 20
FREEZE_F32, FREEZE_BF16 = 0, 1

_lib = None


class FreezeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().freeze_strerror(code).decode() if _lib is not None else str(code)
        super().__init__(f"{where}: {msg} ({code})")


def lib():
    """Load libfreeze_hip.so (built by `python -m paper_2002_02645_amd.build` / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build the HIP library first "
                           "(python -m paper_2002_02645_amd.build); there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    p, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    L.freeze_create.restype = i32
    L.freeze_create.argtypes = [ctypes.POINTER(p), i32]
    L.freeze_destroy.restype = i32
    L.freeze_destroy.argtypes = [p]
    L.freeze_cache_storage_bytes.restype = sz
    L.freeze_cache_storage_bytes.argtypes = [i64, i64, i32]
    L.freeze_cache_build.restype = i32
    L.freeze_cache_build.argtypes = [p, i32, p, i32, i64, i64, p, ctypes.c_int32, p, sz, p]
    L.freeze_set_centring.restype = i32
    L.freeze_set_centring.argtypes = [p, i32]
    L.freeze_lookup_workspace_bytes.restype = sz
    L.freeze_lookup_workspace_bytes.argtypes = [p, i32, i64, i32, i32]
    L.freeze_lookup.restype = i32
    L.freeze_lookup.argtypes = [p, i32, p, i64, i32, i32, i32, p, p, p, p, p, p, sz, p]
    L.freeze_lookup_static.restype = i32
    L.freeze_lookup_static.argtypes = [p, i32, p, i64, i32, i32, i32, p, p, p, p, p, p]
    L.freeze_cascade_workspace_bytes.restype = sz
    L.freeze_cascade_workspace_bytes.argtypes = [p, i32, p, i64, i32, i32]
    L.freeze_lookup_cascade.restype = i32
    L.freeze_lookup_cascade.argtypes = [p, i32, p, p, i64, i32, p, i32, p, p, p, p, sz, p]
    L.freeze_compact_misses.restype = i32
    L.freeze_compact_misses.argtypes = [p, p, i64, p, p, p]
    L.freeze_lookup_confidence.restype = i32
    L.freeze_lookup_confidence.argtypes = [p, i32, p, i64, i32, ctypes.c_float, i32, p, p, p, p, p, p, p, sz, p]
    L.freeze_lookup_cascade_confidence.restype = i32
    L.freeze_lookup_cascade_confidence.argtypes = [p, i32, p, p, i64, i32, p, i32, p, p, p, p, sz, p]
    L.freeze_kmeans_storage_bytes.restype = sz
    L.freeze_kmeans_storage_bytes.argtypes = [i64, i64]
    L.freeze_kmeans_workspace_bytes.restype = sz
    L.freeze_kmeans_workspace_bytes.argtypes = [p, i64, i64, i64]
    L.freeze_kmeans_build.restype = i32
    L.freeze_kmeans_build.argtypes = [p, i32, p, i64, i64, p, ctypes.c_int32, p, i64, i32, p, sz, p, sz, p]
    L.freeze_kmeans_read.restype = i32
    L.freeze_kmeans_read.argtypes = [p, i32, p, p, p, p]
    L.freeze_projection_storage_bytes.restype = sz
    L.freeze_projection_storage_bytes.argtypes = [i64, i64, i32]
    L.freeze_projection_build.restype = i32
    L.freeze_projection_build.argtypes = [p, i32, p, i32, i64, i64, p, p, sz, p, sz, p]
    L.freeze_project_workspace_bytes.restype = sz
    L.freeze_project_workspace_bytes.argtypes = [p, i32, i64]
    L.freeze_project.restype = i32
    L.freeze_project.argtypes = [p, i32, p, i64, i32, p, p, sz, p]
    L.freeze_gather_rows.restype = i32
    L.freeze_gather_rows.argtypes = [p, i64, p, p, i64, p, p]
    L.freeze_compute_thresholds.restype = i32
    L.freeze_compute_thresholds.argtypes = [p, i32, p, p, i64, i32, i32, p, p, p, sz, p]
    L.freeze_lookup_stats_attach.restype = i32
    L.freeze_lookup_stats_attach.argtypes = [p, p]
    L.freeze_profile_enable.restype = i32
    L.freeze_profile_enable.argtypes = [p, i32]
    L.freeze_profile_read.restype = i32
    L.freeze_profile_read.argtypes = [p, p, p]
    L.freeze_profile_read_calls.restype = i32
    L.freeze_profile_read_calls.argtypes = [p, p, i32, p]
    L.freeze_calibrate_mfma.restype = i32
    L.freeze_calibrate_mfma.argtypes = [p, sz, p, p]
    L.freeze_calibrate_hbm_read.restype = i32
    L.freeze_calibrate_hbm_read.argtypes = [p, sz, p]
    L.freeze_strerror.restype = ctypes.c_char_p
    L.freeze_strerror.argtypes = [i32]
    _lib = L
    return L


def _ptr(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc: int, where: str):
    if rc != FREEZE_OK:
        raise FreezeError(rc, where)


# ---- functions with the names of the C entry points ---------------------------------------------

def freeze_strerror(code: int) -> str:
    return lib().freeze_strerror(code).decode()


def freeze_create(num_layers: int) -> ctypes.c_void_p:
    h = ctypes.c_void_p()
    _check(lib().freeze_create(ctypes.byref(h), num_layers), "freeze_create")
    return h


def freeze_destroy(ctx) -> None:
    _check(lib().freeze_destroy(ctx), "freeze_destroy")


def freeze_cache_storage_bytes(n: int, d: int, entries_dtype: int) -> int:
    return int(lib().freeze_cache_storage_bytes(n, d, entries_dtype))


def freeze_cache_build(ctx, layer: int, entries: torch.Tensor, labels: torch.Tensor, num_classes: int,
                       storage: torch.Tensor, stream=None) -> None:
    assert entries.is_cuda and entries.is_contiguous() and entries.dim() == 2
    assert labels.is_cuda and labels.dtype == torch.int32 and labels.is_contiguous()
    dt = {torch.float32: FREEZE_F32, torch.bfloat16: FREEZE_BF16}[entries.dtype]
    n, d = entries.shape
    assert labels.numel() == n
    _check(lib().freeze_cache_build(ctx, layer, _ptr(entries), dt, n, d, _ptr(labels), num_classes, _ptr(storage),
                                    storage.numel() * storage.element_size(), _stream(stream)), "freeze_cache_build")


def freeze_set_centring(ctx, mode: int) -> None:
    """0: caches built from now on are never centred, 1: when their mean dominates their spread (default), 2: always."""
    _check(lib().freeze_set_centring(ctx, mode), "freeze_set_centring")


def freeze_lookup_workspace_bytes(ctx, layer: int, b: int, k: int, rescore_r: int = 0) -> int:
    return int(lib().freeze_lookup_workspace_bytes(ctx, layer, b, k, rescore_r))


def freeze_lookup(ctx, layer: int, queries: torch.Tensor, k: int, vote_threshold: int, rescore_r: int,
                  out_labels: torch.Tensor, out_hit: torch.Tensor, out_votes: torch.Tensor,
                  out_nbr_idx: torch.Tensor, out_nbr_dist: torch.Tensor, workspace: torch.Tensor,
                  stream=None) -> None:
    assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous() and queries.dim() == 2
    b = queries.shape[0]
    _check(lib().freeze_lookup(ctx, layer, _ptr(queries), b, k, vote_threshold, rescore_r, _ptr(out_labels),
                               _ptr(out_hit), _ptr(out_votes), _ptr(out_nbr_idx), _ptr(out_nbr_dist),
                               _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "freeze_lookup")


def freeze_lookup_static(ctx, layer: int, queries: torch.Tensor, k: int, vote_threshold: int, rescore_r: int,
                         out_labels: torch.Tensor, out_hit: torch.Tensor, out_votes: torch.Tensor,
                         out_nbr_idx: torch.Tensor, out_nbr_dist: torch.Tensor, stream=None) -> None:
    assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous() and queries.dim() == 2
    b = queries.shape[0]
    _check(lib().freeze_lookup_static(ctx, layer, _ptr(queries), b, k, vote_threshold, rescore_r, _ptr(out_labels),
                                      _ptr(out_hit), _ptr(out_votes), _ptr(out_nbr_idx), _ptr(out_nbr_dist),
                                      _stream(stream)), "freeze_lookup_static")


def freeze_cascade_workspace_bytes(ctx, layers: Sequence[int], b: int, k: int, rescore_r: int = 0) -> int:
    arr = (ctypes.c_int * len(layers))(*layers)
    return int(lib().freeze_cascade_workspace_bytes(ctx, len(layers), arr, b, k, rescore_r))


def freeze_lookup_cascade(ctx, layers: Sequence[int], queries_per_layer: Sequence[torch.Tensor], k: int,
                          vote_thresholds: Sequence[int], rescore_r: int, out_labels: torch.Tensor,
                          out_exit_layer: torch.Tensor, out_hits_per_layer: torch.Tensor, workspace: torch.Tensor,
                          stream=None) -> None:
    nl = len(layers)
    assert len(queries_per_layer) == nl and len(vote_thresholds) == nl
    b = queries_per_layer[0].shape[0]
    for q in queries_per_layer:
        assert q.is_cuda and q.dtype == torch.float32 and q.is_contiguous() and q.shape[0] == b
    larr = (ctypes.c_int * nl)(*layers)
    tarr = (ctypes.c_int * nl)(*vote_thresholds)
    qarr = (ctypes.c_void_p * nl)(*[q.data_ptr() for q in queries_per_layer])
    _check(lib().freeze_lookup_cascade(ctx, nl, larr, qarr, b, k, tarr, rescore_r, _ptr(out_labels),
                                       _ptr(out_exit_layer), _ptr(out_hits_per_layer), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream)),
           "freeze_lookup_cascade")


def freeze_lookup_confidence(ctx, layer: int, queries: torch.Tensor, k: int, conf_threshold: float, rescore_r: int,
                             out_labels: torch.Tensor, out_hit: torch.Tensor, out_conf: torch.Tensor,
                             out_votes: torch.Tensor, out_nbr_idx: torch.Tensor, out_nbr_dist: torch.Tensor,
                             workspace: torch.Tensor, stream=None) -> None:
    assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous() and queries.dim() == 2
    b = queries.shape[0]
    _check(lib().freeze_lookup_confidence(ctx, layer, _ptr(queries), b, k, conf_threshold, rescore_r,
                                          _ptr(out_labels), _ptr(out_hit), _ptr(out_conf), _ptr(out_votes),
                                          _ptr(out_nbr_idx), _ptr(out_nbr_dist), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)),
           "freeze_lookup_confidence")


def _cascade_arrays(layers, queries_per_layer):
    nl = len(layers)
    assert len(queries_per_layer) == nl
    b = queries_per_layer[0].shape[0]
    for q in queries_per_layer:
        assert q.is_cuda and q.dtype == torch.float32 and q.is_contiguous() and q.shape[0] == b
    larr = (ctypes.c_int * nl)(*layers)
    qarr = (ctypes.c_void_p * nl)(*[q.data_ptr() for q in queries_per_layer])
    return nl, b, larr, qarr


def freeze_lookup_cascade_confidence(ctx, layers: Sequence[int], queries_per_layer: Sequence[torch.Tensor], k: int,
                                     conf_thresholds: Sequence[float], rescore_r: int, out_labels: torch.Tensor,
                                     out_exit_layer: torch.Tensor, out_hits_per_layer: torch.Tensor,
                                     workspace: torch.Tensor, stream=None) -> None:
    nl, b, larr, qarr = _cascade_arrays(layers, queries_per_layer)
    assert len(conf_thresholds) == nl
    tarr = (ctypes.c_float * nl)(*conf_thresholds)
    _check(lib().freeze_lookup_cascade_confidence(ctx, nl, larr, qarr, b, k, tarr, rescore_r, _ptr(out_labels),
                                                  _ptr(out_exit_layer), _ptr(out_hits_per_layer), _ptr(workspace),
                                                  workspace.numel() * workspace.element_size(), _stream(stream)),
           "freeze_lookup_cascade_confidence")


def freeze_compute_thresholds(ctx, layers: Sequence[int], queries_per_layer: Sequence[torch.Tensor], k: int,
                              rescore_r: int, model_labels: torch.Tensor, out_thresholds: torch.Tensor,
                              workspace: torch.Tensor, stream=None) -> None:
    nl, b, larr, qarr = _cascade_arrays(layers, queries_per_layer)
    assert model_labels.is_cuda and model_labels.dtype == torch.int32 and model_labels.numel() == b
    assert out_thresholds.is_cuda and out_thresholds.dtype == torch.float32 and out_thresholds.numel() == nl
    _check(lib().freeze_compute_thresholds(ctx, nl, larr, qarr, b, k, rescore_r, _ptr(model_labels),
                                           _ptr(out_thresholds), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream(stream)),
           "freeze_compute_thresholds")


def freeze_kmeans_storage_bytes(num_centers: int, d: int) -> int:
    return int(lib().freeze_kmeans_storage_bytes(num_centers, d))


def freeze_kmeans_workspace_bytes(ctx, n: int, d: int, num_centers: int) -> int:
    return int(lib().freeze_kmeans_workspace_bytes(ctx, n, d, num_centers))


def freeze_kmeans_build(ctx, layer: int, points: torch.Tensor, labels: torch.Tensor, num_classes: int,
                        init_centers: torch.Tensor, iters: int, storage: torch.Tensor, workspace: torch.Tensor,
                        stream=None) -> None:
    assert points.is_cuda and points.dtype == torch.float32 and points.is_contiguous() and points.dim() == 2
    assert init_centers.is_cuda and init_centers.dtype == torch.float32 and init_centers.is_contiguous()
    assert init_centers.shape[1] == points.shape[1]
    assert labels.is_cuda and labels.dtype == torch.int32 and labels.numel() == points.shape[0]
    n, d = points.shape
    _check(lib().freeze_kmeans_build(ctx, layer, _ptr(points), n, d, _ptr(labels), num_classes, _ptr(init_centers),
                                     init_centers.shape[0], iters, _ptr(storage),
                                     storage.numel() * storage.element_size(), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)),
           "freeze_kmeans_build")


def freeze_kmeans_read(ctx, layer: int, out_centers: torch.Tensor, out_majority: torch.Tensor,
                       out_fraction: torch.Tensor, stream=None) -> None:
    _check(lib().freeze_kmeans_read(ctx, layer, _ptr(out_centers), _ptr(out_majority), _ptr(out_fraction),
                                    _stream(stream)), "freeze_kmeans_read")


def freeze_projection_storage_bytes(m: int, d: int, weights_dtype: int) -> int:
    return int(lib().freeze_projection_storage_bytes(m, d, weights_dtype))


def freeze_projection_build(ctx, slot: int, weights: torch.Tensor, bias: torch.Tensor, storage: torch.Tensor,
                            workspace: torch.Tensor, stream=None) -> None:
    assert weights.is_cuda and weights.is_contiguous() and weights.dim() == 2
    assert bias.is_cuda and bias.dtype == torch.float32 and bias.numel() == weights.shape[0]
    dtype = {torch.float32: FREEZE_F32, torch.bfloat16: FREEZE_BF16}[weights.dtype]
    _check(lib().freeze_projection_build(ctx, slot, _ptr(weights), dtype, weights.shape[0], weights.shape[1], _ptr(bias),
                                         _ptr(storage), storage.numel() * storage.element_size(), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "freeze_projection_build")


def freeze_project_workspace_bytes(ctx, slot: int, b: int) -> int:
    return int(lib().freeze_project_workspace_bytes(ctx, slot, b))


def freeze_project(ctx, slot: int, x: torch.Tensor, relu: bool, out: torch.Tensor, workspace: torch.Tensor,
                   stream=None) -> None:
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 2
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.shape[0] == x.shape[0]
    _check(lib().freeze_project(ctx, slot, _ptr(x), x.shape[0], int(relu), _ptr(out), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)), "freeze_project")


def freeze_gather_rows(x: torch.Tensor, sel: torch.Tensor, count: Optional[torch.Tensor], out: torch.Tensor,
                       stream=None) -> None:
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 2
    assert sel.dtype == torch.int32 and out.dtype == torch.float32 and out.is_contiguous()
    assert out.shape[0] >= sel.numel() and out.shape[1] == x.shape[1]
    _check(lib().freeze_gather_rows(_ptr(x), x.shape[1], _ptr(sel), _ptr(count), sel.numel(), _ptr(out),
                                    _stream(stream)), "freeze_gather_rows")


def freeze_compact_misses(hit: torch.Tensor, sel_in: Optional[torch.Tensor], sel_out: torch.Tensor,
                          out_count: torch.Tensor, stream=None) -> None:
    assert hit.is_cuda and hit.dtype == torch.uint8
    _check(lib().freeze_compact_misses(_ptr(hit), _ptr(sel_in), hit.numel(), _ptr(sel_out), _ptr(out_count),
                                       _stream(stream)), "freeze_compact_misses")


def freeze_lookup_stats_attach(ctx, counters: Optional[torch.Tensor]) -> None:
    """counters: device tensor of three int64 (confirmed at once, after the wider re-scoring, exact scans) or None."""
    if counters is not None:
        assert counters.is_cuda and counters.dtype == torch.int64 and counters.numel() >= 3 and counters.is_contiguous()
    _check(lib().freeze_lookup_stats_attach(ctx, _ptr(counters)), "freeze_lookup_stats_attach")


def freeze_profile_enable(ctx, enable) -> None:
    """enable: 0 / False off, 1 / True events at every stage boundary, 2 events around the distance pass only,
    3 the same for every eighth look-up."""
    _check(lib().freeze_profile_enable(ctx, int(enable)), "freeze_profile_enable")


def freeze_profile_read(ctx):
    """Returns ([prep_ms, dist_ms, finish_ms] summed, number of look-ups covered)."""
    ms = (ctypes.c_float * 3)()
    calls = ctypes.c_int(0)
    _check(lib().freeze_profile_read(ctx, ctypes.cast(ms, ctypes.c_void_p), ctypes.cast(ctypes.byref(calls),
                                                                                     ctypes.c_void_p)),
           "freeze_profile_read")
    return [float(x) for x in ms], int(calls.value)


def freeze_profile_read_calls(ctx, max_calls: int = 256):
    """Returns a list of [prep_ms, dist_ms, finish_ms], one per recorded look-up, in call order."""
    ms = (ctypes.c_float * (3 * max_calls))()
    calls = ctypes.c_int(0)
    _check(lib().freeze_profile_read_calls(ctx, ctypes.cast(ms, ctypes.c_void_p), max_calls,
                                           ctypes.cast(ctypes.byref(calls), ctypes.c_void_p)),
           "freeze_profile_read_calls")
    return [[float(ms[3 * c + i]) for i in range(3)] for c in range(calls.value)]


def freeze_calibrate_mfma(scratch: torch.Tensor):
    """Returns (sustained bf16 MFMA TFLOP/s, shader clock in MHz under that load)."""
    tf, mhz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().freeze_calibrate_mfma(_ptr(scratch), scratch.numel() * scratch.element_size(),
                                       ctypes.cast(ctypes.byref(tf), ctypes.c_void_p),
                                       ctypes.cast(ctypes.byref(mhz), ctypes.c_void_p)), "freeze_calibrate_mfma")
    return float(tf.value), float(mhz.value)


def freeze_calibrate_hbm_read(buffer: torch.Tensor) -> float:
    """Returns the sustained read rate over `buffer` in GB/s."""
    gbs = ctypes.c_double(0.0)
    _check(lib().freeze_calibrate_hbm_read(_ptr(buffer), buffer.numel() * buffer.element_size(),
                                           ctypes.cast(ctypes.byref(gbs), ctypes.c_void_p)),
           "freeze_calibrate_hbm_read")
    return float(gbs.value)


# ---- convenience holder: owns the context, the per-layer storage and a reusable workspace ---------

class FreezeCache:
    def __init__(self, num_layers: int, device="cuda:0"):
        self.device = torch.device(device)
        self.ctx = freeze_create(num_layers)
        self.storage: Dict[int, torch.Tensor] = {}
        self.meta: Dict[int, tuple] = {}
        self._ws: Optional[torch.Tensor] = None

    def close(self):
        if self.ctx is not None:
            freeze_destroy(self.ctx)
            self.ctx = None

    def _workspace(self, nbytes: int) -> torch.Tensor:
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        return self._ws

    def build_layer(self, layer: int, entries: torch.Tensor, labels: torch.Tensor, num_classes: int):
        n, d = entries.shape
        dt = FREEZE_F32 if entries.dtype == torch.float32 else FREEZE_BF16
        nbytes = freeze_cache_storage_bytes(n, d, dt)
        if nbytes == 0:
            raise FreezeError(FREEZE_EINVAL, "freeze_cache_storage_bytes")
        st = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        freeze_cache_build(self.ctx, layer, entries, labels, num_classes, st)
        self.storage[layer] = st
        self.meta[layer] = (n, d, num_classes)

    def alloc_outputs(self, b: int, k: int):
        dev = self.device
        return dict(label=torch.empty(b, dtype=torch.int32, device=dev),
                    hit=torch.empty(b, dtype=torch.uint8, device=dev),
                    votes=torch.empty(b, dtype=torch.int32, device=dev),
                    idx=torch.empty((b, k), dtype=torch.int32, device=dev),
                    dist=torch.empty((b, k), dtype=torch.float32, device=dev))

    def lookup(self, layer: int, queries: torch.Tensor, k: int, vote_threshold: int, rescore_r: int = 0,
               out: Optional[dict] = None) -> dict:
        b = queries.shape[0]
        if out is None:
            out = self.alloc_outputs(b, k)
        nbytes = freeze_lookup_workspace_bytes(self.ctx, layer, b, k, rescore_r)
        ws = self._workspace(nbytes)
        freeze_lookup(self.ctx, layer, queries, k, vote_threshold, rescore_r, out["label"], out["hit"], out["votes"],
                      out["idx"], out["dist"], ws)
        return out

    def lookup_cascade(self, layers: Sequence[int], queries_per_layer: List[torch.Tensor], k: int,
                       vote_thresholds: Sequence[int], rescore_r: int = 0, out: Optional[dict] = None) -> dict:
        b = queries_per_layer[0].shape[0]
        if out is None:
            out = dict(label=torch.empty(b, dtype=torch.int32, device=self.device),
                       exit_layer=torch.empty(b, dtype=torch.int32, device=self.device),
                       hits_per_layer=torch.empty(len(layers), dtype=torch.int64, device=self.device))
        nbytes = freeze_cascade_workspace_bytes(self.ctx, layers, b, k, rescore_r)
        if nbytes == 0:
            raise FreezeError(FREEZE_EINVAL, "freeze_cascade_workspace_bytes")
        ws = self._workspace(nbytes)
        freeze_lookup_cascade(self.ctx, layers, queries_per_layer, k, vote_thresholds, rescore_r, out["label"],
                              out["exit_layer"], out["hits_per_layer"], ws)
        return out

    def lookup_confidence(self, layer: int, queries: torch.Tensor, k: int, conf_threshold: float, rescore_r: int = 0,
                          out: Optional[dict] = None) -> dict:
        b = queries.shape[0]
        if out is None:
            out = self.alloc_outputs(b, k)
            out["conf"] = torch.empty(b, dtype=torch.float32, device=self.device)
        nbytes = freeze_lookup_workspace_bytes(self.ctx, layer, b, k, rescore_r)
        ws = self._workspace(nbytes)
        freeze_lookup_confidence(self.ctx, layer, queries, k, conf_threshold, rescore_r, out["label"], out["hit"],
                                 out["conf"], out["votes"], out["idx"], out["dist"], ws)
        return out

    def lookup_cascade_confidence(self, layers: Sequence[int], queries_per_layer: List[torch.Tensor], k: int,
                                  conf_thresholds: Sequence[float], rescore_r: int = 0) -> dict:
        b = queries_per_layer[0].shape[0]
        out = dict(label=torch.empty(b, dtype=torch.int32, device=self.device),
                   exit_layer=torch.empty(b, dtype=torch.int32, device=self.device),
                   hits_per_layer=torch.empty(len(layers), dtype=torch.int64, device=self.device))
        nbytes = freeze_cascade_workspace_bytes(self.ctx, layers, b, k, rescore_r)
        if nbytes == 0:
            raise FreezeError(FREEZE_EINVAL, "freeze_cascade_workspace_bytes")
        ws = self._workspace(nbytes)
        freeze_lookup_cascade_confidence(self.ctx, layers, queries_per_layer, k, conf_thresholds, rescore_r,
                                         out["label"], out["exit_layer"], out["hits_per_layer"], ws)
        return out

    def compute_thresholds(self, layers: Sequence[int], queries_per_layer: List[torch.Tensor], k: int,
                           model_labels: torch.Tensor, rescore_r: int = 0) -> torch.Tensor:
        b = queries_per_layer[0].shape[0]
        thr = torch.empty(len(layers), dtype=torch.float32, device=self.device)
        nbytes = freeze_cascade_workspace_bytes(self.ctx, layers, b, k, rescore_r)
        if nbytes == 0:
            raise FreezeError(FREEZE_EINVAL, "freeze_cascade_workspace_bytes")
        ws = self._workspace(nbytes)
        freeze_compute_thresholds(self.ctx, layers, queries_per_layer, k, rescore_r, model_labels, thr, ws)
        return thr

    def build_kmeans_layer(self, layer: int, points: torch.Tensor, labels: torch.Tensor, num_classes: int,
                           init_centers: torch.Tensor, iters: int) -> dict:
        """k-means cache of `points` (Sec. 4); returns the centres, majority labels and shares."""
        n, d = points.shape
        kc = init_centers.shape[0]
        nbytes = freeze_kmeans_storage_bytes(kc, d)
        if nbytes == 0:
            raise FreezeError(FREEZE_EINVAL, "freeze_kmeans_storage_bytes")
        st = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        wbytes = freeze_kmeans_workspace_bytes(self.ctx, n, d, kc)
        if wbytes == 0:
            raise FreezeError(FREEZE_EINVAL, "freeze_kmeans_workspace_bytes")
        ws = self._workspace(wbytes)
        freeze_kmeans_build(self.ctx, layer, points, labels, num_classes, init_centers, iters, st, ws)
        self.storage[layer] = st
        self.meta[layer] = (kc, d, num_classes)
        out = dict(centers=torch.empty((kc, d), dtype=torch.float32, device=self.device),
                   majority=torch.empty(kc, dtype=torch.int32, device=self.device),
                   fraction=torch.empty(kc, dtype=torch.float32, device=self.device))
        freeze_kmeans_read(self.ctx, layer, out["centers"], out["majority"], out["fraction"])
        return out

    def build_projection(self, slot: int, weights: torch.Tensor, bias: torch.Tensor):
        """A dense layer y = W x + bias in front of a look-up (Sec. 3); occupies one slot of the context."""
        m, d = weights.shape
        dtype = FREEZE_BF16 if weights.dtype == torch.bfloat16 else FREEZE_F32
        nbytes = freeze_projection_storage_bytes(m, d, dtype)
        if nbytes == 0:
            raise FreezeError(FREEZE_EINVAL, "freeze_projection_storage_bytes")
        st = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        ws = self._workspace(256 + 4 * m)
        freeze_projection_build(self.ctx, slot, weights, bias, st, ws)
        self.storage[slot] = st
        self.meta[slot] = (m, d, 0)

    def project(self, slot: int, x: torch.Tensor, relu: bool = False) -> torch.Tensor:
        m = self.meta[slot][0]
        out = torch.empty((x.shape[0], m), dtype=torch.float32, device=self.device)
        nbytes = freeze_project_workspace_bytes(self.ctx, slot, x.shape[0])
        if nbytes == 0:
            raise FreezeError(FREEZE_EINVAL, "freeze_project_workspace_bytes")
        freeze_project(self.ctx, slot, x, relu, out, self._workspace(nbytes))
        return out
