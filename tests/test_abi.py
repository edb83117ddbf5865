"""CPU-side checks of the C-ABI library: it loads, exports every function include/freeze.h
declares, and its host-side argument checks answer without a GPU (no compute is launched)."""
import ctypes
import os
import re

import pytest

from paper_2002_02645_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "freeze.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(freeze_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"freeze_create", "freeze_destroy", "freeze_cache_build", "freeze_lookup", "freeze_lookup_cascade",
            "freeze_compact_misses", "freeze_cache_storage_bytes", "freeze_lookup_workspace_bytes",
            "freeze_cascade_workspace_bytes", "freeze_strerror"} <= set(names)
    L = binding.lib()
    for name in names:
        assert getattr(L, name) is not None, name


def test_binding_has_the_same_names():
    for name in _declared_functions():
        assert hasattr(binding, name), name


def test_host_side_checks_without_gpu():
    L = binding.lib()
    assert L.freeze_strerror(0) == b"ok"
    for code in range(-6, 0):
        assert L.freeze_strerror(code) not in (b"ok", b"unknown error")
    h = ctypes.c_void_p()
    assert L.freeze_create(ctypes.byref(h), 0) == binding.FREEZE_EINVAL
    assert L.freeze_create(None, 2) == binding.FREEZE_EINVAL
    assert L.freeze_create(ctypes.byref(h), 2) == binding.FREEZE_OK
    try:
        # layout arithmetic: tiled bf16 rows padded to 256 entries x 64 elements, norms, labels, row-major copy
        n, d = 1000, 100
        n_pad, d_pad = 1024, 128
        up = lambda x: (x + 255) // 256 * 256
        base = up(n_pad * d_pad * 2) + up(n_pad * 4) + up(n * 4) + up(d_pad * 4) + up(d_pad * 16)   # ... mean vector, column statistics
        assert L.freeze_cache_storage_bytes(n, d, binding.FREEZE_BF16) == base + up(n * d_pad * 2)
        assert L.freeze_cache_storage_bytes(n, d, binding.FREEZE_F32) == base + up(n * d_pad * 4)
        assert L.freeze_cache_storage_bytes(0, d, binding.FREEZE_BF16) == 0
        assert L.freeze_cache_storage_bytes(n, 0, binding.FREEZE_BF16) == 0
        assert L.freeze_cache_storage_bytes(n, d, 7) == 0
        # look-ups on layers that are out of range / not built are refused before any launch
        assert L.freeze_lookup_workspace_bytes(h, 0, 16, 5, 0) == 0
        dummy = ctypes.c_void_p(256)
        args = (dummy, 4, 5, 3, 0, dummy, dummy, dummy, dummy, dummy, dummy, 1 << 20, None)
        assert L.freeze_lookup(h, 9, *args) == binding.FREEZE_ELAYER
        assert L.freeze_lookup(h, 1, *args) == binding.FREEZE_ENOTBUILT
        assert L.freeze_lookup(None, 0, *args) == binding.FREEZE_EINVAL
        assert L.freeze_cache_build(h, 7, dummy, 0, 10, 10, dummy, 2, dummy, 1 << 20, None) == binding.FREEZE_ELAYER
        assert L.freeze_cache_build(h, 0, dummy, 0, 10, 10, dummy, 2, dummy, 16, None) == binding.FREEZE_EWORKSPACE
        assert L.freeze_cache_build(h, 0, None, 0, 10, 10, dummy, 2, dummy, 1 << 20, None) == binding.FREEZE_EINVAL
        assert L.freeze_compact_misses(None, None, 4, dummy, dummy, None) == binding.FREEZE_EINVAL
        # the entry point with the built-in scratch checks its arguments the same way, before touching the GPU
        sargs = (dummy, 4, 5, 3, 0, dummy, dummy, dummy, dummy, dummy, None)
        assert L.freeze_lookup_static(h, 9, *sargs) == binding.FREEZE_ELAYER
        assert L.freeze_lookup_static(h, 1, *sargs) == binding.FREEZE_ENOTBUILT
        assert L.freeze_lookup_static(None, 0, *sargs) == binding.FREEZE_EINVAL
        assert L.freeze_lookup_static(h, 0, dummy, 4, 5, 9, 0, dummy, dummy, dummy, dummy, dummy, None) == binding.FREEZE_EINVAL
        assert L.freeze_lookup_stats_attach(None, None) == binding.FREEZE_EINVAL
        assert L.freeze_lookup_stats_attach(h, ctypes.c_void_p(12)) == binding.FREEZE_EINVAL     # misaligned
        assert L.freeze_lookup_stats_attach(h, None) == binding.FREEZE_OK
        assert L.freeze_set_centring(h, 3) == binding.FREEZE_EINVAL and L.freeze_set_centring(None, 1) == binding.FREEZE_EINVAL
        assert L.freeze_set_centring(h, 0) == binding.FREEZE_OK and L.freeze_set_centring(h, 1) == binding.FREEZE_OK
        assert L.freeze_profile_enable(h, 4) == binding.FREEZE_EINVAL
        assert L.freeze_profile_enable(h, 2) == binding.FREEZE_OK and L.freeze_profile_enable(h, 3) == binding.FREEZE_OK
        assert L.freeze_profile_enable(h, 0) == binding.FREEZE_OK
    finally:
        assert L.freeze_destroy(h) == binding.FREEZE_OK
    assert L.freeze_destroy(None) == binding.FREEZE_EINVAL


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libfreeze_hip.so")
    with pytest.raises(RuntimeError):
        binding.lib()
