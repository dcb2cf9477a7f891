"""Loader of the HIP library.  There is no CPU fallback: a missing library is an error."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int32, c_int64, c_size_t, c_uint8, c_uint32, c_uint64, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaasd.so")

_lib = None


class LibraryMissing(RuntimeError):
    pass


def load():
    """Load libaasd.so (built beforehand by ``paper_2505_13204_amd.build``) and declare its ABI."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise LibraryMissing(
            f"{LIB_PATH} is missing: build it with `python -m paper_2505_13204_amd.build` "
            "(hipcc, gfx950). The AASD hot path has no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    i32p, u8p, f32p, u32p = POINTER(c_int32), POINTER(c_uint8), POINTER(c_float), POINTER(c_uint32)
    lib.aasd_version.restype = c_char_p
    lib.aasd_version.argtypes = []
    lib.aasd_last_error.restype = c_char_p
    lib.aasd_last_error.argtypes = []
    lib.aasd_hook_sweep_events.restype = None
    lib.aasd_hook_sweep_events.argtypes = [c_void_p, c_void_p]
    lib.aasd_hook_draw_events.restype = None
    lib.aasd_hook_draw_events.argtypes = [c_void_p, c_void_p]
    lib.aasd_hook_sweep_plan.restype = c_int32
    lib.aasd_hook_sweep_plan.argtypes = [c_int32, c_int32, c_int32]
    lib.aasd_hook_verify_launches.restype = c_int32
    lib.aasd_hook_verify_launches.argtypes = [c_int32, c_int32, c_int32, c_int32, c_int32, c_uint32]
    lib.aasd_align_sample.restype = c_int32
    lib.aasd_align_sample.argtypes = [
        c_void_p, c_int32, c_int64, c_int32, c_int64, c_void_p, c_int32, c_int32, c_int32, c_uint64, c_uint64,
        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
        c_void_p, c_size_t, c_void_p]
    lib.aasd_align_sample_workspace_bytes.restype = c_size_t
    lib.aasd_align_sample_workspace_bytes.argtypes = [c_int64, c_int32, c_int32]
    lib.aasd_retrieve_drafts.restype = c_int32
    lib.aasd_retrieve_drafts.argtypes = [
        c_void_p, c_int64, c_void_p, c_void_p, c_int32, c_int32, c_int32, c_int32, c_int32,
        c_void_p, c_void_p, c_int32, c_int64,
        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.aasd_verify_workspace_bytes.restype = c_size_t
    lib.aasd_verify_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, c_int32, c_int32]
    lib.aasd_verify.restype = c_int32
    lib.aasd_verify.argtypes = [
        c_void_p, c_int32, c_int32, c_int32, c_int32, c_int32, c_int64, c_int64,
        c_void_p, c_void_p, c_void_p, c_float, c_float, c_uint32,
        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
        c_void_p, c_size_t, c_void_p]
    lib.aasd_verify_static_max_bytes.restype = c_size_t
    lib.aasd_verify_static_max_bytes.argtypes = []
    lib.aasd_verify_static.restype = c_int32
    lib.aasd_verify_static.argtypes = list(lib.aasd_verify.argtypes[:23]) + [c_void_p]
    lib.aasd_pool_bytes.restype = c_size_t
    lib.aasd_pool_bytes.argtypes = [c_int32, c_int32, c_int32, c_int32]
    lib.aasd_pool_update.restype = c_int32
    lib.aasd_pool_update.argtypes = [c_void_p, c_size_t, c_int32, c_int32, c_int32, c_int32, c_void_p, c_int64, c_void_p,
                                     c_int32, c_void_p]
    lib.aasd_pool_retrieve.restype = c_int32
    lib.aasd_pool_retrieve.argtypes = [
        c_void_p, c_size_t, c_int32, c_int32, c_int32, c_int32, c_void_p, c_int64, c_void_p, c_void_p, c_int32, c_int32,
        c_void_p, c_void_p, c_int32, c_int64,
        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.aasd_pool_step.restype = c_int32
    lib.aasd_pool_step.argtypes = list(lib.aasd_pool_retrieve.argtypes)
    lib.aasd_verify_topk_workspace_bytes.restype = c_size_t
    lib.aasd_verify_topk_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, c_int32, c_int32]
    lib.aasd_verify_topk.restype = c_int32
    lib.aasd_verify_topk.argtypes = [
        c_void_p, c_int32, c_int32, c_int32, c_int32, c_int32, c_int64, c_int64,
        c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.aasd_build_tree.restype = c_int32
    lib.aasd_build_tree.argtypes = [
        c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_int32, c_int32, c_int32, c_int32,
        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.aasd_verify_tree_workspace_bytes.restype = c_size_t
    lib.aasd_verify_tree_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, c_int32]
    lib.aasd_verify_tree.restype = c_int32
    lib.aasd_verify_tree.argtypes = [
        c_void_p, c_int32, c_int32, c_int32, c_int32, c_int64, c_int64,
        c_void_p, c_void_p, c_void_p, c_void_p, c_float, c_float, c_uint32,
        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
        c_void_p, c_size_t, c_void_p]
    _lib = lib
    return lib
