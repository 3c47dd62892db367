"""ctypes loader for libginex.so; declares every entry point of include/ginex.h."""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libginex.so")

i32, i64, u32, u64, vp, sz = C.c_int32, C.c_int64, C.c_uint32, C.c_uint64, C.c_void_p, C.c_size_t


class CsrDesc(C.Structure):
    _fields_ = [("num_nodes", i64), ("num_edges", i64), ("offsets", vp), ("offsets_64", i32),
                ("indices", vp), ("nc_address_table", vp), ("nc_cache_array", vp)]


class CacheDesc(C.Structure):
    _fields_ = [("rows", vp), ("cap", i64), ("row_bytes", i64), ("addr", vp),
                ("num_nodes", i64), ("slow", vp)]


SIGNATURES = {
    "ginex_last_error": (C.c_char_p, []),
    "ginex_version": (i32, []),
    "ginex_sample_workspace_bytes": (sz, [i64, i32, i64, vp, i32]),
    "ginex_sample_superbatch": (i32, [C.POINTER(CsrDesc), vp, vp, i32, vp, i32, u64, u32,
                                      vp, i64, vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, sz, vp]),
    "ginex_neighbor_cache_workspace_bytes": (sz, [i64]),
    "ginex_neighbor_cache_build": (i32, [C.POINTER(CsrDesc), i64, vp, vp, vp, vp, vp, sz, vp]),
    "ginex_changeset_workspace_bytes": (sz, [i64, i64, i32, i64]),
    "ginex_changeset": (i32, [i64, vp, vp, i32, i64, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp,
                              vp, sz, vp]),
    "ginex_changeset_noalloc": (i32, [i64, vp, vp, i32, i64, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp,
                                      vp, vp]),
    "ginex_changeset_lru": (i32, [i64, vp, vp, i32, i64, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp,
                                  vp, vp, sz, vp]),
    "ginex_changeset_resume": (i32, [i64, vp, vp, i32, i64, vp, vp, vp, vp, vp, i64, vp, vp, vp,
                                     vp, vp, sz, vp]),
    "ginex_cache_init": (i32, [C.POINTER(CacheDesc), vp, i64, vp]),
    "ginex_cache_init_part": (i32, [C.POINTER(CacheDesc), vp, i64, i64, vp]),
    "ginex_cache_init_warm": (i32, [C.POINTER(CacheDesc), C.POINTER(CacheDesc), vp, i64, i64, vp]),
    "ginex_gather": (i32, [C.POINTER(CacheDesc), vp, i64, vp, vp, vp, vp, i64, vp]),
    "ginex_gather_lines": (i32, [C.POINTER(CacheDesc), vp, vp, i64, i64, vp, vp, vp, vp, i64, vp]),
    "ginex_cache_update": (i32, [C.POINTER(CacheDesc), vp, vp, vp, vp, i64, vp]),
    "ginex_static_select_workspace_bytes": (sz, [i64]),
    "ginex_static_select": (i32, [C.POINTER(CsrDesc), i64, vp, vp, vp, sz, vp]),
    "ginex_cache_count_misses": (i32, [C.POINTER(CacheDesc), vp, i64, vp, vp]),
}

_lib = None


def stale() -> bool:
    """True if the library is missing or older than any of its sources."""
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    csrc = os.path.join(_PKG, "csrc")
    sources = [os.path.join(csrc, f) for f in os.listdir(csrc)
               if f.endswith((".hip", ".hpp", ".cpp"))]
    sources.append(os.path.join(os.path.dirname(_PKG), "include", "ginex.h"))
    return any(os.path.getmtime(s) > built for s in sources if os.path.exists(s))


def load():
    """Loads the built library.  A library that is missing, or older than one of its sources
    (csrc/*, include/ginex.h), is rebuilt first where the compiler is installed; where it is
    not, a stale library is an error rather than a silent run of old kernels."""
    global _lib
    if _lib is None:
        if stale():
            from .build import HIPCC, build
            if os.path.exists(HIPCC):
                build()
            elif os.path.exists(LIB_PATH):
                raise RuntimeError(f"{LIB_PATH} is older than its sources and {HIPCC} is not "
                                   "installed here: rebuild with python -m paper_2208_09151_amd.build")
            else:
                raise RuntimeError(f"{LIB_PATH} has not been built and {HIPCC} is not installed")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)     # AttributeError if the library lacks a declared symbol
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib
