"""ctypes binding with the same names as the C ABI (kfac_update_factors, kfac_invert_batch,
kfac_precondition).  Tensors are anything with .data_ptr() (torch tensors on the GPU) or
plain integer device addresses."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

KFAC_OK, KFAC_ERR_INVALID_ARG, KFAC_ERR_NOT_SPD, KFAC_ERR_WORKSPACE, KFAC_ERR_DEVICE = range(5)

# every symbol include/kfac.h declares
EXPORTS = [
    "kfac_create", "kfac_destroy", "kfac_last_error",
    "kfac_layer_dA", "kfac_layer_dG", "kfac_layer_rows",
    "kfac_workspace_bytes_factors", "kfac_workspace_bytes_invert", "kfac_workspace_bytes_precondition",
    "kfac_update_factors", "kfac_update_factors_packed", "kfac_invert_batch", "kfac_invert_batch_packed", "kfac_check_info", "kfac_precondition",
    "kfac_packed_elems", "kfac_pack_triangles", "kfac_unpack_triangles", "kfac_place_inversions",
    "kfac_get_plan_stats", "kfac_timing_enable", "kfac_timing_read",
    "kfac_set_option", "kfac_get_option", "kfac_precondition_noalloc",
]

# kfac_option, in the order of the header
OPTIONS = ["inv_groups", "inv_agg", "inv_agg_chain", "inv_fuse", "inv_side_pad",
           "factor_lag", "factor_vec11", "factor_xcd", "factor_kjob", "inv_chain_pad", "inv_side", "inv_split_long", "inv_yield", "inv_quarter"]

KERNEL_CLASSES = ["factor_tiles", "factor_reduce", "inv_small", "inv_init", "inv_pivot", "inv_panel",
                  "inv_update", "inv_finish", "precond_left", "precond_right", "tri_pack"]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class KfacError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"kfac status {status}: {msg}")
        self.status = status


class layer_struct(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("kind", "n", "c_in", "h", "w", "c_out", "kh", "kw", "stride", "pad_h", "pad_w", "rows", "has_bias")]


class cost_model(C.Structure):
    _fields_ = [("alpha_inv", C.c_double), ("beta_inv", C.c_double), ("alpha_bcast", C.c_double),
                ("beta_bcast", C.c_double), ("weight_power", C.c_int32)]


class plan_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("n_jobs", "n_launches", "n_split", "mfma_flops", "ws_bytes")]


def lib_path() -> str:
    # KFAC_HIP_LIBRARY: another build of the same library (the host-sanitized one of build.py), for tests
    return os.environ.get("KFAC_HIP_LIBRARY") or os.path.join(_HERE, "libkfac_hip.so")


def is_built() -> bool:
    return os.path.exists(lib_path())


def load():
    """dlopen libkfac_hip.so (built in-tree by paper_2107_06533_amd.build / __graft_entry__.build)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not is_built():
        raise RuntimeError(f"{lib_path()} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    # PyTorch ships its own HIP runtime (same soname).  Import it first so that the loader binds this
    # library to that one runtime; two runtimes in one process do not share devices, streams or memory.
    import torch  # noqa: F401
    lib = C.CDLL(lib_path())
    vp, i32p, fpp = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_void_p)
    lp = C.POINTER(layer_struct)
    lib.kfac_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.kfac_create.restype = C.c_int
    lib.kfac_destroy.argtypes = [vp]
    lib.kfac_destroy.restype = None
    lib.kfac_last_error.argtypes = [vp]
    lib.kfac_last_error.restype = C.c_char_p
    for f in ("kfac_layer_dA", "kfac_layer_dG"):
        getattr(lib, f).argtypes = [lp]
        getattr(lib, f).restype = C.c_int32
    lib.kfac_layer_rows.argtypes = [lp]
    lib.kfac_layer_rows.restype = C.c_int64
    lib.kfac_workspace_bytes_factors.argtypes = [vp, C.c_int, lp]
    lib.kfac_workspace_bytes_factors.restype = C.c_size_t
    lib.kfac_workspace_bytes_invert.argtypes = [vp, C.c_int, i32p]
    lib.kfac_workspace_bytes_invert.restype = C.c_size_t
    lib.kfac_workspace_bytes_precondition.argtypes = [vp, C.c_int, i32p, i32p]
    lib.kfac_workspace_bytes_precondition.restype = C.c_size_t
    lib.kfac_update_factors.argtypes = [vp, C.c_int, lp, fpp, fpp, fpp, fpp, C.c_float, C.c_float, C.c_float, vp]
    lib.kfac_update_factors.restype = C.c_int
    lib.kfac_update_factors_packed.argtypes = [vp, C.c_int, lp, fpp, fpp, fpp, fpp, C.c_float, C.c_float, C.c_float, vp, vp]
    lib.kfac_update_factors_packed.restype = C.c_int
    lib.kfac_invert_batch.argtypes = [vp, C.c_int, i32p, fpp, fpp, C.c_float, vp, vp]
    lib.kfac_invert_batch.restype = C.c_int
    lib.kfac_invert_batch_packed.argtypes = [vp, C.c_int, i32p, fpp, fpp, vp, C.c_float, vp, vp]
    lib.kfac_invert_batch_packed.restype = C.c_int
    lib.kfac_check_info.argtypes = [vp, C.c_int, vp, i32p, vp]
    lib.kfac_check_info.restype = C.c_int
    lib.kfac_precondition.argtypes = [vp, C.c_int, i32p, i32p, fpp, fpp, fpp, fpp, vp]
    lib.kfac_precondition.restype = C.c_int
    lib.kfac_precondition_noalloc.argtypes = [vp, C.c_int, i32p, i32p, fpp, fpp, fpp, fpp, vp]
    lib.kfac_precondition_noalloc.restype = C.c_int
    lib.kfac_packed_elems.argtypes = [C.c_int, i32p, C.POINTER(C.c_int64)]
    lib.kfac_packed_elems.restype = C.c_size_t
    lib.kfac_pack_triangles.argtypes = [vp, C.c_int, i32p, fpp, vp, vp]
    lib.kfac_pack_triangles.restype = C.c_int
    lib.kfac_unpack_triangles.argtypes = [vp, C.c_int, i32p, vp, fpp, vp]
    lib.kfac_unpack_triangles.restype = C.c_int
    lib.kfac_place_inversions.argtypes = [C.c_int, i32p, C.c_int, C.POINTER(cost_model), i32p, C.POINTER(C.c_double)]
    lib.kfac_place_inversions.restype = C.c_int
    lib.kfac_get_plan_stats.argtypes = [vp, C.c_int, C.POINTER(plan_stats)]
    lib.kfac_get_plan_stats.restype = None
    lib.kfac_timing_enable.argtypes = [vp, C.c_uint32]
    lib.kfac_timing_enable.restype = None
    lib.kfac_timing_read.argtypes = [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int]
    lib.kfac_timing_read.restype = C.c_int
    lib.kfac_set_option.argtypes = [vp, C.c_int, C.c_int]
    lib.kfac_set_option.restype = C.c_int
    lib.kfac_get_option.argtypes = [vp, C.c_int, C.POINTER(C.c_int)]
    lib.kfac_get_option.restype = C.c_int
    _LIB = lib
    return lib


def make_layer(l) -> layer_struct:
    """From any object with the fields of synth.shapes.Layer (or a dict)."""
    has = (lambda k: k in l) if isinstance(l, dict) else (lambda k: hasattr(l, k))
    get = (lambda k: l[k]) if isinstance(l, dict) else (lambda k: getattr(l, k))

    def field(name):
        # objects that carry one `pad` (and optionally `pad_w`, negative = same) are accepted too
        if name == "pad_h" and not has("pad_h"):
            return get("pad")
        if name == "pad_w" and (not has("pad_w") or int(get("pad_w")) < 0):
            return get("pad_h") if has("pad_h") else get("pad")
        return get(name)

    return layer_struct(*[int(field(n)) for n, _ in layer_struct._fields_])


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _ptr_array(xs: Optional[Sequence], n: int):
    if xs is None:
        return None
    assert len(xs) == n
    return (C.c_void_p * n)(*[_ptr(x) for x in xs])


def _i32_array(xs: Sequence[int]):
    return (C.c_int32 * len(xs))(*[int(v) for v in xs])


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        try:
            import torch
            if torch.cuda.is_available():
                return int(torch.cuda.current_stream().cuda_stream) or None
        except Exception:
            pass
        return None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def place_inversions(dims, n_workers, alpha_inv, beta_inv, alpha_bcast, beta_bcast, weight_power=1, check=True):
    """(status, owner list, overall time) of kfac_place_inversions (pure host, no context)."""
    lib = load()
    n = len(dims)
    m = cost_model(alpha_inv, beta_inv, alpha_bcast, beta_bcast, weight_power)
    owner = (C.c_int32 * max(n, 1))()
    t = C.c_double()
    st = lib.kfac_place_inversions(n, _i32_array(dims) if n else None, n_workers, C.byref(m), owner, C.byref(t))
    if check and st != 0:
        raise KfacError(st, lib.kfac_last_error(None).decode())
    return st, [int(owner[i]) for i in range(n)], t.value


class Context:
    """Owns one kfac_ctx.  device=-1 gives a host-only context (validation and planning)."""

    def __init__(self, device: int = 0):
        self.lib = load()
        h = C.c_void_p()
        st = self.lib.kfac_create(C.byref(h), int(device))
        if st != KFAC_OK:
            raise KfacError(st, self.lib.kfac_last_error(None).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.kfac_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return self.lib.kfac_last_error(self.h).decode()

    def _check(self, st: int):
        if st != KFAC_OK:
            raise KfacError(st, self.last_error())

    # -- the three calls of the hot path (same names as the C ABI) -------------------------
    def kfac_update_factors(self, layers, act, gout, A, G, xi: float, scale_a: float = 0.0,
                            scale_g: float = 0.0, stream=None, check: bool = True) -> int:
        n = len(layers)
        arr = (layer_struct * max(n, 1))(*[make_layer(l) for l in layers])
        st = self.lib.kfac_update_factors(self.h, n, arr, _ptr_array(act, n), _ptr_array(gout, n),
                                          _ptr_array(A, n), _ptr_array(G, n),
                                          float(xi), float(scale_a), float(scale_g), _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def kfac_update_factors_packed(self, layers, act, gout, A, G, xi: float, packed, scale_a: float = 0.0,
                                   scale_g: float = 0.0, stream=None, check: bool = True) -> int:
        n = len(layers)
        arr = (layer_struct * max(n, 1))(*[make_layer(l) for l in layers])
        st = self.lib.kfac_update_factors_packed(self.h, n, arr, _ptr_array(act, n), _ptr_array(gout, n),
                                                 _ptr_array(A, n), _ptr_array(G, n),
                                                 float(xi), float(scale_a), float(scale_g), _ptr(packed), _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def kfac_invert_batch(self, dims, F, X, gamma: float, info=None, stream=None, check: bool = True) -> int:
        n = len(dims)
        st = self.lib.kfac_invert_batch(self.h, n, _i32_array(dims) if n else None, _ptr_array(F, n),
                                        _ptr_array(X, n), float(gamma), _ptr(info), _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def kfac_invert_batch_packed(self, dims, F, X, packed, gamma: float, info=None, stream=None, check: bool = True) -> int:
        n = len(dims)
        st = self.lib.kfac_invert_batch_packed(self.h, n, _i32_array(dims) if n else None, _ptr_array(F, n),
                                               _ptr_array(X, n), _ptr(packed), float(gamma), _ptr(info),
                                               _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def kfac_check_info(self, n: int, info, stream=None):
        host = (C.c_int32 * max(n, 1))()
        st = self.lib.kfac_check_info(self.h, n, _ptr(info), host, _stream_handle(stream))
        return st, list(host)[:n]

    def kfac_precondition(self, dG, dA, Ginv, Ainv, gradW, out, stream=None, check: bool = True) -> int:
        n = len(dG)
        st = self.lib.kfac_precondition(self.h, n, _i32_array(dG) if n else None, _i32_array(dA) if n else None,
                                        _ptr_array(Ginv, n), _ptr_array(Ainv, n), _ptr_array(gradW, n),
                                        _ptr_array(out, n), _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def kfac_precondition_noalloc(self, dG, dA, Ginv, Ainv, gradW, out, stream=None, check: bool = True) -> int:
        n = len(dG)
        st = self.lib.kfac_precondition_noalloc(self.h, n, _i32_array(dG) if n else None, _i32_array(dA) if n else None,
                                                _ptr_array(Ginv, n), _ptr_array(Ainv, n), _ptr_array(gradW, n),
                                                _ptr_array(out, n), _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def kfac_pack_triangles(self, dims, M, packed, stream=None, check: bool = True) -> int:
        n = len(dims)
        st = self.lib.kfac_pack_triangles(self.h, n, _i32_array(dims) if n else None, _ptr_array(M, n), _ptr(packed),
                                          _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def kfac_unpack_triangles(self, dims, packed, M, stream=None, check: bool = True) -> int:
        n = len(dims)
        st = self.lib.kfac_unpack_triangles(self.h, n, _i32_array(dims) if n else None, _ptr(packed), _ptr_array(M, n),
                                            _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def packed_elems(self, dims):
        """(total floats, offsets[n+1]) of the concatenated packed upper triangles."""
        n = len(dims)
        off = (C.c_int64 * (n + 1))()
        tot = int(self.lib.kfac_packed_elems(n, _i32_array(dims) if n else None, off))
        return tot, [int(v) for v in off]

    def set_option(self, name: str, value: int, check: bool = True) -> int:
        """name: one of OPTIONS (kfac_option without its prefix, lower case)."""
        st = self.lib.kfac_set_option(self.h, OPTIONS.index(name), int(value))
        if check:
            self._check(st)
        return st

    def get_option(self, name: str) -> int:
        v = C.c_int()
        self._check(self.lib.kfac_get_option(self.h, OPTIONS.index(name), C.byref(v)))
        return v.value

    # -- host-side queries -------------------------------------------------------------------
    def workspace_bytes_factors(self, layers) -> int:
        arr = (layer_struct * max(len(layers), 1))(*[make_layer(l) for l in layers])
        return int(self.lib.kfac_workspace_bytes_factors(self.h, len(layers), arr))

    def workspace_bytes_invert(self, dims) -> int:
        return int(self.lib.kfac_workspace_bytes_invert(self.h, len(dims), _i32_array(dims)))

    def workspace_bytes_precondition(self, dG, dA) -> int:
        return int(self.lib.kfac_workspace_bytes_precondition(self.h, len(dG), _i32_array(dG), _i32_array(dA)))

    def timing_enable(self, classes=()):
        """classes: iterable of names from KERNEL_CLASSES (empty = timing off)."""
        mask = 0
        for c in classes:
            mask |= 1 << KERNEL_CLASSES.index(c)
        self.lib.kfac_timing_enable(self.h, mask)

    def timing_read(self, kclass: str, reset: bool = True):
        """(total milliseconds, launches) of one kernel class since the last reset."""
        ms, n = C.c_double(), C.c_int64()
        self._check(self.lib.kfac_timing_read(self.h, KERNEL_CLASSES.index(kclass), C.byref(ms), C.byref(n), int(reset)))
        return ms.value, n.value

    def plan_stats(self, which: int) -> dict:
        s = plan_stats()
        self.lib.kfac_get_plan_stats(self.h, which, C.byref(s))
        return {n: int(getattr(s, n)) for n, _ in plan_stats._fields_}
