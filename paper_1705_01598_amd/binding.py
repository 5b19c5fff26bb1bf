"""ctypes binding of libtperm.so: same names as the C ABI in include/tperm.h (the product
boundary) and include/tperm_tuning.h (overrides, candidate enumeration and the host-side index
map, for tests and sweeps).

Argument marshalling only.  Every step of the transpose runs in the library's kernels;
there is no Python or CPU fallback: if the shared library is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtperm.so")

TPERM_MAX_RANK = 16

# status codes
OK, ERR_NULL, ERR_RANK, ERR_DIMS, ERR_PERM, ERR_ELEM_SIZE, ERR_TOO_LARGE, ERR_ALIAS, ERR_ALIGN, \
    ERR_HIP, ERR_NOMEM, ERR_KERNEL, ERR_INTERNAL = range(13)

# kernel classes
KERNEL_AUTO, KERNEL_COPY, KERNEL_ROWCOPY, KERNEL_TILED, KERNEL_PACKED, KERNEL_NAIVE = range(6)
KERNEL_NAMES = {KERNEL_AUTO: "auto", KERNEL_COPY: "copy", KERNEL_ROWCOPY: "rowcopy",
                KERNEL_TILED: "tiled", KERNEL_PACKED: "packed", KERNEL_NAIVE: "naive"}

# include/tperm.h
EXPORTS = ["tperm_plan_create", "tperm_plan_create_forced", "tperm_plan_create_measured",
           "tperm_plan_create_measured_cold",
           "tperm_execute", "tperm_execute_accumulate", "tperm_execute_verified", "tperm_execute_verified_static",
           "tperm_plan_describe", "tperm_plan_destroy",
           "tperm_status_string", "tperm_copy_bytes", "tperm_transpose", "tperm_transpose_accumulate",
           "tperm_cache_tune", "tperm_cache_stats", "tperm_cache_clear"]
# include/tperm_tuning.h
TUNING_EXPORTS = ["tperm_plan_create_ex", "tperm_plan_candidate_count", "tperm_plan_create_candidate",
                  "tperm_plan_index_map", "tperm_plan_model", "tperm_multiset_compare",
                  "tperm_device_memory_info"]


class PlanOpts(ctypes.Structure):
    _fields_ = [("kernel_class", ctypes.c_int), ("m", ctypes.c_int), ("tile_in", ctypes.c_int64),
                ("k", ctypes.c_int), ("tile_out", ctypes.c_int64), ("lds_pad", ctypes.c_int),
                ("grid_mode", ctypes.c_int), ("blocks_per_cu", ctypes.c_int),
                ("cache_policy", ctypes.c_int), ("window_in", ctypes.c_int),
                ("window_out", ctypes.c_int), ("threads", ctypes.c_int),
                ("lds_buffers", ctypes.c_int), ("align_out", ctypes.c_int),
                ("tile_order", ctypes.c_int), ("loads_first", ctypes.c_int),
                ("vec2", ctypes.c_int), ("pair_elems", ctypes.c_int), ("selector", ctypes.c_int),
                ("large", ctypes.c_int)]


class Model(ctypes.Structure):
    """tperm_model_t: analytical estimate of a plan (Section 2.3 re-derived for MI355X)."""
    _fields_ = [(n, ctypes.c_double) for n in
                ("ld_tran", "st_tran", "ld_req", "st_req", "cl_full", "cl_part", "ld_runs", "st_runs", "tpr_mem", "mem_lat", "mlp",
                 "mwp", "tpr_lds", "cycles_mem", "cycles_lds", "cycles_ac", "n_iter", "cycles_total",
                 "microseconds", "useful_bytes_per_tile")]


class PlanInfo(ctypes.Structure):
    _fields_ = [("kernel_class", ctypes.c_int), ("elem_size", ctypes.c_int), ("rank", ctypes.c_int),
                ("canon_rank", ctypes.c_int), ("canon_dims", ctypes.c_int64 * TPERM_MAX_RANK),
                ("canon_perm", ctypes.c_int * TPERM_MAX_RANK), ("volume", ctypes.c_int64),
                ("tile_extent", ctypes.c_int64 * TPERM_MAX_RANK), ("tile_volume", ctypes.c_int64),
                ("run_in", ctypes.c_int64), ("run_out", ctypes.c_int64),
                ("num_tiles", ctypes.c_int64), ("m", ctypes.c_int), ("k", ctypes.c_int),
                ("nreg", ctypes.c_int), ("threads", ctypes.c_int), ("lds_bytes", ctypes.c_int),
                ("lds_pad", ctypes.c_int), ("score", ctypes.c_double),
                ("blocks_per_cu", ctypes.c_int), ("cache_policy", ctypes.c_int),
                ("align_out", ctypes.c_int), ("paired", ctypes.c_int),
                ("loads_first", ctypes.c_int), ("vec2", ctypes.c_int), ("large", ctypes.c_int),
                ("reserved", ctypes.c_int * 1)]


class TpermError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libtperm.so (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1705_01598_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        i64p = ctypes.POINTER(ctypes.c_int64)
        ip = ctypes.POINTER(ctypes.c_int)
        L.tperm_plan_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, ip, ctypes.c_size_t]
        L.tperm_plan_create_forced.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, ip, ctypes.c_size_t,
                                               ctypes.c_int]
        L.tperm_plan_create_ex.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, ip,
                                           ctypes.c_size_t, ctypes.POINTER(PlanOpts)]
        L.tperm_plan_create_measured.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, ip,
                                                 ctypes.c_size_t, vp, vp, vp, ctypes.c_int]
        L.tperm_plan_create_measured_cold.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, ip,
                                                      ctypes.c_size_t, vp, vp, vp, ctypes.c_int,
                                                      vp, ctypes.c_size_t]
        L.tperm_plan_candidate_count.argtypes = [ctypes.c_int, i64p, ip, ctypes.c_size_t, ip]
        L.tperm_plan_create_candidate.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, ip,
                                                  ctypes.c_size_t, ctypes.c_int]
        L.tperm_execute.argtypes = [vp, vp, vp, vp]
        L.tperm_execute_accumulate.argtypes = [vp, vp, vp, vp]
        L.tperm_execute_verified.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_size_t]
        L.tperm_execute_verified_static.argtypes = [vp, vp, vp, vp, vp]
        L.tperm_multiset_compare.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_size_t, vp, vp, ctypes.c_size_t, vp]
        L.tperm_plan_describe.argtypes = [vp, ctypes.POINTER(PlanInfo)]
        L.tperm_plan_index_map.argtypes = [vp, i64p]
        L.tperm_plan_model.argtypes = [vp, ctypes.POINTER(Model)]
        L.tperm_device_memory_info.argtypes = [ip, ip, ip]
        L.tperm_plan_destroy.argtypes = [vp]
        L.tperm_copy_bytes.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.tperm_transpose.argtypes = [ctypes.c_int, i64p, ip, ctypes.c_size_t, vp, vp, vp]
        L.tperm_transpose_accumulate.argtypes = [ctypes.c_int, i64p, ip, ctypes.c_size_t, vp, vp, vp]
        L.tperm_cache_tune.argtypes = [ctypes.c_int, i64p, ip, ctypes.c_size_t, vp, vp, vp]
        L.tperm_cache_stats.argtypes = [i64p, i64p, i64p]
        L.tperm_cache_clear.argtypes = []
        L.tperm_status_string.argtypes = [ctypes.c_int]
        L.tperm_status_string.restype = ctypes.c_char_p
        for name in EXPORTS + TUNING_EXPORTS:
            if name != "tperm_status_string":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().tperm_status_string(int(status)).decode()


def _marshal(dims: Sequence[int], perm: Sequence[int]):
    rank = len(dims)
    cd = (ctypes.c_int64 * max(rank, 1))(*[int(d) for d in dims])
    cp = (ctypes.c_int * max(rank, 1))(*[int(p) for p in perm])
    return rank, cd, cp


class Plan:
    """Owns one tperm_plan_t."""

    def __init__(self, handle: ctypes.c_void_p):
        self._h = handle

    @property
    def handle(self):
        return self._h

    def describe(self) -> PlanInfo:
        return tperm_plan_describe(self)

    def execute(self, in_ptr: int, out_ptr: int, stream: int = 0) -> None:
        tperm_execute(self, in_ptr, out_ptr, stream)

    def destroy(self) -> None:
        if self._h is not None:
            lib().tperm_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def tperm_plan_create(dims: Sequence[int], perm: Sequence[int], elem_size: int) -> Plan:
    rank, cd, cp = _marshal(dims, perm)
    h = ctypes.c_void_p()
    st = lib().tperm_plan_create(ctypes.byref(h), rank, cd, cp, int(elem_size))
    if st != OK:
        raise TpermError(st, "tperm_plan_create")
    return Plan(h)


def tperm_plan_create_forced(dims: Sequence[int], perm: Sequence[int], elem_size: int,
                             kernel_class: int) -> Plan:
    rank, cd, cp = _marshal(dims, perm)
    h = ctypes.c_void_p()
    st = lib().tperm_plan_create_forced(ctypes.byref(h), rank, cd, cp, int(elem_size), int(kernel_class))
    if st != OK:
        raise TpermError(st, "tperm_plan_create_forced")
    return Plan(h)


def tperm_plan_create_ex(dims: Sequence[int], perm: Sequence[int], elem_size: int,
                         kernel_class: int = KERNEL_AUTO, m: int = 0, tile_in: int = 0, k: int = 0,
                         tile_out: int = 0, lds_pad: int = -1, grid_mode: int = 0,
                         blocks_per_cu: int = 0, cache_policy: int = 0, window_in: int = 0,
                         window_out: int = 0, threads: int = 0, lds_buffers: int = 0,
                         align_out: int = 0, tile_order: int = 0, pair_elems: int = 0,
                         loads_first: int = 0, vec2: int = 0, selector: int = 0, large: int = 0) -> Plan:
    rank, cd, cp = _marshal(dims, perm)
    opts = PlanOpts(kernel_class=int(kernel_class), m=int(m), tile_in=int(tile_in), k=int(k),
                    tile_out=int(tile_out), lds_pad=int(lds_pad), grid_mode=int(grid_mode),
                    blocks_per_cu=int(blocks_per_cu), cache_policy=int(cache_policy),
                    window_in=int(window_in), window_out=int(window_out), threads=int(threads),
                    lds_buffers=int(lds_buffers), align_out=int(align_out),
                    tile_order=int(tile_order), pair_elems=int(pair_elems),
                    loads_first=int(loads_first), vec2=int(vec2), selector=int(selector), large=int(large))
    h = ctypes.c_void_p()
    st = lib().tperm_plan_create_ex(ctypes.byref(h), rank, cd, cp, int(elem_size), ctypes.byref(opts))
    if st != OK:
        raise TpermError(st, "tperm_plan_create_ex")
    return Plan(h)


def tperm_plan_create_measured(dims: Sequence[int], perm: Sequence[int], elem_size: int,
                               in_ptr: int, out_ptr: int, stream: int = 0,
                               max_candidates: int = 0) -> Plan:
    rank, cd, cp = _marshal(dims, perm)
    h = ctypes.c_void_p()
    st = lib().tperm_plan_create_measured(ctypes.byref(h), rank, cd, cp, int(elem_size),
                                          ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr),
                                          ctypes.c_void_p(stream), int(max_candidates))
    if st != OK:
        raise TpermError(st, "tperm_plan_create_measured")
    return Plan(h)


def tperm_plan_create_measured_cold(dims: Sequence[int], perm: Sequence[int], elem_size: int,
                                    in_ptr: int, out_ptr: int, stream: int, scratch_ptr: int,
                                    scratch_bytes: int, max_candidates: int = 0) -> Plan:
    rank, cd, cp = _marshal(dims, perm)
    h = ctypes.c_void_p()
    st = lib().tperm_plan_create_measured_cold(ctypes.byref(h), rank, cd, cp, int(elem_size),
                                               ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr),
                                               ctypes.c_void_p(stream), int(max_candidates),
                                               ctypes.c_void_p(scratch_ptr), int(scratch_bytes))
    if st != OK:
        raise TpermError(st, "tperm_plan_create_measured_cold")
    return Plan(h)


def tperm_plan_candidate_count(dims: Sequence[int], perm: Sequence[int], elem_size: int) -> int:
    rank, cd, cp = _marshal(dims, perm)
    n = ctypes.c_int(0)
    st = lib().tperm_plan_candidate_count(rank, cd, cp, int(elem_size), ctypes.byref(n))
    if st != OK:
        raise TpermError(st, "tperm_plan_candidate_count")
    return int(n.value)


def tperm_plan_create_candidate(dims: Sequence[int], perm: Sequence[int], elem_size: int,
                                index: int) -> Plan:
    rank, cd, cp = _marshal(dims, perm)
    h = ctypes.c_void_p()
    st = lib().tperm_plan_create_candidate(ctypes.byref(h), rank, cd, cp, int(elem_size), int(index))
    if st != OK:
        raise TpermError(st, "tperm_plan_create_candidate")
    return Plan(h)


def tperm_execute(plan: Plan, in_ptr: int, out_ptr: int, stream: int = 0) -> None:
    st = lib().tperm_execute(plan.handle, ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr),
                             ctypes.c_void_p(stream))
    if st != OK:
        raise TpermError(st, "tperm_execute")


def tperm_execute_accumulate(plan: Plan, in_ptr: int, out_ptr: int, stream: int = 0) -> None:
    st = lib().tperm_execute_accumulate(plan.handle, ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr),
                                        ctypes.c_void_p(stream))
    if st != OK:
        raise TpermError(st, "tperm_execute_accumulate")


VERIFY_CHUNK_ELEMS = 16384


def verify_workspace_bytes(volume: int) -> int:
    """TPERM_VERIFY_WORKSPACE_BYTES of the header."""
    return 64 * ((int(volume) + VERIFY_CHUNK_ELEMS - 1) // VERIFY_CHUNK_ELEMS)


def tperm_execute_verified(plan: Plan, in_ptr: int, out_ptr: int, stream: int, verdict_ptr: int,
                           workspace_ptr: int, workspace_bytes: int) -> None:
    st = lib().tperm_execute_verified(plan.handle, ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr),
                                      ctypes.c_void_p(stream), ctypes.c_void_p(verdict_ptr),
                                      ctypes.c_void_p(workspace_ptr), int(workspace_bytes))
    if st != OK:
        raise TpermError(st, "tperm_execute_verified")


VERIFY_STATIC_MAX_ELEMS = 1 << 27


def tperm_execute_verified_static(plan: Plan, in_ptr: int, out_ptr: int, stream: int, verdict_ptr: int) -> None:
    st = lib().tperm_execute_verified_static(plan.handle, ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr),
                                             ctypes.c_void_p(stream), ctypes.c_void_p(verdict_ptr))
    if st != OK:
        raise TpermError(st, "tperm_execute_verified_static")


def tperm_multiset_compare(a_ptr: int, b_ptr: int, count: int, elem_size: int, verdict_ptr: int,
                           workspace_ptr: int, workspace_bytes: int, stream: int = 0) -> None:
    st = lib().tperm_multiset_compare(ctypes.c_void_p(a_ptr), ctypes.c_void_p(b_ptr), int(count), int(elem_size),
                                      ctypes.c_void_p(verdict_ptr), ctypes.c_void_p(workspace_ptr),
                                      int(workspace_bytes), ctypes.c_void_p(stream))
    if st != OK:
        raise TpermError(st, "tperm_multiset_compare")


def tperm_plan_describe(plan: Plan) -> PlanInfo:
    info = PlanInfo()
    st = lib().tperm_plan_describe(plan.handle, ctypes.byref(info))
    if st != OK:
        raise TpermError(st, "tperm_plan_describe")
    return info


def tperm_plan_index_map(plan: Plan):
    """out_to_in map evaluated on the host from the plan's descriptors (numpy int64)."""
    import numpy as np
    info = tperm_plan_describe(plan)
    # one entry per element of the problem as given (a paired plan reports volume in pairs)
    buf = np.empty(int(info.volume) * (2 if info.paired else 1), dtype=np.int64)
    st = lib().tperm_plan_index_map(plan.handle, buf.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)))
    if st != OK:
        raise TpermError(st, "tperm_plan_index_map")
    return buf


def tperm_device_memory_info() -> dict:
    """Memory bus width (bits), peak memory clock (kHz) and compute units of the current device."""
    w, c, n = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    st = lib().tperm_device_memory_info(ctypes.byref(w), ctypes.byref(c), ctypes.byref(n))
    if st != OK:
        raise TpermError(st, "tperm_device_memory_info")
    return {"memory_bus_width_bits": w.value, "memory_clock_kHz": c.value, "compute_units": n.value}


def tperm_plan_model(plan: Plan) -> Model:
    m = Model()
    st = lib().tperm_plan_model(plan.handle, ctypes.byref(m))
    if st != OK:
        raise TpermError(st, "tperm_plan_model")
    return m


def tperm_transpose(dims: Sequence[int], perm: Sequence[int], elem_size: int, in_ptr: int,
                    out_ptr: int, stream: int = 0, accumulate: bool = False) -> None:
    """Cached-plan transpose (tperm_transpose / tperm_transpose_accumulate)."""
    rank, cd, cp = _marshal(dims, perm)
    fn = lib().tperm_transpose_accumulate if accumulate else lib().tperm_transpose
    st = fn(rank, cd, cp, int(elem_size), ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr),
            ctypes.c_void_p(stream))
    if st != OK:
        raise TpermError(st, "tperm_transpose")


def tperm_cache_tune(dims: Sequence[int], perm: Sequence[int], elem_size: int, in_ptr: int,
                     out_ptr: int, stream: int = 0) -> None:
    rank, cd, cp = _marshal(dims, perm)
    st = lib().tperm_cache_tune(rank, cd, cp, int(elem_size), ctypes.c_void_p(in_ptr),
                                ctypes.c_void_p(out_ptr), ctypes.c_void_p(stream))
    if st != OK:
        raise TpermError(st, "tperm_cache_tune")


def tperm_cache_stats() -> dict:
    e, h, m = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    st = lib().tperm_cache_stats(ctypes.byref(e), ctypes.byref(h), ctypes.byref(m))
    if st != OK:
        raise TpermError(st, "tperm_cache_stats")
    return {"entries": e.value, "hits": h.value, "misses": m.value}


def tperm_cache_clear() -> None:
    st = lib().tperm_cache_clear()
    if st != OK:
        raise TpermError(st, "tperm_cache_clear")


def tperm_plan_destroy(plan: Plan) -> None:
    plan.destroy()


def tperm_copy_bytes(in_ptr: int, out_ptr: int, nbytes: int, stream: int = 0) -> None:
    st = lib().tperm_copy_bytes(ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr), int(nbytes),
                                ctypes.c_void_p(stream))
    if st != OK:
        raise TpermError(st, "tperm_copy_bytes")


def info_dict(info: PlanInfo) -> dict:
    r = info.canon_rank
    return {"kernel": KERNEL_NAMES.get(info.kernel_class, "?"), "canon_dims": list(info.canon_dims[:r]),
            "canon_perm": list(info.canon_perm[:r]), "tile": list(info.tile_extent[:r]),
            "tile_volume": info.tile_volume, "run_in": info.run_in, "run_out": info.run_out,
            "num_tiles": info.num_tiles, "nreg": info.nreg, "threads": info.threads, "lds_bytes": info.lds_bytes,
            "lds_pad": info.lds_pad, "score": round(info.score, 4),
            "blocks_per_cu": info.blocks_per_cu, "cache_policy": info.cache_policy,
            "align_out": info.align_out, "paired": info.paired,
            "loads_first": info.loads_first, "vec2": info.vec2, "large": info.large}
