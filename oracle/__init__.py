"""CPU oracle for the rank-n tensor transpose  B[perm(i)] = A[i].

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does.  It
shares no code with the HIP library.

Conventions (0-based restatement of Section 2 of the paper):

* a tensor is a flat buffer; ``dims[0]`` is the stride-1 dimension;
* ``perm[j]`` is the input dimension found at output position ``j`` (the
  paper's ``w_{j+1} - 1``); output extents are ``dims[perm[j]]``.

Four independent forms of the same definition live here:

``transpose``            C, gather form (inverse scalar position per output element)
``transpose_scatter``    C, scatter form (Eq. (1), walking the input)
``transpose_numpy``      the library special case: ``numpy.transpose`` on a
                         Fortran-ordered view
``transpose_bruteforce`` pure-Python nested loops over every multi-index
``transpose_accumulate`` C, out + transposed in (the paper's accumulate mode)
``contract``             C, D + L * R as a direct loop nest (the contraction of Section 3.4)

All forms move raw bytes (arrays are viewed as unsigned integers of the element
size), so results are compared bit for bit.
"""
from __future__ import annotations

import ctypes
import itertools
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tt_oracle.c")
_LIB = os.path.join(_HERE, "libtt_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``tt_oracle.c`` with gcc + OpenMP into ``libtt_oracle.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i32p = ctypes.POINTER(ctypes.c_int)
        lib.tto_transpose_gather.argtypes = [ctypes.c_int, i64p, i32p, ctypes.c_size_t,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.tto_transpose_gather.restype = ctypes.c_int
        lib.tto_transpose_scatter.argtypes = [ctypes.c_int, i64p, i32p, ctypes.c_size_t,
                                              ctypes.c_void_p, ctypes.c_void_p]
        lib.tto_transpose_scatter.restype = ctypes.c_int
        lib.tto_transpose_accumulate.argtypes = [ctypes.c_int, i64p, i32p, ctypes.c_size_t,
                                                 ctypes.c_void_p, ctypes.c_void_p]
        lib.tto_transpose_accumulate.restype = ctypes.c_int
        lib.tto_input_position.argtypes = [ctypes.c_int, i64p, i32p, ctypes.c_int64]
        lib.tto_input_position.restype = ctypes.c_int64
        lib.tto_sample.argtypes = [ctypes.c_int, i64p, i32p, ctypes.c_size_t, ctypes.c_void_p,
                                   ctypes.c_int64, i64p, ctypes.c_void_p]
        lib.tto_sample.restype = ctypes.c_int
        lib.tto_contract.argtypes = [ctypes.c_int, i64p, ctypes.c_int, i32p, ctypes.c_int, i32p,
                                     ctypes.c_int, i32p, ctypes.c_size_t, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_void_p]
        lib.tto_contract.restype = ctypes.c_int
        lib.tto_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _marshal(dims: Sequence[int], perm: Sequence[int]):
    rank = len(dims)
    if len(perm) != rank:
        raise ValueError("perm and dims differ in length")
    cd = (ctypes.c_int64 * rank)(*[int(d) for d in dims])
    cp = (ctypes.c_int * rank)(*[int(p) for p in perm])
    return rank, cd, cp


def _flat_bytes(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a).reshape(-1)
    if a.dtype.itemsize not in (1, 2, 4, 8):
        raise ValueError("unsupported element size")
    return a


def out_dims(dims: Sequence[int], perm: Sequence[int]) -> list:
    """Extents of the output tensor: position j holds input dimension perm[j]."""
    return [int(dims[p]) for p in perm]


def inverse_perm(perm: Sequence[int]) -> list:
    """inv with inv[perm[j]] = j."""
    inv = [0] * len(perm)
    for j, p in enumerate(perm):
        inv[p] = j
    return inv


def max_threads() -> int:
    return int(_load().tto_max_threads())


def transpose(a: np.ndarray, dims: Sequence[int], perm: Sequence[int], nthreads: int = 0) -> np.ndarray:
    """Gather form in C.  ``a`` is the flat input; returns the flat output."""
    lib = _load()
    a = _flat_bytes(a)
    rank, cd, cp = _marshal(dims, perm)
    if a.size != int(np.prod([int(d) for d in dims], dtype=object)):
        raise ValueError("buffer size does not match dims")
    out = np.empty_like(a)
    rc = lib.tto_transpose_gather(rank, cd, cp, a.dtype.itemsize, a.ctypes.data, out.ctypes.data,
                                  int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return out


def transpose_scatter(a: np.ndarray, dims: Sequence[int], perm: Sequence[int]) -> np.ndarray:
    """Scatter form in C (Eq. (1)): linear walk over the input."""
    lib = _load()
    a = _flat_bytes(a)
    rank, cd, cp = _marshal(dims, perm)
    if a.size != int(np.prod([int(d) for d in dims], dtype=object)):
        raise ValueError("buffer size does not match dims")
    out = np.empty_like(a)
    rc = lib.tto_transpose_scatter(rank, cd, cp, a.dtype.itemsize, a.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return out


def transpose_accumulate(a: np.ndarray, b: np.ndarray, dims: Sequence[int],
                         perm: Sequence[int]) -> np.ndarray:
    """Accumulating form in C: returns b + transpose(a) with one IEEE addition per element.
    ``a`` and ``b`` are float32 or float64 flat buffers of the same dtype; ``b`` is not
    modified."""
    lib = _load()
    a = np.ascontiguousarray(a).reshape(-1)
    out = np.array(b, copy=True).reshape(-1)
    if a.dtype != out.dtype or a.dtype not in (np.float32, np.float64):
        raise ValueError("accumulate needs float32 or float64 buffers of one dtype")
    rank, cd, cp = _marshal(dims, perm)
    if a.size != out.size or a.size != int(np.prod([int(d) for d in dims], dtype=object)):
        raise ValueError("buffer size does not match dims")
    rc = lib.tto_transpose_accumulate(rank, cd, cp, a.dtype.itemsize, a.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return out


def contract(d_labels: str, l_labels: str, r_labels: str, extents: dict, l: np.ndarray,
             r: np.ndarray, d: np.ndarray) -> np.ndarray:
    """Binary tensor contraction as a direct loop nest: returns d + l * r.

    Tensors are flat float64 (or float32) buffers; the label strings name their dimensions,
    first label = stride-1 dimension.  Labels shared by ``l_labels`` and ``r_labels`` and absent
    from ``d_labels`` are summed over, in double precision and in a fixed order; every other
    label occurs in ``d_labels`` and in exactly one input.  ``d`` is not modified."""
    lib = _load()
    names = sorted(set(d_labels + l_labels + r_labels))
    num = {c: i for i, c in enumerate(names)}
    ext = (ctypes.c_int64 * len(names))(*[int(extents[c]) for c in names])
    idx = lambda s: (ctypes.c_int * len(s))(*[num[c] for c in s])
    l = np.ascontiguousarray(l).reshape(-1)
    r = np.ascontiguousarray(r).reshape(-1)
    out = np.array(d, copy=True).reshape(-1)
    if not (l.dtype == r.dtype == out.dtype) or out.dtype not in (np.float32, np.float64):
        raise ValueError("contract needs float32 or float64 buffers of one dtype")
    vol = lambda s: int(np.prod([int(extents[c]) for c in s], dtype=object))
    if l.size != vol(l_labels) or r.size != vol(r_labels) or out.size != vol(d_labels):
        raise ValueError("buffer size does not match the labels' extents")
    rc = lib.tto_contract(len(names), ext, len(d_labels), idx(d_labels), len(l_labels), idx(l_labels),
                          len(r_labels), idx(r_labels), out.dtype.itemsize, l.ctypes.data, r.ctypes.data,
                          out.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle rejected the contraction (code {rc})")
    return out


def input_position(dims: Sequence[int], perm: Sequence[int], o: int) -> int:
    """Input scalar position of the element stored at output scalar position ``o``."""
    rank, cd, cp = _marshal(dims, perm)
    return int(_load().tto_input_position(rank, cd, cp, int(o)))


def sample(a: np.ndarray, dims: Sequence[int], perm: Sequence[int], positions: np.ndarray) -> np.ndarray:
    """Values of the output at the given output scalar positions, one by one."""
    lib = _load()
    a = _flat_bytes(a)
    rank, cd, cp = _marshal(dims, perm)
    pos = np.ascontiguousarray(positions, dtype=np.int64)
    vals = np.empty(pos.size, dtype=a.dtype)
    rc = lib.tto_sample(rank, cd, cp, a.dtype.itemsize, a.ctypes.data, pos.size,
                        pos.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), vals.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return vals


def transpose_numpy(a: np.ndarray, dims: Sequence[int], perm: Sequence[int]) -> np.ndarray:
    """Library special case: with dims[0] fastest the buffer is a Fortran-ordered
    array of shape ``dims``; moving axis perm[j] to position j and reading the
    result back in Fortran order is the whole operation."""
    a = _flat_bytes(a)
    t = np.transpose(a.reshape(tuple(int(d) for d in dims), order="F"), tuple(int(p) for p in perm))
    return np.ascontiguousarray(t.ravel(order="F"))


def transpose_bruteforce(a: Sequence, dims: Sequence[int], perm: Sequence[int]) -> list:
    """Pure-Python nested loops over every input multi-index y (tiny tensors only).

    in  position = sum_z y[z] * prod_{t<z} dims[t]
    out position = sum_j y[perm[j]] * prod_{t<j} dims[perm[t]]
    """
    rank = len(dims)
    vol = 1
    for d in dims:
        vol *= int(d)
    out = [None] * vol
    for y in itertools.product(*[range(int(d)) for d in dims]):
        pin = 0
        stride = 1
        for z in range(rank):
            pin += y[z] * stride
            stride *= int(dims[z])
        pout = 0
        stride = 1
        for j in range(rank):
            pout += y[perm[j]] * stride
            stride *= int(dims[perm[j]])
        out[pout] = a[pin]
    return out
