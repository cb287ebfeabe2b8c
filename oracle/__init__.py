"""CPU oracle for the MiCS per-GPU data path -- TEST INFRASTRUCTURE ONLY.

A thin numpy/ctypes front for ``mics_oracle.c`` (plain scalar C written from
the paper's definitions, Sections 3.1-3.4).  Only the tests, the smoke check
and the bench's ``cpu_baseline`` leg may import this package; the product
package never does, and this package imports nothing from the product.

Arrays are numpy: bf16 data travels as ``uint16`` bit patterns, 4-byte
parameter elements as ``float32`` or ``uint32``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mics_oracle.c")
_LIB = os.path.join(_HERE, "libmics_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = True, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared object."""
    if force or not os.path.exists(out):
        tmp = out + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *CFLAGS, f"-I{_HERE}", "-o", tmp, src, "-lm"], check=True)
        os.replace(tmp, out)
    return out


_lib = None
_lib_path = _LIB


def use_library(path: str) -> None:
    """Load the oracle from another shared object from now on.  Only the mutation test
    (tests/test_oracle_mutants.py, through the --oracle-lib option of tests/conftest.py) calls
    this, with deliberately broken builds, to show that the pins notice; nothing reads the
    environment."""
    global _lib, _lib_path
    _lib, _lib_path = None, path


def _load():
    global _lib
    if _lib is None:
        if _lib_path == _LIB and not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_lib_path)
        vp, sz, i32, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
        lib.orc_set_threads.argtypes = [i32]
        lib.orc_set_threads.restype = i32
        lib.orc_bf16_narrow_array.argtypes = [vp, vp, sz]
        lib.orc_bf16_narrow_array.restype = None
        lib.orc_bf16_widen_array.argtypes = [vp, vp, sz]
        lib.orc_bf16_widen_array.restype = None
        lib.orc_stage1_gather.argtypes = [vp, vp, sz, i32, i32, i32, i32]
        lib.orc_naive_intra_gather.argtypes = [vp, vp, sz, i32, i32, i32]
        lib.orc_concat_shards.argtypes = [vp, vp, sz, sz, i32, i32]
        lib.orc_hier_gather_reorder.argtypes = [vp, vp, sz, sz, i32, i32, i32]
        lib.orc_reduce_scatter_accum.argtypes = [vp, vp, sz, sz, i32, i32]
        lib.orc_reduce_scatter_accum_f64.argtypes = [vp, vp, sz, sz, i32, i32]
        lib.orc_reduce_scatter_accum_typed.argtypes = [vp, vp, sz, sz, i32, i32, i32]
        lib.orc_f16_widen_array.argtypes = [vp, vp, sz]
        lib.orc_f16_widen_array.restype = None
        lib.orc_f16_narrow_array.argtypes = [vp, vp, sz]
        lib.orc_f16_narrow_array.restype = None
        lib.orc_replica_average.argtypes = [vp, vp, sz, i32, f32]
        adam = [vp, vp, vp, vp, vp, sz, f32, f32, f32, f32, f32, i32]
        lib.orc_adam_shard.argtypes = adam
        lib.orc_adam_shard_f32.argtypes = adam
        _lib = lib
    return _lib


def set_threads(n: int) -> int:
    return _load().orc_set_threads(int(n))


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _table(arrs: Sequence[np.ndarray]):
    return (ctypes.c_void_p * len(arrs))(*[_ptr(a) for a in arrs])


def _check(rc: int, name: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {name}: bad arguments (rc={rc})")


def _c(a, dtype=None) -> np.ndarray:
    a = np.asarray(a)
    if dtype is not None and a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("array must be C-contiguous")
    return a


def _elem_bytes(a: np.ndarray) -> int:
    if a.dtype.itemsize not in (2, 4):
        raise TypeError("parameter elements are 2 or 4 bytes wide")
    return a.dtype.itemsize


# ---- bfloat16 ---------------------------------------------------------------

def bf16_narrow(x) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().orc_bf16_narrow_array(_ptr(out), _ptr(x), x.size)
    return out


def bf16_widen(b) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exact."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    out = np.empty(b.shape, dtype=np.float32)
    _load().orc_bf16_widen_array(_ptr(out), _ptr(b), b.size)
    return out


# ---- hierarchical all-gather (Section 3.3) ------------------------------------

def stage1_gather(shards: Sequence[np.ndarray], k: int, l: int) -> np.ndarray:
    """Stage 1: T_l = [C_l, C_{k+l}, ...] for local rank ``l``."""
    shards = [_c(s) for s in shards]
    p, S, eb = len(shards), shards[0].size, _elem_bytes(shards[0])
    if any(s.size != S or s.dtype != shards[0].dtype for s in shards):
        raise ValueError("all shards must have the same length and dtype")
    if k < 1 or p % k:
        raise ValueError("p must be divisible by k")
    out = np.empty((p // k) * S, dtype=shards[0].dtype)
    _check(_load().orc_stage1_gather(_ptr(out), _table(shards), S, p, k, l, eb), "stage1_gather")
    return out


def naive_intra_gather(T: Sequence[np.ndarray], p: int) -> np.ndarray:
    """The wrong layout: intra-node all-gather applied directly to stage-1 outputs."""
    T = [_c(t) for t in T]
    k, eb = len(T), _elem_bytes(T[0])
    S = T[0].size * k // p
    out = np.empty(p * S, dtype=T[0].dtype)
    _check(_load().orc_naive_intra_gather(_ptr(out), _table(T), S, p, k, eb), "naive_intra_gather")
    return out


def concat_shards(shards: Sequence[np.ndarray], n_valid: int) -> np.ndarray:
    """The correct gathered parameter by definition: [C_0 .. C_{p-1}] cut to n_valid."""
    shards = [_c(s) for s in shards]
    p, S, eb = len(shards), shards[0].size, _elem_bytes(shards[0])
    out = np.empty(n_valid, dtype=shards[0].dtype)
    _check(_load().orc_concat_shards(_ptr(out), _table(shards), n_valid, S, p, eb), "concat_shards")
    return out


def hier_gather_reorder(T: Sequence[np.ndarray], n_valid: int, S: int, p: int) -> np.ndarray:
    """Stage-1 outputs -> contiguous flat parameter (first n_valid elements)."""
    T = [_c(t) for t in T]
    k, eb = len(T), _elem_bytes(T[0])
    if k < 1 or p % k or any(t.size < (p // k) * S for t in T):
        raise ValueError("stage-1 buffers do not match (p, k, S)")
    out = np.empty(n_valid, dtype=T[0].dtype)
    _check(_load().orc_hier_gather_reorder(_ptr(out), _table(T), n_valid, S, p, k, eb),
           "hier_gather_reorder")
    return out


def hier_gather_reorder_coalesced(T: Sequence[np.ndarray], segs, p: int, out: np.ndarray) -> np.ndarray:
    """Many tensors gathered at once (the paper's coalesced all-gather, Section 4): the per-tensor
    reorder applied to each tensor in turn.  ``segs`` = (numel, shard_elems, src_offset,
    dst_offset) per tensor; tensor t occupies (p/k)*shard_elems elements from src_offset in every
    stage-1 buffer and numel elements from dst_offset in ``out`` (written in place)."""
    k = len(T)
    for numel, S, src_off, dst_off in segs:
        sub = [np.ascontiguousarray(t[src_off:src_off + (p // k) * S]) for t in T]
        out[dst_off:dst_off + numel] = hier_gather_reorder(sub, numel, S, p)
    return out


# ---- 2-hop gradient synchronisation (Section 3.4) -------------------------------

def reduce_scatter_accum_coalesced(acc, grads: Sequence[np.ndarray], segs, accumulate: bool) -> np.ndarray:
    """Many tensors reduced at once (coalesced reduce-scatter, Section 4): for every segment
    (count, _, src_offset, dst_offset) the plain reduce-scatter-accumulate of elements
    [src_offset, src_offset+count) of the rank buffers into acc[dst_offset:dst_offset+count]."""
    acc = _c(acc, np.float32)
    for count, _, src_off, dst_off in segs:
        reduce_scatter_accum(acc[dst_off:dst_off + count], grads, src_off, accumulate)
    return acc


DTYPE_BF16, DTYPE_F16, DTYPE_F32 = 0, 1, 2


def f16_widen(h) -> np.ndarray:
    """IEEE binary16 bit patterns (uint16) -> float32, exact."""
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    _load().orc_f16_widen_array(_ptr(out), _ptr(h), h.size)
    return out


def f16_narrow(x) -> np.ndarray:
    """float32 -> IEEE binary16 bit patterns (uint16), round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().orc_f16_narrow_array(_ptr(out), _ptr(x), x.size)
    return out


def reduce_scatter_accum_typed(acc, grads: Sequence[np.ndarray], elem_offset: int, accumulate: bool,
                               dtype: int) -> np.ndarray:
    """reduce_scatter_accum for gradients stored as bf16 / binary16 bit patterns (uint16 arrays)
    or as float32 arrays; in place on ``acc`` (float32)."""
    acc = _c(acc, np.float32)
    want = np.float32 if dtype == DTYPE_F32 else np.uint16
    grads = [_c(g, want) for g in grads]
    if any(g.size < elem_offset + acc.size for g in grads):
        raise ValueError("gradient buffer shorter than elem_offset + count")
    _check(_load().orc_reduce_scatter_accum_typed(_ptr(acc), _table(grads), elem_offset, acc.size,
                                                  len(grads), int(bool(accumulate)), dtype),
           "reduce_scatter_accum_typed")
    return acc


def reduce_scatter_accum_coalesced_typed(acc, grads: Sequence[np.ndarray], segs, accumulate: bool,
                                         dtype: int) -> np.ndarray:
    """reduce_scatter_accum_coalesced for bf16 / binary16 / float32 gradient buffers: the typed
    reduction, segment by segment."""
    acc = _c(acc, np.float32)
    for count, _, src_off, dst_off in segs:
        reduce_scatter_accum_typed(acc[dst_off:dst_off + count], grads, src_off, accumulate, dtype)
    return acc


def reduce_scatter_accum(acc, grads: Sequence[np.ndarray], elem_offset: int, accumulate: bool,
                         f64: bool = False) -> np.ndarray:
    """In place on ``acc`` (float32, or float64 with ``f64=True``); returns it."""
    acc = _c(acc, np.float64 if f64 else np.float32)
    grads = [_c(g, np.uint16) for g in grads]
    count = acc.size
    if any(g.size < elem_offset + count for g in grads):
        raise ValueError("gradient buffer shorter than elem_offset + count")
    fn = _load().orc_reduce_scatter_accum_f64 if f64 else _load().orc_reduce_scatter_accum
    _check(fn(_ptr(acc), _table(grads), elem_offset, count, len(grads), int(bool(accumulate))),
           "reduce_scatter_accum")
    return acc


def replica_average(copies: Sequence[np.ndarray], scale: float, out=None) -> np.ndarray:
    copies = [_c(c, np.float32) for c in copies]
    count = copies[0].size
    if any(c.size != count for c in copies):
        raise ValueError("replica copies differ in length")
    if out is None:
        out = np.empty(count, dtype=np.float32)
    out = _c(out, np.float32)
    _check(_load().orc_replica_average(_ptr(out), _table(copies), count, len(copies),
                                       float(np.float32(scale))), "replica_average")
    return out


# ---- mixed-precision Adam ---------------------------------------------------------

def adam_shard(master, exp_avg, exp_avg_sq, grad, *, lr, beta1, beta2, eps, weight_decay, step,
               want_bf16: bool = True, f32: bool = False, param_dtype: str = "bf16"):
    """In place on master / exp_avg / exp_avg_sq (float32).  Returns the low-precision parameter
    bit patterns (uint16; bf16, or binary16 with ``param_dtype="f16"``: the new master rounded
    to nearest even) or None.  ``f32=True`` selects the strict binary32 variant."""
    if param_dtype not in ("bf16", "f16"):
        raise ValueError("param_dtype must be 'bf16' or 'f16'")
    as_f16 = want_bf16 and param_dtype == "f16"
    want_bf16 = want_bf16 and not as_f16
    w, m, v = _c(master, np.float32), _c(exp_avg, np.float32), _c(exp_avg_sq, np.float32)
    g = _c(grad, np.float32)
    count = w.size
    if not (m.size == v.size == g.size == count):
        raise ValueError("Adam state arrays differ in length")
    pb = np.empty(count, dtype=np.uint16) if want_bf16 else None
    fn = _load().orc_adam_shard_f32 if f32 else _load().orc_adam_shard
    _check(fn(_ptr(w), _ptr(m), _ptr(v), _ptr(pb) if pb is not None else None, _ptr(g), count,
              float(np.float32(lr)), float(np.float32(beta1)), float(np.float32(beta2)),
              float(np.float32(eps)), float(np.float32(weight_decay)), int(step)), "adam_shard")
    return f16_narrow(w) if as_f16 else pb
