"""MI355X-native per-GPU data path of MiCS partitioned data parallelism.

Thin ctypes binding over ``libmics.so`` (see ``include/mics.h`` for the contract of each
call, ``include/mics_tuning.h`` for the two measurement knobs).  The functions here only marshal arguments -- device pointers, sizes and the
current HIP stream; every step of the path runs in the library's HIP kernels.  There is
no CPU fallback: if the library is missing, importing this package fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmics.so")

MICS_OK = 0
MICS_ERR_INVALID_ARG = -1
MICS_ERR_ALIGNMENT = -2
MICS_ERR_UNSUPPORTED = -3
MICS_ERR_HIP = -4
MICS_MAX_GROUP = 128

EXPORTS = (
    "mics_version", "mics_last_error", "mics_shard_elems", "mics_set_blocks_per_cu",
    "mics_set_stream_threshold_bytes", "mics_set_launch_shape",
    "mics_hier_gather_reorder", "mics_reduce_scatter_accum", "mics_replica_average",
    "mics_adam_shard", "mics_hier_gather_reorder_coalesced", "mics_reduce_scatter_accum_coalesced",
    "mics_replica_average_adam_shard", "mics_reduce_scatter_accum_typed",
    "mics_adam_shard_typed", "mics_replica_average_adam_shard_typed",
    "mics_reduce_scatter_accum_coalesced_typed",
)
MICS_DTYPE_BF16, MICS_DTYPE_F16, MICS_DTYPE_F32 = 0, 1, 2


class MicsError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libmics error {code}: {message}")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is not built. Run `python -c 'import __graft_entry__ as g; g.build()'` "
        "(or `python paper_2205_00119_amd/build.py`) first; there is no fallback path.")

# PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  It must be in the process before
# libmics.so is opened, so that the library binds to that one runtime -- the one that owns the
# device memory and streams the caller passes in -- instead of loading a second copy.
import torch  # noqa: E402,F401

lib = ctypes.CDLL(LIB_PATH)

_vp, _sz, _i, _f = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
lib.mics_version.argtypes = []
lib.mics_version.restype = _i
lib.mics_last_error.argtypes = []
lib.mics_last_error.restype = ctypes.c_char_p
lib.mics_shard_elems.argtypes = [_sz, _i, _sz]
lib.mics_shard_elems.restype = _sz
lib.mics_set_blocks_per_cu.argtypes = [_i]
lib.mics_set_blocks_per_cu.restype = _i
lib.mics_set_stream_threshold_bytes.argtypes = [_sz]
lib.mics_set_stream_threshold_bytes.restype = _i
lib.mics_set_launch_shape.argtypes = [_i, _i, _i]
lib.mics_set_launch_shape.restype = _i
lib.mics_hier_gather_reorder.argtypes = [_vp, _vp, _sz, _sz, _i, _i, _i, _vp]
lib.mics_hier_gather_reorder.restype = _i
lib.mics_reduce_scatter_accum.argtypes = [_vp, _vp, _sz, _sz, _i, _i, _vp]
lib.mics_reduce_scatter_accum.restype = _i
lib.mics_replica_average.argtypes = [_vp, _vp, _sz, _i, _f, _vp]
lib.mics_replica_average.restype = _i
lib.mics_adam_shard.argtypes = [_vp, _vp, _vp, _vp, _vp, _sz, _f, _f, _f, _f, _f, _i, _vp]
lib.mics_adam_shard.restype = _i


class mics_segment(ctypes.Structure):
    """One separately sharded tensor of a coalesced call (offsets and sizes in elements)."""
    _fields_ = [("numel", ctypes.c_size_t), ("shard_elems", ctypes.c_size_t),
                ("src_offset", ctypes.c_size_t), ("dst_offset", ctypes.c_size_t)]


lib.mics_hier_gather_reorder_coalesced.argtypes = [_vp, _vp, ctypes.POINTER(mics_segment), _i, _i, _i,
                                                   _i, _vp]
lib.mics_hier_gather_reorder_coalesced.restype = _i
lib.mics_reduce_scatter_accum_coalesced.argtypes = [_vp, _vp, ctypes.POINTER(mics_segment), _i, _i, _i,
                                                    _vp]
lib.mics_reduce_scatter_accum_coalesced.restype = _i


lib.mics_replica_average_adam_shard.argtypes = [_vp, _vp, _vp, _vp, _vp, _sz, _i, _f, _f, _f, _f, _f, _f,
                                                _i, _vp]
lib.mics_replica_average_adam_shard.restype = _i


lib.mics_reduce_scatter_accum_coalesced_typed.argtypes = [_vp, _vp, ctypes.POINTER(mics_segment), _i, _i, _i, _i,
                                                          _vp]
lib.mics_reduce_scatter_accum_coalesced_typed.restype = _i
lib.mics_adam_shard_typed.argtypes = [_vp, _vp, _vp, _vp, _i, _vp, _sz, _f, _f, _f, _f, _f, _i, _vp]
lib.mics_adam_shard_typed.restype = _i
lib.mics_replica_average_adam_shard_typed.argtypes = [_vp, _vp, _vp, _vp, _i, _vp, _sz, _i, _f, _f, _f, _f, _f,
                                                      _f, _i, _vp]
lib.mics_replica_average_adam_shard_typed.restype = _i
lib.mics_reduce_scatter_accum_typed.argtypes = [_vp, _vp, _sz, _sz, _i, _i, _i, _vp]
lib.mics_reduce_scatter_accum_typed.restype = _i


def _segments(segs) -> ctypes.Array:
    """(numel, shard_elems, src_offset, dst_offset) tuples -> C array of mics_segment."""
    return (mics_segment * len(segs))(*[mics_segment(*map(int, sg)) for sg in segs])


def _check(rc: int) -> None:
    if rc != MICS_OK:
        raise MicsError(rc, lib.mics_last_error().decode("utf-8", "replace"))


def _dev_ptr(x) -> Optional[int]:
    """Device address of a torch tensor (must be contiguous), or a raw integer address."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return x.data_ptr()


def _table(items: Sequence) -> ctypes.Array:
    return (ctypes.c_void_p * len(items))(*[_dev_ptr(t) for t in items])


def _stream(stream) -> Optional[int]:
    """hipStream_t handle: explicit integer, a torch stream, or torch's current stream."""
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def mics_version() -> int:
    return lib.mics_version()


def mics_last_error() -> str:
    return lib.mics_last_error().decode("utf-8", "replace")


def mics_shard_elems(n: int, p: int, align_elems: int = 8) -> int:
    return lib.mics_shard_elems(n, p, align_elems)


def mics_set_blocks_per_cu(blocks_per_cu: int) -> None:
    _check(lib.mics_set_blocks_per_cu(blocks_per_cu))


def mics_set_stream_threshold_bytes(nbytes: int) -> None:
    _check(lib.mics_set_stream_threshold_bytes(nbytes))


MICS_KERNELS_REORDER, MICS_KERNELS_REDUCE, MICS_KERNELS_AVERAGE, MICS_KERNELS_ADAM, MICS_KERNELS_FUSED = range(5)


def mics_set_launch_shape(kernel_family: int, lanes: int = 0, waves_per_cu: int = 0) -> None:
    _check(lib.mics_set_launch_shape(kernel_family, lanes, waves_per_cu))


def mics_hier_gather_reorder(dst_flat, stage1_bufs: Sequence, n_valid: int, shard_elems: int,
                             p: int, k: int, elem_bytes: int, stream=None) -> None:
    """Stage-1 buffers of the hierarchical all-gather -> contiguous flat parameter."""
    if len(stage1_bufs) != k:
        raise ValueError(f"expected k = {k} stage-1 buffers, got {len(stage1_bufs)}")
    _check(lib.mics_hier_gather_reorder(_dev_ptr(dst_flat), _table(stage1_bufs), n_valid,
                                        shard_elems, p, k, elem_bytes, _stream(stream)))


def mics_reduce_scatter_accum(acc, grads_bf16: Sequence, elem_offset: int, count: int,
                              accumulate: bool, stream=None) -> None:
    """acc[0:count] (+)= sum over the p rank buffers of elements [elem_offset, +count)."""
    _check(lib.mics_reduce_scatter_accum(_dev_ptr(acc), _table(grads_bf16), elem_offset, count,
                                         len(grads_bf16), int(bool(accumulate)), _stream(stream)))


def mics_replica_average(out, acc_copies: Sequence, count: int, scale: float, stream=None) -> None:
    """out = (sum over the r replica copies) * scale."""
    _check(lib.mics_replica_average(_dev_ptr(out), _table(acc_copies), count, len(acc_copies),
                                    scale, _stream(stream)))


def mics_adam_shard(master, exp_avg, exp_avg_sq, param_bf16, grad, count: int, *, lr: float,
                    beta1: float, beta2: float, eps: float, weight_decay: float, step: int,
                    stream=None) -> None:
    """Mixed-precision Adam step in place on the fp32 shard; writes the bf16 parameter."""
    _check(lib.mics_adam_shard(_dev_ptr(master), _dev_ptr(exp_avg), _dev_ptr(exp_avg_sq),
                               _dev_ptr(param_bf16), _dev_ptr(grad), count, lr, beta1, beta2, eps,
                               weight_decay, step, _stream(stream)))


def mics_hier_gather_reorder_coalesced(dst_flat, stage1_bufs: Sequence, segs, p: int, k: int,
                                       elem_bytes: int, stream=None) -> None:
    """The gather reorder for many separately sharded tensors in one call; ``segs`` holds
    (numel, shard_elems, src_offset, dst_offset) per tensor."""
    if len(stage1_bufs) != k:
        raise ValueError(f"expected k = {k} stage-1 buffers, got {len(stage1_bufs)}")
    arr = segs if isinstance(segs, ctypes.Array) else _segments(segs)
    _check(lib.mics_hier_gather_reorder_coalesced(_dev_ptr(dst_flat), _table(stage1_bufs), arr, len(arr),
                                                  p, k, elem_bytes, _stream(stream)))


def mics_reduce_scatter_accum_coalesced(acc, grads_bf16: Sequence, segs, accumulate: bool,
                                        stream=None) -> None:
    """Reduce-scatter-accumulate for many tensors in one call; ``segs`` holds
    (count, 0, src_offset, dst_offset) per tensor."""
    arr = segs if isinstance(segs, ctypes.Array) else _segments(segs)
    _check(lib.mics_reduce_scatter_accum_coalesced(_dev_ptr(acc), _table(grads_bf16), arr, len(arr),
                                                   len(grads_bf16), int(bool(accumulate)),
                                                   _stream(stream)))


def mics_replica_average_adam_shard(master, exp_avg, exp_avg_sq, param_bf16, acc_copies: Sequence,
                                    count: int, scale: float, *, lr: float, beta1: float, beta2: float,
                                    eps: float, weight_decay: float, step: int, stream=None) -> None:
    """Replica average and Adam step in one pass; same results as the two separate calls."""
    _check(lib.mics_replica_average_adam_shard(
        _dev_ptr(master), _dev_ptr(exp_avg), _dev_ptr(exp_avg_sq), _dev_ptr(param_bf16),
        _table(acc_copies), count, len(acc_copies), scale, lr, beta1, beta2, eps, weight_decay, step,
        _stream(stream)))


def mics_reduce_scatter_accum_coalesced_typed(acc, grads: Sequence, segs, accumulate: bool, grad_dtype: int,
                                              stream=None) -> None:
    """mics_reduce_scatter_accum_coalesced for bf16 / fp16 / fp32 gradient buffers (MICS_DTYPE_*)."""
    arr = segs if isinstance(segs, ctypes.Array) else _segments(segs)
    _check(lib.mics_reduce_scatter_accum_coalesced_typed(_dev_ptr(acc), _table(grads), arr, len(arr), len(grads),
                                                         int(bool(accumulate)), grad_dtype, _stream(stream)))


def mics_adam_shard_typed(master, exp_avg, exp_avg_sq, param_out, param_dtype: int, grad, count: int, *,
                          lr: float, beta1: float, beta2: float, eps: float, weight_decay: float, step: int,
                          stream=None) -> None:
    """mics_adam_shard writing the 16-bit parameter as bf16 or binary16 (MICS_DTYPE_*)."""
    _check(lib.mics_adam_shard_typed(_dev_ptr(master), _dev_ptr(exp_avg), _dev_ptr(exp_avg_sq),
                                     _dev_ptr(param_out), param_dtype, _dev_ptr(grad), count, lr, beta1, beta2,
                                     eps, weight_decay, step, _stream(stream)))


def mics_replica_average_adam_shard_typed(master, exp_avg, exp_avg_sq, param_out, param_dtype: int,
                                          acc_copies: Sequence, count: int, scale: float, *, lr: float,
                                          beta1: float, beta2: float, eps: float, weight_decay: float,
                                          step: int, stream=None) -> None:
    """mics_replica_average_adam_shard writing the 16-bit parameter as bf16 or binary16."""
    _check(lib.mics_replica_average_adam_shard_typed(
        _dev_ptr(master), _dev_ptr(exp_avg), _dev_ptr(exp_avg_sq), _dev_ptr(param_out), param_dtype,
        _table(acc_copies), count, len(acc_copies), scale, lr, beta1, beta2, eps, weight_decay, step,
        _stream(stream)))


def mics_reduce_scatter_accum_typed(acc, grads: Sequence, elem_offset: int, count: int,
                                    accumulate: bool, grad_dtype: int, stream=None) -> None:
    """mics_reduce_scatter_accum for bf16 / fp16 / fp32 gradient buffers (MICS_DTYPE_*)."""
    _check(lib.mics_reduce_scatter_accum_typed(_dev_ptr(acc), _table(grads), elem_offset, count,
                                               len(grads), int(bool(accumulate)), grad_dtype,
                                               _stream(stream)))
