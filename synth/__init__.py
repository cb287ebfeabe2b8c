"""Seeded synthetic inputs for the MiCS data path: configurations and generators.

This module serves both the HIP library's tests/bench and the CPU oracle's tests.
It holds none of the method's arithmetic: values are entries of a quantised-normal
table picked by an integer hash of (stream key, element index), so a window of any
buffer can be produced on the host without materialising the rest, and the device
twin produces identical bytes.

The flat buffers stand in for the transformer layers of the paper's BERT variants
(Table 1): 12*h^2 + 13*h elements per layer; fp32 master ~ N(0, 0.02), bf16 gradients
~ N(0, sigma) per configuration (optionally 1 % of elements scaled by 100).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_HOST_LIB = os.path.join(_HERE, "libsynth_host.so")
_DEV_LIB = os.path.join(_HERE, "libsynth_dev.so")

MASK64 = (1 << 64) - 1
TABLE_SLOTS = 1 << 16

# stream roles
ROLE_PARAM, ROLE_MASTER, ROLE_GRAD, ROLE_ACC, ROLE_MISC = 1, 2, 3, 4, 5


# ---- configurations ----------------------------------------------------------------

def layer_elems(h: int) -> int:
    """Elements of one transformer layer with hidden size h and intermediate size 4h
    (Table 1): 4h^2 attention + 8h^2 feed-forward + 9h biases + 4h LayerNorm."""
    return 12 * h * h + 13 * h


def shard_elems(n: int, p: int, align: int = 8) -> int:
    """Workload geometry: how the synthetic layers are cut into p shards (equal parts, rounded up
    to `align` elements, the tail padded).  The paper leaves the padding rule open; this is the
    caller-side convention of the configurations, not arithmetic on data."""
    per = -(-n // p)
    return -(-per // align) * align


@dataclass(frozen=True)
class Config:
    name: str
    N: int            # logical elements of the flat parameter
    p: int            # partition group size
    k: int            # devices per node
    r: int            # replication factor
    s: int            # micro-steps per step
    sigma_grad: float
    seed: int
    outlier_frac: float = 0.0
    outlier_scale: float = 100.0
    align: int = 8
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    sigma_master: float = 0.02

    @property
    def S(self) -> int:
        return shard_elems(self.N, self.p, self.align)

    @property
    def N_pad(self) -> int:
        return self.S * self.p

    @property
    def nodes(self) -> int:
        return self.p // self.k


CONFIGS = {
    "tiny": Config("tiny", 1 << 20, p=4, k=2, r=2, s=2, sigma_grad=1e-2, seed=1001),
    "h2560": Config("h2560", layer_elems(2560), p=8, k=8, r=4, s=4, sigma_grad=1e-3, seed=1002),
    "h4096": Config("h4096", layer_elems(4096), p=16, k=8, r=2, s=8, sigma_grad=1e-3, seed=1003),
    # h = 5120 divides by p = 32 exactly, so the ragged tail is made by dropping 13 elements
    "h5120": Config("h5120", layer_elems(5120) - 13, p=32, k=8, r=2, s=4, sigma_grad=1e-3,
                    seed=1004, outlier_frac=0.01),
    # stress variant: odd shard length, chunk starts only element-aligned
    "h5120_odd": Config("h5120_odd", layer_elems(5120) + 5, p=32, k=8, r=2, s=4, sigma_grad=1e-3,
                        seed=1004, outlier_frac=0.01, align=1),
    "h8192": Config("h8192", layer_elems(8192), p=16, k=8, r=8, s=12, sigma_grad=1e-4, seed=1005),
    # the h = 8192 layer in the partition group the paper trains its 50B model with (8 nodes of
    # 8 devices, Section 5) and the 4 micro-steps of its large-scale run
    "h8192_p64": Config("h8192_p64", layer_elems(8192), p=64, k=8, r=2, s=4, sigma_grad=1e-4, seed=1006),
}


# ---- one layer as its tensors (coalesced collectives, Section 4) -------------------------

def layer_tensors(h: int):
    """(name, elements) of the 16 tensors of one transformer layer (Table 1: intermediate = 4h)."""
    t = []
    for name in ("attn.q", "attn.k", "attn.v", "attn.out"):
        t += [(name + ".weight", h * h), (name + ".bias", h)]
    t += [("ln1.weight", h), ("ln1.bias", h)]
    t += [("ffn.up.weight", 4 * h * h), ("ffn.up.bias", 4 * h)]
    t += [("ffn.down.weight", 4 * h * h), ("ffn.down.bias", h)]
    t += [("ln2.weight", h), ("ln2.bias", h)]
    assert sum(n for _, n in t) == layer_elems(h)
    return t


@dataclass(frozen=True)
class CoalescedLayout:
    """Where each separately sharded tensor lives in the four kinds of buffer.  All offsets
    are in elements.  S[t] = shard size of tensor t."""
    numel: tuple      # logical elements per tensor
    S: tuple          # shard elements per tensor
    stage1_off: tuple  # in every stage-1 buffer: (p/k)*S[t] elements from here
    flat_off: tuple    # in the gathered flat parameter: numel[t] elements from here
    grad_off: tuple    # in every rank's gradient buffer: p*S[t] elements from here
    shard_off: tuple   # in a rank's shard buffers (acc, master, ...): S[t] elements from here

    @property
    def stage1_len(self):
        return self.stage1_off[-1] if self.stage1_off else 0

    def reorder_segments(self):
        return [(self.numel[t], self.S[t], self.stage1_off[t], self.flat_off[t]) for t in range(len(self.S))]

    def reduce_segments(self, g: int):
        return [(self.S[t], 0, self.grad_off[t] + g * self.S[t], self.shard_off[t]) for t in range(len(self.S))]


def coalesced_layout(numels, p: int, k: int, align: int = 8, flat_align: int = 1) -> CoalescedLayout:
    S = [shard_elems(n, p, align) for n in numels]
    stage1, flat, grad, shard = [0], [0], [0], [0]
    for n, s in zip(numels, S):
        stage1.append(stage1[-1] + (p // k) * s)
        flat.append(-(-(flat[-1] + n) // flat_align) * flat_align)
        grad.append(grad[-1] + p * s)
        shard.append(shard[-1] + s)
    return CoalescedLayout(tuple(numels), tuple(S), tuple(stage1), tuple(flat), tuple(grad), tuple(shard))


# ---- tables --------------------------------------------------------------------------

def _bf16_grid_bits(x: np.ndarray) -> np.ndarray:
    """Bit patterns of bf16 values for the table: the upper half of each float32 (the lower half
    is cut off).  This only puts the table entries on the bf16 grid -- it is deliberately not the
    round-to-nearest-even narrowing that the method's Adam step performs, which lives in the
    library and in the oracle, each on its own."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def normal_table(sigma: float, elem: str) -> np.ndarray:
    """65,536 mid-quantiles of N(0, sigma): 'bf16' -> uint16 bit patterns, 'f32' -> float32."""
    from scipy.special import ndtri
    q = ndtri((np.arange(TABLE_SLOTS, dtype=np.float64) + 0.5) / TABLE_SLOTS) * float(sigma)
    f = q.astype(np.float32)
    if elem == "f32":
        return f
    if elem == "bf16":
        return _bf16_grid_bits(f)
    raise ValueError(elem)


def small_int_table(lo: int, hi: int, elem: str) -> np.ndarray:
    """Table of integers in [lo, hi] (exactly representable): sums over them are exact."""
    vals = (lo + (np.arange(TABLE_SLOTS) % (hi - lo + 1))).astype(np.float32)
    return vals if elem == "f32" else _bf16_grid_bits(vals)


# ---- stream keys -----------------------------------------------------------------------

def _mix64(z: int) -> int:
    z &= MASK64
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & MASK64
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & MASK64
    z ^= z >> 31
    return z


def stream_key(seed: int, role: int, c: int = 0, t: int = 0, q: int = 0) -> int:
    """One independent stream per (seed, role, replica c, micro-step t, rank q)."""
    z = _mix64(seed)
    for part in (role, c, t, q):
        z = _mix64(z + part + 1)
    return z


def outlier_threshold(frac: float) -> int:
    return int(round(frac * (1 << 32)))


# ---- native twins ------------------------------------------------------------------------

def build_host(force: bool = True) -> str:
    if force or not os.path.exists(_HOST_LIB):
        tmp = _HOST_LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall",
                        "-o", tmp, os.path.join(_CSRC, "synth_host.c")], check=True)
        os.replace(tmp, _HOST_LIB)
    return _HOST_LIB


def build_device(force: bool = True) -> str:
    if force or not os.path.exists(_DEV_LIB):
        tmp = _DEV_LIB + f".tmp{os.getpid()}"
        res = subprocess.run(["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O3", "-shared",
                              "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                              "-o", tmp, os.path.join(_CSRC, "synth_dev.hip")],
                             capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
        os.replace(tmp, _DEV_LIB)
    return _DEV_LIB


_host = None
_dev = None


def _host_lib():
    global _host
    if _host is None:
        if not os.path.exists(_HOST_LIB):
            build_host()
        _host = ctypes.CDLL(_HOST_LIB)
        _host.synth_fill_host.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_size_t,
                                          ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_uint32, ctypes.c_int, ctypes.c_int]
    return _host


def _dev_lib():
    global _dev
    if _dev is None:
        if not os.path.exists(_DEV_LIB):
            raise RuntimeError(f"{_DEV_LIB} is not built; run __graft_entry__.build() first")
        import torch  # noqa: F401  (its HIP runtime must be the one this library binds to)
        _dev = ctypes.CDLL(_DEV_LIB)
        _dev.synth_fill_device.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_size_t,
                                           ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_uint32, ctypes.c_int, ctypes.c_void_p]
    return _dev


def fill_host(key: int, x0: int, n: int, table: np.ndarray,
              outlier_table: Optional[np.ndarray] = None, outlier_frac: float = 0.0,
              threads: int = 0) -> np.ndarray:
    """Elements [x0, x0+n) of stream ``key`` as a numpy array of the table's dtype."""
    table = np.ascontiguousarray(table)
    assert table.size == TABLE_SLOTS and table.dtype.itemsize in (2, 4)
    if outlier_table is not None:
        outlier_table = np.ascontiguousarray(outlier_table, dtype=table.dtype)
    out = np.empty(n, dtype=table.dtype)
    rc = _host_lib().synth_fill_host(
        out.ctypes.data, x0, n, key, table.ctypes.data,
        outlier_table.ctypes.data if outlier_table is not None else None,
        outlier_threshold(outlier_frac) if outlier_table is not None else 0,
        table.dtype.itemsize, threads or min(16, os.cpu_count() or 1))
    if rc != 0:
        raise ValueError("synth_fill_host: bad arguments")
    return out


def fill_device(out_ptr: int, key: int, x0: int, n: int, table_ptr: int, elem_bytes: int,
                outlier_table_ptr: int = 0, outlier_frac: float = 0.0, stream: int = 0) -> None:
    """Write elements [x0, x0+n) of stream ``key`` to device memory at ``out_ptr``.
    ``table_ptr`` / ``outlier_table_ptr`` are device copies of the tables."""
    rc = _dev_lib().synth_fill_device(
        out_ptr, x0, n, key, table_ptr, outlier_table_ptr or None,
        outlier_threshold(outlier_frac) if outlier_table_ptr else 0, elem_bytes, stream or None)
    if rc != 0:
        raise RuntimeError(f"synth_fill_device failed (rc={rc})")
