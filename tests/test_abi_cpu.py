"""The C ABI without a GPU: exported symbols match the header, and every argument error is
reported by the host-side checks before any HIP call (fake device addresses are never
dereferenced)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", name) for name in ("mics.h", "mics_tuning.h")]

mics = pytest.importorskip("paper_2205_00119_amd", reason="libmics.so is not built")

A = 0x7F0000000000          # a 16-byte aligned pretend device address
BUF = 1 << 24                # pretend buffers are spaced far apart


def declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"\b(mics_\w+)\s*\(", text)


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert len(names) >= 11
    for name in names:
        assert hasattr(mics.lib, name), f"{name} declared in mics.h but not exported"
    assert sorted(set(names)) == sorted(mics.EXPORTS)


def test_version_and_shard_elems():
    assert mics.mics_version() >= 100
    assert mics.mics_shard_elems(805412864, 16, 8) == 50338304
    assert mics.mics_shard_elems(314639347, 32, 8) == 9832480
    assert mics.mics_shard_elems(314639365, 32, 1) == 9832481
    assert mics.mics_shard_elems(10, 4, 8) == 8
    assert mics.mics_shard_elems(0, 4, 8) == 0
    assert mics.mics_shard_elems(10, 0, 8) == 0


def expect(code, fragment, fn, *args, **kw):
    with pytest.raises(mics.MicsError) as ei:
        fn(*args, **kw)
    assert ei.value.code == code, str(ei.value)
    assert fragment in str(ei.value), str(ei.value)
    assert fragment in mics.mics_last_error()


def test_reorder_argument_errors():
    f = mics.mics_hier_gather_reorder
    T = [A + BUF * (i + 1) for i in range(8)]
    expect(mics.MICS_ERR_INVALID_ARG, "not divisible", f, A, T[:3], 10, 10, 4, 3, 2, stream=0)
    expect(mics.MICS_ERR_UNSUPPORTED, "elem_bytes", f, A, T[:2], 10, 10, 4, 2, 8, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "n_valid", f, A, T[:2], 41, 10, 4, 2, 2, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "p = 0", f, A, [], 0, 10, 0, 0, 2, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "p = 256", f, A, T[:2], 10, 10, 256, 2, 2, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "k = 8", f, A, T[:8], 10, 10, 4, 8, 2, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "dst_flat is NULL", f, None, T[:2], 10, 10, 4, 2, 2, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "stage1_bufs[1] is NULL", f, A, [T[0], None], 10, 10, 4, 2, 2, stream=0)
    expect(mics.MICS_ERR_ALIGNMENT, "dst_flat", f, A + 1, T[:2], 10, 10, 4, 2, 2, stream=0)
    expect(mics.MICS_ERR_ALIGNMENT, "stage1_bufs[0]", f, A, [T[0] + 2, T[1]], 10, 10, 4, 2, 4, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overlaps", f, A, [A + 16, T[1]], 40, 10, 4, 2, 2, stream=0)
    # nothing to do is not an error and needs no GPU
    f(A, T[:2], 0, 10, 4, 2, 2, stream=0)


def test_reduce_scatter_accum_argument_errors():
    f = mics.mics_reduce_scatter_accum
    G = [A + BUF * (i + 1) for i in range(4)]
    expect(mics.MICS_ERR_INVALID_ARG, "p = 0", f, A, [], 0, 8, False, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "p = 129", f, A, [G[0]] * 129, 0, 8, False, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "acc is NULL", f, None, G, 0, 8, False, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "grads_bf16[2] is NULL", f, A, [G[0], G[1], None], 0, 8, False, stream=0)
    expect(mics.MICS_ERR_ALIGNMENT, "acc", f, A + 2, G, 0, 8, False, stream=0)
    expect(mics.MICS_ERR_ALIGNMENT, "grads_bf16[1]", f, A, [G[0], G[1] + 1], 0, 8, False, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overlaps", f, A, [G[0], A - 32], 32, 64, False, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overflows", f, A, G, 1 << 63, 1 << 63, False, stream=0)
    f(A, G, 0, 0, False, stream=0)


def test_replica_average_argument_errors():
    f = mics.mics_replica_average
    C = [A + BUF * (i + 1) for i in range(4)]
    expect(mics.MICS_ERR_INVALID_ARG, "r = 0", f, A, [], 8, 1.0, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "out is NULL", f, None, C, 8, 1.0, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "acc_copies[1] is NULL", f, A, [C[0], None], 8, 1.0, stream=0)
    expect(mics.MICS_ERR_ALIGNMENT, "acc_copies[0]", f, A, [C[0] + 2], 8, 1.0, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overlaps acc_copies[1]", f, A, [C[0], A], 8, 1.0, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overlaps acc_copies[0]", f, A, [A + 16, C[1]], 8, 1.0, stream=0)
    f(A, C, 0, 1.0, stream=0)


def test_adam_argument_errors():
    f = mics.mics_adam_shard
    w, m, v, g, pb = (A + BUF * i for i in range(5))
    hp = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)
    expect(mics.MICS_ERR_INVALID_ARG, "step = 0", f, w, m, v, pb, g, 8, step=0, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "non-NULL", f, w, None, v, pb, g, 8, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_ALIGNMENT, "exp_avg_sq", f, w, m, v + 2, pb, g, 8, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_ALIGNMENT, "param_bf16", f, w, m, v, pb + 1, g, 8, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "master overlaps exp_avg", f, w, w + 16, v, pb, g, 8, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "param_bf16 overlaps grad", f, w, m, v, g + 8, g, 8, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "beta1", f, w, m, v, pb, g, 8, step=1, stream=0, **dict(hp, beta1=1.0))
    f(w, m, v, pb, g, 0, step=1, stream=0, **hp)


def test_coalesced_argument_errors():
    f = mics.mics_hier_gather_reorder_coalesced
    T = [A + BUF * (i + 1) for i in range(2)]
    ok = [(40, 10, 0, 0), (8, 2, 40, 40)]
    expect(mics.MICS_ERR_INVALID_ARG, "not divisible", f, A, T + [T[0]], ok, 4, 3, 2, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "segment 1: numel", f, A, T, [(40, 10, 0, 0), (9, 2, 40, 40)], 4, 2, 2, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overflow", f, A, T, [(40, 1 << 62, 0, 0)], 4, 2, 2, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overlaps", f, A, [A + 64, T[1]], ok, 4, 2, 2, stream=0)
    expect(mics.MICS_ERR_UNSUPPORTED, "elem_bytes", f, A, T, ok, 4, 2, 3, stream=0)
    f(A, T, [], 4, 2, 2, stream=0)
    f(A, T, [(0, 10, 0, 0)], 4, 2, 2, stream=0)
    g = mics.mics_reduce_scatter_accum_coalesced
    G = [A + BUF * (i + 1) for i in range(4)]
    expect(mics.MICS_ERR_INVALID_ARG, "grads_bf16[3] is NULL", g, A, G[:3] + [None], [(8, 0, 0, 0)], False, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overflow", g, A, G, [(1 << 61, 0, 0, 0)], False, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overlaps", g, A, [G[0], A], [(8, 0, 8, 0)], False, stream=0)
    expect(mics.MICS_ERR_ALIGNMENT, "acc", g, A + 1, G, [(8, 0, 0, 0)], False, stream=0)
    g(A, G, [(0, 0, 5, 7)], True, stream=0)


def test_fused_average_adam_argument_errors():
    f = mics.mics_replica_average_adam_shard
    w, m, v, pb = (A + BUF * i for i in range(4))
    C = [A + BUF * (5 + i) for i in range(3)]
    hp = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)
    expect(mics.MICS_ERR_INVALID_ARG, "step = 0", f, w, m, v, pb, C, 8, 0.5, step=0, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "r = 0", f, w, m, v, pb, [], 8, 0.5, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "acc_copies[2] is NULL", f, w, m, v, pb, C[:2] + [None], 8, 0.5, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "exp_avg overlaps acc_copies[1]", f, w, m, v, pb, [C[0], m + 4], 8, 0.5, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_ALIGNMENT, "acc_copies[0]", f, w, m, v, pb, [C[0] + 2], 8, 0.5, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "non-NULL", f, None, m, v, pb, C, 8, 0.5, step=1, stream=0, **hp)
    f(w, m, v, pb, C, 0, 0.5, step=1, stream=0, **hp)


def test_typed_coalesced_reduce_argument_errors():
    g = mics.mics_reduce_scatter_accum_coalesced_typed
    G = [A + BUF * (i + 1) for i in range(4)]
    expect(mics.MICS_ERR_UNSUPPORTED, "grad_dtype = 9", g, A, G, [(8, 0, 0, 0)], False, 9, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "mics_reduce_scatter_accum_coalesced_typed: grads[3] is NULL", g, A,
           G[:3] + [None], [(8, 0, 0, 0)], False, mics.MICS_DTYPE_F16, stream=0)
    expect(mics.MICS_ERR_ALIGNMENT, "grads[1] not aligned to 4 bytes", g, A, [G[0], G[1] + 2, G[2]], [(8, 0, 0, 0)],
           False, mics.MICS_DTYPE_F32, stream=0)
    g(A, [G[0], G[1] + 2, G[2]], [(0, 0, 0, 0)], False, mics.MICS_DTYPE_F16, stream=0)
    # binary32 elements are twice as long: the same segment overlaps the accumulator only then
    expect(mics.MICS_ERR_INVALID_ARG, "acc overlaps grads[0]", g, A + 48, [A, G[1]], [(16, 0, 0, 0)], False,
           mics.MICS_DTYPE_F32, stream=0)
    expect(mics.MICS_ERR_INVALID_ARG, "overlap", g, A, G, [(8, 0, 0, 0), (8, 0, 64, 4)], False,
           mics.MICS_DTYPE_F16, stream=0)


def test_typed_adam_argument_errors():
    w, m, v, g, po = (A + BUF * i for i in range(5))
    C = [A + BUF * (5 + i) for i in range(3)]
    hp = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)
    f = mics.mics_adam_shard_typed
    expect(mics.MICS_ERR_UNSUPPORTED, "mics_adam_shard_typed: param_dtype = MICS_DTYPE_F32", f, w, m, v, po,
           mics.MICS_DTYPE_F32, g, 8, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "param_dtype = 7", f, w, m, v, po, 7, g, 8, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_ALIGNMENT, "mics_adam_shard_typed: param_out", f, w, m, v, po + 1, mics.MICS_DTYPE_F16, g, 8,
           step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "param_out overlaps grad", f, w, m, v, g + 8, mics.MICS_DTYPE_F16, g, 8,
           step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "step = 0", f, w, m, v, po, mics.MICS_DTYPE_F16, g, 8, step=0, stream=0, **hp)
    f(w, m, v, po, mics.MICS_DTYPE_F16, g, 0, step=1, stream=0, **hp)
    f(w, m, v, None, mics.MICS_DTYPE_BF16, g, 0, step=1, stream=0, **hp)
    f = mics.mics_replica_average_adam_shard_typed
    expect(mics.MICS_ERR_UNSUPPORTED, "mics_replica_average_adam_shard_typed: param_dtype", f, w, m, v, po,
           mics.MICS_DTYPE_F32, C, 8, 0.5, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "param_out overlaps acc_copies[1]", f, w, m, v, po, mics.MICS_DTYPE_F16,
           [C[0], po + 4], 8, 0.5, step=1, stream=0, **hp)
    expect(mics.MICS_ERR_INVALID_ARG, "r = 0", f, w, m, v, po, mics.MICS_DTYPE_F16, [], 8, 0.5, step=1, stream=0, **hp)
    f(w, m, v, po, mics.MICS_DTYPE_F16, C, 0, 0.5, step=1, stream=0, **hp)


def test_launch_knob_range():
    mics.mics_set_blocks_per_cu(0)
    with pytest.raises(mics.MicsError):
        mics.mics_set_blocks_per_cu(4097)
    with pytest.raises(mics.MicsError):
        mics.mics_set_blocks_per_cu(-1)
    mics.mics_set_stream_threshold_bytes(1)
    mics.mics_set_stream_threshold_bytes(0)
    for fam in range(5):
        mics.mics_set_launch_shape(fam, 128, 8)
        mics.mics_set_launch_shape(fam, 0, 0)
    for bad in [(5, 64, 8), (-1, 64, 8), (1, 96, 8), (1, 1024, 8), (1, 64, 33), (1, 64, -1)]:
        with pytest.raises(mics.MicsError):
            mics.mics_set_launch_shape(*bad)


def test_header_is_valid_c99_and_cxx(tmp_path):
    import subprocess
    c = tmp_path / "use.c"
    c.write_text('#include "mics.h"\n#include "mics_tuning.h"\nint f(void) { mics_segment s = {1, 1, 0, 0}; (void)s; '
                 'return mics_version() + MICS_MAX_GROUP + MICS_ERR_HIP + MICS_DTYPE_F32; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", f"-I{inc}", str(c)],
                   check=True)
    cxx = tmp_path / "use.cpp"
    cxx.write_text(c.read_text())
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", f"-I{inc}", str(cxx)], check=True)
