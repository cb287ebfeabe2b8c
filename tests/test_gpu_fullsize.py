"""The five benchmark configurations at full size, in the launch configuration bench.py times
(rank view, and the whole-group view for the largest): the HIP path runs on device-generated
inputs, the oracle recomputes sampled windows (all chunk boundaries, both ends, the ragged tail,
random windows) from the host twin of the generator.  Same bars as the element-wise tests."""
import os

import numpy as np
import pytest
import torch

from util import adam_rel_err, bf16_ulp_distance

pytestmark = pytest.mark.gpu

mics = pytest.importorskip("paper_2205_00119_amd")

DEV = "cuda:0"
WIN = 1 << 15


@pytest.fixture(scope="module", autouse=True)
def _need_gpu(gen):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    yield
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


def windows(n, extra_points=(), seed=0, n_random=None, win=WIN):
    """Element ranges [a, b) inside [0, n): both ends, around the given points, and random ones
    that cover 1 % of the range (at least 6 of them) unless n_random says otherwise."""
    rng = np.random.default_rng(seed)
    if n_random is None:
        n_random = max(6, -(-n // (100 * win)))
    starts = {0, max(n - win, 0)}
    for pt in extra_points:
        starts.add(min(max(pt - win // 2, 0), max(n - win, 0)))
    for _ in range(n_random):
        starts.add(int(rng.integers(0, max(n - win, 1))))
    return sorted((a, min(a + win, n)) for a in starts)


class Tables:
    def __init__(self, gen, cfg):
        self.gen, self.cfg = gen, cfg
        self.host = {
            "grad": gen.normal_table(cfg.sigma_grad, "bf16"),
            "grad_out": gen.normal_table(cfg.sigma_grad * cfg.outlier_scale, "bf16") if cfg.outlier_frac else None,
            "param": gen.normal_table(cfg.sigma_master, "bf16"),
            "master": gen.normal_table(cfg.sigma_master, "f32"),
            "acc": gen.normal_table(cfg.sigma_grad * (cfg.p * cfg.s) ** 0.5, "f32"),
        }
        self.dev = {}
        for name, tab in self.host.items():
            if tab is None:
                self.dev[name] = None
            elif tab.dtype == np.uint16:
                self.dev[name] = torch.from_numpy(tab.view(np.int16)).to(DEV)
            else:
                self.dev[name] = torch.from_numpy(tab).to(DEV)

    def fill_dev(self, t, key, x0, name, outl=None, frac=0.0):
        tab = self.dev[name]
        o = self.dev[outl] if outl else None
        self.gen.fill_device(t.data_ptr(), key, x0, t.numel(), tab.data_ptr(), tab.element_size(),
                             o.data_ptr() if o is not None else 0, frac,
                             torch.cuda.current_stream().cuda_stream)

    def fill_host(self, key, x0, n, name, outl=None, frac=0.0):
        return self.gen.fill_host(key, x0, n, self.host[name], self.host[outl] if outl else None, frac)


def grad_key(gen, cfg, c, t, q):
    return gen.stream_key(cfg.seed, gen.ROLE_GRAD, c, t, q)


def test_device_generator_matches_host_twin(gen):
    cfg = gen.CONFIGS["h5120"]
    tb = Tables(gen, cfg)
    n = 3_000_001
    for name, outl, frac, dtype in (("grad", "grad_out", cfg.outlier_frac, torch.int16),
                                    ("master", None, 0.0, torch.float32)):
        t = torch.empty(n, dtype=dtype, device=DEV)
        key = gen.stream_key(cfg.seed, gen.ROLE_MISC, 1, 2, 3)
        tb.fill_dev(t, key, 12345, name, outl, frac)
        torch.cuda.synchronize()
        want = tb.fill_host(key, 12345, n, name, outl, frac)
        got = t.cpu().numpy()
        assert np.array_equal(got.view(want.dtype), want)
    w = gen.fill_host(gen.stream_key(1, 2), 0, 1 << 20, tb.host["master"])
    assert abs(float(w.std()) / cfg.sigma_master - 1) < 0.01 and abs(float(w.mean())) < 1e-4


@pytest.mark.parametrize("name", ["h2560", "h4096", "h5120", "h5120_odd", "h8192", "h8192_p64"])
def test_reorder_full_size(orc, gen, name):
    cfg = gen.CONFIGS[name]
    p, k, S, N, n_pad = cfg.p, cfg.k, cfg.S, cfg.N, cfg.N_pad
    nodes = p // k
    tb = Tables(gen, cfg)
    # the gathered-but-unordered buffer W = [T_0 .. T_{k-1}], T_l = [C_l, C_{k+l}, ...]
    W = torch.empty(n_pad, dtype=torch.int16, device=DEV)
    for g in range(p):
        j, l = divmod(g, k)
        slot = (l * nodes + j) * S
        tb.fill_dev(W[slot:slot + S], gen.stream_key(cfg.seed, gen.ROLE_PARAM, 0, 0, g), 0, "param")
    F = torch.full((n_pad + 64,), 0x5A5A, dtype=torch.int16, device=DEV)
    views = [W[l * nodes * S:(l + 1) * nodes * S] for l in range(k)]
    mics.mics_hier_gather_reorder(F, views, N, S, p, k, 2)
    torch.cuda.synchronize()
    # everything at or beyond N is untouched
    assert bool((F[N:] == 0x5A5A).all())
    # sampled windows: every chunk boundary, both ends, random places
    for a, b in windows(N, extra_points=[g * S for g in range(1, p)], seed=cfg.seed):
        got = F[a:b].cpu().numpy().view(np.uint16)
        # the definition: flat element x is element x mod S of chunk x div S
        parts = []
        x = a
        while x < b:
            g, i = divmod(x, S)
            m = min(b - x, S - i)
            parts.append(tb.fill_host(gen.stream_key(cfg.seed, gen.ROLE_PARAM, 0, 0, g), i, m, "param"))
            x += m
        want = np.concatenate(parts)
        assert np.array_equal(got, want), (name, a, b)
    # and a property that holds at any size: the multiset of 64-bit words per chunk is preserved
    for g in (0, p // 2, p - 1):
        j, l = divmod(g, k)
        valid = min(S, max(N - g * S, 0)) // 4 * 4
        if valid == 0:
            continue
        src = W[(l * nodes + j) * S:(l * nodes + j) * S + valid]
        dst = F[g * S:g * S + valid]
        if src.data_ptr() % 8 == 0 and dst.data_ptr() % 8 == 0:
            assert int(src.view(torch.int64).sum()) == int(dst.view(torch.int64).sum())
        else:
            assert int(src.to(torch.int64).sum()) == int(dst.to(torch.int64).sum())


def run_rank_pipeline(orc, gen, cfg, rank, count, offset, boundaries=(), n_random=None):
    """s reduce-scatter-accumulates, the replica average and one Adam step on `count` elements
    starting at global element `offset`, checked on sampled windows."""
    p, r, s = cfg.p, cfg.r, cfg.s
    tb = Tables(gen, cfg)
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, weight_decay=cfg.weight_decay)
    scale = float(np.float32(1.0 / (r * p * s)))
    grads = torch.empty((p, count), dtype=torch.int16, device=DEV)
    acc = torch.full((count,), float("nan"), dtype=torch.float32, device=DEV)
    for t in range(s):
        for q in range(p):
            tb.fill_dev(grads[q], grad_key(gen, cfg, 0, t, q), offset, "grad",
                        "grad_out" if cfg.outlier_frac else None, cfg.outlier_frac)
        mics.mics_reduce_scatter_accum(acc, [grads[q] for q in range(p)], 0, count, t > 0)
    others = torch.empty((r - 1, count), dtype=torch.float32, device=DEV)
    for c in range(1, r):
        tb.fill_dev(others[c - 1], gen.stream_key(cfg.seed, gen.ROLE_ACC, c), offset, "acc")
    avg = torch.empty(count, dtype=torch.float32, device=DEV)
    mics.mics_replica_average(avg, [acc] + [others[c] for c in range(r - 1)], count, scale)
    master = torch.empty(count, dtype=torch.float32, device=DEV)
    tb.fill_dev(master, gen.stream_key(cfg.seed, gen.ROLE_MASTER), offset, "master")
    m = torch.zeros(count, dtype=torch.float32, device=DEV)
    v = torch.zeros(count, dtype=torch.float32, device=DEV)
    pb = torch.empty(count, dtype=torch.int16, device=DEV)
    mics.mics_adam_shard(master, m, v, pb, avg, count, step=1, **hp)
    torch.cuda.synchronize()

    checked = 0
    # MICS_TEST_FULL=1 checks every element instead of sampled windows (minutes of oracle time)
    spans = ([(a, min(a + (1 << 22), count)) for a in range(0, count, 1 << 22)]
             if os.environ.get("MICS_TEST_FULL") == "1" else
             windows(count, extra_points=[count // 2, *boundaries], seed=cfg.seed + rank, n_random=n_random))
    for a, b in spans:
        n = b - a
        acc_ref = np.empty(n, np.float32)
        for t in range(s):
            host = [tb.fill_host(grad_key(gen, cfg, 0, t, q), offset + a, n, "grad",
                                 "grad_out" if cfg.outlier_frac else None, cfg.outlier_frac)
                    for q in range(p)]
            orc.reduce_scatter_accum(acc_ref, host, 0, t > 0)
        assert np.array_equal(acc[a:b].cpu().numpy().view(np.uint32), acc_ref.view(np.uint32)), (cfg.name, a)
        copies = [acc_ref] + [tb.fill_host(gen.stream_key(cfg.seed, gen.ROLE_ACC, c), offset + a, n, "acc")
                              for c in range(1, r)]
        avg_ref = orc.replica_average(copies, scale)
        assert np.array_equal(avg[a:b].cpu().numpy().view(np.uint32), avg_ref.view(np.uint32)), (cfg.name, a)
        w0 = tb.fill_host(gen.stream_key(cfg.seed, gen.ROLE_MASTER), offset + a, n, "master")
        w64, m64, v64 = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
        pb64 = orc.adam_shard(w64, m64, v64, avg_ref, step=1, **hp)
        w32, m32, v32 = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
        pb32 = orc.adam_shard(w32, m32, v32, avg_ref, step=1, f32=True, **hp)
        gw = master[a:b].cpu().numpy()
        assert adam_rel_err(gw, w64, w0).max() <= 1e-6
        assert np.array_equal(gw.view(np.uint32), w32.view(np.uint32))
        assert np.array_equal(m[a:b].cpu().numpy().view(np.uint32), m32.view(np.uint32))
        assert np.array_equal(v[a:b].cpu().numpy().view(np.uint32), v32.view(np.uint32))
        gpb = pb[a:b].cpu().numpy().view(np.uint16)
        assert bf16_ulp_distance(gpb, pb64).max() <= 1
        assert np.array_equal(gpb, pb32)
        checked += n
    # a property at any size: the accumulator is finite everywhere (no element was skipped)
    assert bool(torch.isfinite(acc).all())
    return checked


@pytest.mark.parametrize("name,rank", [("h2560", 3), ("h4096", 15), ("h5120", 31), ("h5120_odd", 7),
                                       ("h8192", 5), ("h8192_p64", 41)])
def test_rank_view_pipeline_full_size(orc, gen, name, rank):
    cfg = gen.CONFIGS[name]
    assert run_rank_pipeline(orc, gen, cfg, rank, cfg.S, rank * cfg.S) >= min(cfg.S // 100, 6 * WIN)


def test_group_view_full_size_h8192(orc, gen):
    # all p shards in one call: N_pad = 805,412,864 elements per launch, 25.8 GB of gradients
    cfg = gen.CONFIGS["h8192"]
    checked = run_rank_pipeline(orc, gen, cfg, 0, cfg.N_pad, 0, boundaries=[g * cfg.S for g in range(1, cfg.p)])
    assert checked >= cfg.N_pad // 100


def test_coalesced_layer_full_size_h8192(orc, gen):
    """The h = 8192 layer as its 16 separately sharded tensors (biases of h/p = 512 elements next
    to 4h^2-element matrices), rank view, through the coalesced entry points."""
    cfg = gen.CONFIGS["h8192"]
    p, k, s, rank = cfg.p, cfg.k, 2, 11
    nodes = p // k
    tb = Tables(gen, cfg)
    lay = gen.coalesced_layout([n for _, n in gen.layer_tensors(8192)], p, k, align=8)
    assert lay.shard_off[-1] == cfg.S and lay.flat_off[-1] == cfg.N
    n_t = len(lay.S)

    # reorder
    T = [torch.empty(lay.stage1_off[-1], dtype=torch.int16, device=DEV) for _ in range(k)]
    for t, St in enumerate(lay.S):
        for g in range(p):
            j, l = divmod(g, k)
            at = lay.stage1_off[t] + j * St
            tb.fill_dev(T[l][at:at + St], gen.stream_key(cfg.seed, gen.ROLE_PARAM, t, 0, g), 0, "param")
    F = torch.full((cfg.N + 64,), 0x5A5A, dtype=torch.int16, device=DEV)
    mics.mics_hier_gather_reorder_coalesced(F, T, lay.reorder_segments(), p, k, 2)
    torch.cuda.synchronize()
    assert bool((F[cfg.N:] == 0x5A5A).all())
    for t in range(n_t):
        St, n = lay.S[t], lay.numel[t]
        wins = [(0, n)] if n <= 4 * WIN else windows(n, extra_points=[g * St for g in range(1, p)],
                                                     seed=t, n_random=2)
        for a, b in wins:
            got = F[lay.flat_off[t] + a:lay.flat_off[t] + b].cpu().numpy().view(np.uint16)
            parts, x = [], a
            while x < b:
                g, i = divmod(x, St)
                m = min(b - x, St - i)
                parts.append(tb.fill_host(gen.stream_key(cfg.seed, gen.ROLE_PARAM, t, 0, g), i, m, "param"))
                x += m
            assert np.array_equal(got, np.concatenate(parts)), (t, a, b)

    # reduce-scatter-accumulate over full-length rank buffers
    del T, F
    grads = torch.empty((p, lay.grad_off[-1]), dtype=torch.int16, device=DEV)
    acc = torch.full((cfg.S,), float("nan"), dtype=torch.float32, device=DEV)
    segs = lay.reduce_segments(rank)
    for ts in range(s):
        for q in range(p):
            tb.fill_dev(grads[q], grad_key(gen, cfg, 0, ts, q), 0, "grad")
        mics.mics_reduce_scatter_accum_coalesced(acc, [grads[q] for q in range(p)], segs, ts > 0)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(acc).all())
    for t in range(n_t):
        St = lay.S[t]
        wins = [(0, St)] if St <= 4 * WIN else windows(St, seed=100 + t, n_random=2)
        for a, b in wins:
            ref = np.empty(b - a, np.float32)
            src0 = lay.grad_off[t] + rank * St + a
            for ts in range(s):
                host = [tb.fill_host(grad_key(gen, cfg, 0, ts, q), src0, b - a, "grad") for q in range(p)]
                orc.reduce_scatter_accum(ref, host, 0, ts > 0)
            got = acc[lay.shard_off[t] + a:lay.shard_off[t] + b].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (t, a, b)


def test_binary16_pipeline_full_size_h8192(orc, gen):
    """Mixed precision without bf16 (the paper's V100 runs, Section 5) on the h = 8192 shard:
    loss-scaled binary16 gradients through the typed reduction, the loss scale undone in the
    averaging factor, and the fused average + Adam step writing binary16 parameters."""
    cfg = gen.CONFIGS["h8192"]
    p, r, s, count, rank = cfg.p, cfg.r, 3, cfg.S, 9
    offset = rank * cfg.S
    loss_scale = 1024.0
    tb = Tables(gen, cfg)
    tb.host["grad16"] = gen.normal_table(cfg.sigma_grad * loss_scale, "f32").astype(np.float16).view(np.uint16)
    tb.dev["grad16"] = torch.from_numpy(tb.host["grad16"].view(np.int16)).to(DEV)
    tb.host["acc16"] = gen.normal_table(cfg.sigma_grad * loss_scale * (p * s) ** 0.5, "f32")
    tb.dev["acc16"] = torch.from_numpy(tb.host["acc16"]).to(DEV)
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, weight_decay=cfg.weight_decay)
    scale = float(np.float32(1.0 / (r * p * s * loss_scale)))
    grads = torch.empty((p, count), dtype=torch.int16, device=DEV)
    acc = torch.full((count,), float("nan"), dtype=torch.float32, device=DEV)
    for t in range(s):
        for q in range(p):
            tb.fill_dev(grads[q], grad_key(gen, cfg, 7, t, q), offset, "grad16")
        mics.mics_reduce_scatter_accum_typed(acc, [grads[q] for q in range(p)], 0, count, t > 0, mics.MICS_DTYPE_F16)
    others = [torch.empty(count, dtype=torch.float32, device=DEV) for _ in range(r - 1)]
    for c in range(1, r):
        tb.fill_dev(others[c - 1], gen.stream_key(cfg.seed, gen.ROLE_ACC, 7, c), offset, "acc16")
    master = torch.empty(count, dtype=torch.float32, device=DEV)
    tb.fill_dev(master, gen.stream_key(cfg.seed, gen.ROLE_MASTER), offset, "master")
    m = torch.zeros(count, dtype=torch.float32, device=DEV)
    v = torch.zeros(count, dtype=torch.float32, device=DEV)
    ph = torch.empty(count, dtype=torch.int16, device=DEV)
    mics.mics_replica_average_adam_shard_typed(master, m, v, ph, mics.MICS_DTYPE_F16, [acc] + others, count, scale,
                                               step=1, **hp)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(acc).all())
    checked = 0
    for a, b in windows(count, extra_points=[count // 2], seed=77):
        n = b - a
        acc_ref = np.empty(n, np.float32)
        for t in range(s):
            host = [tb.fill_host(grad_key(gen, cfg, 7, t, q), offset + a, n, "grad16") for q in range(p)]
            orc.reduce_scatter_accum_typed(acc_ref, host, 0, t > 0, orc.DTYPE_F16)
        assert np.array_equal(acc[a:b].cpu().numpy().view(np.uint32), acc_ref.view(np.uint32)), a
        copies = [acc_ref] + [tb.fill_host(gen.stream_key(cfg.seed, gen.ROLE_ACC, 7, c), offset + a, n, "acc16")
                              for c in range(1, r)]
        avg_ref = orc.replica_average(copies, scale)
        w0 = tb.fill_host(gen.stream_key(cfg.seed, gen.ROLE_MASTER), offset + a, n, "master")
        w32, m32, v32 = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
        p32 = orc.adam_shard(w32, m32, v32, avg_ref, step=1, f32=True, param_dtype="f16", **hp)
        w64, m64, v64 = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
        orc.adam_shard(w64, m64, v64, avg_ref, step=1, want_bf16=False, **hp)
        gw = master[a:b].cpu().numpy()
        assert adam_rel_err(gw, w64, w0).max() <= 1e-6
        assert np.array_equal(gw.view(np.uint32), w32.view(np.uint32))
        assert np.array_equal(m[a:b].cpu().numpy().view(np.uint32), m32.view(np.uint32))
        assert np.array_equal(v[a:b].cpu().numpy().view(np.uint32), v32.view(np.uint32))
        assert np.array_equal(ph[a:b].cpu().numpy().view(np.uint16), p32)
        checked += n
    assert checked >= min(count // 100, 6 * WIN)


def test_element_indices_beyond_32_bits(orc, gen):
    """The largest calls: more than 2^32 elements per buffer, so that element indices, byte offsets
    and lane counts all leave 32 bits.  Windows at both ends, around 2^31 and 2^32 and at random."""
    n = (1 << 32) + 4096 + 40
    # reorder: 4 chunks of 2^30 + 1034 elements (byte offsets of the later chunks exceed 2^32)
    p, k = 4, 2
    S = n // p
    assert S * p == n
    cfg = gen.Config("beyond32", n - 5, p=p, k=k, r=2, s=2, sigma_grad=1e-3, seed=1099)
    tb = Tables(gen, cfg)
    nodes = p // k
    W = torch.empty(n, dtype=torch.int16, device=DEV)
    for g in range(p):
        j, l = divmod(g, k)
        slot = (l * nodes + j) * S
        tb.fill_dev(W[slot:slot + S], gen.stream_key(cfg.seed, gen.ROLE_PARAM, 0, 0, g), 0, "param")
    F = torch.full((n,), 0x5A5A, dtype=torch.int16, device=DEV)
    mics.mics_hier_gather_reorder(F, [W[l * nodes * S:(l + 1) * nodes * S] for l in range(k)], cfg.N, S, p, k, 2)
    torch.cuda.synchronize()
    assert bool((F[cfg.N:] == 0x5A5A).all())
    for a, b in windows(cfg.N, extra_points=[g * S for g in range(1, p)] + [1 << 31, 1 << 32], seed=5, n_random=6):
        got = F[a:b].cpu().numpy().view(np.uint16)
        parts, x = [], a
        while x < b:
            g, i = divmod(x, S)
            m = min(b - x, S - i)
            parts.append(tb.fill_host(gen.stream_key(cfg.seed, gen.ROLE_PARAM, 0, 0, g), i, m, "param"))
            x += m
        assert np.array_equal(got, np.concatenate(parts)), (a, b)
    del W, F
    torch.cuda.empty_cache()
    # reduce (p = 2 buffers, 2 micro-steps), average over 2 copies, Adam: one call of n - 3 elements each
    cfg2 = gen.Config("beyond32", n, p=2, k=2, r=2, s=2, sigma_grad=1e-3, seed=1098)
    checked = run_rank_pipeline(orc, gen, cfg2, 0, n - 3, 16, boundaries=[1 << 31, 1 << 32], n_random=6)
    assert checked >= 8 * WIN
