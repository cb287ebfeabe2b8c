"""Pins for the oracle's mixed-precision Adam step (the paper names only "Adam optimizer using
mixed-precision" with 16 bytes of model state per parameter, Section 3.2; the update rule is
the textbook bias-corrected Adam with decoupled weight decay)."""
import numpy as np
import pytest
import torch

from util import adam_rel_err, state_rel_err

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)


def fresh(gen, n, seed=21):
    w = gen.fill_host(gen.stream_key(seed, gen.ROLE_MASTER), 0, n, gen.normal_table(0.02, "f32"))
    return w, np.zeros(n, np.float32), np.zeros(n, np.float32)


@pytest.mark.parametrize("f32", [False, True])
def test_constant_gradient_has_a_closed_form(orc, gen, f32):
    # zero-initialised moments and a constant gradient c: m_hat = c and v_hat = c^2 at every
    # step, so w_T = w_0 - T * lr * c / (|c| + eps)
    n, T = 512, 20
    w, m, v = fresh(gen, n)
    w0 = w.astype(np.float64)
    c = gen.fill_host(gen.stream_key(22, gen.ROLE_ACC), 0, n, gen.normal_table(1e-3, "f32"))
    c[c == 0] = 1e-3
    for t in range(1, T + 1):
        orc.adam_shard(w, m, v, c, step=t, f32=f32, **HP)
    c64 = c.astype(np.float64)
    want = w0 - T * float(np.float32(HP["lr"])) * c64 / (np.abs(c64) + float(np.float32(HP["eps"])))
    assert adam_rel_err(w, want, w0).max() < 1e-6
    # and the moments are geometric sums: m_T = (1 - b1^T) c, v_T = (1 - b2^T) c^2
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
    assert state_rel_err(m, (1 - b1 ** T) * c64, 1e-30).max() < 1e-5
    assert state_rel_err(v, (1 - b2 ** T) * c64 ** 2, 1e-30).max() < 1e-5


@pytest.mark.parametrize("f32", [False, True])
def test_zero_gradient_leaves_everything_unchanged_and_decay_is_decoupled(orc, gen, f32):
    n, T = 256, 7
    w, m, v = fresh(gen, n)
    w0 = w.copy()
    zero = np.zeros(n, np.float32)
    orc.adam_shard(w, m, v, zero, step=1, f32=f32, **HP)
    assert np.array_equal(w, w0) and not m.any() and not v.any()
    hp = dict(HP, weight_decay=0.1, lr=1e-2)
    for t in range(1, T + 1):
        orc.adam_shard(w, m, v, zero, step=t, f32=f32, **hp)
    shrink = (1.0 - float(np.float32(1e-2)) * float(np.float32(0.1))) ** T
    assert np.allclose(w, w0.astype(np.float64) * shrink, rtol=1e-6, atol=0)


@pytest.mark.parametrize("f32", [False, True])
def test_update_is_an_odd_function_of_gradient_and_weight(orc, gen, f32):
    n = 300
    w, m, v = fresh(gen, n)
    g = gen.fill_host(gen.stream_key(23, gen.ROLE_ACC), 0, n, gen.normal_table(1e-3, "f32"))
    hp = dict(HP, weight_decay=0.01)
    wn, mn, vn = -w, m.copy(), v.copy()
    for t in (1, 2, 3):
        pb = orc.adam_shard(w, m, v, g, step=t, f32=f32, **hp)
        pbn = orc.adam_shard(wn, mn, vn, -g, step=t, f32=f32, **hp)
    assert np.array_equal(wn, -w) and np.array_equal(mn, -m) and np.array_equal(vn, v)
    assert np.array_equal(pbn ^ 0x8000, pb)


def library_adamw_step(w, m, v, g, step, hp):
    """One step of torch.optim.AdamW in double precision from the given binary32 state."""
    wt = torch.from_numpy(w.astype(np.float64)).requires_grad_(True)
    opt = torch.optim.AdamW([wt], lr=float(np.float32(hp["lr"])),
                            betas=(float(np.float32(hp["beta1"])), float(np.float32(hp["beta2"]))),
                            eps=float(np.float32(hp["eps"])),
                            weight_decay=float(np.float32(hp["weight_decay"])))
    opt.state[wt] = {"step": torch.tensor(float(step - 1)),
                     "exp_avg": torch.from_numpy(m.astype(np.float64)),
                     "exp_avg_sq": torch.from_numpy(v.astype(np.float64))}
    wt.grad = torch.from_numpy(g.astype(np.float64))
    opt.step()
    st = opt.state[wt]
    return wt.detach().numpy(), st["exp_avg"].numpy(), st["exp_avg_sq"].numpy()


@pytest.mark.parametrize("wd", [0.0, 0.05])
@pytest.mark.parametrize("f32", [False, True])
def test_against_the_library_optimizer_in_double_precision(orc, gen, wd, f32):
    # every step starts both sides from the same binary32 state, so the only differences are
    # the final roundings to binary32 (and, for the single-precision variant, its own steps)
    n, T = 4000, 6
    w, m, v = fresh(gen, n)
    hp = dict(HP, weight_decay=wd, lr=1e-3)
    table = gen.normal_table(1e-3, "f32")
    b1 = float(np.float32(hp["beta1"]))
    for t in range(1, T + 1):
        g = gen.fill_host(gen.stream_key(24, gen.ROLE_ACC, t), 0, n, table)
        w_lib, m_lib, v_lib = library_adamw_step(w, m, v, g, t, hp)
        w_before = w.copy()
        m_terms = b1 * np.abs(m.astype(np.float64)) + (1 - b1) * np.abs(g.astype(np.float64))
        orc.adam_shard(w, m, v, g, step=t, f32=f32, **hp)
        assert adam_rel_err(w, w_lib, w_before).max() < 1e-6
        assert (np.abs(m - m_lib) / m_terms).max() < 2e-7
        assert state_rel_err(v, v_lib, 1e-30).max() < 2e-7


def test_single_precision_variant_tracks_the_double_precision_one(orc, gen):
    n, T = 50000, 4
    w, m, v = fresh(gen, n)
    w2, m2, v2 = w.copy(), m.copy(), v.copy()
    table = gen.normal_table(2.6e-6, "f32")      # scale of a mean over 1536 gradients of 1e-4
    worst_ulp = 0
    for t in range(1, T + 1):
        g = gen.fill_host(gen.stream_key(25, gen.ROLE_ACC, t), 0, n, table)
        before, before_m = w.copy(), m.copy()
        pb = orc.adam_shard(w, m, v, g, step=t, **HP)
        pb2 = orc.adam_shard(w2, m2, v2, g, step=t, f32=True, **HP)
        assert adam_rel_err(w2, w, before).max() < 1e-6
        m_terms = 0.9 * np.abs(before_m.astype(np.float64)) + 0.1 * np.abs(g.astype(np.float64))
        assert (np.abs(m2.astype(np.float64) - m) / m_terms).max() < 2e-7
        assert state_rel_err(v2, v, 1e-30).max() < 3e-7
        from util import bf16_ulp_distance
        worst_ulp = max(worst_ulp, int(bf16_ulp_distance(pb, pb2).max()))
        w2[:], m2[:], v2[:] = w, m, v            # compare one step at a time
    assert worst_ulp <= 1


def test_bf16_parameter_is_the_rounded_master_and_state_is_16_bytes_per_parameter(orc, gen):
    n = 4096
    w, m, v = fresh(gen, n)
    g = gen.fill_host(gen.stream_key(26, gen.ROLE_ACC), 0, n, gen.normal_table(1e-3, "f32"))
    pb = orc.adam_shard(w, m, v, g, step=1, **HP)
    lib = torch.from_numpy(w.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(pb, lib)
    grad_bf16_bytes = 2
    per_param = pb.itemsize + grad_bf16_bytes + w.itemsize + m.itemsize + v.itemsize
    assert per_param == 16          # 10 B parameters <-> about 160 GB of model state
    assert orc.adam_shard(w, m, v, g, step=2, want_bf16=False, **HP) is None


def test_step_must_start_at_one(orc, gen):
    w, m, v = fresh(gen, 8)
    with pytest.raises(ValueError):
        orc.adam_shard(w, m, v, np.zeros(8, np.float32), step=0, **HP)
