"""Pins for the oracle's Adam arithmetic: closed forms of Kingma & Ba's
Algorithm 1, an fp64 evaluation in the textbook (m-hat / v-hat) form, library
Adam / AdamW, exact power-of-two unscaling, overflow-skip bit identity and the
fp16 re-cast.  The paper fixes neither the loss-scale schedule nor the decay
mode; the schedule used here (halve on overflow, double after a run of good
steps, skipped steps do not advance t) is held against PyTorch's own
mixed-precision loop, its floor at 1 and the default decay mode are conventions
whose behaviour is tested."""
import numpy as np
import pytest

from paper_2108_05818_amd import workloads as W

F32 = np.float32


def ulp32(x):
    x = np.abs(np.asarray(x, dtype=np.float32))
    x = np.maximum(x, np.float32(1.1754944e-38))
    return (np.nextafter(x, np.float32(np.inf)) - x).astype(np.float64)


def f16(vals):
    return np.asarray(vals, dtype=np.float16).view(np.uint16).copy()


def state(n, p0=0.0):
    return (np.zeros(n, np.uint16), np.full(n, p0, F32), np.zeros(n, F32), np.zeros(n, F32))


# ---------------------------------------------------------------- closed forms

def test_step1_from_zero_state_moves_by_lr_g_over_absg_plus_eps(orc):
    g = np.array([1e-3, -1e-3, 0.5, -2.0, 3e-5, -7e-4, 60000.0, 6e-8], dtype=np.float16)
    n = g.size
    p16, p, m, v = state(n)
    h = orc.hyper(lr=1e-3, eps=1e-8, weight_decay=0.0, step=1, loss_scale=1.0)
    orc.adam_chunk(g.view(np.uint16).copy(), p16, p, m, v, n, h)
    gd = g.astype(np.float64)
    want = -1e-3 * gd / (np.abs(gd) + 1e-8)
    assert np.allclose(p, want, rtol=2e-6, atol=0)
    # |g| >> eps: the move is lr*sign(g)
    big = np.abs(gd) > 1e-4
    assert np.allclose(p[big], -1e-3 * np.sign(gd[big]), rtol=2e-4)
    b1, b2 = 0.9, 0.999
    assert np.allclose(m, (1 - b1) * gd, rtol=2e-7, atol=0)
    assert np.allclose(v, (1 - b2) * gd * gd, rtol=3e-7, atol=1e-45)
    assert np.array_equal(p16, p.astype(np.float16).view(np.uint16))


def test_zero_grad_zero_state_is_a_fixed_point(orc):
    rng = np.random.default_rng(1)
    n = 257
    p0 = W.params_np(n, 3)
    p16 = rng.integers(0, 1000, n).astype(np.uint16)
    p, m, v = p0.copy(), np.zeros(n, F32), np.zeros(n, F32)
    for t in (1, 2, 50):
        orc.adam_chunk(np.zeros(n, np.uint16), p16, p, m, v, n,
                       orc.hyper(weight_decay=0.0, step=t, loss_scale=1024.0))
        assert p.tobytes() == p0.tobytes()
        assert not m.any() and not v.any()
    assert np.array_equal(p16, p0.astype(np.float16).view(np.uint16))


@pytest.mark.parametrize("gval", [1e-3, -1e-3, 0.25, -3.0])
def test_constant_grad_moves_lr_sign_g_every_step(orc, gval):
    # m_t=(1-b1^t)g, v_t=(1-b2^t)g^2 => bias-corrected ratio is g/|g| at every t
    n, T, lr = 4, 25, 1e-3
    g = f16([gval] * n)
    p16, p, m, v = state(n, 0.5)
    gd = float(np.float16(gval))
    b1, b2 = 0.9, 0.999
    for t in range(1, T + 1):
        orc.adam_chunk(g, p16, p, m, v, n, orc.hyper(lr=lr, weight_decay=0.0, step=t))
        assert np.allclose(p, 0.5 - t * lr * np.sign(gd), rtol=0, atol=t * lr * 3e-5 + 1e-7)
        assert np.allclose(m, (1 - b1 ** t) * gd, rtol=1e-5)
        assert np.allclose(v, (1 - b2 ** t) * gd * gd, rtol=1e-5)


# ---------------------------------------------------------------- fp64 textbook form

def kingma_fp64(g16_bits, p, m, v, lr, b1, b2, eps, wd, adamw, t, scale):
    g = g16_bits.view(np.float16).astype(np.float64) / scale
    p = p.astype(np.float64); m = m.astype(np.float64); v = v.astype(np.float64)
    if wd != 0 and not adamw:
        g = g + wd * p
    if wd != 0 and adamw:
        p = p * (1 - lr * wd)
    m = b1 * m + (1 - b1) * g
    v = b2 * v + (1 - b2) * g * g
    mhat = m / (1 - b1 ** t)
    vhat = v / (1 - b2 ** t)
    upd = lr * mhat / (np.sqrt(vhat) + eps)
    return p - upd, m, v, upd


@pytest.mark.parametrize("wd,adamw", [(0.0, 0), (0.01, 0), (0.01, 1), (0.1, 1)])
@pytest.mark.parametrize("scale", [1.0, 1024.0, 65536.0])
def test_against_fp64_textbook_form_per_step(orc, wd, adamw, scale):
    n = 10000
    lr, b1, b2, eps = 1e-3, 0.9, 0.999, 1e-8
    p = W.params_np(n, 21)
    m = np.zeros(n, F32); v = np.zeros(n, F32)
    p16 = np.zeros(n, np.uint16)
    for t in range(1, 13):
        g = W.grads_f16_np(n, 100 + t, scale)
        if t == 5:
            g[:100] = 0                       # exact zeros
        if t == 6:
            g[:64] = np.arange(1, 65)         # fp16 subnormal grads
        p_old = p.copy(); m_old = m.copy(); v_old = v.astype(np.float64)
        want_p, want_m, want_v, upd = kingma_fp64(g, p, m, v, float(lr), float(b1), float(b2),
                                                  float(eps), wd, adamw, t, scale)
        orc.adam_chunk(g, p16, p, m, v, n,
                       orc.hyper(lr=lr, beta1=b1, beta2=b2, eps=eps, weight_decay=wd,
                                 adamw_mode=adamw, step=t, loss_scale=scale))
        # beta1*m and (1-beta1)*g may cancel: the error floor is an ulp of the operands
        gmag = np.abs(g.view(np.float16).astype(np.float64)) / scale + wd * np.abs(p_old)
        assert np.all(np.abs(m - want_m) <= 2 * ulp32(np.maximum(np.abs(m_old), gmag)) + 1e-45)
        # g (rounded once) enters squared, then three more roundings: a few ulp against exact
        # (with L2 decay g + wd*p may cancel; its absolute error then enters through 2*g*dg)
        geff = np.sqrt(np.maximum(want_v - float(b2) * v_old, 0) / (1 - float(b2)))
        assert np.all(np.abs(v - want_v) <= 4 * ulp32(want_v) + 4e-3 * geff * ulp32(gmag) + 1e-45)
        # p: ulps of the operands, relative error of the update, and m's cancellation error
        # carried through lr/(1-b1^t)/(sqrt(vhat)+eps)
        gain = float(lr) / (1 - float(b1) ** t) / (np.sqrt(want_v / (1 - float(b2) ** t)) + float(eps))
        tol = (2 * ulp32(np.maximum(np.abs(p_old), np.abs(want_p))) + 2e-6 * np.abs(upd)
               + gain * 2 * ulp32(np.maximum(np.abs(m_old), gmag)))
        assert np.all(np.abs(p - want_p) <= tol)
        assert np.array_equal(p16, p.astype(np.float16).view(np.uint16))


# ---------------------------------------------------------------- library Adam / AdamW

@pytest.mark.parametrize("adamw", [0, 1])
def test_against_torch_optim(orc, adamw):
    import torch
    n, T, wd, scale = 4096, 8, 0.01, 1024.0
    p0 = W.params_np(n, 33)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    cls = torch.optim.AdamW if adamw else torch.optim.Adam
    opt = cls([tp], lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
    p = p0.copy(); m = np.zeros(n, F32); v = np.zeros(n, F32); p16 = np.zeros(n, np.uint16)
    for t in range(1, T + 1):
        g = W.grads_f16_np(n, 200 + t, scale)
        tp.grad = torch.from_numpy(g.view(np.float16).astype(np.float32) / np.float32(scale))
        opt.step()
        m_old = m.copy()
        orc.adam_chunk(g, p16, p, m, v, n,
                       orc.hyper(weight_decay=wd, adamw_mode=adamw, step=t, loss_scale=scale))
        st = opt.state[tp]
        # tolerances are relative to the operands: beta1*m + (1-beta1)*g and g + wd*p may cancel
        gmag = np.abs(tp.grad.numpy()) + wd * np.abs(p)
        assert np.all(np.abs(m - st["exp_avg"].numpy()) <= 1e-6 * np.maximum(np.abs(m_old), gmag))
        assert np.all(np.abs(v - st["exp_avg_sq"].numpy()) <= 1e-5 * v + 1e-9 * gmag * gmag)
        assert np.allclose(p, tp.detach().numpy(), rtol=0, atol=t * 5e-8)


# ---------------------------------------------------------------- unscale, skip, re-cast

def test_power_of_two_unscale_is_exact(orc):
    rng = np.random.default_rng(4)
    n = 4096
    base = (rng.standard_normal(n) * 1e-3).astype(np.float16)
    base = np.where(np.abs(base) < 6.2e-5, np.float16(1e-3), base)       # keep fp16-normal
    outs = []
    for scale in (1.0, 1024.0, 65536.0 / 64):
        g = (base.astype(np.float32) * F32(scale)).astype(np.float16)
        assert np.array_equal(g.astype(np.float32) / F32(scale), base.astype(np.float32))
        p = W.params_np(n, 8); m = np.zeros(n, F32); v = np.zeros(n, F32); p16 = np.zeros(n, np.uint16)
        for t in (1, 2):
            orc.adam_chunk(g.view(np.uint16).copy(), p16, p, m, v, n,
                           orc.hyper(weight_decay=0.01, step=t, loss_scale=scale))
        outs.append((p.tobytes(), m.tobytes(), v.tobytes(), p16.tobytes()))
    assert outs[0] == outs[1] == outs[2]


@pytest.mark.parametrize("alias", [False, True])
def test_overflow_step_leaves_state_bit_identical(orc, alias):
    n_chunks, C = 3, 512
    used = np.array([512, 300, 77], np.uint64)
    for special in W.specials_f16():
        for (c, k) in [(0, 0), (1, 299), (2, 76), (0, 511)]:
            p = [W.params_np(C, 40 + i) for i in range(n_chunks)]
            m = [np.abs(W.params_np(C, 50 + i)) for i in range(n_chunks)]
            v = [np.abs(W.params_np(C, 60 + i)) for i in range(n_chunks)]
            g = [W.grads_f16_np(C, 70 + i, 1024.0) for i in range(n_chunks)]
            g[c][k] = special
            p16 = g if alias else [np.full(C, 0x1234, np.uint16) for _ in range(n_chunks)]
            snap = [x.copy() for x in p + m + v]
            flag = orc.chunk_adam_step(g, p16, p, m, v, used, orc.hyper(step=3, loss_scale=1024.0))
            assert flag == 1
            for a, b in zip(p + m + v, snap):
                assert a.tobytes() == b.tobytes()
            for i in range(n_chunks):
                u = int(used[i])
                if alias:      # grads were sitting in the param fp16 chunk: params restored
                    assert np.array_equal(p16[i][:u], p[i][:u].astype(np.float16).view(np.uint16))
                else:
                    assert np.all(p16[i] == 0x1234)


def test_special_in_padding_does_not_skip(orc):
    C = 64
    used = np.array([40], np.uint64)
    g = [W.grads_f16_np(C, 1, 1024.0)]
    g[0][40] = 0x7C00
    g[0][63] = 0x7E00
    p = [W.params_np(C, 2)]; m = [np.zeros(C, F32)]; v = [np.zeros(C, F32)]
    p16 = [np.zeros(C, np.uint16)]
    p0 = p[0].copy()
    flag = orc.chunk_adam_step(g, p16, p, m, v, used, orc.hyper(step=1, loss_scale=1024.0))
    assert flag == 0
    assert np.all(p[0][:40] != p0[:40])
    assert p[0][40:].tobytes() == p0[40:].tobytes()            # padding never written
    assert not m[0][40:].any() and not v[0][40:].any() and not p16[0][40:].any()


def test_recast_is_rne_of_fp32_params(orc):
    p = np.concatenate([W.params_np(5000, 9), F32([0, -0.0, 65504, 65520, 1e-8, -1e-8, 6e-8, 1e5])])
    p16 = np.zeros(p.size, np.uint16)
    orc.recast_chunk(p16, p.astype(F32), p.size)
    with np.errstate(over="ignore"):
        assert np.array_equal(p16, p.astype(F32).astype(np.float16).view(np.uint16))


# ---------------------------------------------------------------- scalars

def test_step_scalars(orc):
    for t in (1, 2, 10, 1000, 100000):
        h = orc.hyper(lr=1e-3, beta1=0.9, beta2=0.999, weight_decay=0.01, step=t, loss_scale=65536.0)
        s = orc.adam_prepare(h)
        b1, b2, lr = 0.9, 0.999, 1e-3
        assert s.step_size == pytest.approx(lr / (1 - b1 ** t), rel=2e-7)
        assert s.c2 == pytest.approx((1 - b2 ** t) ** -0.5, rel=2e-7)
        assert s.inv_scale == 2.0 ** -16
        assert s.omb1 == pytest.approx(1 - b1, rel=1e-7) and s.omb2 == pytest.approx(1 - b2, rel=1e-7)
        assert s.decay == pytest.approx(1 - lr * 0.01, rel=1e-7)


# ---------------------------------------------------------------- the whole loop against library mixed-precision training

def test_skip_and_loss_scale_against_library_amp(orc):
    """Overflow test, skipped update, unscaling, Adam and the loss-scale schedule together, against PyTorch's own
    mixed-precision loop on the CPU (torch.amp.GradScaler around torch.optim.Adam): after every step the scale,
    the run of good steps and the optimizer's step count must be the library's, and the parameters its
    parameters.  (The library has no floor at 1; the scale stays far above it here.)"""
    import torch
    n, gi = 64, 3
    coeff = (np.arange(n) % 13 - 6).astype(np.float32) / np.float32(1024.0)       # exact in fp16 at every scale used
    p0 = W.params_np(n, 71)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.Adam([tp], lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.0)
    amp = torch.amp.GradScaler("cpu", init_scale=1024.0, growth_factor=2.0, backoff_factor=0.5, growth_interval=gi)
    s = orc.scaler(1024.0, gi)
    g16 = [np.zeros(n, np.uint16)]
    p16, p, m, v = [np.zeros(n, np.uint16)], [p0.copy()], [np.zeros(n, F32)], [np.zeros(n, F32)]
    used = np.array([n], np.uint64)
    bad_steps = {4, 5, 11, 20, 21, 22}
    seen = set()
    for it in range(30):
        c = coeff * np.float32(1 + it % 3)
        ct = torch.from_numpy(c.copy())
        if it in bad_steps:
            ct[it % n] = float("inf") if it % 2 else float("nan")
        opt.zero_grad()
        amp.scale((tp * ct).sum()).backward()
        amp.step(opt)
        amp.update()
        with np.errstate(over="ignore", invalid="ignore"):
            g16[0][:] = (ct.numpy() * np.float32(s.scale)).astype(np.float16).view(np.uint16)
        flag = orc.chunk_adam_step(g16, p16, p, m, v, used, orc.hyper(weight_decay=0.0, step=s.step, loss_scale=s.scale))
        orc.scaler_update(s, flag)
        assert flag == int(it in bad_steps)
        assert s.scale == amp.get_scale() and s.good_steps == int(amp._growth_tracker.item())
        assert s.step - 1 == (int(opt.state[tp]["step"]) if tp in opt.state else 0)
        assert np.allclose(p[0], tp.detach().numpy(), rtol=0, atol=(it + 1) * 5e-8)
        seen.add(s.scale)
    assert len(seen) >= 3 and s.step == 31 - len(bad_steps)       # the scale both grew and shrank on the way


# ---------------------------------------------------------------- loss-scale convention (unpinned by the paper)

def test_scaler_halves_floors_and_grows(orc):
    s = orc.scaler(scale=4.0, growth_interval=3)
    orc.scaler_update(s, 1)
    assert (s.scale, s.good_steps, s.step) == (2.0, 0, 1)          # t not advanced on a skipped step
    orc.scaler_update(s, 1); orc.scaler_update(s, 1); orc.scaler_update(s, 1)
    assert s.scale == 1.0                                          # floor
    for k in range(1, 3):
        orc.scaler_update(s, 0)
        assert (s.scale, s.good_steps, s.step) == (1.0, k, 1 + k)
    orc.scaler_update(s, 0)
    assert (s.scale, s.good_steps, s.step) == (2.0, 0, 4)          # doubled after 3 good steps
    orc.scaler_update(s, 0); orc.scaler_update(s, 1)
    assert (s.scale, s.good_steps, s.step) == (1.0, 0, 5)          # an overflow resets the run
