"""Pins of oracle/optim.py: closed forms of AdamW's first step, a hand-run second step, torch.optim.AdamW, and
the straggling-rate rule on a trace that mirrors the paper's straggler situations.  CPU only."""
import numpy as np
import pytest

from oracle import optim as oo


def test_first_step_is_lr_times_sign_when_eps_and_decay_vanish():
    """t = 1: mhat = g, vhat = g^2, so the update is lr * g/|g| whatever the betas."""
    g = np.array([3.0, -0.25, 1e-3, -7.0])
    w, m, v = oo.adamw_step(np.zeros(4), np.zeros(4), np.zeros(4), g, 1, 0.1, 0.9, 0.999, 0.0, 0.0)
    assert np.allclose(w, -0.1 * np.sign(g), rtol=1e-15)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_zero_gradient_only_decays_the_weights():
    w0 = np.array([2.0, -4.0])
    w, m, v = oo.adamw_step(w0, np.zeros(2), np.zeros(2), np.zeros(2), 1, 0.5, 0.9, 0.999, 1e-8, 0.1)
    assert np.allclose(w, w0 * (1 - 0.5 * 0.1)) and not m.any() and not v.any()


def test_second_step_by_hand():
    """g = 1 then g = -1 with b1 = 0.5, b2 = 0.75, eps = 0, no decay, lr = 1:
    m1 = .5, v1 = .25, w1 = -1;  m2 = .25 - .5 = -.25, v2 = .1875 + .25 = .4375, mhat = -.25/.75, vhat = .4375/.4375 = 1
    -> w2 = -1 + 1/3."""
    w, m, v = oo.adamw_step(np.zeros(1), np.zeros(1), np.zeros(1), np.ones(1), 1, 1.0, 0.5, 0.75, 0.0, 0.0)
    w, m, v = oo.adamw_step(w, m, v, -np.ones(1), 2, 1.0, 0.5, 0.75, 0.0, 0.0)
    assert w[0] == pytest.approx(-1.0 + 1.0 / 3.0, rel=1e-15) and m[0] == -0.25 and v[0] == 0.4375


def test_matches_torch_adamw_over_several_steps():
    import torch
    rng = np.random.default_rng(0)
    w0 = rng.standard_normal(50)
    p = torch.nn.Parameter(torch.tensor(w0))
    opt = torch.optim.AdamW([p], lr=3e-2, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    w, m, v = w0.copy(), np.zeros(50), np.zeros(50)
    for t in range(1, 6):
        g = rng.standard_normal(50) * 10.0 ** rng.integers(-3, 2)
        p.grad = torch.tensor(g)
        opt.step()
        w, m, v = oo.adamw_step(w, m, v, g, t, 3e-2, 0.9, 0.95, 1e-8, 0.1)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_straggling_rate_rule():
    """Reference 5 ms per unit.  Steps: normal, normal, a level-1 straggler appears (x = 2.62 as in Table 4's 32B case),
    stays, drifts by 4 % (no shift), disappears."""
    tau = 5.0
    units = [16, 16, 16, 16, 8, 16]
    x = [1.0, 1.02, 2.62, 2.62, 2.62 * 1.04, 1.0]
    elapsed = [xi * tau * u for xi, u in zip(x, units)]
    rates, shifts = oo.straggling_rates(elapsed, units, tau, 0.05)
    assert np.allclose(rates, x, rtol=1e-14)
    assert shifts == [False, False, True, False, False, True]


def test_library_probe_replay_matches_the_rule():
    """mls_probe_feed is host code: the same trace through the library (no GPU needed)."""
    import paper_2410_13333_amd as mls
    tau = 5.0
    units = [(4, 4), (4, 4), (2, 8), (4, 4), (8, 1), (4, 4)]
    x = [1.0, 1.02, 2.62, 2.62, 2.62 * 1.04, 1.0]
    elapsed = [xi * tau * l * m for xi, (l, m) in zip(x, units)]
    want_r, want_s = oo.straggling_rates(elapsed, [l * m for l, m in units], tau, 0.05)
    pr = mls.Probe(tau, 0.05)
    for e, (l, m), r, s in zip(elapsed, units, want_r, want_s):
        got_r, got_s = pr.feed(e, l, m)
        assert got_r == pytest.approx(r, rel=1e-14) and got_s == s
    with pytest.raises(mls.MlsError):
        pr.feed(1.0, 0, 4)
    pr.close()
    with pytest.raises(mls.MlsError):
        mls.Probe(0.0)
