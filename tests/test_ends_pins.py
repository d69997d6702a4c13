"""Pins of the first/last-stage oracle (oracle/ends.py) against what the mathematics and a library routine fix:
closed forms, invariants, finite differences, the adjoint identity, torch's cross-entropy and autograd.  CPU only."""
import numpy as np
import pytest

import synth
from oracle import ends as oe

SH = synth.EndsShape(hidden=24, vocab=40, seq=7, micro_batch=2, microbatches=1, dtype="fp32")


def _setup(seed=5, sh=SH):
    _, flat = synth.make_ends_params(sh, seed)
    p = synth.split_ends_params(sh, flat)
    rng = np.random.default_rng(seed)
    y = rng.standard_normal((sh.tokens, sh.hidden))
    tgt = synth.make_targets(sh, seed + 1, 0)
    return p, y, tgt


def test_zero_head_gives_log_vocab():
    """All logits equal -> every token's loss is log V."""
    p, y, tgt = _setup()
    p = dict(p, w_lm=np.zeros_like(p["w_lm"]))
    loss, _ = oe.head_forward(y, tgt, p, 1e-5)
    assert loss == pytest.approx(np.log(SH.vocab), rel=1e-14)


def test_confident_correct_prediction_has_vanishing_loss_and_wrong_one_the_margin():
    """One logit far above the rest: loss ~ 0 when it is the target, ~ the margin when it is not."""
    h, V = 4, 6
    p = dict(gamma_f=np.ones(h), w_lm=np.zeros((h, V)))
    p["w_lm"][0, 2] = 50.0
    y = np.tile(np.array([[1.0, 0, 0, 0]]), (3, 1))          # nrm = y * 2 (rms = 1/2) -> logit 100 for class 2
    assert oe.head_forward(y, np.array([2, 2, 2]), p, 0.0)[0] == pytest.approx(0.0, abs=1e-30)
    assert oe.head_forward(y, np.array([1, 1, 1]), p, 0.0)[0] == pytest.approx(100.0, rel=1e-12)


def test_loss_matches_torch_cross_entropy_and_ignored_targets():
    import torch
    p, y, tgt = _setup()
    tgt = tgt.copy().reshape(-1)
    tgt[3] = -100                      # ignored
    tgt[5] = SH.vocab + 7              # out of range: ignored as well
    loss, c = oe.head_forward(y, tgt, p, 1e-5)
    t_tgt = torch.tensor(np.where((tgt >= 0) & (tgt < SH.vocab), tgt, -100), dtype=torch.long)
    ref = torch.nn.functional.cross_entropy(torch.tensor(c["logits"]), t_tgt, ignore_index=-100, reduction="sum")
    assert loss == pytest.approx(float(ref) / tgt.size, rel=1e-13)


def test_head_backward_matches_torch_autograd():
    import torch
    p, y, tgt = _setup()
    tgt = tgt.reshape(-1).copy()
    tgt[2] = -1
    w = 0.25
    loss, c = oe.head_forward(y, tgt, p, 1e-5)
    dy, g, _ = oe.head_backward(c, p, w)
    ty = torch.tensor(y, requires_grad=True)
    tg = torch.tensor(p["gamma_f"], requires_grad=True)
    tw = torch.tensor(p["w_lm"], requires_grad=True)
    nrm = ty * torch.rsqrt((ty * ty).mean(-1, keepdim=True) + 1e-5) * tg
    t_tgt = torch.tensor(np.where(tgt >= 0, tgt, -100), dtype=torch.long)
    tl = torch.nn.functional.cross_entropy(nrm @ tw, t_tgt, ignore_index=-100, reduction="sum") / tgt.size
    (w * tl).backward()
    assert np.allclose(dy, ty.grad.numpy(), rtol=1e-11, atol=1e-15)
    assert np.allclose(g["w_lm"], tw.grad.numpy(), rtol=1e-11, atol=1e-15)
    assert np.allclose(g["gamma_f"], tg.grad.numpy(), rtol=1e-11, atol=1e-15)


def test_head_backward_finite_differences():
    p, y, tgt = _setup(seed=9)
    w = 1.0
    loss, c = oe.head_forward(y, tgt, p, 1e-5)
    dy, g, _ = oe.head_backward(c, p, w)
    rng = np.random.default_rng(0)
    for name, arr, grad in (("y", y, dy), ("w_lm", p["w_lm"], g["w_lm"]), ("gamma_f", p["gamma_f"], g["gamma_f"])):
        d = rng.standard_normal(arr.shape)
        eps = 1e-6
        def f(a):
            q = dict(p)
            yy = y
            if name == "y":
                yy = a
            else:
                q[name] = a
            return oe.head_forward(yy, tgt, q, 1e-5)[0]
        fd = (f(arr + eps * d) - f(arr - eps * d)) / (2 * eps)
        assert fd == pytest.approx(float(np.sum(grad * d)), rel=1e-6), name


def test_logit_gradient_rows_sum_to_zero_and_scale_with_the_weight():
    p, y, tgt = _setup()
    tgt = tgt.reshape(-1).copy()
    tgt[0] = -5
    _, c = oe.head_forward(y, tgt, p, 1e-5)
    _, _, d1 = oe.head_backward(c, p, 1.0)
    _, _, d2 = oe.head_backward(c, p, 0.125)
    assert np.allclose(d1.sum(axis=1), 0.0, atol=1e-16)
    assert np.all(d1[0] == 0.0)                              # ignored token: no gradient
    assert np.allclose(d2, 0.125 * d1, rtol=1e-15)
    # every entry but the target's is positive, the target's is negative
    rows = np.arange(1, tgt.size)
    assert np.all(d1[rows, tgt[1:]] < 0) and np.all(np.delete(d1[1], tgt[1]) > 0)


def test_embedding_gather_adjoint_and_duplicates():
    sh = SH
    _, flat = synth.make_ends_params(sh, 3)
    E = synth.split_ends_params(sh, flat)["embed"]
    tok = np.array([3, 3, 39, 0, 3, -1, 40, 17, 0, 5, 5, 5, 5, 12], dtype=np.int32)
    x = oe.embed_forward(tok, E)
    assert np.array_equal(x[0], E[3]) and np.array_equal(x[2], E[39]) and np.all(x[5] == 0) and np.all(x[6] == 0)
    rng = np.random.default_rng(1)
    dx = rng.standard_normal(x.shape)
    g = oe.embed_backward(tok, dx, sh.vocab)
    # adjoint identity <gather(E), dx> = <E, scatter(dx)>
    assert float(np.sum(x * dx)) == pytest.approx(float(np.sum(E * g)), rel=1e-13)
    assert np.allclose(g[3], dx[0] + dx[1] + dx[4]) and np.allclose(g[5], dx[9:13].sum(axis=0))
    assert np.all(g[1] == 0) and np.count_nonzero(np.abs(g).sum(axis=1)) == 6


def test_store_hook_identity_changes_nothing_and_rounding_is_small():
    p, y, tgt = _setup()
    a = oe.head_forward(y, tgt, p, 1e-5)
    b = oe.head_forward(y, tgt, p, 1e-5, store=lambda name, v: v)
    assert a[0] == b[0]
    from tests.helpers import bf16_store
    c = oe.head_forward(y, tgt, p, 1e-5, store=bf16_store)
    assert abs(c[0] - a[0]) / a[0] < 1e-2


def test_generated_tokens_are_in_range_and_reproducible():
    sh = synth.ENDS_CONFIGS["tiny"]
    t0, t1 = synth.make_tokens(sh, 2100, 0), synth.make_tokens(sh, 2100, 1)
    assert t0.shape == (sh.micro_batch, sh.seq) and t0.dtype == np.int32
    assert t0.min() >= 0 and t0.max() < sh.vocab and not np.array_equal(t0, t1)
    assert np.array_equal(t0, synth.make_tokens(sh, 2100, 0))
    sk = synth.make_tokens(sh, 2100, 0, skew=True)
    assert sk.max() < sh.vocab // 64 + 1 and len(np.unique(sk)) < sk.size / 4
