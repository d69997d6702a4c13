"""Pins of the CPU oracle against what mathematics fixes (no GPU, no HIP code).

The paper prints no worked numeric example of the decoder layer, so every pin here is a closed form, an
invariant, a special case that reduces to a library routine, brute force on tiny inputs, or finite
differences."""
import math

import numpy as np
import pytest

import synth
from oracle import stage as O

TINY = synth.StageShape(hidden=16, n_q_heads=4, n_kv_heads=2, head_dim=4, ffn=24, seq=6, micro_batch=2,
                        layers=2, microbatches=2, dtype="fp32")


def _weights(sh, seed, scale=0.3):
    """fp64 weights with a larger spread than the workload's 0.02 so every term matters in the pins."""
    rng = np.random.default_rng(seed)
    ws = []
    for _ in range(sh.layers):
        ws.append(dict(
            gamma1=1.0 + 0.2 * rng.standard_normal(sh.hidden),
            w_qkv=scale * rng.standard_normal((sh.hidden, sh.q_dim + 2 * sh.kv_dim)),
            w_o=scale * rng.standard_normal((sh.q_dim, sh.hidden)),
            gamma2=1.0 + 0.2 * rng.standard_normal(sh.hidden),
            w_gu=scale * rng.standard_normal((sh.hidden, 2 * sh.ffn)),
            w_d=scale * rng.standard_normal((sh.ffn, sh.hidden))))
    return ws


def _xdy(sh, seed):
    rng = np.random.default_rng(seed)
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    return rng.standard_normal(shape), rng.standard_normal(shape)

# ------------------------------------------------------------------ finite differences (whole stage)


def test_finite_differences_every_parameter_and_dx():
    sh = TINY
    W = _weights(sh, 1)
    x, dy = _xdy(sh, 2)
    y, caches = O.stage_forward(x, W, sh)
    dx, grads = O.stage_backward(dy, W, caches, sh)
    loss = lambda xx, ww: float(np.sum(O.stage_forward(xx, ww, sh)[0] * dy))
    eps = 1e-5
    rng = np.random.default_rng(3)
    # dX: every element
    num = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        num[idx] = (loss(xp, W) - loss(xm, W)) / (2 * eps)
    assert np.linalg.norm(num - dx) / np.linalg.norm(dx) < 1e-6
    # every parameter tensor of every layer: 40 random elements each (all of the gains)
    for l in range(sh.layers):
        for name, g in grads[l].items():
            flat = W[l][name].reshape(-1)
            picks = np.arange(flat.size) if flat.size <= 40 else rng.choice(flat.size, 40, replace=False)
            num = np.empty(len(picks))
            for n, i in enumerate(picks):
                old = flat[i]
                flat[i] = old + eps
                lp = loss(x, W)
                flat[i] = old - eps
                lm = loss(x, W)
                flat[i] = old
                num[n] = (lp - lm) / (2 * eps)
            ref = g.reshape(-1)[picks]
            assert np.linalg.norm(num - ref) / np.linalg.norm(ref) < 1e-6, (l, name)


def test_adjoint_identity_random_directions():
    """<dY, J v> = <J^T dY, v> for input and weight directions (J v by central differences)."""
    sh = TINY
    W = _weights(sh, 4)
    x, dy = _xdy(sh, 5)
    rng = np.random.default_rng(6)
    _, caches = O.stage_forward(x, W, sh)
    dx, grads = O.stage_backward(dy, W, caches, sh)
    e = 1e-6
    v = rng.standard_normal(x.shape)
    jv = (O.stage_forward(x + e * v, W, sh)[0] - O.stage_forward(x - e * v, W, sh)[0]) / (2 * e)
    assert abs(np.sum(dy * jv) - np.sum(dx * v)) / abs(np.sum(dx * v)) < 1e-7
    V = [{n: rng.standard_normal(a.shape) for n, a in w.items()} for w in W]
    Wp = [{n: a + e * V[l][n] for n, a in w.items()} for l, w in enumerate(W)]
    Wm = [{n: a - e * V[l][n] for n, a in w.items()} for l, w in enumerate(W)]
    jv = (O.stage_forward(x, Wp, sh)[0] - O.stage_forward(x, Wm, sh)[0]) / (2 * e)
    rhs = sum(np.sum(grads[l][n] * V[l][n]) for l in range(sh.layers) for n in V[l])
    assert abs(np.sum(dy * jv) - rhs) / abs(rhs) < 1e-7

# ------------------------------------------------------------------ softmax / causality


def test_softmax_rows_sum_to_one_and_mask_is_exact():
    rng = np.random.default_rng(7)
    q, k, v = rng.standard_normal((2, 9, 4, 8)), rng.standard_normal((2, 9, 2, 8)), rng.standard_normal((2, 9, 2, 8))
    _, p = O.attention_fwd(3 * q, 3 * k, v)
    assert np.all(p >= 0)
    assert np.max(np.abs(p.sum(-1) - 1)) < 1e-12
    iu = np.triu_indices(9, 1)
    assert np.all(p[:, :, iu[0], iu[1]] == 0.0)


def test_causality_forward_and_backward():
    sh = TINY
    W = _weights(sh, 8)
    x, dy = _xdy(sh, 9)
    t0 = 3
    y0, c0 = O.stage_forward(x, W, sh)
    x2 = x.copy()
    x2[:, t0 + 1:, :] += np.random.default_rng(10).standard_normal(x2[:, t0 + 1:, :].shape)
    y2, _ = O.stage_forward(x2, W, sh)
    assert np.array_equal(y0[:, :t0 + 1], y2[:, :t0 + 1])          # bit for bit
    assert not np.allclose(y0[:, t0 + 1:], y2[:, t0 + 1:])
    # batch rows never see each other
    x3 = x.copy()
    x3[1] += 1.0
    assert np.array_equal(O.stage_forward(x3, W, sh)[0][0], y0[0])
    # dX[t] depends on dY[>= t] only
    dx0, _ = O.stage_backward(dy, W, c0, sh)
    dy2 = dy.copy()
    dy2[:, :t0, :] += 1.0
    dx2, _ = O.stage_backward(dy2, W, c0, sh)
    assert np.allclose(dx0[:, t0:], dx2[:, t0:], rtol=0, atol=1e-12)
    assert not np.allclose(dx0[:, :t0], dx2[:, :t0])

# ------------------------------------------------------------------ RoPE


def test_rope_is_a_rotation_with_relative_position_property():
    rng = np.random.default_rng(11)
    S, d = 12, 8
    ang = O.rope_angles(S, d, 10000.0)
    # angles: closed form
    assert ang[0].tolist() == [0.0] * (d // 2)
    assert math.isclose(ang[5, 1], 5 * 10000.0 ** (-2.0 / d), rel_tol=1e-15)
    assert math.isclose(ang[7, 3], 7 * 10000.0 ** (-6.0 / d), rel_tol=1e-15)
    u = rng.standard_normal((2, S, 3, d))
    r = O.rope_apply(u, ang)
    assert np.max(np.abs(np.linalg.norm(r, axis=-1) - np.linalg.norm(u, axis=-1))) < 1e-12
    assert np.array_equal(r[:, 0], u[:, 0])                                      # position 0: identity
    # complex-number formulation: (u_i + j u_{i+d/2}) * exp(j p theta_i)
    z = (u[..., :d // 2] + 1j * u[..., d // 2:]) * np.exp(1j * ang)[None, :, None, :]
    assert np.allclose(r, np.concatenate([z.real, z.imag], -1), rtol=0, atol=1e-13)
    # <R_m q, R_n k> depends on m - n only
    qv, kv = rng.standard_normal(d), rng.standard_normal(d)
    tile = lambda w: np.broadcast_to(w, (1, S, 1, d)).copy()
    rq, rk = O.rope_apply(tile(qv), ang)[0, :, 0], O.rope_apply(tile(kv), ang)[0, :, 0]
    assert abs(rq[7] @ rk[4] - rq[10] @ rk[7]) < 1e-12
    assert abs(rq[3] @ rk[3] - qv @ kv) < 1e-12
    # backward = rotation by the negated angle = inverse = transpose
    assert np.allclose(O.rope_apply(r, ang, sign=-1.0), u, rtol=0, atol=1e-13)
    w = rng.standard_normal(u.shape)
    assert abs(np.sum(O.rope_apply(u, ang) * w) - np.sum(u * O.rope_apply(w, ang, sign=-1.0))) < 1e-10

# ------------------------------------------------------------------ RMSNorm


def test_rmsnorm_closed_forms():
    rng = np.random.default_rng(12)
    h, eps = 32, 1e-5
    gamma = 1 + 0.1 * rng.standard_normal(h)
    c = 1.7
    a, r = O.rmsnorm_fwd(np.full((3, h), c), gamma, eps)
    assert np.allclose(a, gamma * c / math.sqrt(c * c + eps), rtol=1e-15)
    x = rng.standard_normal((5, h))
    a, r = O.rmsnorm_fwd(x, np.ones(h), 0.0)
    assert np.allclose(np.mean(a * a, -1), 1.0, rtol=1e-14)
    a2, _ = O.rmsnorm_fwd(1000.0 * x, np.ones(h), 0.0)
    assert np.allclose(a, a2, rtol=1e-13)
    # one hand-computed row: x = (3,4), gamma = (2,5), eps = 0 -> rms = sqrt(12.5)
    a, r = O.rmsnorm_fwd(np.array([[3.0, 4.0]]), np.array([2.0, 5.0]), 0.0)
    assert np.allclose(a, [[6 / math.sqrt(12.5), 20 / math.sqrt(12.5)]], rtol=1e-15)
    # backward: dx is orthogonal to x when eps = 0; finite differences with eps > 0
    da = rng.standard_normal((5, h))
    _, r0 = O.rmsnorm_fwd(x, gamma, 0.0)
    dx, dg = O.rmsnorm_bwd(da, x, gamma, r0)
    assert np.max(np.abs(np.sum(dx * x, -1))) < 1e-12
    _, r = O.rmsnorm_fwd(x, gamma, eps)
    dx, dg = O.rmsnorm_bwd(da, x, gamma, r)
    f = lambda xx, gg: np.sum(O.rmsnorm_fwd(xx, gg, eps)[0] * da)
    e = 1e-6
    for idx in [(0, 0), (2, 7), (4, 31)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += e
        xm[idx] -= e
        assert abs((f(xp, gamma) - f(xm, gamma)) / (2 * e) - dx[idx]) < 1e-8
    for i in [0, 13]:
        gp, gm = gamma.copy(), gamma.copy()
        gp[i] += e
        gm[i] -= e
        assert abs((f(x, gp) - f(x, gm)) / (2 * e) - dg[i]) < 1e-8

# ------------------------------------------------------------------ attention special cases / brute force


def test_attention_special_cases():
    rng = np.random.default_rng(13)
    # S = 1: O = V of the group's KV head
    q, k, v = rng.standard_normal((2, 1, 4, 8)), rng.standard_normal((2, 1, 2, 8)), rng.standard_normal((2, 1, 2, 8))
    o, _ = O.attention_fwd(q, k, v)
    assert np.allclose(o[:, :, 0], v[:, :, 0]) and np.allclose(o[:, :, 1], v[:, :, 0])
    assert np.allclose(o[:, :, 2], v[:, :, 1]) and np.allclose(o[:, :, 3], v[:, :, 1])
    # all keys equal: O_i = mean of V_{<= i}
    S = 7
    q, v = rng.standard_normal((1, S, 2, 4)), rng.standard_normal((1, S, 2, 4))
    k = np.broadcast_to(rng.standard_normal((1, 1, 2, 4)), (1, S, 2, 4)).copy()
    o, _ = O.attention_fwd(q, k, v)
    run = np.cumsum(v, axis=1) / np.arange(1, S + 1)[None, :, None, None]
    assert np.allclose(o, run, rtol=0, atol=1e-13)


def test_attention_brute_force_scalar_loops_gqa():
    rng = np.random.default_rng(14)
    b, S, nq, nkv, d = 2, 5, 4, 2, 3
    q, k, v = rng.standard_normal((b, S, nq, d)), rng.standard_normal((b, S, nkv, d)), rng.standard_normal((b, S, nkv, d))
    o, _ = O.attention_fwd(q, k, v)
    for bi in range(b):
        for hq in range(nq):
            hk = hq // (nq // nkv)
            for i in range(S):
                sc = [sum(q[bi, i, hq, c] * k[bi, j, hk, c] for c in range(d)) / math.sqrt(d) for j in range(i + 1)]
                den = sum(math.exp(s) for s in sc)
                for c in range(d):
                    ref = sum(math.exp(sc[j]) / den * v[bi, j, hk, c] for j in range(i + 1))
                    assert abs(ref - o[bi, i, hq, c]) < 1e-12


def test_attention_backward_finite_differences_gqa():
    rng = np.random.default_rng(15)
    b, S, nq, nkv, d = 1, 6, 4, 2, 4
    q, k, v = rng.standard_normal((b, S, nq, d)), rng.standard_normal((b, S, nkv, d)), rng.standard_normal((b, S, nkv, d))
    do = rng.standard_normal((b, S, nq, d))
    o, p = O.attention_fwd(q, k, v)
    dq, dk, dv = O.attention_bwd(do, q, k, v, p)
    f = lambda qq, kk, vv: np.sum(O.attention_fwd(qq, kk, vv)[0] * do)
    e = 1e-6
    for arr, grad, pos in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(*arr.shape):
            args = [q, k, v]
            ap, am = arr.copy(), arr.copy()
            ap[idx] += e
            am[idx] -= e
            args[pos] = ap
            fp = f(*args)
            args[pos] = am
            num[idx] = (fp - f(*args)) / (2 * e)
        assert np.linalg.norm(num - grad) / np.linalg.norm(grad) < 1e-7

# ------------------------------------------------------------------ SwiGLU


def test_swiglu_values_and_derivative():
    assert O.swiglu_fwd(np.array([0.0]), np.array([3.0]))[0] == 0.0
    dg, du = O.swiglu_bwd(np.array([1.0]), np.array([0.0]), np.array([3.0]))
    assert dg[0] == 1.5 and du[0] == 0.0                       # silu'(0) = 1/2
    assert math.isclose(O.swiglu_fwd(np.array([2.0]), np.array([-1.5]))[0], -1.5 * 2.0 / (1 + math.exp(-2.0)), rel_tol=1e-15)
    rng = np.random.default_rng(16)
    g, u, dz = rng.standard_normal(50) * 3, rng.standard_normal(50), rng.standard_normal(50)
    dg, du = O.swiglu_bwd(dz, g, u)
    e = 1e-6
    assert np.allclose((O.swiglu_fwd(g + e, u) - O.swiglu_fwd(g - e, u)) / (2 * e) * dz, dg, atol=1e-8)
    assert np.allclose((O.swiglu_fwd(g, u + e) - O.swiglu_fwd(g, u - e)) / (2 * e) * dz, du, atol=1e-8)

# ------------------------------------------------------------------ layer / stage structure


def test_zero_output_projections_make_the_layer_an_identity():
    sh = TINY
    W = _weights(sh, 17)
    for w in W:
        w["w_o"][:] = 0
        w["w_d"][:] = 0
    x, dy = _xdy(sh, 18)
    y, caches = O.stage_forward(x, W, sh)
    dx, grads = O.stage_backward(dy, W, caches, sh)
    assert np.array_equal(y, x) and np.array_equal(dx, dy)
    for g in grads:
        for n in ("gamma1", "w_qkv", "gamma2", "w_gu"):
            assert not g[n].any()
        assert g["w_o"].any() and g["w_d"].any()


def test_zero_layers_is_identity():
    sh = TINY
    x, dy = _xdy(sh, 19)
    y, caches = O.stage_forward(x, _weights(sh, 20), sh, k_layers=0)
    assert np.array_equal(y, x) and caches == []
    dx, grads = O.stage_backward(dy, [], caches, sh)
    assert np.array_equal(dx, dy) and grads == []


def test_composition_of_stages():
    sh = TINY.with_(layers=3)
    W = _weights(sh, 21)
    x, dy = _xdy(sh, 22)
    y, c = O.stage_forward(x, W, sh)
    y1, c1 = O.stage_forward(x, W[:1], sh)
    y2, c2 = O.stage_forward(y1, W[1:], sh)
    assert np.array_equal(y, y2)
    dx, g = O.stage_backward(dy, W, c, sh)
    dmid, g2 = O.stage_backward(dy, W[1:], c2, sh)
    dx1, g1 = O.stage_backward(dmid, W[:1], c1, sh)
    assert np.array_equal(dx, dx1)
    assert np.array_equal(g[0]["w_gu"], g1[0]["w_gu"]) and np.array_equal(g[2]["w_d"], g2[1]["w_d"])


def test_gradient_accumulation_is_a_sum_over_microbatches():
    sh = TINY
    W = _weights(sh, 23)
    xs, dys = zip(*[_xdy(sh, 30 + i) for i in range(3)])
    _, _, tot = O.stage_step(list(xs), list(dys), W, sh)
    singles = [O.stage_step([x], [dy], W, sh)[2] for x, dy in zip(xs, dys)]
    for l in range(sh.layers):
        for n in tot[l]:
            s = singles[0][l][n] + singles[1][l][n] + singles[2][l][n]
            assert np.allclose(tot[l][n], s, rtol=1e-13, atol=1e-13)
    _, _, rep = O.stage_step([xs[0]] * 4, [dys[0]] * 4, W, sh)
    assert np.allclose(rep[1]["w_qkv"], 4 * singles[0][1]["w_qkv"], rtol=1e-13)
    _, _, rev = O.stage_step(list(xs)[::-1], list(dys)[::-1], W, sh)
    assert np.allclose(rev[0]["w_d"], tot[0]["w_d"], rtol=1e-12, atol=1e-12)

# ------------------------------------------------------------------ library cross-check (independent autodiff)


def test_layer_against_library_routines_and_autograd():
    """The same layer assembled from a CPU tensor library's own routines (rms_norm, fused causal
    attention, silu) and differentiated by its autograd engine; RoPE in its complex-number form."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    sh = TINY.with_(layers=1)
    W = _weights(sh, 40)[0]
    x, dy = _xdy(sh, 41)
    b, S, h = x.shape
    nq, nkv, d, f = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.ffn
    tw = {n: torch.tensor(a, dtype=torch.float64, requires_grad=True) for n, a in W.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    a = F.rms_norm(tx, (h,), tw["gamma1"], sh.rms_eps)
    qkv = a @ tw["w_qkv"]
    q, k, v = qkv.split([nq * d, nkv * d, nkv * d], dim=-1)
    inv = sh.rope_base ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    rot = torch.polar(torch.ones(S, d // 2, dtype=torch.float64), torch.arange(S, dtype=torch.float64)[:, None] * inv)

    def rope(u, n):
        u = u.reshape(b, S, n, d)
        z = torch.complex(u[..., :d // 2], u[..., d // 2:]) * rot[None, :, None, :]
        return torch.cat([z.real, z.imag], -1)
    q, k, v = rope(q, nq).transpose(1, 2), rope(k, nkv).transpose(1, 2), v.reshape(b, S, nkv, d).transpose(1, 2)
    k, v = k.repeat_interleave(nq // nkv, dim=1), v.repeat_interleave(nq // nkv, dim=1)
    o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(b, S, nq * d)
    hmid = tx + o @ tw["w_o"]
    g, u = (F.rms_norm(hmid, (h,), tw["gamma2"], sh.rms_eps) @ tw["w_gu"]).split([f, f], dim=-1)
    y = hmid + (F.silu(g) * u) @ tw["w_d"]
    y.backward(torch.tensor(dy))
    oy, cache = O.layer_forward(x, W, sh)
    odx, og = O.layer_backward(dy, W, cache, sh)
    rel = lambda p, r: np.linalg.norm(p - r) / np.linalg.norm(r)
    assert rel(oy, y.detach().numpy()) < 1e-13
    assert rel(odx, tx.grad.numpy()) < 1e-12
    for n in W:
        assert rel(og[n], tw[n].grad.numpy()) < 1e-12, n


def test_rounding_hook_sees_every_named_tensor_and_identity_changes_nothing():
    from tests.helpers import bf16_store
    sh = TINY
    W = _weights(sh, 50)
    x, dy = _xdy(sh, 51)
    seen = []

    def spy(name, t):
        seen.append(name)
        return t
    y0, c0 = O.stage_forward(x, W, sh)
    y1, c1 = O.stage_forward(x, W, sh, store=spy)
    dx0, g0 = O.stage_backward(dy, W, c0, sh)
    dx1, g1 = O.stage_backward(dy, W, c1, sh, store=spy)
    assert np.array_equal(y0, y1) and np.array_equal(dx0, dx1) and np.array_equal(g0[1]["w_qkv"], g1[1]["w_qkv"])
    heads = sh.micro_batch * sh.n_q_heads
    fwd = ["a", "qk_pre", "qk", "v"] + ["p"] * heads + ["o", "h", "b", "gu", "z", "y", "gu_kept"]
    bwd = ["dz", "dgu", "db", "dh", "dc"] + ["p_dv", "ds"] * heads + ["dqk_pre", "dqk_pre", "dv", "dqk", "dqk", "da", "dx"]
    assert seen == fwd * 2 + bwd * 2 and set(seen) == set(O.ROUNDING_POINTS)
    y2, c2 = O.stage_forward(x, W, sh, store=bf16_store)
    dx2, g2 = O.stage_backward(dy, W, c2, sh, store=bf16_store)
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)
    assert 1e-4 < rel(y2, y0) < 3e-2 and 1e-4 < rel(dx2, dx0) < 3e-2
    # every stored tensor is exactly representable in bf16
    from synth import round_to_storage
    assert np.array_equal(round_to_storage(y2.reshape(-1), "bf16")[1], y2.reshape(-1))


def test_oracle_regression_values_tiny_stage():
    """Stored oracle outputs (written by tests/golden/make_golden.py, which calls only the oracle)."""
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.values()
    stored = {}
    for line in open(os.path.join(here, "golden", "tiny_stage_fp64.txt")):
        if not line.startswith("#"):
            k, v = line.rstrip("\n").split("\t")
            stored[k] = float(v)
    assert set(got) == set(stored)
    for k in stored:
        assert math.isclose(got[k], stored[k], rel_tol=1e-9, abs_tol=1e-12), k
