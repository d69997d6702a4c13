"""GPU parity of the first/last-stage layers (include/mls_ends.h) against oracle/ends.py, through the C ABI.

Bars (relative Frobenius error per tensor, fp64 metric; loss: relative error of the scalar):
  fp32 storage: 1e-4 for the loss, dY and every gradient;
  bf16 storage: 1e-2 for dY and the gradients against the oracle with the stored tensors rounded to bf16 (and against
  the exact oracle: the chain is short, no softmax over rounded queries and keys); 2e-3 for the loss;
  embedding: gather and gradient are exact in fp32 (sums of <= a few rows in the same order) -- compared at 1e-6."""
import numpy as np
import pytest

import synth
from oracle import ends as oe
from tests.helpers import bf16_store, rel_err, storage_bits, to_device, to_host64

pytestmark = pytest.mark.gpu

TINY = synth.ENDS_CONFIGS["tiny"]
# nothing a multiple of a tile: vocab 8*173, hidden 8*23, 3 micro-batches
RAGGED = synth.EndsShape(hidden=184, vocab=1384, seq=75, micro_batch=2, microbatches=3)


def _params(sh, seed):
    bits, flat = synth.make_ends_params(sh, seed)
    return bits, synth.split_ends_params(sh, flat)


def _inputs(sh, mb, skew=False, ignore=True):
    import torch
    tok = synth.make_tokens(sh, 2100, mb, skew=skew).reshape(-1).copy()
    tgt = synth.make_targets(sh, 2200, mb).reshape(-1).copy()
    if ignore:
        tok[1], tok[-1] = -3, sh.vocab          # padding ids: zero rows, no gradient
        tgt[0], tgt[-2] = -100, sh.vocab + 5    # ignored targets
    ysh = synth.StageShape(sh.hidden, 1, 1, 64, 8, sh.seq, sh.micro_batch, 1, 1, dtype=sh.dtype)
    ybits, y = synth.make_x(ysh, 2300, mb)
    dbits, dx = synth.make_dy(ysh, 2400, mb)
    return tok, tgt, ybits, y.reshape(sh.tokens, sh.hidden), dbits, dx.reshape(sh.tokens, sh.hidden)


def _run_head(sh, n, weight):
    import torch
    import paper_2410_13333_amd as mls
    en = mls.Ends.from_shape(sh, seed=1100, max_inflight=n)
    bits, p = _params(sh, 1100)
    assert np.array_equal(storage_bits(en.get_params()), bits)
    losses = torch.zeros(n, dtype=torch.float32, device="cuda")
    grads = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
    dy = torch.empty((n, sh.micro_batch, sh.seq, sh.hidden), dtype=en.tdtype, device="cuda")
    ins = [_inputs(sh, mb) for mb in range(n)]
    for mb, (tok, tgt, ybits, y, _, _) in enumerate(ins):
        en.head_forward(to_device(ybits, sh.dtype), torch.from_numpy(tgt).cuda(), weight, losses[mb:mb + 1])
    assert en.inflight == (0, n)
    dlog0 = to_host64(en.debug_dlogits(0))
    en.head_backward(grads, n, dy)
    torch.cuda.synchronize()
    assert en.inflight == (0, 0)
    out = dict(loss=losses.cpu().numpy().astype(np.float64), dy=to_host64(dy).reshape(n, sh.tokens, sh.hidden),
               grads=to_host64(grads), dlog0=dlog0, layout={k: en.param_layout(k) for k in ("embed", "gamma_f", "w_lm")})
    en.close()
    return out, p, ins


def _check_head(sh, n, weight, tol, tol_loss):
    got, p, ins = _run_head(sh, n, weight)
    refs = [("exact", None)] + ([("stored", bf16_store)] if sh.dtype == "bf16" else [])
    for kind, store in refs:
        g_w, g_g = 0.0, 0.0
        for mb, (tok, tgt, _, y, _, _) in enumerate(ins):
            loss, cache = oe.head_forward(y, tgt, p, sh.rms_eps, store)
            dy, g, dlog = oe.head_backward(cache, p, weight, store)
            g_w, g_g = g_w + g["w_lm"], g_g + g["gamma_f"]
            e_loss = abs(got["loss"][mb] - loss) / loss
            e_dy = rel_err(got["dy"][mb], dy)
            assert e_loss <= tol_loss and e_dy <= tol, (kind, mb, e_loss, e_dy)
            if mb == 0:
                assert rel_err(got["dlog0"], dlog) <= tol, (kind, rel_err(got["dlog0"], dlog))
        off, r, c = got["layout"]["w_lm"]
        e_w = rel_err(got["grads"][off:off + r * c].reshape(r, c), g_w)
        off, r, c = got["layout"]["gamma_f"]
        e_g = rel_err(got["grads"][off:off + c], g_g)
        print(f"[{sh.dtype} h={sh.hidden} V={sh.vocab} n={n}] vs {kind}: w_lm {e_w:.2e} gamma_f {e_g:.2e}")
        assert e_w <= tol and e_g <= tol, (kind, e_w, e_g)
        off, r, c = got["layout"]["embed"]
        assert not got["grads"][off:off + r * c].any()          # the head never touches the embedding gradient


def test_head_fp32_matches_oracle_1e4():
    _check_head(TINY.with_(dtype="fp32"), 2, 0.5, 1e-4, 1e-5)
    _check_head(RAGGED.with_(dtype="fp32"), 3, 1.0 / 3, 1e-4, 1e-5)


def test_head_bf16_matches_oracle_1e2():
    _check_head(TINY, 2, 0.5, 1e-2, 2e-3)
    _check_head(RAGGED, 3, 1.0 / 3, 1e-2, 2e-3)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_embedding_gather_and_deterministic_gradient(dtype):
    import torch
    import paper_2410_13333_amd as mls
    sh = RAGGED.with_(dtype=dtype)
    n = 3
    en = mls.Ends.from_shape(sh, seed=1100, max_inflight=n)
    _, p = _params(sh, 1100)
    ins = [_inputs(sh, mb, skew=True) for mb in range(n)]
    x = torch.empty((sh.tokens, sh.hidden), dtype=en.tdtype, device="cuda")
    for mb, (tok, *_rest) in enumerate(ins):
        en.embed_forward(torch.from_numpy(tok).cuda(), x)
        assert np.array_equal(to_host64(x), oe.embed_forward(tok, p["embed"]))       # a copy: exact
    dX = torch.stack([to_device(i[4], dtype).reshape(sh.tokens, sh.hidden) for i in ins])
    ref = sum(oe.embed_backward(i[0], i[5], sh.vocab) for i in ins)
    res = []
    for rep in range(2):
        grads = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
        if rep == 1:                                   # same entries again: forwards repeated, backward in two calls
            for tok, *_rest in ins:
                en.embed_forward(torch.from_numpy(tok).cuda(), x)
            en.embed_backward(dX[:1], grads, 1)
            en.embed_backward(dX[1:], grads, 2)
        else:
            en.embed_backward(dX, grads, n)
        torch.cuda.synchronize()
        off, r, c = en.param_layout("embed")
        g = to_host64(grads)
        assert rel_err(g[off:off + r * c].reshape(r, c), ref) <= 1e-6
        assert not g[off + r * c:].any()
        res.append(g)
    assert rel_err(res[1], res[0]) < 1e-6
    # run-to-run bitwise reproducibility of one call
    for tok, *_rest in ins:
        en.embed_forward(torch.from_numpy(tok).cuda(), x)
    grads = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
    en.embed_backward(dX, grads, n)
    assert np.array_equal(to_host64(grads), res[0])
    en.close()


def test_ends_errors_and_stash_accounting():
    import torch
    import paper_2410_13333_amd as mls
    sh = TINY
    en = mls.Ends.from_shape(sh, seed=1, max_inflight=1)
    tok = torch.zeros(sh.tokens, dtype=torch.int32, device="cuda")
    x = torch.empty((sh.tokens, sh.hidden), dtype=en.tdtype, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    grads = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
    en.embed_forward(tok, x)
    with pytest.raises(mls.MlsError) as e:
        en.embed_forward(tok, x)
    assert e.value.code == -4
    en.head_forward(x, tok, 1.0, loss)
    with pytest.raises(mls.MlsError) as e:
        en.head_forward(x, tok, 1.0, loss)
    assert e.value.code == -4
    with pytest.raises(mls.MlsError) as e:
        en.head_backward(grads, 2, x)
    assert e.value.code == -4
    en.head_backward(grads, 0, x)                       # zero micro-batches: legal no-op
    en.head_backward(grads, 1, x.view(1, sh.micro_batch, sh.seq, sh.hidden))
    en.embed_backward(x, grads, 1)
    assert en.inflight == (0, 0)
    en.close()
    with pytest.raises(mls.MlsError) as e:
        mls.Ends(hidden=100, vocab=1000, seq=8, micro_batch=1, max_inflight=1)
    assert e.value.code == -1


def test_ends_set_params_reaches_every_copy_of_the_weights():
    """The head's forward product reads a transposed copy of w_lm: a handle whose parameters were replaced by another
    handle's must give that handle's loss and gradients bit for bit."""
    import torch
    import paper_2410_13333_amd as mls
    sh = TINY
    a = mls.Ends.from_shape(sh, seed=1, max_inflight=1)
    b = mls.Ends.from_shape(sh, seed=2, max_inflight=1)
    b.set_params(a.get_params())
    g = torch.Generator(device="cpu").manual_seed(3)
    y = torch.randn(sh.tokens, sh.hidden, generator=g).to(a.tdtype).cuda()
    tgt = torch.randint(0, sh.vocab, (sh.tokens,), generator=g, dtype=torch.int32).cuda()
    out = []
    for en in (a, b):
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        grads = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
        dy = torch.empty((1, sh.micro_batch, sh.seq, sh.hidden), dtype=en.tdtype, device="cuda")
        en.head_forward(y, tgt, 1.0, loss)
        en.head_backward(grads, 1, dy)
        torch.cuda.synchronize()
        out.append((loss, grads, dy))
        en.close()
    for u, v in zip(*out):
        assert torch.equal(u, v)
    assert float(out[0][0]) > 0


def test_whole_model_step_embedding_stage_head():
    """tokens -> embedding -> 2 decoder layers -> head -> loss and back, against the oracles chained the same way."""
    import torch
    import paper_2410_13333_amd as mls
    from oracle import stage as O
    ssh = synth.CONFIGS["tiny"].with_(dtype="fp32")
    esh = synth.EndsShape(ssh.hidden, 1000, ssh.seq, ssh.micro_batch, 1, dtype="fp32")
    st = mls.Stage.from_shape(ssh, seed=1000, max_inflight=1)
    en = mls.Ends.from_shape(esh, seed=1100, max_inflight=1)
    tok, tgt, *_ = _inputs(esh, 0, ignore=False)
    shape = (ssh.micro_batch, ssh.seq, ssh.hidden)
    x, y, dy, dx = (torch.empty(shape, dtype=torch.float32, device="cuda") for _ in range(4))
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    gs = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
    ge = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
    en.embed_forward(torch.from_numpy(tok).cuda(), x)
    st.forward(x, 2, y)
    en.head_forward(y, torch.from_numpy(tgt).cuda(), 1.0, loss)
    en.head_backward(ge, 1, dy.view((1,) + shape))
    st.backward(dy.view((1,) + shape), gs, 1, dx.view((1,) + shape))
    en.embed_backward(dx, ge, 1)
    torch.cuda.synchronize()
    # oracle chain
    _, pe = _params(esh, 1100)
    _, flat = synth.make_params(ssh, 1000)
    W = [synth.split_params(ssh, flat, l) for l in range(2)]
    x0 = oe.embed_forward(tok, pe["embed"]).reshape(shape)
    yo, caches = O.stage_forward(x0, W, ssh, 2)
    lo, cache = oe.head_forward(yo.reshape(ssh.tokens, ssh.hidden), tgt, pe, esh.rms_eps)
    dyo, gh, _ = oe.head_backward(cache, pe, 1.0)
    dxo, gl = O.stage_backward(dyo.reshape(shape), W, caches, ssh)
    geo = oe.embed_backward(tok, dxo.reshape(ssh.tokens, ssh.hidden), esh.vocab)
    assert abs(float(loss) - lo) / lo <= 1e-5
    off, r, c = en.param_layout("embed")
    assert rel_err(to_host64(ge)[off:off + r * c].reshape(r, c), geo) <= 1e-4
    off, r, c = en.param_layout("w_lm")
    assert rel_err(to_host64(ge)[off:off + r * c].reshape(r, c), gh["w_lm"]) <= 1e-4
    off, r, c = st.param_layout(0, "w_qkv")
    assert rel_err(to_host64(gs)[off:off + r * c].reshape(r, c), gl[0]["w_qkv"]) <= 1e-4
    st.close()
    en.close()


def test_fullsize_7b_head_and_embedding():
    """The LLaMA-2-7B shaped first/last-stage layers (hidden 4096, vocabulary 32000, 4096 tokens), one micro-batch
    through the head and two through the embedding, in the launch configuration the benchmark times."""
    import torch
    import paper_2410_13333_amd as mls
    sh = synth.ENDS_CONFIGS["7b"]
    en = mls.Ends.from_shape(sh, seed=1101, max_inflight=2)
    bits, p = _params(sh, 1101)
    assert np.array_equal(storage_bits(en.get_params()), bits)
    tok, tgt, ybits, y, dbits, dxv = _inputs(sh, 0)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    grads = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
    dy = torch.empty((1, sh.micro_batch, sh.seq, sh.hidden), dtype=en.tdtype, device="cuda")
    en.head_forward(to_device(ybits, "bf16"), torch.from_numpy(tgt).cuda(), 0.25, loss)
    en.head_backward(grads, 1, dy)
    torch.cuda.synchronize()
    g = to_host64(grads)
    off, r, c = en.param_layout("w_lm")
    gw = g[off:off + r * c].reshape(r, c)
    offg, _, cg = en.param_layout("gamma_f")
    for kind, store in (("exact", None), ("stored", bf16_store)):
        lo, cache = oe.head_forward(y, tgt, p, sh.rms_eps, store)
        dyo, go, _ = oe.head_backward(cache, p, 0.25, store)
        e = (abs(float(loss) - lo) / lo, rel_err(to_host64(dy).reshape(sh.tokens, sh.hidden), dyo), rel_err(gw, go["w_lm"]),
             rel_err(g[offg:offg + cg], go["gamma_f"]))
        print(f"[7b ends] vs {kind}: loss {e[0]:.2e} dy {e[1]:.2e} w_lm {e[2]:.2e} gamma_f {e[3]:.2e}")
        assert e[0] <= 2e-3 and max(e[1:]) <= 1e-2, (kind, e)
    # embedding: two micro-batches, one of them with heavily repeated tokens
    ins = [_inputs(sh, 0), _inputs(sh, 1, skew=True)]
    x = torch.empty((sh.tokens, sh.hidden), dtype=en.tdtype, device="cuda")
    for i in ins:
        en.embed_forward(torch.from_numpy(i[0]).cuda(), x)
    assert np.array_equal(to_host64(x), oe.embed_forward(ins[1][0], p["embed"]))
    dX = torch.stack([to_device(i[4], "bf16").reshape(sh.tokens, sh.hidden) for i in ins])
    grads.zero_()
    en.embed_backward(dX, grads, 2)
    torch.cuda.synchronize()
    ref = sum(oe.embed_backward(i[0], i[5], sh.vocab) for i in ins)
    off, r, c = en.param_layout("embed")
    assert rel_err(to_host64(grads)[off:off + r * c].reshape(r, c), ref) <= 1e-6
    en.close()
