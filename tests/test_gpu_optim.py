"""GPU parity of the optimizer step and the event-based probe (include/mls_optim.h) against oracle/optim.py.

The kernel computes in fp32 on fp32 state; the oracle in fp64 from the same fp32 inputs: bar 1e-6 relative
Frobenius error for master weights and moments after several steps; the storage-type output is the master weight
rounded once (checked exactly against rounding the kernel's own master copy)."""
import numpy as np
import pytest

import synth
from oracle import optim as oo
from tests.helpers import rel_err, storage_bits, to_device, to_host64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_adamw_steps_match_oracle(dtype):
    import torch
    import paper_2410_13333_amd as mls
    n = 8 * 12345
    bits, w0 = synth.round_to_storage(0.02 * synth.normal(77, 40, 0, n), dtype)
    p = to_device(bits, dtype)
    opt = mls.Optim(p)
    hp = dict(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    w, m, v = w0.copy(), np.zeros(n), np.zeros(n)
    out = torch.empty_like(p)
    for t in range(1, 5):
        g32 = (synth.normal(78, 41, t, n) * 10.0 ** (t - 3)).astype(np.float32)
        opt.step(torch.from_numpy(g32).cuda(), out, grad_scale=0.25, **hp)
        w, m, v = oo.adamw_step(w, m, v, 0.25 * g32.astype(np.float64), t, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                                hp["weight_decay"])
    torch.cuda.synchronize()
    assert opt.steps == 4
    gw = to_host64(opt.read("w"))
    assert rel_err(gw, w) <= 1e-6 and rel_err(to_host64(opt.read("m")), m) <= 1e-6
    assert rel_err(to_host64(opt.read("v")), v) <= 1e-6
    want_bits, _ = synth.round_to_storage(gw, dtype)      # the output is the kernel's master copy rounded once
    assert np.array_equal(storage_bits(out), want_bits)
    opt.close()


def test_optimizer_updates_a_stage_and_the_loss_goes_down():
    """embedding -> 1 layer -> head; three AdamW steps on the stage's and the ends' parameters lower the loss."""
    import torch
    import paper_2410_13333_amd as mls
    ssh = synth.CONFIGS["tiny"].with_(layers=1)
    esh = synth.EndsShape(ssh.hidden, 1000, ssh.seq, ssh.micro_batch, 1)
    st = mls.Stage.from_shape(ssh, seed=1000, max_inflight=1)
    en = mls.Ends.from_shape(esh, seed=1100, max_inflight=1)
    ps, pe = st.get_params(), en.get_params()
    os_, oe_ = mls.Optim(ps), mls.Optim(pe)
    tok = torch.from_numpy(synth.make_tokens(esh, 2100, 0).reshape(-1)).cuda()
    tgt = torch.from_numpy(synth.make_targets(esh, 2200, 0).reshape(-1)).cuda()
    shape = (ssh.micro_batch, ssh.seq, ssh.hidden)
    x, y, dy, dx = (torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(4))
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    losses = []
    for it in range(4):
        gs = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
        ge = torch.zeros(en.grad_elems, dtype=torch.float32, device="cuda")
        en.embed_forward(tok, x)
        st.forward(x, 1, y)
        en.head_forward(y, tgt, 1.0, loss)
        en.head_backward(ge, 1, dy.view((1,) + shape))
        st.backward(dy.view((1,) + shape), gs, 1, dx.view((1,) + shape))
        en.embed_backward(dx, ge, 1)
        losses.append(float(loss))
        os_.step(gs, ps, lr=2e-3, weight_decay=0.0)
        oe_.step(ge, pe, lr=2e-3, weight_decay=0.0)
        st.set_params(ps)
        en.set_params(pe)
    assert losses[0] == pytest.approx(np.log(1000), rel=0.1)
    assert losses[3] < losses[2] < losses[1] < losses[0] - 0.05
    for h in (os_, oe_, st, en):
        h.close()


def test_probe_brackets_a_stage_step():
    """The probe's tau for a tiny stage step equals the wall time per unit, a first step gives no shift, a step
    with a layer count halved at the same elapsed work per unit gives none either, and an artificial reference
    makes the rate scale."""
    import torch
    import paper_2410_13333_amd as mls
    sh = synth.CONFIGS["tiny"]
    st = mls.Stage.from_shape(sh, seed=1000, max_inflight=2)
    x = to_device(synth.make_x(sh, 2000, 0)[0], "bf16")
    dy = torch.stack([to_device(synth.make_dy(sh, 3000, 0)[0], "bf16")] * 2)
    y, dx = torch.empty_like(x), torch.empty_like(dy)
    g = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
    pr = mls.Probe(1.0, 0.05, torch.cuda.current_stream().cuda_stream)
    with pytest.raises(mls.MlsError):
        pr.read()
    for _ in range(3):                                    # warm up
        st.forward(x, 2, y); st.forward(x, 2, y); st.backward(dy, g, 2, dx)
    pr.begin()
    st.forward(x, 2, y); st.forward(x, 2, y); st.backward(dy, g, 2, dx)
    pr.end(2, 2)
    rate, tau, shift = pr.read()
    assert tau > 0 and rate == pytest.approx(tau / 1.0) and shift is False
    assert pr.read() == (rate, tau, shift)                # reading twice changes nothing
    pr2 = mls.Probe(tau / 3.0, 0.05, torch.cuda.current_stream().cuda_stream)
    pr2.begin()
    st.forward(x, 2, y); st.forward(x, 2, y); st.backward(dy, g, 2, dx)
    pr2.end(2, 2)
    r2, t2, _ = pr2.read()
    assert r2 == pytest.approx(3.0 * t2 / tau)
    st.close(); pr.close(); pr2.close()
