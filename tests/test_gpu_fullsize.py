"""Full-size parity: one layer x one micro-batch at the real 7B, 13B and 70B-shard (grouped KV heads) shapes, i.e.
every kernel in exactly the launch configuration the benchmark times, compared with the fp64 oracle on the
same seeded bf16 inputs: the full y, dX and every parameter gradient (tolerance 1e-2, relative Frobenius)."""
import time

import numpy as np
import pytest

import synth
from tests.helpers import bf16_store, gpu_step, grad_errors, oracle_step, rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-2      # relative Frobenius error of bf16 outputs and gradients against the exact fp64 oracle


@pytest.mark.parametrize("name", ["7b", "13b", "70b_tp4"])
@pytest.mark.timeout(400)
def test_full_shape_single_layer(name):
    sh = synth.CONFIGS[name].with_(layers=1, microbatches=1)
    t0 = time.time()
    _, p64 = synth.make_params(sh, 1001)
    print(f"[{name}] weights generated in {time.time() - t0:.1f} s", flush=True)
    ys, dxs, g, st = gpu_step(sh, 1001, 2001, 3001, [1])
    from tests.helpers import storage_bits
    # the library drew the same weights from its own generator: compare a slice bit for bit
    got = storage_bits(st.get_params()[:1 << 20])
    ref_bits, _ = synth.round_to_storage(p64[:1 << 20], "bf16")
    assert np.array_equal(got, ref_bits)
    st.close()
    t0 = time.time()
    rys, rdxs, rg = oracle_step(sh, 1001, 2001, 3001, [1], params64=p64)
    ey, ex = rel_err(ys[0], rys[0]), rel_err(dxs[0], rdxs[0])
    eg, errs = grad_errors(sh, g, rg, 1)
    print(f"[{name}] vs exact oracle ({time.time() - t0:.1f} s): y={ey:.2e} dx={ex:.2e} grads(max)={eg:.2e} "
          f"{sorted(errs.items(), key=lambda kv: -kv[1])[:3]}", flush=True)
    assert ey <= TOL and ex <= TOL, (ey, ex)
    assert eg <= TOL, sorted(errs.items(), key=lambda kv: -kv[1])[:3]


@pytest.mark.parametrize("name", ["7b", "13b", "70b_tp4"])
@pytest.mark.timeout(600)
def test_full_configuration_all_layers_all_microbatches(name):
    """The benchmark's own launch configurations (7B: 4 layers x 4 micro-batches; 13B: 5 x 7; 70B shard: 3 x 8), one
    backward call in overwrite mode.
    (1) The weight gradients of layer 0, sampled, against fp64 sums over the captured bf16 operands of all the
    micro-batches: 1e-4.
    (2) Properties that hold at any size: y and dX of every micro-batch are bitwise what a one-at-a-time execution
    gives, and the batched weight gradient equals the sum of the single ones to fp32 summation order.
    (3) Parity at full depth (7B: four layers; 70B shard: three layers with grouped KV heads; 13B is left out, its
    oracle pass takes too long): micro-batch 0 through all layers against the oracle in storage-rounded mode (y,
    dX, and the gradients of a run that holds only micro-batch 0).  The 1e-2 bound is a one-layer bound: bf16 storage
    noise grows with depth, and the oracle's own storage-rounded mode stands, for 7B, 1.04e-2 (y), 1.41e-2 (dX)
    and 2.63e-2 (largest gradient distance, gamma1 / w_qkv of the last layer) from its exact mode on these very
    inputs, for the shard 1.55e-2 / 2.95e-2 / 4.72e-2 (measured on the CPU, oracle only).  Two bf16 executions that
    round in different orders sit at that distance from each other too, so the bounds here are 1.5 times those
    floors."""
    import torch
    import paper_2410_13333_amd as mls
    from tests.helpers import to_device, to_host64
    sh = synth.CONFIGS[name]
    K, M = sh.layers, sh.microbatches
    st = mls.Stage.from_shape(sh, seed=1001)
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    xs = [to_device(synth.make_x(sh, 2001, mb)[0], "bf16") for mb in range(M)]
    dy = torch.stack([to_device(synth.make_dy(sh, 3001, mb)[0], "bf16") for mb in range(M)])
    ys = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(M)]
    dx = torch.empty_like(dy)
    grads = torch.full((st.grad_elems,), float("nan"), dtype=torch.float32, device="cuda")
    for mb in range(M):
        st.forward(xs[mb], K, ys[mb])
    # operand capture (layer 0): sampled rows of the weight = sampled columns of its activation operand
    pairs = (("w_d", "z", "dy"), ("w_gu", "b", "dgu"), ("w_o", "o", "dh"), ("w_qkv", "a", "dqkv"))
    rng = np.random.default_rng(7)

    def pick(n):  # both ends (the last columns belong to the narrower tail tiles) and a random spread
        return np.unique(np.concatenate([np.arange(8), np.arange(n - 8, n), rng.integers(0, n, 48)]))
    sel = {}
    for w, _, _ in pairs:
        _, rows, cols = st.param_layout(0, w)
        sel[w] = (pick(rows), pick(cols))
    act = {w: [to_host64(st.debug_read(a, 0, mb)[:, torch.from_numpy(sel[w][0]).cuda()]) for mb in range(M)] for w, a, _ in pairs}
    st.backward(dy, grads, M, dx, overwrite=True)
    torch.cuda.synchronize()
    # the 1e-4 bar of the fp32-accumulated weight gradients at full size, all micro-batches in one call:
    # sampled entries rebuilt in fp64 from exactly the captured bf16 operands
    gl0 = grads[:st.grad_elems // st.cfg.max_layers]
    for w, _, b in pairs:
        off, rows, cols = st.param_layout(0, w)
        R, Cc = sel[w]
        ref = sum(act[w][mb].T @ to_host64(st.debug_read(b, 0, mb)[:, torch.from_numpy(Cc).cuda()]) for mb in range(M))
        got = to_host64(gl0[off:off + rows * cols].reshape(rows, cols)[torch.from_numpy(R).cuda()][:, torch.from_numpy(Cc).cuda()])
        e = rel_err(got, ref)
        print(f"[{name} {K}x{M}] {w} sampled {len(R)}x{len(Cc)} entries vs fp64 from captured operands: {e:.2e}", flush=True)
        assert e <= 1e-4, (w, e)
    del act
    # one at a time
    y1, dx1 = torch.empty_like(ys[0]), torch.empty_like(dy[:1])
    gsum = torch.zeros_like(grads)
    g0 = None
    for mb in range(M):
        g1 = torch.empty_like(grads)
        st.forward(xs[mb], K, y1)
        st.backward(dy[mb:mb + 1], g1, 1, dx1, overwrite=True)
        torch.cuda.synchronize()
        assert torch.equal(y1, ys[mb]) and torch.equal(dx1[0], dx[mb])
        gsum += g1
        if mb == 0:
            g0 = to_host64(g1)
    # the orders differ (one register accumulation over M*T terms vs M rounded fp32 sums): about 1e-6 at M = 7, 8
    assert rel_err(to_host64(grads), to_host64(gsum)) < 1e-5
    del gsum, g1
    y0, dx0 = to_host64(ys[0]), to_host64(dx[0])
    st.close()
    # bf16 depth floors: oracle storage-rounded mode against oracle exact mode on these inputs (CPU, oracle only)
    floors = {"7b": (1.04e-2, 1.41e-2, 2.63e-2), "70b_tp4": (1.55e-2, 2.95e-2, 4.72e-2)}
    if name not in floors:
        return
    t0 = time.time()
    rys, rdxs, rg = oracle_step(sh.with_(microbatches=1), 1001, 2001, 3001, [K], store=bf16_store)
    ey, ex = rel_err(y0, rys[0]), rel_err(dx0, rdxs[0])
    eg, errs = grad_errors(sh, g0, rg, K)
    print(f"[{name} {K} layers] vs stored oracle ({time.time() - t0:.1f} s): y={ey:.2e} dx={ex:.2e} grads(max)={eg:.2e}", flush=True)
    fy, fx, fg = floors[name]
    assert ey <= 1.5 * fy and ex <= 1.5 * fx and eg <= 1.5 * fg, (ey, ex, sorted(errs.items(), key=lambda kv: -kv[1])[:3])
