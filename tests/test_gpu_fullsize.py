"""Full-size parity at the real 7B, 13B and 70B-shard (grouped KV heads) shapes, i.e. every kernel in exactly the launch
configuration the benchmark times, compared with the EXACT fp64 oracle on the same seeded bf16 inputs: the full y, dX
and every parameter gradient, relative Frobenius error.

The bar is the benchmark spec's tolerance, 1e-2.  Where bf16 matrix operands cannot reach it, the bound of the regression
guard comes from tests/golden/bf16_rounding_distances.txt (written by tests/golden/make_bf16_floors.py from the oracle
alone): the distance of the oracle from itself when the tensors the library keeps in bf16 are rounded ("library"
set), times 1.1.  Which quantities exceed 1e-2 at which depth is printed by the tests and stated in the design notes."""
import importlib.util
import os
import time

import numpy as np
import pytest

import synth
from tests.helpers import gpu_step, grad_errors, oracle_step, rel_err, storage_bits, to_device, to_host64

pytestmark = pytest.mark.gpu

TOL = 1e-2      # relative Frobenius error of bf16 outputs and gradients against the exact fp64 oracle
GUARD = 1.1     # regression guard: this many times the oracle-only distance of the library's set of bf16 tensors


def _floors(name, layers):
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_bf16_floors", os.path.join(here, "golden", "make_bf16_floors.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    y, dx, g, _ = mod.read()[(name, layers, 0, "library")]
    return y, dx, g


def _assert_parity(tag, name, layers, ey, ex, eg, errs):
    """1e-2 wherever bf16 storage of the library's tensors alone stays below it; the guard bound elsewhere."""
    fy, fx, fg = _floors(name, layers)
    by, bx, bg = (TOL if f <= TOL else GUARD * f for f in (fy, fx, fg))
    missed = [q for q, e in (("y", ey), ("dX", ex), ("gradients", eg)) if e > TOL]
    print(f"[{tag}] vs exact oracle: y={ey:.2e} dx={ex:.2e} grads(max)={eg:.2e}; bounds {by:.2e} {bx:.2e} {bg:.2e}"
          + (f"; north-star tolerance 1e-2 not met at depth {layers} for: {', '.join(missed)}" if missed else ""), flush=True)
    assert ey <= by and ex <= bx, (tag, ey, ex)
    assert eg <= bg, (tag, sorted(errs.items(), key=lambda kv: -kv[1])[:3])


@pytest.mark.parametrize("name", ["7b", "13b", "70b_tp4"])
@pytest.mark.timeout(400)
def test_full_shape_single_layer(name):
    sh = synth.CONFIGS[name].with_(layers=1, microbatches=1)
    t0 = time.time()
    _, p64 = synth.make_params(sh, 1001)
    print(f"[{name}] weights generated in {time.time() - t0:.1f} s", flush=True)
    ys, dxs, g, st = gpu_step(sh, 1001, 2001, 3001, [1])
    # the library drew the same weights from its own generator: compare a slice bit for bit
    got = storage_bits(st.get_params()[:1 << 20])
    ref_bits, _ = synth.round_to_storage(p64[:1 << 20], "bf16")
    assert np.array_equal(got, ref_bits)
    st.close()
    rys, rdxs, rg = oracle_step(sh, 1001, 2001, 3001, [1], params64=p64)
    eg, errs = grad_errors(sh, g, rg, 1)
    _assert_parity(f"{name} 1 layer", name, 1, rel_err(ys[0], rys[0]), rel_err(dxs[0], rdxs[0]), eg, errs)


@pytest.mark.parametrize("name", ["7b", "13b", "70b_tp4"])
@pytest.mark.timeout(900)
def test_full_configuration_all_layers_all_microbatches(name):
    """The benchmark's own launch configurations (7B: 4 layers x 4 micro-batches; 13B: 5 x 7; 70B shard: 3 x 8), one
    backward call in overwrite mode.
    (1) The weight gradients of layer 0, sampled, against fp64 sums over the captured bf16 operands of all the
    micro-batches: 1e-4.
    (2) Properties that hold at any size: y and dX of every micro-batch are bitwise what a one-at-a-time execution
    gives, and the batched weight gradient equals the sum of the single ones to fp32 summation order.
    (3) Parity at full depth against the exact oracle: the first and the last micro-batch through all layers (y, dX,
    and the gradients of a run that holds only that micro-batch)."""
    import torch
    import paper_2410_13333_amd as mls
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
    single = {}
    for mb in range(M):
        g1 = torch.empty_like(grads)
        st.forward(xs[mb], K, y1)
        st.backward(dy[mb:mb + 1], g1, 1, dx1, overwrite=True)
        torch.cuda.synchronize()
        assert torch.equal(y1, ys[mb]) and torch.equal(dx1[0], dx[mb])
        gsum += g1
        if mb in (0, M - 1):
            single[mb] = (to_host64(ys[mb]), to_host64(dx[mb]), to_host64(g1))
    # the orders differ (one register accumulation over M*T terms vs M rounded fp32 sums): about 1e-6 at M = 7, 8
    assert rel_err(to_host64(grads), to_host64(gsum)) < 1e-5
    del gsum, g1
    st.close()
    torch.cuda.empty_cache()
    # (3) first and last micro-batch through all K layers against the exact oracle
    _, p64 = synth.make_params(sh, 1001)
    W = [synth.split_params(sh, p64, l) for l in range(K)]
    per = synth.layer_param_elems(sh)
    from oracle import stage as O
    for mb, (y0, dx0, g0) in single.items():
        t0 = time.time()
        _, x = synth.make_x(sh, 2001, mb)
        _, dyr = synth.make_dy(sh, 3001, mb)
        ry, caches = O.stage_forward(x, W, sh, K)
        ey = rel_err(y0, ry)
        rdx, rgl = O.stage_backward(dyr, W, caches, sh)
        del caches
        rg = np.zeros(K * per)
        for l in range(K):
            for pname, tid, r, c, off in synth.param_layout(sh):
                rg[l * per + off: l * per + off + r * c] = rgl[l][pname].reshape(-1)
        del rgl
        eg, errs = grad_errors(sh, g0, rg, K)
        print(f"[{name} {K} layers, micro-batch {mb}] oracle pass {time.time() - t0:.1f} s", flush=True)
        _assert_parity(f"{name} {K} layers, micro-batch {mb}", name, K, ey, rel_err(dx0, rdx), eg, errs)
