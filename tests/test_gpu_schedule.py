"""1F1B-ordered execution with stash accounting, activation recomputation, and the memory report against the
device (Appendix B.4 of the paper for the memory model).

Recomputation runs the same kernels on the same inputs, so its results must equal the kept-activation results
bit for bit; a 1F1B order pops the same entries one at a time, so y and dX are bitwise equal to the
all-forward-then-backward order and the weight gradients differ only in fp32 summation order."""
import numpy as np
import pytest

import synth
from tests.helpers import gpu_step, rel_err, to_device, to_host64

pytestmark = pytest.mark.gpu

RAGGED = synth.StageShape(hidden=192, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=328, seq=200, micro_batch=2,
                          layers=3, microbatches=3)
FUSED = RAGGED.with_(ffn=352)


@pytest.mark.parametrize("sh", [RAGGED, FUSED, RAGGED.with_(dtype="fp32")], ids=["ragged", "fused", "fp32"])
def test_recomputation_is_bit_identical(sh):
    import paper_2410_13333_amd as mls
    ks = [3, 1, 0, 2]
    a = gpu_step(sh, 1000, 2000, 3000, ks)
    a[3].close()
    for interleave in (False, True):
        st = mls.Stage.from_shape(sh, seed=1000, max_inflight=len(ks), recompute=True)
        b = gpu_step(sh, 1000, 2000, 3000, ks, interleave, stage=st)
        for u, v in zip(a[0] + a[1], b[0] + b[1]):
            assert np.array_equal(u, v)
        if interleave:
            assert rel_err(b[2], a[2]) < 1e-6          # one contraction per micro-batch: fp32 order differs
        else:
            assert np.array_equal(a[2], b[2])
        x = to_device(synth.make_x(sh, 2000, 0)[0], sh.dtype)
        st.forward(x, 1, x.clone())
        assert np.array_equal(to_host64(st.debug_read("x")).reshape(-1), to_host64(x).reshape(-1))
        with pytest.raises(mls.MlsError) as e:          # only the layer inputs are kept
            st.debug_read("a")
        assert e.value.code == -3
        st.close()


def _one_f_one_b(st, sh, xs, dy, ys, dx, grads, k, pp, j):
    """Stage j (1-based) of a pp-stage 1F1B pipeline over len(xs) micro-batches: pp - j forwards of warm-up, then
    one forward / one backward, then the cool-down backwards.  Returns the peak number of kept micro-batches."""
    m, warm = len(xs), min(len(xs), pp - j)
    f = b = peak = 0
    for _ in range(warm):
        st.forward(xs[f], k, ys[f]); f += 1
    while b < m:
        if f < m:
            st.forward(xs[f], k, ys[f]); f += 1
        peak = max(peak, st.inflight)
        st.backward(dy[b:b + 1], grads, 1, dx[b:b + 1]); b += 1
    return peak


@pytest.mark.parametrize("pp,j", [(4, 1), (4, 3), (4, 4)])
def test_1f1b_order_keeps_pp_minus_j_plus_one_microbatches(pp, j):
    import torch
    import paper_2410_13333_amd as mls
    sh, m, k = RAGGED, 6, 2
    ref = gpu_step(sh.with_(microbatches=m), 1000, 2000, 3000, [k] * m)
    ref[3].close()
    keep = pp - j + 1
    st = mls.Stage.from_shape(sh, seed=1000, max_layers=k, max_inflight=keep)
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    xs = [to_device(synth.make_x(sh, 2000, mb)[0], sh.dtype) for mb in range(m)]
    dy = torch.stack([to_device(synth.make_dy(sh, 3000, mb)[0], sh.dtype) for mb in range(m)])
    ys = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(m)]
    dx = torch.empty_like(dy)
    grads = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
    peak = _one_f_one_b(st, sh, xs, dy, ys, dx, grads, k, pp, j)
    torch.cuda.synchronize()
    assert peak == keep and st.inflight == 0
    for mb in range(m):
        assert np.array_equal(to_host64(ys[mb]), ref[0][mb]) and np.array_equal(to_host64(dx[mb]), ref[1][mb])
    g = to_host64(grads)
    assert rel_err(g, ref[2][:g.size]) < 1e-6 and not ref[2][g.size:].any()
    st.close()
    if keep > 1:                                   # one entry fewer than the schedule needs: the stash says so
        st = mls.Stage.from_shape(sh, seed=1000, max_layers=k, max_inflight=keep - 1)
        with pytest.raises(mls.MlsError) as e:
            _one_f_one_b(st, sh, xs, dy, ys, dx, torch.zeros_like(grads), k, pp, j)
        assert e.value.code == -4
        st.close()


@pytest.mark.parametrize("recompute", [False, True])
def test_memory_report_matches_the_device(recompute):
    """hipMalloc rounds each of the ~15 allocations up to its granule: the free-memory drop must lie between the
    report and the report plus 1 % + 64 MiB of slack."""
    import torch
    import paper_2410_13333_amd as mls
    sh = synth.CONFIGS["7b"].with_(layers=2, microbatches=2)
    want = mls.Stage.memory(sh, recompute=recompute)["total_bytes"]
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    st = mls.Stage.from_shape(sh, seed=1, recompute=recompute)
    free1, _ = torch.cuda.mem_get_info()
    used = free0 - free1
    st.close()
    assert want <= used <= want * 1.01 + 64 * 2 ** 20, (want, used)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_stage_step_replays_from_a_hip_graph(dtype):
    """A whole stage step (forwards with different layer counts, one backward) captured into a HIP graph on the
    stage's stream replays bit for bit: the library allocates nothing, synchronises nothing and records no memset on
    the hot path, and the stash ring returns to its starting slot after a step that fills it.  Replays alternate
    with eager steps on other inputs and with synchronisations; every replay is compared with the eager result."""
    import torch
    import paper_2410_13333_amd as mls
    sh = synth.StageShape(hidden=192, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=352, seq=200, micro_batch=2,
                          layers=3, microbatches=3, dtype=dtype)
    ks = [3, 1, 2]
    side = torch.cuda.Stream()
    st = mls.Stage.from_shape(sh, seed=1000, stream=side)
    M = len(ks)
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    xs = [to_device(synth.make_x(sh, 2000, mb)[0], dtype) for mb in range(M)]
    other = [to_device(synth.make_x(sh, 2100, mb)[0], dtype) for mb in range(M)]
    dy = torch.stack([to_device(synth.make_dy(sh, 3000, mb)[0], dtype) for mb in range(M)])
    xin = [x.clone() for x in xs]  # the graph reads these buffers; their contents may change between replays
    ys = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(M)]
    dx = torch.empty_like(dy)
    grads = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")

    def step():
        for mb in range(M):
            st.forward(xin[mb], ks[mb], ys[mb])
        st.backward(dy, grads, M, dx, overwrite=True)

    def run_eager():
        with torch.cuda.stream(side):
            step()
        side.synchronize()
        return [y.clone() for y in ys], dx.clone(), grads.clone()
    torch.cuda.synchronize()
    ref = run_eager()                      # also the warm-up that sets the kernels' attributes
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(3):
        for a, b in zip(xin, other):       # eager work on other inputs between the replays
            a.copy_(b)
        torch.cuda.synchronize()
        got_other = run_eager()
        assert not torch.equal(got_other[1], ref[1])
        for a, b in zip(xin, xs):
            a.copy_(b)
        grads.fill_(float("nan"))
        dx.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        side.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(ys, ref[0])), rep
        assert torch.equal(dx, ref[1]) and torch.equal(grads, ref[2]), rep
    assert st.inflight == 0
    del graph
    st.close()
