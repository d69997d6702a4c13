"""GPU parity of the HIP decoder stage against the CPU oracle, through the C ABI (ctypes binding).

Tolerances (relative Frobenius error per tensor, fp64 metric):
  fp32 storage: 1e-4 for every output and gradient (validates the algorithm with no bf16 in the way);
  bf16 storage: 1e-2 for y, dX and the parameter gradients against the oracle fed the same bf16 inputs;
  weight-gradient contraction + fp32 accumulation given identical bf16 operands: 1e-4."""
import numpy as np
import pytest

import synth
from tests.helpers import (gpu_step, grad_errors, oracle_step, rel_err, round_bf16, storage_bits, to_device,
                           to_host64)

pytestmark = pytest.mark.gpu

TINY = synth.CONFIGS["tiny"]
# grouped KV heads, ragged everything: seq not a multiple of any tile, ffn = 8*41, 3 layers, 3 micro-batches
RAGGED = synth.StageShape(hidden=192, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=328, seq=200, micro_batch=2,
                          layers=3, microbatches=3)
# ffn a multiple of 32 (SwiGLU runs fused into the contractions around it), 2 ffn = 704 not a multiple of any tile
FUSED_RAGGED = synth.StageShape(hidden=192, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=352, seq=200, micro_batch=2,
                                layers=3, microbatches=3)
GQA128 = synth.StageShape(hidden=256, n_q_heads=4, n_kv_heads=1, head_dim=128, ffn=512, seq=328, micro_batch=1,
                          layers=1, microbatches=2)


def _check(sh, ks, tol, interleave=False):
    ys, dxs, g, st = gpu_step(sh, 1000, 2000, 3000, ks, interleave)
    assert st.inflight == 0
    st.close()
    refs = [("exact", tol, oracle_step(sh, 1000, 2000, 3000, ks))]     # the exact fp64 oracle is the only bar
    for kind, t, (rys, rdxs, rg) in refs:
        ey = max(rel_err(ys[mb], rys[mb]) for mb in range(len(ks)))
        ex = max(rel_err(dxs[mb], rdxs[mb]) for mb in range(len(ks)))
        worst, errs = grad_errors(sh, g, rg, max(ks) if ks else 0)
        print(f"[{sh.dtype} h={sh.hidden} S={sh.seq} ks={ks}] vs {kind} oracle: y {ey:.2e} dx {ex:.2e} grads {worst:.2e}")
        assert ey <= t and ex <= t, (kind, ey, ex)
        assert worst <= t, (kind, sorted(errs.items(), key=lambda kv: -kv[1])[:4])
    return ys, dxs, g


def test_weights_match_the_generator_bit_for_bit():
    import paper_2410_13333_amd as mls
    for dtype in ("bf16", "fp32"):
        sh = TINY.with_(dtype=dtype)
        st = mls.Stage.from_shape(sh, seed=1000)
        bits, _ = synth.make_params(sh, 1000)
        assert np.array_equal(storage_bits(st.get_params()), bits)
        off, r, c = st.param_layout(1, "w_gu")
        per = synth.layer_param_elems(sh)
        assert (off, r, c) == (per + 2 * 256 + 256 * 768 + 256 * 256, 256, 1376) and st.grad_elems == 2 * per
        st.close()


def test_tiny_fp32_matches_oracle_1e4():
    _check(TINY.with_(dtype="fp32"), [2], 1e-4)


def test_tiny_bf16_matches_oracle_1e2():
    _check(TINY, [2], 1e-2)


def test_ragged_gqa_fp32_and_bf16_multi_microbatch():
    _check(RAGGED.with_(dtype="fp32"), [3, 3, 3], 1e-4)
    _check(RAGGED, [3, 3, 3], 1e-2)


def test_ragged_shape_with_fused_swiglu():
    """ffn % 32 == 0 switches w_gu, gu and dgu to the interleaved gate/up column order inside the library; weights
    (generator and get/set), the captured gu / dgu operands and the w_gu gradient must still come out in the
    public order."""
    import paper_2410_13333_amd as mls
    sh = FUSED_RAGGED
    st = mls.Stage.from_shape(sh, seed=1000)
    bits, _ = synth.make_params(sh, 1000)
    assert np.array_equal(storage_bits(st.get_params()), bits)
    p = st.get_params()
    st.set_params(p.flip(0).contiguous())
    assert np.array_equal(storage_bits(st.get_params()), bits[::-1])
    st.close()
    _check(sh, [3, 3, 3], 1e-2)
    _check(sh, [1, 3, 2], 1e-2, interleave=True)


def test_set_params_reaches_every_copy_of_the_weights():
    """The library keeps transposed copies of the weight matrices for its forward products: a stage whose parameters
    were replaced by another stage's must give that stage's output and input gradient bit for bit."""
    import torch
    import paper_2410_13333_amd as mls
    sh = FUSED_RAGGED
    a = mls.Stage.from_shape(sh, seed=1000)
    b = mls.Stage.from_shape(sh, seed=4321)
    x = to_device(synth.make_x(sh, 2000, 0)[0], "bf16")
    dy = to_device(synth.make_dy(sh, 3000, 0)[0], "bf16")
    out = []
    for st in (a, b):
        if st is b:
            st.set_params(a.get_params())
        y, dx = torch.empty_like(x), torch.empty_like(dy)
        g = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
        st.forward(x, sh.layers, y)
        st.backward(dy.unsqueeze(0), g, 1, dx.unsqueeze(0))
        torch.cuda.synchronize()
        out.append((y, dx, g))
    for u, v in zip(*out):
        assert torch.equal(u, v)
    a.close()
    b.close()


def test_head_dim_128_gqa_single_kv_head():
    _check(GQA128.with_(dtype="fp32"), [1, 1], 1e-4)
    _check(GQA128, [1, 1], 1e-2)


def test_uneven_layer_counts_and_interleaved_order_agree():
    """Entries forwarded with different layer counts (including zero) may be mixed; one-forward-one-backward
    order gives the same y and dX bit for bit as all forwards then one backward; the weight gradients differ only
    in fp32 summation order (one contraction over all micro-batches vs one per micro-batch)."""
    ks = [2, 0, 1]
    a = _check(TINY, ks, 1e-2)
    b = _check(TINY, ks, 1e-2, interleave=True)
    for u, v in zip(a[0] + a[1], b[0] + b[1]):
        assert np.array_equal(u, v)
    assert rel_err(a[2], b[2]) < 1e-6


def test_run_to_run_bitwise_determinism():
    a = gpu_step(RAGGED, 1000, 2000, 3000, [3, 2])
    b = gpu_step(RAGGED, 1000, 2000, 3000, [3, 2])
    for u, v in zip(a[0] + a[1], b[0] + b[1]):
        assert np.array_equal(u, v)
    assert np.array_equal(a[2], b[2])
    a[3].close()
    b[3].close()


def test_gradients_accumulate_and_are_never_zeroed():
    import torch
    import paper_2410_13333_amd as mls
    sh = TINY
    st = mls.Stage.from_shape(sh, seed=1000, max_inflight=2)
    x = to_device(synth.make_x(sh, 2000, 0)[0], "bf16")
    dy = to_device(synth.make_dy(sh, 3000, 0)[0], "bf16")[None]
    y, dx = torch.empty_like(x), torch.empty_like(dy)
    g1 = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
    st.forward(x, 2, y)
    st.backward(dy, g1, 1, dx)
    g2 = torch.full((st.grad_elems,), 7.0, dtype=torch.float32, device="cuda")
    st.forward(x, 2, y)
    st.forward(x, 2, y)
    st.backward(torch.cat([dy, dy]), g2, 2, torch.empty(2, *x.shape, dtype=x.dtype, device="cuda"))
    torch.cuda.synchronize()
    ref = 7.0 + 2.0 * to_host64(g1)
    assert rel_err(to_host64(g2), ref) < 1e-6
    st.close()


def test_zero_layers_zero_microbatches_and_errors():
    import torch
    import paper_2410_13333_amd as mls
    sh = TINY
    st = mls.Stage.from_shape(sh, seed=1, max_inflight=2)
    x = to_device(synth.make_x(sh, 2000, 0)[0], "bf16")
    y = torch.empty_like(x)
    g = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
    st.backward(None, None, 0, None)                      # n = 0: no-op even with null buffers
    st.forward(x, 0, y)                                   # k = 0: identity, still one stash entry
    assert st.inflight == 1
    dy = to_device(synth.make_dy(sh, 3000, 0)[0], "bf16")[None]
    dx = torch.empty_like(dy)
    st.backward(dy, g, 1, dx)
    torch.cuda.synchronize()
    assert torch.equal(y, x) and torch.equal(dx, dy) and not g.any()
    with pytest.raises(mls.MlsError) as e:
        st.backward(dy, g, 1, dx)                         # nothing stashed
    assert e.value.code == -4
    with pytest.raises(mls.MlsError) as e:
        st.forward(x, 3, y)                               # beyond max_layers
    assert e.value.code == -3
    st.forward(x, 1, y)
    st.forward(x, 1, y)
    with pytest.raises(mls.MlsError) as e:
        st.forward(x, 1, y)                               # stash full
    assert e.value.code == -4
    with pytest.raises(mls.MlsError) as e:
        st.forward(None, 1, y)
    assert e.value.code == -2
    st.reset()
    assert st.inflight == 0
    st.close()
    with pytest.raises(mls.MlsError) as e:
        mls.Stage(hidden=100, n_q_heads=4, n_kv_heads=3, head_dim=64, ffn=688, seq=8, micro_batch=1, max_layers=1,
                  max_inflight=1)
    assert e.value.code == -1


@pytest.mark.parametrize("batched", [0, 3, 17])
@pytest.mark.parametrize("base", ["ragged", "fused"])
def test_weight_gradient_contraction_given_identical_operands_1e4(base, batched):
    """The 1e-4 bar of the fp32-accumulated weight gradients: capture the bf16 operand pairs of every
    weight-gradient contraction of layer 0 and rebuild sum_mb X^T dY in fp64 from exactly those operands.
    batched = n > 0: n micro-batches go through ONE backward call (one contraction per weight over all of them, in a
    two-layer stage; 17 is one more than a launch's 16 segments, so every weight takes a second, accumulating launch);
    batched = 0: three micro-batches, one call per micro-batch accumulates into the same gradient vector."""
    import torch
    import paper_2410_13333_amd as mls
    sh = (RAGGED if base == "ragged" else FUSED_RAGGED).with_(layers=2 if batched else 1)
    n, K = batched or 3, sh.layers
    st = mls.Stage.from_shape(sh, seed=1000, max_inflight=n if batched else 1)
    g = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
    ref = {k: 0.0 for k in ("w_d", "w_gu", "w_o", "w_qkv")}
    pairs = (("w_d", "z", "dy"), ("w_gu", "b", "dgu"), ("w_o", "o", "dh"), ("w_qkv", "a", "dqkv"))
    xs = [to_device(synth.make_x(sh, 2000, mb)[0], "bf16") for mb in range(n)]
    dys = torch.stack([to_device(synth.make_dy(sh, 3000, mb)[0], "bf16") for mb in range(n)])
    y, dx = torch.empty_like(xs[0]), torch.empty_like(dys)
    if batched:
        for mb in range(n):
            st.forward(xs[mb], K, y)
        ops = [{k: to_host64(st.debug_read(k, 0, mb)) for _, k, _ in pairs} for mb in range(n)]
        st.backward(dys, g, n, dx)
        for mb in range(n):
            for w, a, b in pairs:
                ref[w] = ref[w] + ops[mb][a].T @ to_host64(st.debug_read(b, 0, mb))
        with pytest.raises(mls.MlsError):
            st.debug_read("dy", 0, n)  # beyond the micro-batches of that call
    else:
        for mb in range(n):
            st.forward(xs[mb], K, y)
            ops = {k: to_host64(st.debug_read(k)) for _, k, _ in pairs}
            st.backward(dys[mb:mb + 1], g, 1, dx[mb:mb + 1])
            for w, a, b in pairs:
                ref[w] = ref[w] + ops[a].T @ to_host64(st.debug_read(b))
    torch.cuda.synchronize()
    gh = to_host64(g)
    for name, r in ref.items():
        off, rows, cols = st.param_layout(0, name)
        e = rel_err(gh[off:off + rows * cols].reshape(rows, cols), r)
        assert e <= 1e-4, (name, e)
    st.close()


def test_wide_hidden_rows_span_many_chunks():
    """hidden above 4096 and above 8192 exercises the wider register tilings of the RMSNorm kernels."""
    for hidden in (4104, 8200):
        sh = synth.StageShape(hidden=hidden, n_q_heads=2, n_kv_heads=1, head_dim=64, ffn=64, seq=72, micro_batch=1,
                              layers=1, microbatches=2)
        _check(sh, [1, 1], 1e-2)
        _check(sh.with_(dtype="fp32"), [1], 1e-4)


@pytest.mark.parametrize("base", ["ragged", "fused", "fp32"])
def test_overwrite_mode_equals_zeroing_then_accumulating(base):
    """MLS_BWD_OVERWRITE: a gradient vector full of NaN goes in, exactly the gradients of zero-then-accumulate come
    out, layers no entry reached are zero, and a following plain call accumulates on top."""
    import torch
    import paper_2410_13333_amd as mls
    sh = {"ragged": RAGGED, "fused": FUSED_RAGGED, "fp32": RAGGED.with_(dtype="fp32")}[base].with_(layers=4)
    ks = [2, 3, 0, 1]
    ref = gpu_step(sh, 1000, 2000, 3000, ks)
    ref[3].close()
    st = mls.Stage.from_shape(sh, seed=1000, max_inflight=len(ks))
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    xs = [to_device(synth.make_x(sh, 2000, mb)[0], sh.dtype) for mb in range(len(ks))]
    dy = torch.stack([to_device(synth.make_dy(sh, 3000, mb)[0], sh.dtype) for mb in range(len(ks))])
    ys = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in ks]
    dx = torch.empty_like(dy)
    grads = torch.full((st.grad_elems,), float("nan"), dtype=torch.float32, device="cuda")
    for mb, k in enumerate(ks):
        st.forward(xs[mb], k, ys[mb])
    st.backward(dy, grads, len(ks), dx, overwrite=True)
    torch.cuda.synchronize()
    g = to_host64(grads)
    assert np.array_equal(g, ref[2])
    per = synth.layer_param_elems(sh)
    assert not g[3 * per:].any() and g[2 * per:3 * per].any()          # layer 3 untouched, layer 2 reached by one entry
    for u, v in zip(ref[1], dx):
        assert np.array_equal(u, to_host64(v))
    # a second, plain call adds the same gradients once more
    for mb, k in enumerate(ks):
        st.forward(xs[mb], k, ys[mb])
    st.backward(dy, grads, len(ks), dx)
    torch.cuda.synchronize()
    assert rel_err(to_host64(grads), 2 * ref[2]) < 1e-6
    st.backward(dy, grads, 0, dx, overwrite=True)                       # nothing to pop: everything zero
    torch.cuda.synchronize()
    assert not to_host64(grads).any()
    st.close()


@pytest.mark.parametrize("seq,mb", [(37, 1), (1, 1), (3, 3), (65, 2)])
def test_token_counts_that_are_not_multiples_of_eight(seq, mb):
    """Tokens per micro-batch T = seq * micro_batch need not be a multiple of anything: T is the row count of
    every activation and the contraction length of the weight gradients (zero-filled beyond the last row).
    seq = 1: attention over a single position is the identity on v."""
    for ffn in (40, 64):  # separate and fused SwiGLU
        sh = synth.StageShape(hidden=72, n_q_heads=2, n_kv_heads=1, head_dim=64, ffn=ffn, seq=seq, micro_batch=mb,
                              layers=2, microbatches=2)
        _check(sh, [2, 1], 1e-2)
    _check(sh.with_(dtype="fp32", head_dim=16), [2, 1], 1e-4)


@pytest.mark.parametrize("nq,nkv,d,seq,mb", [(30, 2, 128, 4096, 1), (60, 4, 64, 4096, 1), (6, 2, 128, 1000, 3),
                                              (6, 2, 64, 1000, 3)])
def test_rotary_epilogue_of_the_qkv_projection(nq, nkv, d, seq, mb):
    """q|k|v after the rotary step, read back from the stash, against RMSNorm -> projection -> rotation in fp64 where
    only what the matrix unit needs is rounded to bf16: the normalised input before the projection and q|k|v once, after
    the rotation.  The shapes take the projection through every tiling of its kernel: (30, 2, 128) and (60, 4, 64) at
    4096 tokens give 17 column tiles of 256 = a full round of 256x256 tiles plus a 256x128 tail launch; 3000 tokens x
    1280 / 640 columns run on the 128x128 tiles with ragged rows.  The positions restart with every sequence of the
    micro-batch."""
    import paper_2410_13333_amd as mls
    import oracle.stage as O
    sh = synth.StageShape(hidden=256, n_q_heads=nq, n_kv_heads=nkv, head_dim=d, ffn=64, seq=seq, micro_batch=mb,
                          layers=1, microbatches=1)
    st = mls.Stage.from_shape(sh, seed=1000)
    xbits, x = synth.make_x(sh, 2000, 0)
    xd = to_device(xbits, "bf16")
    import torch
    y = torch.empty_like(xd)
    st.forward(xd, 1, y)
    got = to_host64(st.debug_read("qkv"))
    st.close()
    _, p64 = synth.make_params(sh, 1000)
    w = synth.split_params(sh, p64, 0)
    a, _ = O.rmsnorm_fwd(x.reshape(seq * mb, sh.hidden), w["gamma1"], sh.rms_eps)
    pre = round_bf16(a) @ w["w_qkv"]
    qd, kvd = nq * d, nkv * d
    rot = O.rope_apply(pre[:, :qd + kvd].reshape(mb, seq, nq + nkv, d), O.rope_angles(seq, d, sh.rope_base))
    ref = round_bf16(np.concatenate([rot.reshape(seq * mb, qd + kvd), pre[:, qd + kvd:]], axis=1))
    # one rounding on each side; what is left are the elements whose fp32 and fp64 values round to different
    # neighbours (a bf16 step is 2^-8 of the value, and the normalised input already differs that way now and then)
    for name, lo, hi in (("q", 0, qd), ("k", qd, qd + kvd), ("v", qd + kvd, qd + 2 * kvd)):
        e = rel_err(got[:, lo:hi], ref[:, lo:hi])
        print(f"[rotary epilogue nq={nq} d={d}] {name}: {e:.2e}")
        assert e <= 2e-3, (name, e)
    # per-head check on the last head of k and the last rows: a wrong pairing or position would be O(1) there
    assert rel_err(got[-64:, qd + kvd - d:qd + kvd], ref[-64:, qd + kvd - d:qd + kvd]) <= 2e-3
