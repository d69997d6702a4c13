"""Shared plumbing of the GPU parity tests: seeded inputs -> HIP stage and -> CPU oracle, error metric."""
import numpy as np

import synth
from oracle import stage as O


def rel_err(got, ref):
    """Relative Frobenius error, computed in fp64."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    n = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / n) if n > 0 else float(np.linalg.norm(got))


to_device = synth.to_device      # synth storage array -> CUDA tensor of the storage type


def to_host64(t):
    """CUDA tensor (bf16 / fp32) -> fp64 numpy."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def storage_bits(t):
    """CUDA tensor -> numpy array of its raw storage (uint16 for bf16, float32 otherwise)."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def round_bf16(t):
    _, v = synth.round_to_storage(np.ascontiguousarray(t).reshape(-1), "bf16")
    return v.reshape(t.shape)


def rounding_hook(names):
    """Hook for the oracle that rounds the named intermediate tensors (oracle.stage.ROUNDING_POINTS) to bf16 and
    leaves the others exact.  A CPU measuring device: how far do these roundings alone move a result."""
    names = frozenset(names)
    return lambda name, t: round_bf16(t) if name in names else t


def bf16_store(name, t):
    """Hook that rounds every named intermediate tensor to bf16."""
    return round_bf16(t)


def oracle_step(sh, wseed, xseed, dyseed, ks, params64=None, store=None):
    """Oracle stage step with per-micro-batch layer counts ks.  Returns (ys, dxs, grads flat fp64 [max_layers*P]).
    store: None = exact fp64 oracle; bf16_store = the oracle's storage-rounded mode."""
    if params64 is None:
        _, params64 = synth.make_params(sh, wseed)
    W = [synth.split_params(sh, params64, l) for l in range(sh.layers)]
    per = synth.layer_param_elems(sh)
    flat = np.zeros(sh.layers * per)
    ys, dxs = [], []
    for mb, k in enumerate(ks):
        _, x = synth.make_x(sh, xseed, mb)
        _, dy = synth.make_dy(sh, dyseed, mb)
        y, caches = O.stage_forward(x, W, sh, k, store)
        dx, grads = O.stage_backward(dy, W[:k], caches, sh, store)
        for l in range(k):
            for name, tid, r, c, off in synth.param_layout(sh):
                flat[l * per + off: l * per + off + r * c] += grads[l][name].reshape(-1)
        ys.append(y)
        dxs.append(dx)
    return ys, dxs, flat


def gpu_step(sh, wseed, xseed, dyseed, ks, interleave=False, stage=None):
    """HIP stage step on the same seeded inputs.  Returns (ys, dxs, grads fp64, stage)."""
    import torch
    import paper_2410_13333_amd as mls
    st = stage or mls.Stage.from_shape(sh, seed=wseed, max_inflight=max(1, len(ks)))
    n = len(ks)
    shape = (sh.micro_batch, sh.seq, sh.hidden)
    xs = [to_device(synth.make_x(sh, xseed, mb)[0], sh.dtype) for mb in range(n)]
    dy = torch.stack([to_device(synth.make_dy(sh, dyseed, mb)[0], sh.dtype) for mb in range(n)]) if n else \
        torch.empty((0,) + shape, dtype=st.tdtype, device="cuda")
    ys = [torch.empty(shape, dtype=st.tdtype, device="cuda") for _ in range(n)]
    dx = torch.empty_like(dy)
    grads = torch.zeros(st.grad_elems, dtype=torch.float32, device="cuda")
    if interleave:      # one-forward-one-backward order
        for mb in range(n):
            st.forward(xs[mb], ks[mb], ys[mb])
            st.backward(dy[mb:mb + 1], grads, 1, dx[mb:mb + 1])
    else:
        for mb in range(n):
            st.forward(xs[mb], ks[mb], ys[mb])
        st.backward(dy, grads, n, dx)
    torch.cuda.synchronize()
    return [to_host64(y) for y in ys], [to_host64(dx[i]) for i in range(n)], to_host64(grads), st


def grad_errors(sh, got, ref, layers):
    """max over parameter tensors of the per-tensor relative error; returns (max, dict)."""
    per = synth.layer_param_elems(sh)
    errs = {}
    for l in range(layers):
        for name, tid, r, c, off in synth.param_layout(sh):
            sl = slice(l * per + off, l * per + off + r * c)
            errs[(l, name)] = rel_err(got[sl], ref[sl])
    return max(errs.values()) if errs else 0.0, errs
