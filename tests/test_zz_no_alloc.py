"""mls_head_forward_static (the entry point for callers that cannot allocate: its kernels' scratch is a fixed array
inside the library) against mls_head_forward, through the C ABI: loss and logits gradient bit for bit, on two calls
in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

import synth
from tests.helpers import storage_bits, to_device

pytestmark = pytest.mark.gpu

BIG = synth.EndsShape(hidden=184, vocab=1384, seq=75, micro_batch=2, microbatches=1)       # 150 tokens, ragged
SMALL = synth.EndsShape(hidden=64, vocab=520, seq=37, micro_batch=1, microbatches=1)       # 37 tokens


def _inputs(sh, mb):
    import torch
    tgt = synth.make_targets(sh, 2200, mb).reshape(-1).copy()
    tgt[0] = -100                                                                          # an ignored target
    ysh = synth.StageShape(sh.hidden, 1, 1, 64, 8, sh.seq, sh.micro_batch, 1, 1, dtype=sh.dtype)
    ybits, _ = synth.make_x(ysh, 2300, mb)
    return to_device(ybits, sh.dtype), torch.from_numpy(tgt).cuda()


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_static_scratch_head_forward_equals_the_allocating_one(dtype):
    import torch
    import paper_2410_13333_amd as mls
    for sh in (BIG.with_(dtype=dtype), SMALL.with_(dtype=dtype)):     # two calls in a row, the second smaller
        ref = mls.Ends.from_shape(sh, seed=1100, max_inflight=1)
        new = mls.Ends.from_shape(sh, seed=1100, max_inflight=1)
        y, tgt = _inputs(sh, 0)
        loss = torch.full((2,), float("nan"), dtype=torch.float32, device="cuda")
        ref.head_forward(y, tgt, 0.5, loss[0:1])
        new.head_forward_static(y, tgt, 0.5, loss[1:2])
        torch.cuda.synchronize()
        l = loss.cpu().numpy()
        assert np.isfinite(l).all() and l[0] == l[1], l
        assert np.array_equal(storage_bits(ref.debug_dlogits(0)), storage_bits(new.debug_dlogits(0)))
        assert new.inflight == (0, 1)
        ref.close()
        new.close()


def test_static_scratch_rejects_more_tokens_than_it_holds():
    import torch
    import paper_2410_13333_amd as mls
    sh = synth.EndsShape(hidden=8, vocab=8, seq=65544, micro_batch=1, microbatches=1, dtype="fp32")
    en = mls.Ends.from_shape(sh, seed=1, max_inflight=1)
    y = torch.zeros((1, sh.seq, sh.hidden), dtype=torch.float32, device="cuda")
    tgt = torch.zeros(sh.seq, dtype=torch.int32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    with pytest.raises(mls.MlsError) as ei:
        en.head_forward_static(y, tgt, 1.0, loss)
    assert "65536" in str(ei.value)
    en.head_forward(y, tgt, 1.0, loss)          # the allocating entry point takes it
    torch.cuda.synchronize()
    assert abs(float(loss[0]) - np.log(8.0)) < 1e-5   # zero inputs: uniform prediction
    en.close()
