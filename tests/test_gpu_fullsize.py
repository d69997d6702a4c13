"""Full-size parity: one layer x one micro-batch at the real 7B, 13B and 70B-shard (grouped KV heads) shapes, i.e.
every kernel in exactly the launch configuration the benchmark times, compared with the fp64 oracle on the
same seeded bf16 inputs: the full y, dX and every parameter gradient (tolerance 1e-2, relative Frobenius)."""
import time

import numpy as np
import pytest

import synth
from tests.helpers import bf16_store, gpu_step, grad_errors, oracle_step, rel_err

pytestmark = pytest.mark.gpu


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
    # (kind, store hook, tolerance).  Against the exact oracle the 7B layer meets 1e-2.  For the wider layers rounding
    # every stored tensor to bf16 ALONE moves the result past 1e-2 from the exact one (oracle's storage-rounded mode
    # vs its exact mode: dX by 1.2e-2 for the 70B shard, hidden 8192; the QKV-side gradients by about 1e-2 for 13B,
    # hidden 5120), so the exact distance is bounded by 1.5e-2 / 2e-2 there and the sharp check is the one against the
    # storage-rounded mode.
    exact_tol = {"7b": 1e-2, "13b": 1.5e-2, "70b_tp4": 2e-2}[name]
    for kind, store, tol in (("exact", None, exact_tol), ("stored", bf16_store, 1e-2)):
        t0 = time.time()
        rys, rdxs, rg = oracle_step(sh, 1001, 2001, 3001, [1], params64=p64, store=store)
        ey, ex = rel_err(ys[0], rys[0]), rel_err(dxs[0], rdxs[0])
        eg, errs = grad_errors(sh, g, rg, 1)
        print(f"[{name}] vs {kind} oracle ({time.time() - t0:.1f} s): y={ey:.2e} dx={ex:.2e} grads(max)={eg:.2e}", flush=True)
        assert ey <= tol and ex <= tol, (kind, ey, ex)
        assert eg <= tol, (kind, sorted(errs.items(), key=lambda kv: -kv[1])[:3])
