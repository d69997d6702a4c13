"""The paper's cost-model claim on one GPU: stage step time is linear in layers x micro-batches (Sec. 4.2,
t = y * l * tau(b), step ~ m * max t; the paper reports a cost-model error of at most 6.3 %).  All sixteen seeded
plans at the real layer shape (layers 2..9, micro-batches 1..16, seq 2048), the single-micro-batch plan included; the
least-squares line t = alpha + tau * l * m must fit every plan within 5 %."""
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(400)
def test_stage_time_is_linear_in_layers_times_microbatches():
    import bench
    plans = synth.plan_sweep()
    assert len(plans) == 16 and min(m for _, m in plans) == 1
    out = bench.run_plan_sweep(plans, steps=3)
    worst = max(out["plans"], key=lambda p: abs(p["ms"] - (out["alpha_ms"] + out["tau_ms_per_layer_microbatch"] * p["layers"] * p["microbatches"])) / p["ms"])
    print(f"tau {out['tau_ms_per_layer_microbatch']:.3f} ms  alpha {out['alpha_ms']:.3f} ms  max residual "
          f"{out['max_relative_residual']:.4f} at {worst['layers']} x {worst['microbatches']}  R2 {out['r2']:.5f}")
    assert out["max_relative_residual"] <= 0.05
    assert out["r2"] >= 0.999
