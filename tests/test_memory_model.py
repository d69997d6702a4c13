"""The stage's memory report (mls_stage_memory) and the layer cap of the linear memory model (Appendix B.4):
host code, no GPU."""
import pytest

import synth


def test_memory_report_is_linear_in_layers_and_kept_microbatches():
    import paper_2410_13333_amd as mls
    sh = synth.CONFIGS["7b"]
    base = mls.Stage.memory(sh, max_layers=4, max_inflight=4)
    assert base["total_bytes"] == base["param_bytes"] + base["stash_bytes"] + base["workspace_bytes"]
    a_f = base["stash_bytes_per_layer_microbatch"]
    assert base["stash_bytes"] == 4 * 4 * a_f
    # about 0.55 GB per layer and kept micro-batch at the 7B shape: x, a, qkv, o, h, b, gu, z (bf16, padded) + statistics
    T, h, f = 4096, 4096, 11008
    dense = 2 * T * (5 * h + 3 * h + 3 * f)
    assert dense <= a_f <= 1.03 * dense
    more_layers = mls.Stage.memory(sh, max_layers=6, max_inflight=4)
    assert more_layers["param_bytes"] - base["param_bytes"] == 2 * base["param_bytes_per_layer"]
    assert more_layers["stash_bytes"] == 6 * 4 * a_f and more_layers["workspace_bytes"] == base["workspace_bytes"]
    assert base["grad_bytes_per_layer"] == 4 * synth.layer_param_elems(sh)
    # bf16 weights plus the transposed copy of the four matrices that the data-gradient products read
    # (the gains have no copy): just under 4 bytes per parameter, plus padding
    P = synth.layer_param_elems(sh)
    assert 4 * (P - 2 * h) <= base["param_bytes_per_layer"] <= 4.06 * P


def test_recomputation_keeps_only_the_layer_inputs():
    import paper_2410_13333_amd as mls
    sh = synth.CONFIGS["7b"]
    full = mls.Stage.memory(sh, max_layers=4, max_inflight=4)
    rc = mls.Stage.memory(sh, max_layers=4, max_inflight=4, recompute=True)
    assert rc["stash_bytes_per_layer_microbatch"] * 15 < full["stash_bytes_per_layer_microbatch"]
    assert rc["param_bytes"] == full["param_bytes"]
    # the scratch entries the recomputed tensors live in: one full entry per kept micro-batch
    assert rc["workspace_bytes"] - full["workspace_bytes"] == 4 * full["stash_bytes_per_layer_microbatch"]
    assert rc["total_bytes"] < full["total_bytes"]


def test_layer_cap_closed_form_and_bad_input():
    import paper_2410_13333_amd as mls
    # mu = 2*(4-1) + 3 + 5 = 14; room = 100 - 10 - 6 = 84 -> 6 layers; one byte less room -> 5
    assert mls.plan_layer_cap(2, 3, 5, 6, 4, 1, 100, 10) == 6
    assert mls.plan_layer_cap(2, 3, 5, 6.5, 4, 1, 100, 10) == 5
    assert mls.plan_layer_cap(2, 3, 5, 6, 4, 4, 100, 10) == 10          # last stage keeps no earlier micro-batch
    assert mls.plan_layer_cap(2, 3, 5, 200, 4, 1, 100, 10) == 0
    assert mls.plan_layer_cap(2, 3, 5, 6, 4, 5, 100, 10) == -1 and mls.plan_layer_cap(0, 0, 0, 0, 1, 1, 1, 0) == -1


@pytest.mark.parametrize("pp,j", [(4, 1), (4, 3), (8, 8)])
def test_cap_from_the_report_is_the_largest_stage_that_fits(pp, j):
    """Close the loop: coefficients from mls_stage_memory -> mls_plan_layer_cap -> a stage with that many layers and
    pp - j + 1 kept micro-batches fits the capacity, one more layer does not (model states = parameters + fp32
    gradients + 12 B per parameter of optimizer state)."""
    import paper_2410_13333_amd as mls
    sh = synth.CONFIGS["7b"]
    C, G = 288e9, 4096 * 2 ** 20                      # HBM of an MI355X; the paper's reserved gap
    keep = pp - j + 1
    one = mls.Stage.memory(sh, max_layers=1, max_inflight=keep)
    a_f = one["stash_bytes_per_layer_microbatch"]
    s = one["param_bytes_per_layer"] + one["grad_bytes_per_layer"] + 12 * synth.layer_param_elems(sh)
    nu = one["workspace_bytes"]
    cap = mls.plan_layer_cap(a_f, a_f, s, nu, pp, j, C, G)
    assert cap > 0

    def need(layers):
        m = mls.Stage.memory(sh, max_layers=layers, max_inflight=keep)
        return m["total_bytes"] + layers * (m["grad_bytes_per_layer"] + 12 * synth.layer_param_elems(sh))
    assert need(cap) <= C - G < need(cap + 1)
