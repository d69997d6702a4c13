"""The seeded input generator: format conversion pinned to a library's bfloat16, statistics, layout."""
import numpy as np
import pytest

import synth


def test_bf16_round_matches_library_conversion():
    torch = pytest.importorskip("torch")
    a = (np.random.default_rng(0).standard_normal(100000) * np.logspace(-3, 3, 100000)).astype(np.float32)
    bits = synth.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    assert np.array_equal(synth.bf16_bits_to_f32(bits), torch.from_numpy(a).to(torch.bfloat16).float().numpy())
    # single rounding from fp64: a value whose fp32 rounding lands on a bf16 tie must not round twice
    v = np.array([1.0 + 2.0 ** -8 + 2.0 ** -30])           # just above the tie between 1 and 1+2^-7
    b, val = synth.round_to_storage(v, "bf16")
    assert val[0] == 1.0 + 2.0 ** -7
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -0.02 * (1 + 2.0 ** -8)])
    _, val = synth.round_to_storage(ties, "bf16")
    assert val.tolist() == [1.0, 1.0 + 2.0 ** -6, -0.02 * 1.0] or np.allclose(val, [1.0, 1.015625, -0.02], rtol=2 ** -8)


def test_normal_statistics_and_counter_addressing():
    z = synth.normal(1000, synth.TID_WQKV, 0, 1 << 20)
    assert abs(z.mean()) < 4e-3 and abs(z.std() - 1) < 4e-3
    assert abs(np.mean(z ** 3)) < 2e-2 and abs(np.mean(z ** 4) - 3) < 5e-2
    assert np.array_equal(z[1000:1010], synth.normal(1000, synth.TID_WQKV, 0, 10, start=1000))
    assert not np.array_equal(z[:10], synth.normal(1000, synth.TID_WQKV, 1, 10))
    assert not np.array_equal(z[:10], synth.normal(1001, synth.TID_WQKV, 0, 10))
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 5e-3


def test_param_layout_and_scales():
    sh = synth.CONFIGS["tiny"]
    lay = synth.param_layout(sh)
    assert [n for n, *_ in lay] == ["gamma1", "w_qkv", "w_o", "gamma2", "w_gu", "w_d"]
    assert synth.layer_param_elems(sh) == 2 * 256 + sh.matrix_params() == 2 * 256 + 790528
    bits, vals = synth.make_params(sh, 1000)
    assert bits.dtype == np.uint16 and bits.size == 2 * synth.layer_param_elems(sh)
    w = synth.split_params(sh, vals, 1)
    assert w["w_qkv"].shape == (256, 768) and w["w_gu"].shape == (256, 1376) and w["w_d"].shape == (688, 256)
    assert abs(w["w_gu"].std() - 0.02) < 5e-4 and abs(w["gamma1"].mean() - 1) < 5e-3
    f32, vals32 = synth.make_params(sh.with_(dtype="fp32"), 1000)
    assert f32.dtype == np.float32 and np.max(np.abs(vals32 - vals)) < 0.03 * 2 ** -8 + 1.2 * 2 ** -8
    assert synth.CONFIGS["7b"].model_flops_layer_mb() * 16 == pytest.approx(8.618e13, rel=1e-3)


def test_plan_sweep_ranges():
    plans = synth.plan_sweep()
    assert len(plans) == 16 and all(2 <= k <= 9 and 1 <= m <= 16 for k, m in plans)
    assert plans == synth.plan_sweep()
