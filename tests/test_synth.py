"""The input generator: storage formats and reproducibility (no method arithmetic lives there)."""
import numpy as np

import moe_synth as S


def test_bf16_round_to_nearest_even():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -2.5, 0.0], np.float32)
    b = S.f32_to_bf16_bits(f)
    back = S.bf16_bits_to_f32(b)
    assert list(back) == [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7, -2.5, 0.0]
    assert S.to_f64(b).dtype == np.float64 and np.array_equal(S.to_f64(b), back.astype(np.float64))


def test_draws_are_reproducible_and_shaped():
    w = S.WORKLOADS["tiny"]
    a, b = S.draw_all(w), S.draw_all(w)
    for name in ("x", "w_gate", "w1", "w2", "dy"):
        assert np.array_equal(a[name], b[name])
    assert a["x"].shape == (256, 64) and a["w1"].shape == (4, 64, 128) and a["w2"].shape == (4, 128, 64)
    assert a["w3"] is None and a["b_gate"] is None
    assert abs(float(a["x"].std()) - 0.02) < 2e-3 and abs(float(a["w1"].std()) - 0.02) < 1e-3
    sw = S.scaled(S.WORKLOADS["switch"], N=64, M=16, H=32)
    bg = S.draw_b_gate(sw)
    assert bg.dtype == np.float32 and sorted(np.round(np.exp(-bg / 1.1)).astype(int)) == list(range(1, 33))
    g = S.scaled(S.WORKLOADS["gpt2"], N=32, M=16, H=32)
    assert S.draw_x(g).dtype == np.uint16
