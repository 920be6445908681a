"""Input generator: determinism, storage rounding, distribution recipe."""
import numpy as np

from paper_2406_04984_amd import synth


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 0.0], np.float32)
    assert [hex(v) for v in synth.bf16_round(x)] == ["0x3f80", "0x3f80", "0x3f82", "0xc020", "0x7f62", "0x0"]
    assert (synth.bf16_to_f32(synth.bf16_round(x))[:4] == np.array([1.0, 1.0, 1.015625, -2.5], np.float32)).all()


def test_tensors_are_reproducible_and_independent():
    c = synth.CONFIGS["tiny_f32"]
    a, b = synth.make_inputs(c), synth.make_inputs(c)
    for n in ("h", "Wg", "K", "V", "dOut"):
        assert (getattr(a, n) == getattr(b, n)).all()
    assert (synth.make_tensor(c, "V") == a.V).all()
    assert abs(np.corrcoef(a.K.ravel(), a.V.ravel())[0, 1]) < 0.02


def test_recipe_small_bf16():
    c = synth.CONFIGS["small_bf16"]
    h = synth.make_tensor(c, "h")
    ch = synth.outlier_channels(c)
    assert ch.size == 10
    rest = np.setdiff1d(np.arange(c.d), ch)
    assert abs(h[:, rest].std() - 1.0) < 0.02 and abs(h[:, ch].std() - 8.0) < 0.2
    Wg = synth.make_tensor(c, "Wg")
    assert abs(Wg.std() * np.sqrt(c.d) - 1.0) < 0.02
    assert (synth.bf16_to_f32(synth.bf16_round(h)) == h).all()


def test_zipf_bias():
    c = synth.CONFIGS["wide_bf16"]
    b = synth.router_bias(c)
    assert b.shape == (256,) and np.isclose(b.max(), 0.0) and np.isclose(b.min(), -1.1 * np.log(256), rtol=1e-6)
    assert synth.router_bias(synth.CONFIGS["tiny_f32"]) is None
