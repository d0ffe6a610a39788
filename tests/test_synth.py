"""The seeded input generators: determinism, shapes, and bf16 rounding against torch's."""
import numpy as np
import pytest

from paper_2508_12594_amd import synth


def test_bf16_round_matches_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 4096),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], np.float32)])
    ours = synth.bf16_round(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours.view(np.uint32), ref.view(np.uint32))
    bits = synth.bf16_bits(ours)
    assert np.array_equal(synth.bf16_from_bits(bits), ours)
    with pytest.raises(ValueError):
        synth.bf16_bits(np.array([1.001], np.float32))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_shapes_and_determinism(cfg):
    a = synth.make_inputs(cfg, N=257, B=min(2, synth.CONFIGS[cfg]["B"]))
    b = synth.make_inputs(cfg, N=257, B=min(2, synth.CONFIGS[cfg]["B"]))
    c = synth.CONFIGS[cfg]
    assert a["q"].shape == (c["H"], c["M"], c["d"])
    assert a["k"].shape == (a["B"], c["H"], 257, c["d"]) == a["v"].shape
    assert ("dy" in a) == c["backward"]
    for name in ("q", "k", "v"):
        assert a[name].dtype == np.float32 and np.array_equal(a[name], b[name])
        assert np.isfinite(a[name]).all()
        if c["dtype"] == "bf16":
            assert not np.any(a[name].view(np.uint32) & 0xFFFF)
    assert abs(a["scale"] - c["d"] ** -0.5) < 1e-15
    # scores are O(1): the softmaxes are neither uniform nor one-hot
    s = a["scale"] * np.einsum("hmd,bhnd->bhmn", a["q"].astype(np.float64), a["k"].astype(np.float64))
    assert 0.3 < s.std() < 4.0
