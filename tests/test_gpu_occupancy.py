"""W(c), the "SM" of Eq. 6 on this chip (Sec. 4.2): the static wave capacity the cost model uses (derived from what
the compiler reported for each kernel when the library was built) against the HIP runtime's own answer on the device."""
import pytest
import torch

from paper_2604_26039_amd import ramp, synth

pytestmark = pytest.mark.gpu


def test_wave_capacity_agrees_with_the_runtime_occupancy():
    torch.zeros(1, device="cuda:0")
    seen = {}
    for s in synth.SHAPES.values():
        for c in ramp.configs(ramp.Shape(64, s.k, s.E, s.H, s.I)):
            seen.setdefault(c.key(), c)
    assert len(seen) >= 50
    for key, c in seen.items():
        static = ramp.config_wave_capacity(c) // 256
        up, down = ramp.config_runtime_occupancy(c)
        assert up >= 1 and down >= 1, key
        if c.mode & 0x400:
            assert static == 1, key          # persistent kernels launch one workgroup per compute unit
        else:
            assert static == up, f"{key}: static {static}, runtime {up} (up-projection) / {down} (down-projection)"
