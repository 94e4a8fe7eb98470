"""Host-side checks of the seeded workload generator (CPU only)."""
import numpy as np
import torch

from paper_2306_15799_amd import inputs


def test_bf16_rounding_matches_torch_round_to_nearest_even():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(20000) * 10 ** rng.uniform(-6, 6, 20000)).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]      # exact ties and zero
    got = inputs.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, ref)
    bits = inputs.bf16_bits(got)
    assert bits.dtype == np.uint16
    assert np.array_equal(inputs.bf16_bits_to_f32(bits), got)


def test_workload_shapes_scales_and_determinism():
    w = inputs.shrink(inputs.WORKLOADS["C5"], B=2, H=3, n=256, k=32, m=16)
    a = inputs.make_inputs(w, seed=0)
    b = inputs.make_inputs(w, seed=0)
    c = inputs.make_inputs(w, seed=1)
    for key in ["Q", "K", "V", "E", "F", "omega", "dOut"]:
        assert np.array_equal(a[key], b[key])
        assert not np.array_equal(a[key], c[key])
        assert np.array_equal(a[key], inputs.round_to_bf16(a[key]))   # bf16-exact
    assert a["Q"].shape == (2, 3, 256, 64) and a["E"].shape == (32, 256)
    assert a["omega"].shape == (3, 16, 64)
    assert abs(a["Q"].std() - 64 ** -0.25) < 0.01
    assert abs(a["E"].std() - 32 ** -0.5) < 0.01
    assert abs(a["omega"].std() - 1.0) < 0.05
    assert abs(a["dOut"].std() - 1.0) < 0.02


def test_named_workloads_follow_the_benchmark_table():
    W = inputs.WORKLOADS
    assert (W["C1"].B, W["C1"].H, W["C1"].n, W["C1"].d, W["C1"].k, W["C1"].m, W["C1"].dtype) == (1, 1, 512, 64, 64, 64, "f32")
    assert (W["C2"].B, W["C2"].H, W["C2"].n, W["C2"].d, W["C2"].k, W["C2"].m) == (8, 8, 4096, 64, 256, 256)
    assert (W["C3"].B, W["C3"].H, W["C3"].n, W["C3"].d, W["C3"].k, W["C3"].phi) == (4, 16, 16384, 64, 256, inputs.PHI_ELU1)
    assert (W["C4"].B, W["C4"].H, W["C4"].n, W["C4"].d, W["C4"].k, W["C4"].m) == (1, 16, 65536, 128, 512, 256)
    assert (W["C5"].B, W["C5"].H, W["C5"].n, W["C5"].d, W["C5"].k, W["C5"].m, W["C5"].backward) == (4, 12, 8192, 64, 256, 256, True)
    assert inputs.make_inputs(inputs.shrink(W["C3"], B=1, H=1, n=64, k=8))["omega"] is None
