"""The seeded input generator: determinism, distribution, exact bf16 rounding (no GPU)."""
import numpy as np
import torch

from paper_2502_08145_amd import synth


def test_counter_based_and_seeded():
    a = synth.normal_bf16(5, (64, 64))
    assert np.array_equal(a, synth.normal_bf16(5, (64, 64)))
    assert not np.array_equal(a, synth.normal_bf16(6, (64, 64)))
    # chunking does not change the stream
    assert np.array_equal(a, synth.normal_bf16(5, (64, 64), chunk=100))


def test_distribution_moments():
    v = synth.bf16_bits_to_f32(synth.normal_bf16(9, (512, 512))).astype(np.float64)
    assert abs(v.mean()) < 0.01 and abs(v.std() - 1.0) < 0.01
    w = synth.bf16_bits_to_f32(synth.normal_bf16(10, (512, 512), 0.02)).astype(np.float64)
    assert abs(w.std() - 0.02) < 0.0004
    assert np.isfinite(v).all() and np.isfinite(w).all()


def test_rne_rounding_matches_torch_cpu():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]   # ties and a tiny value
    ours = synth.f32_to_bf16_bits(x)
    theirs = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, theirs)
    back = synth.bf16_bits_to_f32(ours)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_integers_exact_and_in_range():
    b = synth.integer_bf16(3, (100, 100), -4, 4)
    v = synth.bf16_bits_to_f32(b)
    assert v.min() == -4 and v.max() == 4 and np.array_equal(v, np.round(v))


def test_workload_shapes():
    g = synth.workload("gpt5b_layer")
    assert len(g) == 12
    assert all(2 * x["M"] * x["N"] * x["K"] in (206158430208, 68719476736, 274877906944) for x in g)
    t = synth.fc_layer_tensors(8, 4, 6, 1)
    for op, lay in [("fwd", "NN"), ("bwd_data", "NT"), ("bwd_weight", "TN")]:
        a, b = synth.operands_for(op, lay, t)
        # natural modes use the cached buffers untouched
        assert a is t["X"] or a is t["dY"]
        assert b is t["W"] or b is t["dY"]
