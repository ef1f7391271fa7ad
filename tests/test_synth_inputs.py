"""CPU-only checks of the seeded input recipes."""
import numpy as np
import torch

from paper_2501_17086_amd import synth


def test_bf16_rounding_matches_torch():
    a = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    a[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]   # ties
    want = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    np.testing.assert_array_equal(synth.round_bf16(a), want)


def test_inputs_are_seeded_and_subsets_agree():
    w = synth.scaled(synth.WORKLOADS["resnet_like"], L=3, N=40, d=64, d_ff=128)
    a = synth.make_inputs(w)
    b = synth.make_inputs(w)
    for k in a:
        if a[k] is not None:
            np.testing.assert_array_equal(a[k], b[k])
    sub = synth.make_inputs(w, tokens=slice(8, 24))
    np.testing.assert_array_equal(sub["x0"], a["x0"][8:24])
    np.testing.assert_array_equal(sub["e"], a["e"][8:24])
    np.testing.assert_array_equal(sub["W1"], a["W1"])
    assert a["lam"].shape == (3, 64) and a["lam"].min() >= 0.9 and a["lam"].max() <= 1.0
    # bf16 storage: values survive a round trip
    np.testing.assert_array_equal(synth.round_bf16(a["W2"]), a["W2"])


def test_rnn_recipe():
    w = synth.scaled(synth.WORKLOADS["gated_rnn"], L=6, N=4, d=64, d_ff=64, d_in=32)
    a = synth.make_inputs(w)
    assert a["W1"].shape == (64, 64) and a["U"].shape == (64, 32)
    assert a["xin"].shape == (6, 4, 32) and a["e"].shape == (7, 4, 64)
    assert np.all(a["e"][0] == 0) and np.all(a["x0"] == 0)
    assert 0.5 < a["lam"].min() and a["lam"].max() < 1.0
    sub = synth.make_inputs(w, tokens=slice(1, 3))
    np.testing.assert_array_equal(sub["xin"], a["xin"][:, 1:3])


def test_weight_statistics():
    w = synth.WORKLOADS["transformer_mlp"]
    W1, W2 = synth.weights_block(w, 3)
    assert abs(W1.std() - 0.02) < 1e-3
    assert abs(W2.std() - 0.02 / np.sqrt(96.0)) < 2e-4
    w = synth.WORKLOADS["resnet_like"]
    W1, W2 = synth.weights_block(w, 0)
    assert abs(W1.std() - 1 / np.sqrt(512)) < 1e-3
    assert abs(W2.std() - 1 / np.sqrt(2048) / np.sqrt(32)) < 2e-4
