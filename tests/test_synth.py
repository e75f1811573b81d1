"""The input generators: seeded, shaped and distributed as stated, and free of method arithmetic."""
import numpy as np

from paper_2512_19720_amd import synth


def test_host_layer_is_deterministic_and_distributed_as_stated():
    a = synth.layer_host(256, 512, 4, synth.F16, "row", synth.seed_for(0))
    b = synth.layer_host(256, 512, 4, synth.F16, "row", synth.seed_for(0))
    for k in ("W_b", "dW", "X"):
        assert a[k].dtype == np.uint16 and np.array_equal(a[k], b[k])
    W = a["W_b"].view(np.float16).astype(np.float64)
    assert abs(W.std() - 0.02) < 5e-4 and abs(W.mean()) < 2e-4
    X = a["X"].view(np.float16).astype(np.float64)
    assert X.shape == (4, 512) and abs(X.std() - 1.0) < 0.05
    d = a["dW"].view(np.float16).astype(np.float64)
    row_rms = np.sqrt((d ** 2).mean(axis=1))
    assert abs(np.log(row_rms).mean() - np.log(1e-3)) < 0.15      # lognormal around 1e-3
    assert 0.35 < np.log(row_rms).std() < 0.65
    c = synth.layer_host(256, 512, 4, synth.F16, "col", synth.seed_for(0))
    col_rms = np.sqrt((c["dW"].view(np.float16).astype(np.float64) ** 2).mean(axis=0))
    assert 0.35 < np.log(col_rms).std() < 0.65


def test_zero_fraction_and_fine_tuned_matrix():
    L = synth.layer_host(128, 256, 1, synth.F16, "row", synth.seed_for(4), zero_frac=0.05, with_wf=True)
    d = L["dW"].view(np.float16)
    assert 0.03 < (d == 0).mean() < 0.08
    wf = L["W_f"].view(np.float16).astype(np.float32)
    want = (L["W_b"].view(np.float16).astype(np.float32) + d.astype(np.float32)).astype(np.float16)
    assert np.array_equal(wf, want.astype(np.float32))


def test_bf16_round_trip_matches_torch():
    import torch
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32) * 3
    bits = synth.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), want.view(torch.int16).numpy())
    assert np.array_equal(synth.bf16_bits_to_f32(bits), want.float().numpy())
    t = synth.bits_to_torch(bits, synth.BF16, "cpu")
    assert t.dtype == torch.bfloat16 and np.array_equal(synth.torch_to_bits(t), bits)


def test_stack_has_224_linears_and_the_stated_weight_count():
    shapes = synth.stack_shapes()
    assert len(shapes) == 224
    assert sum(o * i for _, o, i, _ in shapes) == 6_476_005_376
    assert shapes[0][3] == "row" and shapes[7][3] == "col"


def test_device_generator_runs_on_cpu_device_too():
    L = synth.layer_device(64, 128, synth.F16, "col", 5, "cpu", zero_frac=0.05, with_wf=True)
    assert L["W_b"].shape == (64, 128) and L["W_f"].dtype == L["W_b"].dtype
    assert 0.02 < (L["dW"] == 0).float().mean().item() < 0.09
