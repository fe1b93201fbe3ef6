"""The synthetic-input generator: bit-reproducible, right moments, right shapes."""
import numpy as np
import pytest
import torch

from paper_2501_10375_amd import synth


def test_tensor_elements_match_the_scalar_reference():
    t = synth.normal((5, 7), seed=3, tensor_id=synth.TID_W1, std=1.0, dtype=torch.float32)
    flat = t.flatten()
    for i in (0, 1, 6, 17, 34):
        want = np.float32(synth.element_py(3, synth.TID_W1, i)) * np.float32(1.0 / 131072.0)
        assert flat[i].item() == want
    assert abs(synth.element_py(3, synth.TID_W1, 0)) < 786420


def test_chunking_does_not_change_values():
    a = synth.normal((1000,), 0, 1, 0.5, torch.float32)
    b = synth.normal((1000,), 0, 1, 0.5, torch.float32, chunk=37)
    assert torch.equal(a, b)


def test_moments_and_independence_between_tensors():
    a = synth.normal((200000,), 0, synth.TID_X, 1.0, torch.float32)
    b = synth.normal((200000,), 0, synth.TID_WG, 1.0, torch.float32)
    assert abs(a.mean().item()) < 0.01 and abs(a.std().item() - 1.0) < 0.01
    assert abs((a * b).mean().item()) < 0.01
    assert abs((a[1:] * a[:-1]).mean().item()) < 0.01
    assert a.abs().max().item() <= 6.0
    k = ((a ** 4).mean() / (a ** 2).mean() ** 2).item()  # Irwin-Hall(12) kurtosis = 3 - 0.1
    assert abs(k - 2.9) < 0.05


def test_bf16_rounding_is_round_to_nearest_even_of_the_fp32_value():
    a32 = synth.normal((4096,), 1, 2, 0.3, torch.float32)
    a16 = synth.normal((4096,), 1, 2, 0.3, torch.bfloat16)
    assert torch.equal(a16, a32.to(torch.bfloat16))
    bits = synth.to_numpy(a16)
    assert bits.dtype == np.uint16 and bits.shape == (4096,)


def test_zipf_bias():
    b = synth.zipf_gate_bias(8, 1.2)
    assert b[0].item() == 0.0 and torch.all(b[1:] < b[:-1])
    p = synth.zipf_gate_bias(8, 1.2, perm_seed=5)
    assert torch.equal(torch.sort(p, descending=True).values, b)


@pytest.mark.gpu
def test_gpu_generator_matches_cpu_bits():
    a = synth.normal((3, 1001), 7, synth.TID_W2, 0.02, torch.bfloat16, device="cuda")
    b = synth.normal((3, 1001), 7, synth.TID_W2, 0.02, torch.bfloat16, device="cpu")
    assert torch.equal(a.cpu(), b)
