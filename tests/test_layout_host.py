"""The host-side converters between the row-major and the blocked matrix layout
(what every blocked-layout GPU test is checked through) against the formula
the header documents, element by element; numpy arrays and torch tensors."""
import numpy as np

from paper_1611_04581_amd import workloads as W


def test_layout_converters_are_inverse_and_match_the_documented_formula():
    k, b, nb = 3, 8, 4
    ld = b * nb
    a = np.arange(k * ld, dtype=np.float32).reshape(k, ld)
    blk = W.to_blocked(a, b)
    flat = blk.reshape(-1)
    for i in range(k):
        for j in range(ld):
            assert flat[(j // b) * k * b + i * b + j % b] == a[i, j]
    assert np.array_equal(W.from_blocked(blk, b), a)


def test_layout_converters_on_torch_tensors_match_numpy():
    import torch
    k, b, nb = 5, 16, 3
    a = np.random.default_rng(0).standard_normal((k, b * nb)).astype(np.float32)
    t = torch.from_numpy(a)
    assert np.array_equal(W.to_blocked(t, b).numpy(), W.to_blocked(a, b))
    assert np.array_equal(W.from_blocked(W.to_blocked(t, b), b).numpy(), a)
