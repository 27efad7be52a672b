"""Pins for the oracle's thinning gather (CPU only).

Section 3.4 (Network Thinning): zero structures left by structure pruning are physically removed and
the tensor dimensions of the successors are adjusted.  Pins: numpy fancy indexing, and functional
equivalence of a two-layer convolution before and after thinning (torch's CPU conv2d in float64).
"""
import numpy as np
import torch

import oracle


def test_thin_is_a_gather_along_the_first_two_dimensions():
    rng = np.random.default_rng(40)
    t = rng.standard_normal((7, 5, 3, 3)).astype(np.float32)
    ko, ki = [0, 2, 6], [4, 1]
    got = oracle.thin(t, ko, ki)
    assert got.shape == (3, 2, 3, 3)
    assert np.array_equal(got, t[np.ix_(ko, ki)])
    assert np.array_equal(oracle.thin(t, ko, None), t[ko])
    assert np.array_equal(oracle.thin(t, None, ki), t[:, ki])
    assert np.array_equal(oracle.thin(t, None, None), t)
    lin = rng.standard_normal((6, 9)).astype(np.float32)
    assert np.array_equal(oracle.thin(lin, [5, 1], [0, 8, 3]), lin[np.ix_([5, 1], [0, 8, 3])])
    assert oracle.thin(t, [], ki).shape == (0, 2, 3, 3)


def test_thinned_network_computes_the_same_function():
    """Filter-prune layer 1, thin it and the input channels of layer 2: same output as the masked network."""
    rng = np.random.default_rng(41)
    w1 = rng.standard_normal((8, 3, 3, 3)).astype(np.float32)
    w2 = rng.standard_normal((5, 8, 3, 3)).astype(np.float32)
    x = torch.from_numpy(rng.standard_normal((2, 3, 10, 10))).double()
    res = oracle.filter_prune([w1], 0.5)
    keep = res["keep_idx"]
    assert len(keep) == 4
    full = torch.nn.functional.conv2d(torch.nn.functional.conv2d(x, torch.from_numpy(res["theta"][0]).double(), padding=1),
                                      torch.from_numpy(w2).double(), padding=1)
    t1 = oracle.thin(w1, keep, None)
    t2 = oracle.thin(w2, None, keep)
    thin = torch.nn.functional.conv2d(torch.nn.functional.conv2d(x, torch.from_numpy(t1).double(), padding=1),
                                      torch.from_numpy(t2).double(), padding=1)
    assert torch.allclose(full, thin, rtol=1e-12, atol=1e-12)
    assert t1.size + t2.size == (w1.size + w2.size) // 2
