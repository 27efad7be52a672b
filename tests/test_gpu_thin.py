"""GPU parity: condensa_thin against the oracle's gather, fed by the GPU's own filter pruning."""
import numpy as np
import pytest
import torch

import oracle
import paper_1911_02497_amd as P
import workloads
from gpu_util import DEV, assert_bits_equal, up

pytestmark = pytest.mark.gpu


def test_thin_vgg_after_filter_pruning():
    """VGG-19 convs filter-pruned per layer at sparsity 0.79 (Table 2), then every layer loses its pruned
    filters and the input channels that its predecessor lost (a plain chain, no graph analysis needed)."""
    convs = workloads.vgg19_cifar()[:16]
    dev = up(convs)
    res = P.condensa_filter_prune(dev, 0.21, P.SCOPE_PER_TENSOR)
    torch.cuda.synchronize()
    ora = oracle.filter_prune(convs, 0.21, P.SCOPE_PER_TENSOR)
    recs = P.select_records(res["results"])
    first, pos = 0, 0
    prev_keep_dev, prev_keep_host, prev_first = None, None, 0
    for t, w in enumerate(convs):
        k = recs[t]["k"]
        keep_dev = res["keep_idx"][pos:pos + k].contiguous()
        keep_host = ora["keep_idx"][pos:pos + k] - first
        got = P.condensa_thin(dev[t], keep_dev, prev_keep_dev, keep_out_offset=first, keep_in_offset=prev_first)
        want = oracle.thin(convs[t], keep_host, prev_keep_host)
        assert got.shape == want.shape == (k, w.shape[1] if prev_keep_host is None else len(prev_keep_host), 3, 3)
        assert_bits_equal(got, want, f"layer {t}")
        prev_keep_dev, prev_keep_host, prev_first = keep_dev, keep_host, first
        first += w.shape[0]
        pos += k


def test_thin_linear_identity_and_guards():
    rng = np.random.default_rng(50)
    lin = rng.standard_normal((300, 77)).astype(np.float32)
    d = torch.from_numpy(lin).to(DEV)
    ko = torch.tensor([5, 299, 0, 17], dtype=torch.int32, device=DEV)
    ki = torch.arange(0, 77, 3, dtype=torch.int32, device=DEV)
    assert_bits_equal(P.condensa_thin(d, ko, ki), oracle.thin(lin, ko.cpu().numpy(), ki.cpu().numpy()), "linear")
    assert_bits_equal(P.condensa_thin(d), lin, "identity")
    assert P.condensa_thin(d, ko[:0], ki).shape == (0, 26)
    bad = torch.tensor([1, 300, -4], dtype=torch.int32, device=DEV)       # out-of-range ids give zeros
    got = P.condensa_thin(d, bad, None).cpu().numpy()
    assert np.array_equal(got[0], lin[1]) and np.all(got[1:] == 0)
    import ctypes
    shape = (ctypes.c_int64 * 4)(4, 4, 1, 1)
    assert P.library().condensa_thin(d.data_ptr(), shape, 1, None, 0, 0, None, 0, 0, d.data_ptr(), None) == -4   # ndim
    assert P.library().condensa_thin(d.data_ptr(), shape, 2, None, 0, 0, None, 0, 0, d.data_ptr(), None) == -6   # alias
