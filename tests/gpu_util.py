"""Helpers of the GPU parity tests: upload numpy tensors, compare device results with the oracle."""
import numpy as np
import torch

import paper_1911_02497_amd as P

DEV = "cuda:0"

# The forms of the selection that every element-pruning and L-C case runs through, as per-call
# configurations (condensa_config fields): nothing process-wide is touched by the tests.
FORMS = {
    "auto": {"select_path": 0},          # what a caller gets: small calls finish on a list after the first radix level
    "radix": {"select_path": 1},
    "window": {"select_path": 2},
    "window_narrow": {"select_path": 2, "window_margin": 0},
    "window_two_sweeps": {"select_path": 2, "fused_sweep": 1},
}


class Form:
    """Configuration of the running test case; the fixtures of the test modules set and clear it."""
    config = None


def with_form(fn, **defaults):
    """The binding call ``fn`` with the running case's configuration passed as its ``config`` argument."""
    def call(*a, **k):
        k.setdefault("config", Form.config)
        for name, value in defaults.items():
            k.setdefault(name, value)
        return fn(*a, **k)
    return call


def up(arrs):
    return [torch.from_numpy(np.ascontiguousarray(a)).to(DEV) for a in arrs]


def bits32(x):
    if isinstance(x, torch.Tensor):
        x = x.cpu().numpy()
    return np.ascontiguousarray(x).view(np.uint32)


def assert_bits_equal(got, want, what=""):
    g, w = bits32(got), bits32(want)
    assert g.shape == w.shape, (what, g.shape, w.shape)
    if not np.array_equal(g, w):
        bad = np.flatnonzero(g.reshape(-1) != w.reshape(-1))
        raise AssertionError(f"{what}: {bad.size} of {g.size} differ, first at {bad[:5]}: "
                             f"got {g.reshape(-1)[bad[:5]]} want {w.reshape(-1)[bad[:5]]}")


def assert_select_equal(rec, want, what=""):
    for f in ("n", "k", "n_gt", "n_tie_kept", "n_tie", "threshold_key", "tie_end"):
        assert rec[f] == want[f], (what, f, rec, want)


def check_prune_against_oracle(res, ora, scope, n_tensors, what=""):
    """res: binding output of condensa_prune; ora: oracle.prune output (list over densities)."""
    recs = P.select_records(res["results"])
    for j, o in enumerate(ora):
        if scope == P.SCOPE_GLOBAL:
            assert_select_equal(recs[j], o["select"], f"{what} density {j}")
        else:
            for t in range(n_tensors):
                assert_select_equal(recs[j * n_tensors + t], o["select"][t], f"{what} density {j} tensor {t}")
        for t in range(n_tensors):
            if res["mask"] is not None:
                got = res["mask"][j][t].cpu().numpy()
                assert np.array_equal(got, o["mask"][t]), f"{what} mask d{j} t{t}: {int((got != o['mask'][t]).sum())} differ"
            if res["theta"] is not None:
                assert_bits_equal(res["theta"][j][t], o["theta"][t], f"{what} theta d{j} t{t}")
