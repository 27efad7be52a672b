"""GPU parity: condensa_prune against the oracle (masks, thetas, fp16 thetas, records bit exact)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1911_02497_amd as P
import workloads
from gpu_util import assert_bits_equal, assert_select_equal, check_prune_against_oracle, DEV, Form, FORMS, up, with_form

pytestmark = pytest.mark.gpu

prune = with_form(P.condensa_prune)


@pytest.fixture(params=["auto", "radix", "window", "window_narrow", "window_two_sweeps"], autouse=True)
def select_path(request):
    """Every case runs through the automatic choice (small calls: the first radix level, then a list of the
    keys around the thresholds), the radix levels, the sampled window (selection and apply in one sweep
    where the call allows it), a window whose margin is cut to a couple of sample ranks so that it
    regularly misses and falls back, and the window with separate selection and apply sweeps."""
    Form.config = FORMS[request.param]
    yield request.param
    Form.config = None


def _prune_both(arrs, densities, scope=P.SCOPE_GLOBAL, what="", **kw):
    res = prune(up(arrs), densities, scope=scope, **kw)
    torch.cuda.synchronize()
    ora = oracle.prune(arrs, densities, scope)
    check_prune_against_oracle(res, ora, scope, len(arrs), what)
    return res, ora


def test_single_matrix_density_002_with_fp16():
    (w,) = workloads.single_matrix()
    res, ora = _prune_both([w], [0.02], theta_f16=True)
    rec = P.select_records(res["results"])[0]
    assert rec["k"] == 20972 and int(res["mask"][0][0].sum().item()) == 20972
    q = res["theta_f16"][0][0].cpu().numpy().view(np.uint16)
    oq, _ = oracle.quantize_f16(ora[0]["theta"][0])
    assert np.array_equal(q, oq)
    # unfused: prune then quantize gives the same bits
    q2, _ = P.condensa_quantize(res["theta"][0][0])
    assert np.array_equal(q2.cpu().numpy().view(np.uint16), oq)


CASES = {
    "all_equal": [np.full(1000, 0.5, np.float32)],
    "all_zero": [np.zeros(777, np.float32)],
    "signed_zeros": [np.tile(np.array([0.0, -0.0, 1.0, -0.0], np.float32), 300)],
    "few_values_many_ties": [np.random.default_rng(1).integers(-3, 4, 20001).astype(np.float32)],
    "inf_nan_denormal": [np.array([1.0, np.inf, -np.inf, np.nan, 0.0, -3.0, 1e-40, -1e-40, 2e-45] * 5, np.float32)],
    "ragged_multi": [np.random.default_rng(2).standard_normal(s).astype(np.float32)
                     for s in ((8192 * 2 + 5,), (1,), (3, 7), (0,), (4, 3, 3, 3), (8192,), (8193,))],
    "spans_many_chunks": [np.random.default_rng(3).standard_normal(8192 * 37 + 11).astype(np.float32)],
    "empty_first_and_last": [np.zeros((0,), np.float32), np.arange(100, dtype=np.float32), np.zeros((0, 4), np.float32)],
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("scope", [P.SCOPE_GLOBAL, P.SCOPE_PER_TENSOR])
def test_adversarial_shapes(name, scope):
    arrs = CASES[name]
    _prune_both(arrs, [0.0, 0.001, 0.1, 0.5, 0.9, 1.0], scope=scope, what=name)


def test_ties_planted_across_tensors_and_chunks():
    rng = np.random.default_rng(4)
    a = rng.standard_normal(8192 * 3).astype(np.float32)
    b = rng.standard_normal(5000).astype(np.float32)
    t = np.float32(0.731)
    for arr, pos in ((a, [5, 8191, 8192, 20000]), (b, [0, 4999, 77])):
        for p in pos:
            arr[p] = t if p % 2 else -t
    n = a.size + b.size
    n_gt = int((np.abs(np.concatenate([a, b])) > t).sum())
    for extra in (1, 3, 6, 7):                      # keep only some of the 7 tied magnitudes
        d = (n_gt + extra) / n
        res, ora = _prune_both([a, b], [d])
        assert ora[0]["select"]["n_tie"] == 7 and ora[0]["select"]["n_tie_kept"] == extra


def test_vgg19_shapes_ten_densities_one_call():
    ws = workloads.vgg19_cifar()
    assert sum(w.size for w in ws) == 20024000
    ds = workloads.search_densities()
    dev = up(ws)
    res = prune(dev, ds, theta=False, mask=False)          # thresholds only
    torch.cuda.synchronize()
    ora = oracle.prune(ws, ds)
    recs = P.select_records(res["results"])
    for j in range(len(ds)):
        assert_select_equal(recs[j], ora[j]["select"], f"density {j}")
    # the masks of all ten densities from one call (one selection, one apply sweep writing ten masks)
    res = prune(dev, ds, theta=False, mask=True)
    torch.cuda.synchronize()
    recs = P.select_records(res["results"])
    for j in range(len(ds)):
        assert_select_equal(recs[j], ora[j]["select"], f"density {j} (mask call)")
        for t in range(len(ws)):
            assert np.array_equal(res["mask"][j][t].cpu().numpy(), ora[j]["mask"][t]), f"mask of density {j}, tensor {t}"


def test_in_place_and_misaligned():
    rng = np.random.default_rng(6)
    w = rng.standard_normal(30011).astype(np.float32)
    ora = oracle.prune([w], [0.3])[0]
    dw = torch.from_numpy(w).to(DEV)
    res = prune([dw], [0.3], in_place=True)
    assert_bits_equal(dw, ora["theta"][0], "in place")
    big = torch.from_numpy(np.concatenate([[9.0], w]).astype(np.float32)).to(DEV)
    res = prune([big[1:]], [0.3])
    assert_bits_equal(res["theta"][0][0], ora["theta"][0], "misaligned input")
    assert np.array_equal(res["mask"][0][0].cpu().numpy(), ora["mask"][0])


def test_argument_errors_have_no_side_effects():
    w = torch.ones(16, device=DEV)
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(P.CondensaError) as e:
            prune([w], [bad])
        assert e.value.code == -3
    with pytest.raises(P.CondensaError) as e:
        prune([w], [0.5] * 17)
    assert e.value.code == -2
    with pytest.raises(P.CondensaError) as e:
        prune([w], [0.5], workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == -5
    with pytest.raises(P.CondensaError) as e:
        prune([w], [0.5], scope=7)
    assert e.value.code == -6
    assert torch.all(w == 1)


@pytest.mark.parametrize("levels,n", [(8, (1 << 22) + 12345), (256, (1 << 24) + 77), (3, 300001)])
def test_few_distinct_values_far_apart(levels, n, select_path):
    """Quantised-looking weights: few distinct magnitudes, far apart in key space, each with a huge number
    of ties.  With 256 levels (16M weights) the sampled window spans a few levels whose keys are ~2^19
    apart and the ~65000 ties at the threshold are only partly kept (index search on the tie list); with
    8 or 3 levels one level alone overflows the candidate list and the radix levels take over."""
    rng = np.random.default_rng(levels)
    table = (0.37 * (1.9 if levels <= 8 else 1.05) ** np.arange(levels)).astype(np.float32)
    w = (table[rng.integers(0, levels, n)] * rng.choice(np.array([-1.0, 1.0], np.float32), n)).astype(np.float32)
    for density in ((0.5, 0.123) if levels == 256 else (0.5, 1.0 / levels, 0.123, 0.999)):
        res, _ = _prune_both([w[: n // 3], w[n // 3:]], [density], what=f"{levels} levels d={density}")
        if select_path in ("window", "window_two_sweeps") and levels == 256:
            assert P.select_records(res["results"])[0]["path"] == 2, "expected to resolve inside the window"


@pytest.mark.parametrize("cluster,ties", [(600, 9), (3000, 300), (3000, 700), (20000, 40), (300000, 2)])
def test_ties_among_keys_that_agree_on_all_but_the_last_digit(cluster, ties):
    """The radix levels list the keys that agree with a threshold on every digit but the last and usually find
    the ties in that list.  Clusters of `cluster` magnitudes whose bit patterns differ only in their low ten
    bits, with `ties` copies of one of them, exercise the list (few keys, few ties), the ranking of several
    hundred ties inside it, more ties than the list resolves, more keys than the list holds, and more keys in
    one workgroup's share than it may offer - the last three fall back to the sweep that counts ties per chunk.
    Two densities put their thresholds into the cluster, one of them on the tied magnitude with part of it kept."""
    rng = np.random.default_rng(cluster + ties)
    n = 8192 * 50 + 123
    w = (rng.standard_normal(n) * 0.001).astype(np.float32)
    pos = rng.choice(n, cluster, replace=False)
    bits = (np.uint32(0x3D000000) + rng.integers(0, 1024, cluster).astype(np.uint32))      # |x| ~ 0.031, one bin of 2^10 keys
    tied = np.uint32(0x3D000000 + 517)
    bits[:ties] = tied
    signs = rng.integers(0, 2, cluster).astype(np.uint32) << np.uint32(31)
    w[pos] = (bits | signs).view(np.float32)
    mag = np.abs(w).view(np.uint32)
    n_gt = int((mag > tied).sum())
    n_eq = int((mag == tied).sum())
    assert n_eq >= ties
    d_tied = (n_gt + max(1, n_eq // 2)) / n                     # keeps half of the tied magnitudes
    d_other = (cluster // 3) / n                                # a threshold elsewhere in the cluster
    half = n // 2 + 5
    res, ora = _prune_both([w[:half], w[half:]], [d_tied, d_other], what=f"cluster {cluster} ties {ties}")
    assert ora[0]["select"]["n_tie"] == n_eq and ora[0]["select"]["n_tie_kept"] == max(1, n_eq // 2)


def test_same_call_twice_and_other_launch_shapes_give_the_same_bits():
    """Determinism: the result is a function of the inputs alone.  The same call twice, and calls whose
    launches are shaped differently (sample size and candidate capacity change the grids, the segment counts
    and the order in which candidates are appended), must agree in every output bit and record field."""
    rng = np.random.default_rng(77)
    ws = [(rng.standard_normal(s) * 0.02).astype(np.float32) for s in ((1500, 1111), (8192 * 40 + 17,), (64, 64, 3, 3))]
    ws[1][::97] = np.float32(0.0337)                               # ties at a magnitude near the threshold of d = 0.1
    dev = up(ws)
    fields = ("n", "k", "n_gt", "n_tie_kept", "n_tie", "threshold_key", "tie_end")
    ref = prune(dev, [0.1, 0.4], theta_f16=True)
    torch.cuda.synchronize()
    ref_rec = P.select_records(ref["results"])
    variants = [dict(Form.config), dict(Form.config, sample_log2=16), dict(Form.config, cand_shift=2),
                dict(Form.config, sample_log2=19, cand_shift=4)]
    for cfg in variants:
        got = P.condensa_prune(dev, [0.1, 0.4], theta_f16=True, config=cfg)
        torch.cuda.synchronize()
        rec = P.select_records(got["results"])
        for j in range(2):
            assert all(rec[j][f] == ref_rec[j][f] for f in fields), (cfg, rec[j], ref_rec[j])
            for t in range(len(ws)):
                assert torch.equal(got["theta"][j][t].view(torch.int32), ref["theta"][j][t].view(torch.int32)), (cfg, j, t)
                assert torch.equal(got["theta_f16"][j][t], ref["theta_f16"][j][t]), (cfg, j, t)
                assert torch.equal(got["mask"][j][t], ref["mask"][j][t]), (cfg, j, t)
