"""Pins for the oracle's filter / block aggregation and structure pruning (CPU only).

Table 1: FilterPrune aggregates filters (3-D blocks), BlockPrune aggregates
n-D blocks; Section 3.1: "filter/neuron/block aggregation".  The aggregate is
the squared L2 norm; pins are exact summation (math.fsum), brute-force ranks,
planted exact ties and the Kaiming expectation E[S_f] = 2.
"""
import math

import numpy as np
import pytest

import oracle
import workloads
from test_oracle_select import brute_keep


def test_filter_sumsq_against_exact_summation():
    rng = np.random.default_rng(0)
    t = rng.standard_normal((6, 5, 3, 3)).astype(np.float32)
    s = oracle.filter_sumsq(t)
    for f in range(6):
        exact = math.fsum(float(v) * float(v) for v in t[f].reshape(-1))
        assert abs(s[f] - exact) <= 45 * 2.0**-53 * exact
    # sequential order: same as a plain left-to-right python loop in binary64
    acc = 0.0
    for v in t[2].reshape(-1):
        acc = acc + float(v) * float(v)
    assert s[2] == acc


def test_block_sumsq_layout_and_order():
    rng = np.random.default_rng(1)
    m = rng.standard_normal((6, 8)).astype(np.float32)
    s = oracle.block_sumsq(m, 2, 4)
    assert s.shape == (6,)
    for br in range(3):
        for bc in range(2):
            blk = m[br * 2:(br + 1) * 2, bc * 4:(bc + 1) * 4]
            acc = 0.0
            for v in blk.reshape(-1):          # row-major inside the block
                acc = acc + float(v) * float(v)
            assert s[br * 2 + bc] == acc
    # a transposed operand or swapped block dims would give other values
    assert not np.allclose(oracle.block_sumsq(m, 2, 4), oracle.block_sumsq(np.ascontiguousarray(m.T).reshape(6, 8), 2, 4))
    with pytest.raises(ValueError):
        oracle.block_sumsq(m, 4, 4)


def test_zero_and_duplicate_structures_have_identical_keys():
    rng = np.random.default_rng(2)
    t = rng.standard_normal((5, 4, 3, 3)).astype(np.float32)
    t[1] = 0.0
    t[4] = t[0]
    s = oracle.filter_sumsq(t)
    assert s[1] == 0.0 and s[4] == s[0]
    n = oracle.norms_of(s)
    assert n[1] == 0.0 and np.allclose(n, np.sqrt(s), rtol=1e-7)


def test_filter_prune_matches_brute_force_with_planted_ties():
    rng = np.random.default_rng(3)
    a = rng.standard_normal((6, 2, 3, 3)).astype(np.float32)
    b = rng.standard_normal((4, 6, 3, 3)).astype(np.float32)
    a[3] = a[1]                      # exact tie
    b[2] = 0.0
    for scope in (oracle.SCOPE_GLOBAL, oracle.SCOPE_PER_TENSOR):
        for d in (0.0, 0.2, 0.5, 0.8, 1.0):
            res = oracle.filter_prune([a, b], d, scope)
            sa = [math.fsum(float(v) ** 2 for v in a[f].reshape(-1)) for f in range(6)]
            sb = [math.fsum(float(v) ** 2 for v in b[f].reshape(-1)) for f in range(4)]
            # exact sums decide the same order as the binary64 sums here (gaps are large) except the planted tie
            sa[3] = sa[1]
            if scope == oracle.SCOPE_GLOBAL:
                k = int(math.floor(d * 10 + 0.5))
                want = brute_keep(sa + sb, k)
            else:
                want = brute_keep(sa, int(math.floor(d * 6 + 0.5))) + brute_keep(sb, int(math.floor(d * 4 + 0.5)))
            assert res["structure_mask"].tolist() == want
            assert res["keep_idx"].tolist() == [i for i, m in enumerate(want) if m]
            for t, th, mk, w in ((a, res["theta"][0], res["mask"][0], want[:6]), (b, res["theta"][1], res["mask"][1], want[6:])):
                for f in range(t.shape[0]):
                    if w[f]:
                        assert np.array_equal(th[f].view(np.uint32), t[f].view(np.uint32)) and np.all(mk[f] == 1)
                    else:
                        assert np.all(th[f].view(np.uint32) == 0) and np.all(mk[f] == 0)


def test_block_prune_zeroes_whole_blocks():
    rng = np.random.default_rng(4)
    m = rng.standard_normal((8, 12)).astype(np.float32)
    m[0:4, 4:8] = 0.0
    res = oracle.block_prune([m], 4, 4, 0.5)
    s = oracle.block_sumsq(m, 4, 4)
    want = brute_keep([float(v) for v in s], 3)
    assert res["structure_mask"].tolist() == want and want[1] == 0
    mk = res["mask"][0]
    for b in range(6):
        blk = mk[(b // 3) * 4:(b // 3 + 1) * 4, (b % 3) * 4:(b % 3 + 1) * 4]
        assert np.all(blk == want[b])
    assert np.array_equal(res["theta"][0], m * mk)


def test_resnet_filter_counts_and_kaiming_expectation():
    convs = workloads.resnet56_cifar_convs()
    assert len(convs) == 55 and sum(t.size for t in convs) == 848304
    assert sum(t.shape[0] for t in convs) == 2032
    res = oracle.filter_prune(convs, 0.3, oracle.SCOPE_GLOBAL)
    assert res["select"]["k"] == 610 and len(res["keep_idx"]) == 610
    assert abs(float(res["sumsq"].mean()) - 2.0) < 0.05          # fan_in * 2 / fan_in
    per = oracle.filter_prune(convs, 0.5, oracle.SCOPE_PER_TENSOR)
    assert [s["k"] for s in per["select"]] == [t.shape[0] // 2 for t in convs]


def test_transformer_block_counts():
    shapes = workloads.transformer_base_shapes()
    assert len(shapes) == 96 and sum(r * c for r, c in shapes) == 44040192
    assert sum((r // 8) * (c // 8) for r, c in shapes) == 688128
    assert sum((r // 32) * (c // 32) for r, c in shapes) == 43008
    assert oracle.kept_count(0.25, 688128) == 172032 and oracle.kept_count(0.25, 43008) == 10752


# ---- n-D / ragged blocks, neurons, combined structures (Table 1: NeuronPrune, StructurePrune, BlockPrune) ----

def _py_block_sums(t, block):
    """Blocks cut with python slices; squares added left to right in row-major order, in binary64."""
    import itertools
    pad = 4 - t.ndim
    t4 = t.reshape((1,) * pad + t.shape)
    b4 = (1,) * pad + tuple(block)
    grids = [range(0, t4.shape[k], b4[k]) for k in range(4)]
    out = []
    for o in itertools.product(*grids):
        blk = t4[o[0]:o[0] + b4[0], o[1]:o[1] + b4[1], o[2]:o[2] + b4[2], o[3]:o[3] + b4[3]]
        acc = 0.0
        for v in blk.reshape(-1):
            acc = acc + float(v) * float(v)
        out.append(acc)
    return out


@pytest.mark.parametrize("shape,block", [((10, 15), (5, 5)), ((10, 15), (4, 7)), ((13,), (5,)), ((6, 5, 3, 3), (4, 2, 3, 3)),
                                         ((6, 5, 3, 3), (1, 5, 1, 1)), ((7, 9), (1, 4)), ((3, 4, 5), (2, 2, 2))])
def test_nd_block_sums_against_python_slices(shape, block):
    t = np.random.default_rng(21).standard_normal(shape).astype(np.float32)
    s = oracle.block_sumsq_nd(t, block)
    assert s.tolist() == _py_block_sums(t, block)          # bit exact: same order, same precision


def test_nd_blocks_reduce_to_the_2d_case_when_shapes_divide():
    m = np.random.default_rng(22).standard_normal((12, 20)).astype(np.float32)
    assert np.array_equal(oracle.block_sumsq_nd(m, (4, 5)), oracle.block_sumsq(m, 4, 5))
    a = oracle.block_prune_nd([m], (4, 5), 0.5)
    b = oracle.block_prune([m], 4, 5, 0.5)
    assert np.array_equal(a["mask"][0], b["mask"][0]) and a["select"] == b["select"]


def test_ragged_block_prune_masks_follow_the_structure_mask():
    rng = np.random.default_rng(23)
    m = rng.standard_normal((11, 13)).astype(np.float32)
    res = oracle.block_prune_nd([m], (4, 5), 0.5)
    s = _py_block_sums(m, (4, 5))
    want = brute_keep(s, int(math.floor(0.5 * 9 + 0.5)))
    assert res["structure_mask"].tolist() == want
    for u in range(9):
        r0, c0 = (u // 3) * 4, (u % 3) * 5
        assert np.all(res["mask"][0][r0:r0 + 4, c0:c0 + 5] == want[u])
    assert np.array_equal(res["theta"][0], m * res["mask"][0])


def test_neuron_and_structure_prune():
    rng = np.random.default_rng(24)
    lin = rng.standard_normal((6, 10)).astype(np.float32)
    conv = rng.standard_normal((5, 3, 3, 3)).astype(np.float32)
    res = oracle.neuron_prune([lin], 0.5)
    rows = [math.fsum(float(v) ** 2 for v in lin[r]) for r in range(6)]
    assert res["structure_mask"].tolist() == brute_keep(rows, 3)
    assert np.array_equal(res["mask"][0], np.repeat(res["structure_mask"][:, None], 10, axis=1))
    both = oracle.structure_prune([conv, lin], 0.4)
    filt = [math.fsum(float(v) ** 2 for v in conv[f].reshape(-1)) for f in range(5)]
    assert both["structure_mask"].tolist() == brute_keep(filt + rows, int(math.floor(0.4 * 11 + 0.5)))
    with pytest.raises(ValueError):
        oracle.neuron_prune([conv], 0.5)
