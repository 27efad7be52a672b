"""GPU checks of calls that carry more than 2^32 elements: flat indices, tie positions and launch sizes
beyond 32 bits.  The oracle cannot run at this size within a test's time, so the results are checked
against the properties that define them (computed with plain torch operations on the device): the kept
count, the threshold separating kept from pruned magnitudes, ties kept in flat-index order, theta = w on
kept positions and +0 elsewhere, and the selection record's own counts."""
import numpy as np
import pytest
import torch

import paper_1911_02497_amd as P
from gpu_util import DEV

pytestmark = pytest.mark.gpu

N_EACH = 1 << 30
N_TENSORS = 5                                   # 5 * 2^30 elements: the last tensor starts at flat index 2^32


def _free():
    import gc
    gc.collect()
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def big_weights():
    if torch.cuda.get_device_properties(0).total_memory < 200 * (1 << 30):
        pytest.skip("needs ~140 GiB of device memory")
    g = torch.Generator(device=DEV)
    g.manual_seed(20191102497)
    ws = [torch.randn(N_EACH, device=DEV, generator=g) for _ in range(N_TENSORS)]
    yield ws
    del ws
    _free()


def _key_to_float(key):
    return float(np.array([key], dtype=np.uint32).view(np.float32)[0])


def _check_prune_properties(ws, theta, mask, rec, k, what):
    """Everything the record and the outputs must satisfy, whatever the size."""
    N = sum(w.numel() for w in ws)
    assert rec["n"] == N and rec["k"] == k, (what, rec)
    assert rec["n_gt"] + rec["n_tie_kept"] == k, (what, rec)
    T = _key_to_float(rec["threshold_key"])
    n_gt = n_tie = kept = 0
    tie_flat, tie_kept = [], []
    start = 0
    for w, th, m in zip(ws, theta, mask):
        a = w.abs()
        mb = m.bool()
        gt = a > T
        eq = a == T
        n_gt += int(gt.sum())
        n_tie += int(eq.sum())
        kept += int(mb.sum())
        assert bool((mb | ~gt).all()), f"{what}: a magnitude above the threshold was pruned"
        assert bool((~mb | gt | eq).all()), f"{what}: a magnitude below the threshold was kept"
        pos = eq.nonzero().flatten()
        tie_flat.append(pos + start)
        tie_kept.append(m[pos])
        assert torch.equal(th, torch.where(mb, w, torch.zeros((), device=DEV))), f"{what}: theta"
        assert not bool(torch.signbit(th[~mb]).any()), f"{what}: pruned positions must hold +0"
        start += w.numel()
        del a, mb, gt, eq
    assert kept == k and n_gt == rec["n_gt"] and n_tie == rec["n_tie"], (what, kept, n_gt, n_tie, rec)
    tie_flat = torch.cat(tie_flat).cpu().numpy()
    tie_kept = torch.cat(tie_kept).cpu().numpy()
    r = rec["n_tie_kept"]
    assert tie_kept[:r].all() and not tie_kept[r:].any(), f"{what}: ties are kept in flat-index order"
    want_end = N if r == n_tie else (int(tie_flat[r - 1]) + 1 if r > 0 else 0)
    if k > 0:
        assert rec["tie_end"] == want_end, (what, rec["tie_end"], want_end)
    return T


# (selection path, two sweeps, window margin); a margin of zero makes the sampled window miss, so that the
# one-sweep call ends in the radix levels and the gated full apply
FORMS = {"one_sweep": {"select_path": 2}, "two_sweeps": {"select_path": 2, "fused_sweep": 1},
         "radix": {"select_path": 1}, "window_missed": {"select_path": 2, "window_margin": 0}}


@pytest.mark.parametrize("form", sorted(FORMS))
def test_global_prune_of_more_than_2_32_weights(big_weights, form):
    ws = big_weights
    N = N_EACH * N_TENSORS
    assert N > (1 << 32)
    cfg = FORMS[form]
    try:
        density = 0.1
        res = P.condensa_prune(ws, [density], config=cfg)
        torch.cuda.synchronize()
        rec = P.select_records(res["results"])[0]
        assert rec["path"] in {"radix": (1,), "window_missed": (2, 3)}.get(form, (2,)), rec
        k = int(round(density * N))
        T = _check_prune_properties(ws, res["theta"][0], res["mask"][0], rec, k, form)
        del res
        _free()
        # plant 1000 more magnitudes equal to the threshold at the start of the call and 1000 beyond flat
        # index 2^32, over values far below it, and cut the tie group in the middle
        saved = []
        for t, lo in ((0, 0), (N_TENSORS - 1, N_EACH - (1 << 20))):
            seg = ws[t][lo:lo + (1 << 20)]
            pos = (seg.abs() < T / 2).nonzero().flatten()[:1000]
            assert pos.numel() == 1000
            saved.append((t, lo, pos, seg[pos].clone()))
            sign = torch.where(torch.arange(1000, device=DEV) % 2 == 0, 1.0, -1.0)
            seg[pos] = sign * T
        try:
            k2 = rec["n_gt"] + 1500
            res = P.condensa_prune(ws, [k2 / N], config=cfg)
            torch.cuda.synchronize()
            rec2 = P.select_records(res["results"])[0]
            assert rec2["threshold_key"] == rec["threshold_key"] and rec2["n_tie"] == rec["n_tie"] + 2000, (rec, rec2)
            assert rec2["n_tie_kept"] == 1500 and rec2["tie_end"] > (1 << 32), rec2
            _check_prune_properties(ws, res["theta"][0], res["mask"][0], rec2, k2, form + " planted ties")
            del res
        finally:
            for t, lo, pos, old in saved:
                ws[t][lo:lo + (1 << 20)][pos] = old
    finally:
        _free()


def test_lc_step_of_more_than_2_32_weights_with_zero_multipliers(big_weights):
    """With lambda = 0 the step prunes w itself, and with p = mu (w - theta) rounded once the new multiplier
    is lambda' = -p and the penalty gradient g = p - lambda' = 2 p, exactly; both vanish on kept positions."""
    ws = big_weights
    N = N_EACH * N_TENSORS
    mu, density = 1e-3, 0.07
    lam = [torch.zeros_like(w) for w in ws]
    res = P.condensa_lc_step(ws, lam, mu, density)
    torch.cuda.synchronize()
    rec = P.select_records(res["results"])[0]
    assert rec["path"] == 2 and rec["k"] == int(round(density * N))
    _check_prune_properties(ws, res["theta"], res["mask"], rec, rec["k"], "lc step")
    for w, th, m, lo, g in zip(ws, res["theta"], res["mask"], res["lambda"], res["grad"]):
        mb = m.bool()
        assert not bool(lo[mb].any()) and not bool(g[mb].any())
        p = (w - th)[~mb] * mu
        assert torch.equal(lo[~mb], -p) and torch.equal(g[~mb], 2 * p)
        del mb, p
    del res, lam
    _free()


def _check_structure_result(res, w, s_ref, block_mask_of, k, what):
    rec = P.select_records(res["results"])[0]
    F = s_ref.numel()
    assert rec["n"] == F and rec["k"] == k, (what, rec)
    s = res["sumsq"]
    assert torch.allclose(s, s_ref, rtol=1e-10, atol=0), what + ": aggregates"
    assert torch.allclose(res["norms"].double(), s.sqrt(), rtol=1e-6, atol=0), what + ": norms"
    T = float(np.array([rec["threshold_key"]], dtype=np.uint64).view(np.float64)[0])
    idx = torch.arange(F, device=DEV)
    want = (s > T) | ((s == T) & (idx < rec["tie_end"]))
    assert int(want.sum()) == k and int((s > T).sum()) == rec["n_gt"] and int((s == T).sum()) == rec["n_tie"], (what, rec)
    sm = res["structure_mask"].bool()
    assert torch.equal(sm, want), what + ": structure mask"
    keep = res["keep_idx"]
    assert torch.equal(keep[:k].long(), want.nonzero().flatten()) and bool((keep[k:] == -1).all()), what + ": kept ids"
    em = block_mask_of(sm)
    assert torch.equal(res["mask"][0].bool(), em), what + ": element mask"
    assert torch.equal(res["theta"][0], torch.where(em, w, torch.zeros((), device=DEV))), what + ": theta"


def test_filter_prune_of_one_tensor_with_more_than_2_32_elements():
    if torch.cuda.get_device_properties(0).total_memory < 200 * (1 << 30):
        pytest.skip("needs ~60 GiB of device memory")
    rows, cols = 8200, 524288
    assert rows * cols > (1 << 32)
    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    w = torch.randn(rows, cols, device=DEV, generator=g)
    w[4000] = w[100]                                  # two equal aggregates
    s_ref = torch.cat([w[r:r + 512].double().pow(2).sum(1) for r in range(0, rows, 512)])
    k = int(round(0.3 * rows))
    res = P.condensa_filter_prune([w.view(rows, cols, 1, 1)], 0.3, fill_keep_idx=True)
    torch.cuda.synchronize()
    _check_structure_result(res, w.view(rows, cols, 1, 1), s_ref, lambda sm: sm[:, None, None, None].expand(rows, cols, 1, 1), k,
                            "filters")
    del res, w, s_ref
    _free()


def test_block_prune_of_one_matrix_with_more_than_2_32_elements():
    if torch.cuda.get_device_properties(0).total_memory < 200 * (1 << 30):
        pytest.skip("needs ~80 GiB of device memory")
    rows, cols, b = 65544, 65536, 8
    assert rows * cols > (1 << 32)
    g = torch.Generator(device=DEV)
    g.manual_seed(8)
    w = torch.randn(rows, cols, device=DEV, generator=g)
    gr, gc_ = rows // b, cols // b
    parts = []
    for r in range(0, gr, 1024):
        blk = w[r * b:(r + 1024) * b].view(-1, b, gc_, b).double()
        parts.append(blk.pow(2).sum((1, 3)).flatten())
        del blk
    s_ref = torch.cat(parts)
    del parts
    F = gr * gc_
    k = int(round(0.25 * F))
    res = P.condensa_block_prune([w], b, b, 0.25, fill_keep_idx=True)
    torch.cuda.synchronize()

    def expand(sm):
        return sm.view(gr, 1, gc_, 1).expand(gr, b, gc_, b).reshape(rows, cols)

    _check_structure_result(res, w, s_ref, expand, k, "blocks")
    del res, w, s_ref
    _free()
