"""Full-size check of the L-C step in the launch configuration the benchmark times (1.2 G weights).

The oracle cannot sort 1.2 G keys in test time, so the result is verified through properties that
pin it uniquely at any size (exact counts above / at the threshold, the tie prefix rule, the mask
rule element by element) and through the oracle's element-wise arithmetic on every output value.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1911_02497_amd as P
import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
def test_lc_step_on_the_large_model_workload():
    T, rows, cols = 64, 4096, 4608
    mu, d = workloads.LC_MU, workloads.LC_DENSITY
    dev = "cuda:0"
    w_dev, l_dev = [], []
    for b in range(0, T, 8):
        ws, ls = workloads.lc_stress(indices=range(b, b + 8), threads=16)
        w_dev += [torch.from_numpy(a).to(dev) for a in ws]
        l_dev += [torch.from_numpy(a).to(dev) for a in ls]
        print(f"generated tensors {b}..{b + 7}", flush=True)
    N = T * rows * cols
    res = P.condensa_lc_step(w_dev, l_dev, mu, d)
    torch.cuda.synchronize()
    rec = P.select_records(res["results"])[0]
    print("record", rec, flush=True)
    k = oracle.kept_count(d, N)
    assert rec["n"] == N and rec["k"] == k == 120795955
    assert rec["path"] == 2, "the sampled window is expected to hold the threshold"
    Tkey, tie_end = rec["threshold_key"], rec["tie_end"]
    assert rec["n_gt"] + rec["n_tie_kept"] == k and 1 <= rec["n_tie_kept"] <= rec["n_tie"]

    L = oracle.lib()
    mu32 = float(np.float32(mu))
    n_gt = n_tie = n_tie_below = kept = 0
    flat0 = 0
    for t in range(T):
        w = w_dev[t].cpu().numpy().reshape(-1)
        lam = l_dev[t].cpu().numpy().reshape(-1)
        v = np.empty_like(w)
        L.oracle_lc_shifted(w.ctypes.data, lam.ctypes.data, w.size, mu32, v.ctypes.data)
        key = v.view(np.uint32) & np.uint32(0x7FFFFFFF)
        gt = key > Tkey
        tie = key == Tkey
        n_gt += int(gt.sum())
        n_tie += int(tie.sum())
        tie_idx = np.flatnonzero(tie) + flat0
        n_tie_below += int((tie_idx < tie_end).sum())
        want_mask = gt.copy()
        want_mask[tie_idx[tie_idx < tie_end] - flat0] = True
        mask = res["mask"][t].cpu().numpy().reshape(-1)
        assert np.array_equal(mask.astype(bool), want_mask), f"mask rule, tensor {t}"
        kept += int(mask.sum())
        # oracle arithmetic, element by element, on the GPU's own keep flags
        theta, lam2, grad = np.empty_like(w), np.empty_like(w), np.empty_like(w)
        L.oracle_lc_update(w.ctypes.data, lam.ctypes.data, v.ctypes.data, mask.ctypes.data, w.size, mu32,
                           theta.ctypes.data, lam2.ctypes.data, grad.ctypes.data)
        for name, want in (("theta", theta), ("lambda", lam2), ("grad", grad)):
            got = res[name][t].cpu().numpy().reshape(-1)
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{name}, tensor {t}"
        flat0 += w.size
        if t % 8 == 7:
            print(f"checked tensors ..{t}", flush=True)
    # these counts make threshold_key the k-th largest key and fix the tie split
    assert n_gt == rec["n_gt"] and n_tie == rec["n_tie"] and kept == k
    assert n_gt < k <= n_gt + n_tie
    assert n_tie_below == rec["n_tie_kept"]
    if rec["n_tie_kept"] == rec["n_tie"]:
        assert tie_end == N

    # The benchmark's exact output set and launch configuration: no mask, every output and the workspace
    # preallocated and passed in.  It must reproduce the outputs just verified, bit for bit.
    outputs = {"theta": [torch.empty_like(t) for t in w_dev], "grad": [torch.empty_like(t) for t in w_dev],
               "lambda": [torch.empty_like(t) for t in w_dev],
               "results": torch.zeros((1, 8), dtype=torch.int64, device=dev)}
    ws_bytes = P.condensa_workspace_bytes(P.binding.OP_LC_STEP, N, 0, T, 1, P.SCOPE_GLOBAL)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    for _ in range(2):                                   # the second step reuses the workspace the first one left
        res2 = P.condensa_lc_step(w_dev, l_dev, mu, d, outputs=outputs, mask=False, workspace=workspace)
        torch.cuda.synchronize()
        assert res2["mask"] is None
        rec2 = P.select_records(res2["results"])[0]
        assert rec2 == rec, (rec2, rec)
        for name in ("theta", "lambda", "grad"):
            for t in range(T):
                assert res2[name][t].data_ptr() == outputs[name][t].data_ptr()
                assert torch.equal(res2[name][t].view(torch.int32), res[name][t].view(torch.int32)), f"{name}, tensor {t} (no mask)"


@pytest.mark.timeout(600)
@pytest.mark.parametrize("density", [0.003, 0.1, 0.97])
def test_every_selection_form_gives_the_same_bits_at_full_size(density):
    """1.2 G weights of the benchmark's shape (seeded on the device): the one-sweep form, the two-sweep form
    and the radix levels must agree bit for bit on every output of the L-C step and of global pruning, and
    on every field of the selection record.  (The form that the test above checks against the oracle
    anchors the three.)"""
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(3)
    ws = [torch.randn(4096, 4608, device=dev, generator=g) * 0.01 for _ in range(64)]
    ls = [torch.randn(4096, 4608, device=dev, generator=g) * 0.01 for _ in range(64)]
    fields = ("n", "k", "n_gt", "n_tie_kept", "n_tie", "threshold_key", "tie_end")
    as_bits = lambda t: t.view(torch.int32) if t.dtype == torch.float32 else t  # noqa: E731
    ref = ref_rec = None
    try:
        for name, (path, two) in {"one_sweep": (2, 0), "two_sweeps": (2, 1), "radix": (1, 0)}.items():
            cfg = {"select_path": path, "fused_sweep": two}
            r = P.condensa_lc_step(ws, ls, 1e-3, density, config=cfg)
            p = P.condensa_prune(ws, [density], config=cfg)
            torch.cuda.synchronize()
            cur = (r["theta"], r["lambda"], r["grad"], r["mask"], p["theta"][0], p["mask"][0])
            rec = (P.select_records(r["results"])[0], P.select_records(p["results"])[0])
            assert rec[0]["path"] == rec[1]["path"] == (1 if name == "radix" else 2), (name, rec)
            if ref is None:
                ref, ref_rec = cur, rec
                continue
            for k in fields:
                assert rec[0][k] == ref_rec[0][k] and rec[1][k] == ref_rec[1][k], (name, k, rec, ref_rec)
            for which, (a_list, b_list) in enumerate(zip(cur, ref)):
                for t, (a, b) in enumerate(zip(a_list, b_list)):
                    assert torch.equal(as_bits(a), as_bits(b)), f"{name}: output {which} of tensor {t} differs"
            del r, p, cur
    finally:
        del ref, ws, ls
        torch.cuda.empty_cache()
