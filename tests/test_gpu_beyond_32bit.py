"""Flat indices above 2^32: a prune call over 4.3 G weights with ties planted on both sides of 2^32.

No host oracle can sort this in test time; the result is pinned by counts and the keep rule evaluated with
plain torch comparisons on the exact key patterns (properties that hold at any size)."""
import numpy as np
import pytest
import torch

import paper_1911_02497_amd as P

pytestmark = pytest.mark.gpu


def _keys(t):
    return t.view(torch.int32) & 0x7FFFFFFF        # magnitude pattern; non-negative as int32


@pytest.mark.timeout(600)
def test_prune_with_flat_indices_beyond_32_bits():
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(1911)
    sizes = [1 << 30, 1 << 30, 1 << 30, 1 << 30, (1 << 20) + 5]          # N = 2^32 + 2^20 + 5
    ws = [torch.randn(n, device=dev, generator=gen) for n in sizes]
    N = sum(sizes)
    tval = torch.tensor(1.6448536, dtype=torch.float32)
    tkey = int(tval.view(torch.int32).item())
    for t, w in enumerate(ws):                                            # 200 ties per tensor, the last ones past 2^32
        pos = torch.arange(0, 200, device=dev) * (w.numel() // 200) + 3
        w[pos] = tval if t % 2 == 0 else -tval
    n_gt = sum(int((_keys(w) > tkey).sum().item()) for w in ws)
    n_tie = sum(int((_keys(w) == tkey).sum().item()) for w in ws)
    assert n_tie >= 1000                                                  # planted ones plus natural duplicates
    for extra, path in ((n_tie - 50, 0), (n_tie, 0), (n_tie - 50, 1)):   # last kept tie beyond 2^32 / all kept / radix levels
        P.condensa_set_option(P.OPT_SELECT_PATH, path)
        k = n_gt + extra
        d = k / N
        assert int(np.floor(d * N + 0.5)) == k
        res = P.condensa_prune(ws, [d], theta=False, mask=True)
        torch.cuda.synchronize()
        rec = P.select_records(res["results"])[0]
        print("record", rec, flush=True)
        assert rec["n"] == N and rec["k"] == k and rec["threshold_key"] == tkey
        assert rec["n_gt"] == n_gt and rec["n_tie"] == n_tie and rec["n_tie_kept"] == extra
        flat0, kept, ties_seen = 0, 0, 0
        for t, w in enumerate(ws):
            key = _keys(w)
            tie_pos = torch.nonzero(key == tkey).flatten()
            want = key > tkey
            n_keep_here = max(0, min(tie_pos.numel(), extra - ties_seen))
            want[tie_pos[:n_keep_here]] = True
            assert torch.equal(res["mask"][0][t].bool(), want), f"mask of tensor {t}"
            if n_keep_here and ties_seen + n_keep_here == extra and extra < n_tie:
                assert rec["tie_end"] == flat0 + int(tie_pos[n_keep_here - 1].item()) + 1
                assert rec["tie_end"] > (1 << 32)
            ties_seen += tie_pos.numel()
            kept += int(want.sum().item())
            flat0 += w.numel()
            del key, want
        assert kept == k
        if extra == n_tie:
            assert rec["tie_end"] == N
        assert rec["path"] == (1 if path == 1 else 2)
    P.condensa_set_option(P.OPT_SELECT_PATH, 0)
