"""GPU parity: condensa_quantize / condensa_dequantize against the oracle, bit for bit."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_1911_02497_amd as P
from gpu_util import DEV, assert_bits_equal

pytestmark = pytest.mark.gpu


def _run(x):
    q, dq = P.condensa_quantize(torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    return q.cpu().numpy().view(np.uint16), dq.cpu().numpy()


def _compare(x, what):
    q, dq = _run(x)
    oq, odq = oracle.quantize_f16(x)
    nan = np.isnan(x)
    assert np.array_equal(q[~nan], oq[~nan]), what
    assert np.array_equal(q[nan], oq[nan]), what + " (NaN payload rule)"
    assert_bits_equal(dq, odq, what + " dq")


def test_golden_points():
    path = os.path.join(os.path.dirname(__file__), "golden", "binary16_points.txt")
    pts = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    x = np.array([int(a, 16) for a, _ in pts], np.uint32).view(np.float32)
    q, _ = _run(x)
    assert [hex(v) for v in q.tolist()] == [hex(int(b, 16)) for _, b in pts]


def test_stratified_bit_patterns_and_band_sweeps():
    hi10 = np.array([0, 1, 0x2AA, 0x3FF], np.uint32)
    low = np.arange(1 << 13, dtype=np.uint32)
    se = np.arange(1 << 9, dtype=np.uint32)
    bits = ((se[:, None, None] << 23) | (hi10[None, :, None] << 13) | low[None, None, :]).reshape(-1)
    _compare(bits.view(np.float32), "stratified")
    for e in (101, 102, 112, 113, 142, 143, 255):
        b = np.arange(e << 23, (e + 1) << 23, dtype=np.uint64).astype(np.uint32)
        _compare(b.view(np.float32), f"exponent band {e}")


@pytest.mark.slow
def test_every_binary32_pattern_against_numpy():
    """All 2^32 input patterns (opt-in: CONDENSA_SLOW=1, about four minutes).  The kernels round numbers with the
    conversion instruction; numpy's conversion, against which the oracle is pinned over the same 2^32 patterns on
    the CPU, is the fast independent reference here.  NaN inputs (whose payload rule is the oracle's, not numpy's)
    are compared with the oracle on a sample."""
    step = 1 << 28
    for start in range(0, 1 << 32, step):
        print(f"patterns from {start:#010x}", flush=True)     # (a long quiet test looks hung to a watchdog)
        bits = np.arange(start, start + step, dtype=np.uint64).astype(np.uint32)
        x = bits.view(np.float32)
        q, dq = _run(x)
        nan = np.isnan(x)
        with np.errstate(over="ignore"):
            ref = x.astype(np.float16)
        assert np.array_equal(q[~nan], ref.view(np.uint16)[~nan]), hex(start)
        assert np.array_equal(dq[~nan].view(np.uint32), ref.astype(np.float32).view(np.uint32)[~nan]), hex(start)
        if nan.any():
            idx = np.flatnonzero(nan)[:: 4099]
            oq, odq = oracle.quantize_f16(x[idx])
            assert np.array_equal(q[idx], oq) and np.array_equal(dq[idx].view(np.uint32), odq.view(np.uint32)), hex(start)


def test_ragged_sizes_and_misaligned_views():
    rng = np.random.default_rng(5)
    for n in (1, 2, 3, 5, 255, 1023, 1025, 8191, 70001):
        x = (rng.standard_normal(n) * 0.02).astype(np.float32)
        _compare(x, f"n={n}")
    big = torch.from_numpy((rng.standard_normal(10007) * 3).astype(np.float32)).to(DEV)
    view = big[1:]                                         # 4-byte aligned only: scalar path
    q, dq = P.condensa_quantize(view)
    oq, odq = oracle.quantize_f16(view.cpu().numpy())
    assert np.array_equal(q.cpu().numpy().view(np.uint16), oq)
    assert_bits_equal(dq, odq, "misaligned dq")


def test_empty_and_dequantize_all_patterns():
    q, dq = P.condensa_quantize(torch.empty(0, dtype=torch.float32, device=DEV))
    assert q.numel() == 0 and dq.numel() == 0
    allh = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    got = P.condensa_dequantize(torch.from_numpy(allh.view(np.int16)).to(DEV)).cpu().numpy()
    want = oracle.dequantize_f16(allh)
    assert_bits_equal(got, want, "dequantize")


@pytest.mark.parametrize("n", [1, 7, 511, 512, 513, 1000, 64 * 512 + 3, (1 << 20) + 255])
def test_dequantize_and_codes_only_ragged_sizes(n):
    """Sizes around the 512-code wavefront tile of the wide dequantize and the 8-element thread tile of the
    codes-only quantize, aligned and misaligned storage."""
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * rng.choice(np.array([1e-6, 1.0, 300.0], np.float32), n)).astype(np.float32)
    oq, odq = oracle.quantize_f16(x)
    q, _ = P.condensa_quantize(torch.from_numpy(x).to(DEV), want_dq=False)
    assert np.array_equal(q.cpu().numpy().view(np.uint16), oq)
    assert_bits_equal(P.condensa_dequantize(q), odq, "dequantize aligned")
    big = torch.empty(n + 1, dtype=torch.int16, device=DEV)
    big[1:] = q
    assert_bits_equal(P.condensa_dequantize(big[1:]), odq, "dequantize misaligned")


def test_errors():
    with pytest.raises(P.CondensaError) as e:
        P.condensa_quantize(torch.zeros(4, device=DEV), want_q=False, want_dq=False)
    assert e.value.code == -1


@pytest.mark.parametrize("n", [1, 511, 513, 4097, (1 << 20) + 255])
def test_bfloat16_against_the_oracle(n):
    """bfloat16 quantize / dequantize: random magnitudes over many octaves plus every special class, ragged
    sizes, codes-only and misaligned forms."""
    rng = np.random.default_rng(n + 5)
    with np.errstate(over="ignore"):                   # some magnitudes overflow binary32 on purpose
        x = (rng.standard_normal(n) * np.exp(rng.standard_normal(n) * 25)).astype(np.float32)
    special = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 3.3895314e38, -3.4e38, 1e-40, -2e-45, 1.00390625, 1.01171875],
                       np.float32)
    x[: min(n, special.size)] = special[: min(n, special.size)]
    oq, odq = oracle.quantize_bf16(x)
    dx = torch.from_numpy(x).to(DEV)
    q, dq = P.condensa_quantize_bf16(dx)
    assert np.array_equal(q.cpu().numpy().view(np.uint16), oq)
    assert_bits_equal(dq, odq, "bf16 dq")
    q2, _ = P.condensa_quantize_bf16(dx, want_dq=False)
    assert np.array_equal(q2.cpu().numpy().view(np.uint16), oq)
    assert_bits_equal(P.condensa_dequantize_bf16(q), odq, "bf16 dequantize")
    big = torch.empty(n + 1, dtype=torch.float32, device=DEV)
    big[1:] = dx
    q3, dq3 = P.condensa_quantize_bf16(big[1:])
    assert np.array_equal(q3.cpu().numpy().view(np.uint16), oq)
    assert_bits_equal(dq3, odq, "bf16 misaligned")


def test_bfloat16_all_codes_round_trip():
    allh = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    got = P.condensa_dequantize_bf16(torch.from_numpy(allh.view(np.int16)).to(DEV))
    assert_bits_equal(got, oracle.dequantize_bf16(allh), "bf16 all codes")


# ---- 8-bit floating point ---------------------------------------------------------------------------------

FP8 = {"e4m3": (P.FP8_E4M3, oracle.FP8_E4M3, 448.0), "e5m2": (P.FP8_E5M2, oracle.FP8_E5M2, 57344.0)}


@pytest.mark.parametrize("name", sorted(FP8))
@pytest.mark.parametrize("n", [0, 1, 3, 255, 256, 257, 1024, 1025, 64 * 16 * 7 + 5, 1_000_003])
def test_fp8_matches_the_oracle(name, n):
    """Codes and widened values bit for bit: several workgroups and a ragged tail, weights-like values, every
    binade of the format and beyond (saturation), tie points, specials; all three kernel forms (codes and
    values, codes only, scalar path on misaligned pointers) and the dequantize entry point."""
    fmt, ofmt, vmax = FP8[name]
    rng = np.random.default_rng(n + fmt)
    x = np.where(rng.random(n) < 0.5, rng.standard_normal(n) * 0.02,
                 np.exp(rng.uniform(np.log(vmax) - 45, np.log(vmax) + 3, n)) * rng.choice([-1.0, 1.0], n)).astype(np.float32)
    codes = np.arange(0x7C, dtype=np.uint8)
    vals = oracle.dequantize_fp8(codes, ofmt).astype(np.float64)
    mids = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)
    special = np.concatenate([np.array([0.0, -0.0, np.inf, -np.inf, np.nan, -np.nan, 3.4e38, -3.4e38, 1e-45, -1e-40], np.float32),
                              mids, np.nextafter(mids, np.float32(np.inf)), -np.nextafter(mids, np.float32(0))])
    m = min(n, special.size)
    x[:m] = special[:m]
    oq, odq = oracle.quantize_fp8(x, ofmt)
    dx = torch.from_numpy(x).to(DEV)
    q, dq = P.condensa_quantize_fp8(dx, fmt)
    assert np.array_equal(q.cpu().numpy(), oq)
    assert_bits_equal(dq, odq, f"{name} dq")
    q2, _ = P.condensa_quantize_fp8(dx, fmt, want_dq=False)
    assert np.array_equal(q2.cpu().numpy(), oq)
    _, dq2 = P.condensa_quantize_fp8(dx, fmt, want_q=False)
    assert_bits_equal(dq2, odq, f"{name} dq only")
    assert_bits_equal(P.condensa_dequantize_fp8(q, fmt), odq, f"{name} dequantize")
    big = torch.empty(n + 1, dtype=torch.float32, device=DEV)
    big[1:] = dx
    q3, dq3 = P.condensa_quantize_fp8(big[1:], fmt)
    assert np.array_equal(q3.cpu().numpy(), oq)
    assert_bits_equal(dq3, odq, f"{name} misaligned")
    qb = torch.empty(n + 1, dtype=torch.uint8, device=DEV)
    qb[1:] = q
    assert_bits_equal(P.condensa_dequantize_fp8(qb[1:], fmt), odq, f"{name} dequantize misaligned")


@pytest.mark.parametrize("name", sorted(FP8))
def test_fp8_all_codes_and_errors(name):
    fmt, ofmt, _ = FP8[name]
    codes = np.arange(256, dtype=np.uint8)
    got = P.condensa_dequantize_fp8(torch.from_numpy(codes).to(DEV), fmt)
    assert_bits_equal(got, oracle.dequantize_fp8(codes, ofmt), f"{name} all codes")
    with pytest.raises(P.CondensaError) as e:
        P.condensa_quantize_fp8(torch.ones(8, device=DEV), 2)
    assert e.value.code == -6
