"""Pins for the oracle's 16-bit-storage variants (half and bfloat16 rows): no GPU needed.

The paper works in fp32.  For rows stored in 16 bits the oracle widens exactly and runs the fp32
method; what is pinned here is (a) that the widening is exact, against two decoders that share
nothing with it, (b) the exact mode against brute force and against a library top-k that works on
the 16-bit type itself, and (c) Algorithm 2 against the paper-derived hand traces and the grid
characterisation, whose inputs are representable in both 16-bit types.
"""
import struct

import numpy as np
import pytest
import torch

import oracle
import workloads
from test_oracle_pins import _handtrace_cases, brute_topk

KINDS = ("f16", "bf16")
TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16}


def test_widening_is_exact_for_every_finite_bit_pattern():
    allbits = np.arange(65536, dtype=np.uint16)
    # half: Python's struct 'e' decoder
    with np.errstate(invalid="ignore"):  # signalling-NaN patterns, excluded below
        w = oracle.widen16(allbits, "f16").astype(np.float64)
    ref = np.array([struct.unpack("<e", struct.pack("<H", int(b)))[0] for b in allbits], dtype=np.float64)
    fin = np.isfinite(ref)
    assert np.array_equal(w[fin], ref[fin]) and np.array_equal(np.signbit(w[fin]), np.signbit(ref[fin]))
    # bfloat16: sign, exponent and 7 fraction bits written out
    with np.errstate(invalid="ignore"):
        w = oracle.widen16(allbits, "bf16").astype(np.float64)
    s = np.where(allbits >> 15, -1.0, 1.0)
    e = ((allbits >> 7) & 0xFF).astype(np.int64)
    f = (allbits & 0x7F).astype(np.float64)
    ref = np.where(e == 0, s * f / 128.0 * 2.0 ** -126, s * (1.0 + f / 128.0) * 2.0 ** (e - 127).astype(np.float64))
    fin = e != 255
    assert np.array_equal(w[fin], ref[fin])
    # and torch's own bfloat16 -> float32 conversion
    t = torch.from_numpy(allbits.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert np.array_equal(t[fin].view(np.int32), oracle.widen16(allbits, "bf16")[fin].view(np.int32))


def test_rounding_helpers_round_to_nearest_even():
    x = workloads.normal(200, 64, seed=7)
    b = workloads.to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b, t)
    h = workloads.to_f16_bits(x)
    t = torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(h, t)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("M", [1, 3, 8, 12, 40])
def test_exact16_matches_bruteforce(kind, M):
    # rounding to 16 bits makes ties across the k-th place common
    b = workloads.to_bits16(workloads.normal(400, M, seed=900 + M) * 0.25, kind)
    w = oracle.widen16(b, kind)
    for k in sorted({1, 2, (M + 1) // 2, M}):
        if k > M:
            continue
        vb, idx = oracle.topk_exact_16(b, kind, k)
        for r in range(b.shape[0]):
            assert np.array_equal(idx[r], brute_topk(w[r], k)), (kind, M, k, r)
        assert np.array_equal(vb, np.take_along_axis(b, idx.astype(np.int64), axis=1))


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("M,k", [(64, 8), (256, 32), (768, 96)])
def test_exact16_values_match_torch_topk_on_the_16bit_tensor(kind, M, k):
    b = workloads.to_bits16(workloads.normal(300, M, seed=910 + M), kind)
    vb, idx = oracle.topk_exact_16(b, kind, k)
    t = torch.from_numpy(b.view(np.int16).copy()).view(TORCH_DT[kind])
    tv = torch.topk(t.float(), k, dim=1).values.numpy()           # descending values
    mine = np.sort(oracle.widen16(vb, kind), axis=1)[:, ::-1]
    assert np.array_equal(mine, tv)
    # a second, type-native check where the library supports it on the CPU
    try:
        tv16 = torch.topk(t, k, dim=1).values.float().numpy()
    except RuntimeError:
        return
    assert np.array_equal(mine, tv16)


@pytest.mark.parametrize("kind", KINDS)
def test_alg2_16bit_hand_traces(kind):
    # the hand-traced rows hold small integers and halves: exactly representable in both types
    for v, k, mi, exp in _handtrace_cases():
        b = workloads.to_bits16(v[None, :], kind)
        assert np.array_equal(oracle.widen16(b, kind)[0], v)
        vb, idx = oracle.topk_earlystop_16(b, kind, k, mi)
        assert idx[0].tolist() == exp
        assert np.array_equal(vb[0], b[0][exp])


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("t", [1, 3, 6])
def test_alg2_16bit_grid_characterisation(kind, t):
    # small-integer rows: every midpoint is exact in fp32, so after t steps min is the largest grid
    # point min + D*j/2^t that still has at least k elements at or above it
    x = workloads.small_ints(80, 40, seed=940 + t, span=16)
    b = workloads.to_bits16(x, kind)
    assert np.array_equal(oracle.widen16(b, kind), x)
    for k in (1, 5, 20, 39):
        _, idx = oracle.topk_earlystop_16(b, kind, k, t)
        for r in range(x.shape[0]):
            row = x[r].astype(np.float64)
            mn, mx = row.min(), row.max()
            grid = mn + (mx - mn) * np.arange(2 ** t, dtype=np.float64) / 2 ** t
            cnts = (row[None, :] >= grid[:, None]).sum(axis=1)
            lo = grid[np.nonzero(cnts >= k)[0].max()]
            assert np.array_equal(idx[r], np.nonzero(row >= lo)[0][:k].astype(np.int32))


@pytest.mark.parametrize("kind", KINDS)
def test_alg2_16bit_reaches_exact_result_on_rows_without_ties(kind):
    rng = np.random.Generator(np.random.Philox(77))
    # 64 distinct 16-bit values per row: a permutation of a strictly increasing ladder
    ladder = workloads.to_bits16(np.linspace(-3.0, 3.0, 64, dtype=np.float32)[None, :], kind)[0]
    assert np.unique(ladder).size == 64
    b = np.stack([rng.permutation(ladder) for _ in range(200)])
    for k in (1, 8, 63):
        _, ei = oracle.topk_exact_16(b, kind, k)
        _, si = oracle.topk_earlystop_16(b, kind, k, 64)
        assert np.array_equal(si, ei)
