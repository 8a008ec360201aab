"""Pins for the oracle's MXFP4 conversion and its decoupled scale search (Sec. 4.3, "DSS on
MXFP4"; the format itself from the OCP Microscaling Formats specification v1.0): hand-worked
blocks, the shared-exponent rule and nearest-of-grid rounding written independently in float64,
enumeration of every (beta, stored code) pair, equivariance under powers of two, dequantization."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_12245_amd import synth

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
HERE = os.path.dirname(os.path.abspath(__file__))


def unpack(codes):
    nib = np.stack([codes & 0xF, codes >> 4], axis=-1).reshape(codes.shape[0], -1)
    v = E2M1[nib & 7]
    return np.where(nib & 8, -v, v)


def nearest_grid(x):
    a = np.minimum(np.abs(x), 1e3)
    return np.sign(x) * E2M1[np.abs(a[..., None] - E2M1).argmin(axis=-1)]


def tensor(workload=2, div=32):
    spec = synth.workload_specs(workload, div)[0]
    w = synth.make_weight(spec, "cpu")
    return w, synth.bf16_bits(w)


def test_hand_worked_blocks():
    for line in open(os.path.join(HERE, "golden", "mxfp4_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        vals, code, want = [p.strip() for p in line.split("|")]
        v = [float(x) for x in vals.split()]
        blk = np.zeros((1, 32), dtype=np.float32)
        blk[0, : len(v)] = v
        out = oracle.mxfp4_quantize(blk)
        assert int(out.scales[0, 0]) == int(code), line
        q = unpack(out.codes)[0]
        assert list(q[: len(v)]) == [float(x) for x in want.split()], line
        assert not q[len(v):].any()


@pytest.mark.parametrize("workload,div", [(1, 1), (2, 32), (5, 128)])
def test_plain_conversion_against_the_rule_in_float64(workload, div):
    w, bits = tensor(workload, div)
    out = oracle.mxfp4_quantize(bits)
    wb = w.double().numpy().reshape(-1, 32)
    bmax = np.abs(wb).max(axis=1)
    _, ex = np.frexp(bmax)                                   # bmax = m 2^ex, m in [0.5, 1)
    want = np.where(bmax > 0, np.clip(ex - 1 - 2, -127, 127) + 127, 127)
    assert np.array_equal(out.scales.reshape(-1), want.astype(np.uint8))
    x = wb / np.exp2(want - 127.0)[:, None]
    assert np.abs(x).max() < 8.0 and (np.abs(x) > 6.0).any()  # the format's own saturation zone is exercised
    q = unpack(out.codes).reshape(-1, 32)
    # the scaled values are exact in float64 (division by a power of two): the codes are a nearest grid
    # value everywhere, and differ from "first nearest" only at exact ties, where the even code is taken
    ax = np.minimum(np.abs(x), 6.0)
    near = np.abs(ax[..., None] - E2M1).min(axis=-1)
    assert np.all(np.abs(np.abs(q) - ax) == near)
    differ = q != nearest_grid(x)
    mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    assert np.all(np.isin(np.abs(x[differ]), mids))
    idx = np.abs(np.abs(q[differ])[..., None] - E2M1).argmin(axis=-1)
    assert np.all(idx % 2 == 0)
    e = ((wb - q * np.exp2(want - 127.0)[:, None]) ** 2).sum()
    assert math.isclose(out.sse, float(e), rel_tol=1e-5)
    assert out.status == 0


@pytest.mark.parametrize("K", [0, 1, 2])
def test_search_against_enumeration_of_all_pairs(K):
    w, bits = tensor()
    n_beta = 21
    base = oracle.mxfp4_quantize(bits)
    out = oracle.mxfp4_quantize(bits, True, n_beta, 0.5, 1.5, K)
    wb = w.double().numpy().reshape(-1, 32)
    e0 = base.scales.reshape(-1).astype(np.int64)
    betas = np.array([(0.5 * (n_beta - 1 - k) + 1.5 * k) / (n_beta - 1) for k in range(n_beta)])
    best = np.full(wb.shape[0], np.inf)
    for bt in betas:
        qq = nearest_grid(wb / (np.exp2(e0 - 127.0) * bt)[:, None])
        for o in range(-K, K + 1):
            c = np.clip(e0 + o, 0, 254)
            best = np.minimum(best, ((wb - qq * np.exp2(c - 127.0)[:, None]) ** 2).sum(axis=1))
    chosen = out.scales.reshape(-1).astype(np.int64)
    assert np.all(np.abs(chosen - e0) <= K)
    q = unpack(out.codes).reshape(-1, 32)
    e_out = ((wb - q * np.exp2(chosen - 127.0)[:, None]) ** 2).sum(axis=1)
    ref = (wb * wb).sum(axis=1)
    assert np.mean(e_out <= best + 2e-6 * ref) > 0.999
    assert np.all(e_out <= best * 1.02 + 2e-6 * ref)
    assert math.isclose(out.sse, float(e_out.sum()), rel_tol=1e-5)
    # the plain conversion is the pair (beta = 1, e0): no block may get worse, and the tensor gets better
    q0 = unpack(base.codes).reshape(-1, 32)
    e_base = ((wb - q0 * np.exp2(e0 - 127.0)[:, None]) ** 2).sum(axis=1)
    assert np.all(e_out <= e_base * (1 + 1e-6) + 1e-30)
    if K == 0:
        # with the stored scale fixed, nearest rounding under that very scale is already optimal
        # (an earlier factor may tie on an exactly-half element, so only the error is compared)
        assert out.sse == base.sse
    else:
        assert out.sse < base.sse and (chosen != e0).any()


def test_trivial_search_is_the_plain_conversion():
    _, bits = tensor(1, 1)
    a = oracle.mxfp4_quantize(bits)
    b = oracle.mxfp4_quantize(bits, True, 1, 1.0, 1.0, 0)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales) and a.sse == b.sse


def test_power_of_two_and_sign_equivariance():
    w, bits = tensor(1, 1)
    a = oracle.mxfp4_quantize(bits, True, 11, 0.5, 1.5, 1)
    b = oracle.mxfp4_quantize(synth.bf16_bits((w.float() * 2.0 ** -7).to(torch.bfloat16)), True, 11, 0.5, 1.5, 1)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales.astype(np.int64) - 7, b.scales.astype(np.int64))
    c = oracle.mxfp4_quantize(synth.bf16_bits(-w), True, 11, 0.5, 1.5, 1)
    assert np.array_equal(c.codes, a.codes ^ 0x88) and np.array_equal(c.scales, a.scales)


def test_dequantize_and_edges():
    w, bits = tensor(1, 1)
    out = oracle.mxfp4_quantize(bits)
    back = oracle.mxfp4_dequantize(out.codes, out.scales, oracle.FP32)
    want = unpack(out.codes) * np.repeat(np.exp2(out.scales.astype(np.float64) - 127.0), 32, axis=1)
    assert np.array_equal(back.astype(np.float64), want)
    back16 = oracle.mxfp4_dequantize(out.codes, out.scales, oracle.BF16)
    assert np.array_equal(back16, synth.bf16_bits(torch.from_numpy(back).to(torch.bfloat16)))
    e = ((w.double().numpy() - want) ** 2).sum()
    assert math.isclose(out.sse, float(e), rel_tol=1e-5)
    # zero block, tiny and huge magnitudes, bad shapes
    z = np.zeros((2, 64), dtype=np.float32)
    z[1, 0] = -0.0
    o = oracle.mxfp4_quantize(z)
    assert (o.scales == 127).all() and o.sse == 0.0 and o.codes[1, 0] == 0x08
    t = np.full((1, 32), 2.0 ** -140, dtype=np.float32)
    assert oracle.mxfp4_quantize(t).scales[0, 0] == 0
    h = np.full((1, 32), 3.0e38, dtype=np.float32)
    assert oracle.mxfp4_quantize(h).scales[0, 0] == 127 + 127 - 2
    n = np.zeros((1, 32), dtype=np.float32)
    n[0, 3] = np.nan
    assert oracle.mxfp4_quantize(n).status == oracle.STATUS_NONFINITE
    with pytest.raises(ValueError):
        oracle.mxfp4_quantize(np.zeros((4, 48), dtype=np.float32))


def test_first_pair_wins_an_exact_tie():
    """Blocks of small dyadic values with the factors {0.5, 1}: every quantity of the search is exact in
    binary32 and binary64 alike, so the enumeration below is exact, ties included.  Where two pairs with
    different outputs reach the least error, the earlier one (beta ascending, then e0, e0-1, e0+1) is kept."""
    rng = np.random.default_rng(5)
    ties = 0
    for _ in range(4000):
        blk = np.zeros((1, 32), dtype=np.float32)
        n = rng.integers(1, 4)
        blk[0, :n] = rng.integers(-48, 49, size=n) / 8.0
        if not blk.any():
            continue
        out = oracle.mxfp4_quantize(blk, True, 2, 0.5, 1.0, 1)
        e0 = int(oracle.mxfp4_quantize(blk).scales[0, 0])
        wb = blk.astype(np.float64)[0]
        cands = []
        for bt in (0.5, 1.0):
            x = wb / (2.0 ** (e0 - 127) * bt)
            ax = np.minimum(np.abs(x), 6.0)
            idx = np.abs(ax[:, None] - E2M1).argmin(axis=1)
            # exact ties go to the even code
            d = np.abs(ax[:, None] - E2M1)
            tie = (np.sort(d, axis=1)[:, 0] == np.sort(d, axis=1)[:, 1])
            idx = np.where(tie & (idx % 2 == 1), idx + 1, idx)
            q = np.sign(x) * E2M1[idx]
            for c in (e0, e0 - 1, e0 + 1):
                err = float(((wb - q * 2.0 ** (c - 127)) ** 2).sum())
                cands.append((err, tuple(q), c))
        least = min(c[0] for c in cands)
        winners = [c for c in cands if c[0] == least]
        first = winners[0]
        if any((w[1], w[2]) != (first[1], first[2]) for w in winners[1:]):
            ties += 1
        assert int(out.scales[0, 0]) == first[2], blk[0, :n]
        assert tuple(unpack(out.codes)[0]) == first[1], blk[0, :n]
        assert out.sse == least
    assert ties >= 20
