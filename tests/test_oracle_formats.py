"""Pins for the oracle's number-format primitives (CPU only).

Each check compares the oracle with something that is not the oracle: the
value grids the paper states (Sec. 3.1), brute-force nearest-value search, or a
library cast (torch float8_e4m3fn / bfloat16).
"""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([float(t) for t in line.split()])
    return rows


# ----------------------------------------------------------------------- E2M1
E2M1_MAGS = np.array([v[0] for v in _read_table("e2m1_grid.txt")], dtype=np.float64)


def _brute_e2m1(x: np.ndarray) -> np.ndarray:
    """Nearest of the 8 magnitudes (exact distances in float64; a tie goes to
    the even index), saturating, sign bit from the input."""
    a = np.minimum(np.abs(x.astype(np.float64)), 1e3)   # keeps float64 distances exact
    dist = np.abs(a[:, None] - E2M1_MAGS[None, :])
    best = np.full(a.shape, 0, dtype=np.int64)
    bestd = dist[:, 0].copy()
    for k in range(1, 8):
        dk = dist[:, k]
        better = dk < bestd
        tie = (dk == bestd) & (k % 2 == 0)
        take = better | tie
        best[take] = k
        bestd[take] = dk[take]
    sign = np.signbit(x).astype(np.int64) << 3
    return (sign | best).astype(np.uint8)


def test_e2m1_grid_is_the_papers():
    assert list(E2M1_MAGS) == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    for k, m in enumerate(E2M1_MAGS):
        assert oracle.e2m1_value(k) == m
        assert oracle.e2m1_value(k | 8) == -m or m == 0.0
        assert oracle.e2m1_nibble(float(m)) == k
        assert oracle.e2m1_nibble(-float(m)) == (k | 8)


def test_e2m1_ties_golden():
    for x, want in _read_table("e2m1_ties.txt"):
        assert oracle.e2m1_round(x) == want, (x, want)
        assert oracle.e2m1_round(-x) == -want


def test_e2m1_all_bf16_patterns_times_scales():
    bits = np.arange(65536, dtype=np.uint32)
    x = (bits << 16).view(np.float32)
    x = x[np.isfinite(x)]
    for s in (1.0, 0.37, 3.3, 1.0 / 3.0, 117.0, 2.0 ** -20):
        xs = (x * np.float32(s)).astype(np.float32)
        xs = xs[np.isfinite(xs)]
        got = oracle.e2m1_nibble_many(xs)
        assert np.array_equal(got, _brute_e2m1(xs)), s


def test_e2m1_random_and_neighbourhood_of_thresholds():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(400_000) * 3).astype(np.float32)
    thr = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0, 2.0, 4.0], dtype=np.float32)
    near = []
    for t in thr:
        v = t
        lo = t
        for _ in range(8):
            v = np.nextafter(v, np.float32(np.inf), dtype=np.float32)
            lo = np.nextafter(lo, np.float32(-np.inf), dtype=np.float32)
            near += [v, lo, -v, -lo]
        near += [t, -t]
    x = np.concatenate([x, np.array(near, dtype=np.float32),
                        np.array([0.0, -0.0, 1e-30, -1e-30, 1e30, -1e30, 7.0, 6.0001], np.float32)])
    assert np.array_equal(oracle.e2m1_nibble_many(x), _brute_e2m1(x))


def test_e2m1_monotone_idempotent_saturating():
    x = np.linspace(-8, 8, 20001).astype(np.float32)
    v = np.array([oracle.e2m1_value(int(n)) for n in oracle.e2m1_nibble_many(x)])
    assert np.all(np.diff(v) >= 0)
    assert v.max() == 6.0 and v.min() == -6.0
    again = np.array([oracle.e2m1_value(int(n)) for n in oracle.e2m1_nibble_many(v.astype(np.float32))])
    assert np.array_equal(v, again)
    assert oracle.e2m1_nibble(-0.0) == 8 and oracle.e2m1_nibble(-0.2) == 8 and oracle.e2m1_nibble(0.2) == 0


# ----------------------------------------------------------------------- E4M3
def _torch_e4m3_values():
    codes = torch.arange(0, 128, dtype=torch.uint8)
    return codes.view(torch.float8_e4m3fn).float().numpy()


def test_e4m3_values_match_library_cast_table():
    lib_vals = _torch_e4m3_values()
    for c in range(0, 0x7F):
        assert oracle.e4m3_value(c) == lib_vals[c], c
    assert oracle.e4m3_value(0x7E) == 448.0          # M_FP8 of Sec. 3.1
    assert oracle.e4m3_value(0x01) == 2.0 ** -9
    assert np.isnan(lib_vals[0x7F])


def test_e4m3_roundtrip_all_codes():
    for c in range(1, 0x7F):
        assert oracle.e4m3_project(oracle.e4m3_value(c)) == c


def test_e4m3_project_matches_library_cast_in_range():
    # every float32 between 2^-10 (exclusive) and 464 (exclusive), binade by binade
    for e in range(-10, 9):
        base = np.float32(2.0 ** e).view(np.uint32)
        bits = base + np.arange(0, 1 << 23, 3, dtype=np.uint32)
        y = bits.view(np.float32)
        y = y[(y > np.float32(2.0 ** -10)) & (y < np.float32(464.0))]
        got = oracle.e4m3_project_many(y)
        want = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(got, want), e


def _brute_e4m3(y: np.ndarray) -> np.ndarray:
    vals = _torch_e4m3_values()[1:0x7F].astype(np.float64)      # codes 1..126
    yy = np.clip(y.astype(np.float64), 0.0, 1e6)
    out = np.empty(y.shape, dtype=np.uint8)
    for i, v in enumerate(yy):
        d = np.abs(vals - v)
        k = int(np.argmin(d))
        # tie: even code (= even mantissa)
        ties = np.nonzero(d == d[k])[0]
        if len(ties) > 1:
            k = int([t for t in ties if (t + 1) % 2 == 0][0])
        out[i] = k + 1
    return out


def test_e4m3_project_brute_force_with_clip():
    rng = np.random.default_rng(2)
    y = np.exp(rng.uniform(np.log(1e-5), np.log(2000.0), 20000)).astype(np.float32)
    vals = _torch_e4m3_values()[1:0x7F]
    mids = ((vals[:-1].astype(np.float64) + vals[1:].astype(np.float64)) / 2).astype(np.float32)
    edge = []
    for m in mids:
        edge += [m, np.nextafter(m, np.float32(0)), np.nextafter(m, np.float32(1e9))]
    y = np.concatenate([y, np.array(edge, np.float32),
                        np.array([0.0, 1e-12, 2.0 ** -10, 2.0 ** -9, 448, 464, 465, 480, 1e30], np.float32)])
    # 2^-10 is the midpoint of 0 and 2^-9: after the clip both give code 1
    assert np.array_equal(oracle.e4m3_project_many(y), _brute_e4m3(y))
    assert oracle.e4m3_project(float("inf")) == 0x7E
    assert oracle.e4m3_project(0.0) == 0x01
    assert oracle.e4m3_project(-1.0) == 0x01


# ----------------------------------------------------------------------- bf16
def test_bf16_rounding_matches_library_cast():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(50000) * np.exp(rng.uniform(-20, 20, 50000))).astype(np.float32)
    ties = (np.arange(1, 2000, dtype=np.uint32) << 16 | 0x8000).view(np.float32) + np.float32(0)
    x = np.concatenate([x, ties, -ties])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f32_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
    back = oracle.bf16_to_f32(want)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())
