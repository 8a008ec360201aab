"""Pins for the oracle's max-based NVFP4 with a supplied tensor maximum (Sec. 3.1 as applied
to activations, Appendix B.2): the measured-maximum function as special case, float64
nearest-of-grid with saturation for a maximum that is too small, clipping of the block
scale, exact scaling behaviour, argument checks."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2605_12245_amd import synth

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
E4M3 = torch.arange(0, 128, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)


def unpack(codes):
    nib = np.stack([codes & 0xF, codes >> 4], axis=-1).reshape(codes.shape[0], -1)
    v = E2M1[nib & 7]
    return np.where(nib & 8, -v, v)


def case(workload=2, div=16):
    spec = synth.workload_specs(workload, div)[0]
    w = synth.make_weight(spec, "cpu")
    return w, synth.bf16_bits(w)


def test_true_maximum_reproduces_the_measured_function():
    for workload, div in ((1, 1), (2, 16), (5, 64)):
        w, bits = case(workload, div)
        amax = float(w.float().abs().max())
        a = oracle.quantize(bits, oracle.METHOD_RTN, 0)
        b = oracle.quantize_rtn_amax(bits, amax)
        assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
        assert a.global_scale == b.global_scale and a.sse == b.sse and b.status == 0


@pytest.mark.parametrize("factor", [0.05, 0.3, 1.0, 1.7, 40.0])
def test_against_float64_nearest_of_grid_with_saturation(factor):
    w, bits = case()
    amax = float(np.float32(float(w.float().abs().max()) * factor))
    out = oracle.quantize_rtn_amax(bits, amax)
    alpha = np.float32(amax) / np.float32(2688.0)
    assert out.global_scale == alpha
    wb = w.double().numpy().reshape(-1, 16)
    bmax = np.abs(wb).max(axis=1)
    # block scale: nearest E4M3 to bmax / (6 alpha), clipped to [2^-9, 448]
    target = np.clip(bmax / (6.0 * float(alpha)), E4M3[1], 448.0)
    codes = out.scales.reshape(-1).astype(np.int64)
    dist = np.abs(E4M3[1:0x7F][None, :] - target[:, None])
    assert np.all(np.abs(E4M3[codes] - target) <= dist.min(axis=1) * (1 + 1e-6) + 1e-300)
    if factor < 1.0:
        assert (codes == 0x7E).any()            # blocks above the supplied maximum clip the scale
    # elements: nearest grid value of w / (alpha d), saturating at 6, sign kept
    s = float(alpha) * E4M3[codes]
    x = wb / s[:, None]
    q = unpack(out.codes).reshape(-1, 16)
    near = np.abs(np.minimum(np.abs(x), 1e3)[..., None] - E2M1).min(axis=-1)
    assert np.all(np.abs(np.abs(q) - np.minimum(np.abs(x), 1e3)) <= near + 1e-6)
    assert np.all((q == 0) | (np.sign(q) == np.sign(wb)))
    if factor < 1.0:
        assert (np.abs(x) > 6.0).any() and np.all(np.abs(q)[np.abs(x) > 6.0] == 6.0)
    e = ((wb - q * s[:, None]) ** 2).sum()
    assert math.isclose(out.sse, float(e), rel_tol=1e-5)
    assert oracle.recon_error(bits, out.codes, out.scales, out.global_scale) == out.sse


def test_power_of_two_scaling_of_input_and_maximum():
    w, bits = case(1, 1)
    amax = float(w.float().abs().max()) * 0.75
    a = oracle.quantize_rtn_amax(bits, amax)
    b = oracle.quantize_rtn_amax(synth.bf16_bits((w.float() * 16.0).to(torch.bfloat16)), amax * 16.0)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
    assert b.global_scale == np.float32(a.global_scale * np.float32(16.0))


def test_bad_maximum_is_flagged_and_writes_nothing():
    _, bits = case(1, 1)
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        out = oracle.quantize_rtn_amax(bits, bad)
        assert out.status == oracle.STATUS_BAD_AMAX
        assert not out.codes.any() and not out.scales.any()
    f = np.zeros((4, 24), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.quantize_rtn_amax(f, 1.0)
