"""Pins for the oracle's full Algorithm 1 (T iterations, beta grid, early stop).

Checked against: the already pinned single-step function (special case),
float64 enumeration of every (beta, stored scale) pair, prefix consistency of
the error trace, the early-stop rule evaluated on an unstopped run, the
qualitative statements of the paper's convergence figure, exact equivariances.
"""
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


def tensor(workload, div, shift=0):
    spec = synth.workload_specs(workload, div)[0]
    if shift:
        spec = type(spec)(**{**spec.__dict__, "index": spec.index + shift})
    w = synth.make_weight(spec, "cpu")
    return spec, w, synth.bf16_bits(w)


CASES = [(1, 2), (2, 32), (5, 128)]


@pytest.mark.parametrize("workload,div", CASES)
@pytest.mark.parametrize("K", [0, 1, 4])
def test_single_step_special_case_equals_the_pinned_function(workload, div, K):
    _, _, bits = tensor(workload, div)
    a = oracle.quantize(bits, oracle.METHOD_SOAR, K)
    b = oracle.quantize_iter(bits, 1, 1, 1.0, 1.0, oracle.DD_WINDOW, K, 0.0)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
    assert a.global_scale == b.global_scale and a.sse == b.sse
    assert b.trace["iters_run"] == 1
    assert b.trace["sse_trace"][0] == oracle.quantize(bits, oracle.METHOD_RTN, 0).sse
    assert b.trace["sse_trace"][1] == b.sse


def _nearest_grid(x):
    a = np.minimum(np.abs(x), 1e3)
    idx = np.abs(a[..., None] - E2M1).argmin(axis=-1)
    return np.sign(x) * E2M1[idx]


def _state(bits, t, n_beta, lo, hi, dd_mode, K):
    """(codes, scales, alpha) after t iterations; t = 0 is the Eq. 1-2 state."""
    if t == 0:
        r = oracle.quantize(bits, oracle.METHOD_RTN, 0)
    else:
        r = oracle.quantize_iter(bits, t, n_beta, lo, hi, dd_mode, K, 0.0)
    return r


@pytest.mark.parametrize("t", [1, 2, 4])
@pytest.mark.parametrize("dd_mode", [oracle.DD_WINDOW, oracle.DD_BRACKET])
def test_iteration_t_against_enumeration_of_all_pairs(dd_mode, t):
    """Iteration t with an 11-point beta grid, rebuilt in float64 from the outputs of the
    run that stops one iteration earlier: Eq. 5 from (Q, stored scales) of that state,
    Eq. 6 from its block sums, and per block the chosen (codes, scale) must reach the
    minimum over every (beta, candidate scale) pair."""
    _, w, bits = tensor(2, 32)
    n_beta, lo, hi, K = 11, 0.5, 1.5, 2
    before = _state(bits, t - 1, n_beta, lo, hi, dd_mode, K)
    out = _state(bits, t, n_beta, lo, hi, dd_mode, K)
    wb = w.double().numpy().reshape(-1, 16)
    q = unpack(before.codes).reshape(-1, 16)
    d_before = E4M3[before.scales.reshape(-1)]
    a = (wb * q).sum(axis=1)
    b = (q * q).sum(axis=1)
    alpha = float((a * d_before).sum() / (b * d_before * d_before).sum())          # Eq. 5
    assert math.isclose(float(out.global_scale), alpha, rel_tol=1e-6)
    alpha = float(out.global_scale)
    ds = np.where(b > 0, a / np.where(b > 0, b, 1) / alpha, d_before)               # Eq. 6
    betas = np.array([(lo * (n_beta - 1 - k) + hi * k) / (n_beta - 1) for k in range(n_beta)])
    assert betas[5] == 1.0 and betas[0] == lo and betas[-1] == hi
    floor = np.array([np.nonzero(E4M3[1:0x7F] <= d)[0].max() + 1 if d >= E4M3[1] else 1 for d in ds])
    chosen = out.scales.reshape(-1).astype(np.int64)
    if dd_mode == oracle.DD_WINDOW:
        up = np.minimum(floor + 1, 0x7E)
        centre = np.where(ds - E4M3[floor] <= E4M3[up] - ds, floor, up)
        cands = [np.clip(centre + o, 1, 0x7E) for o in range(-K, K + 1)]
        assert np.mean(np.abs(chosen - centre) <= K) > 0.9999      # float32 vs float64 ties only
    else:
        cands = [floor, np.minimum(floor + 1, 0x7E)]
        assert np.mean((chosen == cands[0]) | (chosen == cands[1])) > 0.9999
    best = np.full(wb.shape[0], np.inf)
    for bt in betas:
        qq = _nearest_grid(wb / (alpha * ds * bt)[:, None])
        for c in cands:
            e = ((wb - qq * (alpha * E4M3[c])[:, None]) ** 2).sum(axis=1)
            best = np.minimum(best, e)
    q_out = unpack(out.codes).reshape(-1, 16)
    e_out = ((wb - q_out * (alpha * E4M3[chosen])[:, None]) ** 2).sum(axis=1)
    scale_ref = (wb * wb).sum(axis=1)
    # what is left: float32 evaluation noise and rounding ties of the float64 re-quantization
    assert np.mean(e_out <= best + 2e-6 * scale_ref) > 0.999
    assert np.all(e_out <= best * 1.02 + 2e-6 * scale_ref)
    assert math.isclose(out.sse, float(e_out.sum()), rel_tol=1e-5)
    if dd_mode == oracle.DD_WINDOW and t == 1:
        # a grid that contains beta = 1 cannot lose to beta = {1} with the same stored-scale candidates
        assert out.sse <= oracle.quantize(bits, oracle.METHOD_SOAR, K).sse


def test_trace_prefix_consistency_and_reported_error():
    _, w, bits = tensor(1, 2)
    full = oracle.quantize_iter(bits, 6, 21, 0.5, 1.5, oracle.DD_BRACKET, 1, 0.0)
    tr = full.trace["sse_trace"]
    assert full.trace["iters_run"] == 6 and not np.isnan(tr).any()
    for t in (1, 3, 6):
        part = oracle.quantize_iter(bits, t, 21, 0.5, 1.5, oracle.DD_BRACKET, 1, 0.0)
        assert part.sse == tr[t]
        assert np.array_equal(part.trace["sse_trace"][: t + 1], tr[: t + 1])
        assert oracle.recon_error(bits, part.codes, part.scales, part.global_scale) == part.sse
        w64 = w.double().numpy()
        q = unpack(part.codes)
        s = np.repeat(E4M3[part.scales], 16, axis=1) * float(part.global_scale)
        assert math.isclose(part.sse, float(((w64 - q * s) ** 2).sum()), rel_tol=1e-5)


@pytest.mark.parametrize("workload,div", CASES)
def test_early_stop_rule(workload, div):
    _, _, bits = tensor(workload, div)
    free = oracle.quantize_iter(bits, 15, 21, 0.5, 1.5, oracle.DD_BRACKET, 1, 0.0)
    tr = free.trace["sse_trace"]
    for rel in (1e-3, 1e-2, 0.2):
        want = 15
        for t in range(15):
            if (tr[t] - tr[t + 1]) < np.float64(np.float32(rel)) * tr[t]:
                want = t + 1
                break
        got = oracle.quantize_iter(bits, 15, 21, 0.5, 1.5, oracle.DD_BRACKET, 1, rel)
        assert got.trace["iters_run"] == want, rel
        same = oracle.quantize_iter(bits, want, 21, 0.5, 1.5, oracle.DD_BRACKET, 1, 0.0)
        assert np.array_equal(got.codes, same.codes) and np.array_equal(got.scales, same.scales)
        assert got.global_scale == same.global_scale and got.sse == same.sse
        assert np.isnan(got.trace["sse_trace"][want + 1:]).all()


@pytest.mark.parametrize("workload,div", CASES)
def test_convergence_statements_of_the_paper(workload, div):
    """Error falls with the iterations, and the decoupled search reaches a lower
    floor than the closed-form steps with beta = 1 alone (paper, convergence figure)."""
    _, _, bits = tensor(workload, div)
    soar = oracle.quantize_iter(bits, 8, 101, 0.5, 1.5, oracle.DD_BRACKET, 1, 0.0)
    plain = oracle.quantize_iter(bits, 8, 1, 1.0, 1.0, oracle.DD_BRACKET, 1, 0.0)
    tr = soar.trace["sse_trace"]
    # the re-assignment step may drop the previous (Q, stored scale) pair from the candidate
    # set, so the fall is not strict: rises stay at rounding-noise size, the net fall is large
    assert np.all(np.diff(tr) <= 1e-4 * tr[0])
    assert np.all(np.diff(tr)[:3] < 0)
    assert tr[-1] < plain.trace["sse_trace"][-1] < tr[0]
    rtn = oracle.quantize(bits, oracle.METHOD_RTN, 0)
    assert tr[0] == rtn.sse and soar.sse < rtn.sse


def test_equivariance_and_degenerate_inputs():
    _, w, bits = tensor(1, 2)
    base = oracle.quantize_iter(bits, 3, 11, 0.5, 1.5, oracle.DD_BRACKET, 1, 0.0)
    up = oracle.quantize_iter(synth.bf16_bits((w.float() * 2.0 ** 5).to(torch.bfloat16)), 3, 11, 0.5, 1.5,
                              oracle.DD_BRACKET, 1, 0.0)
    assert np.array_equal(up.codes, base.codes) and np.array_equal(up.scales, base.scales)
    assert up.global_scale == np.float32(base.global_scale * np.float32(32.0))
    neg = oracle.quantize_iter(synth.bf16_bits(-w), 3, 11, 0.5, 1.5, oracle.DD_BRACKET, 1, 0.0)
    assert np.array_equal(neg.codes, base.codes ^ 0x88) and np.array_equal(neg.scales, base.scales)
    z = np.zeros((4, 32), dtype=np.uint16)
    o = oracle.quantize_iter(z)
    assert o.status & oracle.STATUS_ALLZERO and o.trace["iters_run"] == 0
    with pytest.raises(ValueError):
        oracle.quantize_iter(bits, iters=0)
    with pytest.raises(ValueError):
        oracle.quantize_iter(bits, beta_lo=1.5, beta_hi=0.5)
