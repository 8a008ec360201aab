"""Pins for the two ablation arms of the oracle's iterated function: "+CJSO" alone (Sec. 3.2,
refinement scheme: one block scale, projected onto E4M3, used for assignment and storage) and
"+DSS" alone (Sec. 3.3 (i)-(ii): max-based initialisation, joint search, no closed-form step).
Each iteration is rebuilt in float64 from the outputs of the run that stops one iteration earlier."""
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


def nearest_grid(x):
    a = np.minimum(np.abs(x), 1e3)
    return np.sign(x) * E2M1[np.abs(a[..., None] - E2M1).argmin(axis=-1)]


def tensor(workload=2, div=32):
    spec = synth.workload_specs(workload, div)[0]
    w = synth.make_weight(spec, "cpu")
    return w, synth.bf16_bits(w)


def cjso(bits, t, stop=0.0):
    if t == 0:
        return oracle.quantize(bits, oracle.METHOD_RTN, 0)
    return oracle.quantize_iter(bits, t, 1, 1.0, 1.0, oracle.DD_WINDOW, 0, stop, oracle.ARM_CJSO_ONLY)


def dss(bits, t, n_beta=11, K=2):
    if t == 0:
        return oracle.quantize(bits, oracle.METHOD_RTN, 0)
    return oracle.quantize_iter(bits, t, n_beta, 0.5, 1.5, oracle.DD_WINDOW, K, 0.0, oracle.ARM_DSS_ONLY)


@pytest.mark.parametrize("t", [1, 2, 5])
def test_cjso_only_iteration_rebuilt_in_float64(t):
    w, bits = tensor()
    before, out = cjso(bits, t - 1), cjso(bits, t)
    wb = w.double().numpy().reshape(-1, 16)
    q = unpack(before.codes).reshape(-1, 16)
    d0 = E4M3[before.scales.reshape(-1)]
    a, b = (wb * q).sum(axis=1), (q * q).sum(axis=1)
    alpha = float((a * d0).sum() / (b * d0 * d0).sum())                      # Eq. 5
    assert math.isclose(float(out.global_scale), alpha, rel_tol=1e-6)
    alpha = float(out.global_scale)
    ds = np.where(b > 0, a / np.where(b > 0, b, 1) / alpha, d0)               # Eq. 6
    # projection onto E4M3 (nearest of the 126 codes, clipped)
    target = np.clip(ds, E4M3[1], 448.0)
    code = out.scales.reshape(-1).astype(np.int64)
    dist = np.abs(E4M3[1:0x7F][None, :] - target[:, None]).min(axis=1)
    assert np.all(np.abs(E4M3[code] - target) <= dist * (1 + 1e-6) + 1e-300)
    # ONE scale: the codes are those of the projected scale, not of the unrounded Eq. 6 value
    s = alpha * E4M3[code]
    want = nearest_grid(wb / s[:, None])
    got = unpack(out.codes).reshape(-1, 16)
    assert np.mean(got == want) > 0.9999
    e = ((wb - got * s[:, None]) ** 2).sum()
    assert math.isclose(out.sse, float(e), rel_tol=1e-5)
    assert oracle.recon_error(bits, out.codes, out.scales, out.global_scale) == out.sse
    decoupled = nearest_grid(wb / (alpha * ds)[:, None])
    assert np.mean(got == decoupled) < 0.9999            # the two assignments really differ on this tensor


def test_cjso_only_trace_and_floor_above_soar():
    """Convergence figure of the paper: the closed-form steps alone settle on a higher error than SOAR."""
    for workload, div in ((1, 1), (2, 32), (5, 128)):
        _, bits = tensor(workload, div)
        c = cjso(bits, 8)
        s = oracle.quantize_iter(bits, 8, 101, 0.5, 1.5, oracle.DD_BRACKET, 1, 0.0)
        tr = c.trace["sse_trace"]
        assert tr[0] == oracle.quantize(bits, oracle.METHOD_RTN, 0).sse
        assert tr[-1] < tr[0] and s.trace["sse_trace"][-1] < tr[-1]
        for k in (1, 3):
            assert cjso(bits, k).sse == tr[k]
        stopped = cjso(bits, 8, stop=1e-3)
        n = stopped.trace["iters_run"]
        assert 1 <= n <= 8 and stopped.sse == tr[n]
        assert n == 8 or (tr[n - 1] - tr[n]) < np.float64(np.float32(1e-3)) * tr[n - 1]


def test_cjso_only_takes_no_search_parameters():
    _, bits = tensor(1, 1)
    for kw in (dict(n_beta=3), dict(beta_lo=0.5, beta_hi=0.5), dict(dd_mode=oracle.DD_BRACKET), dict(dss_radius=1)):
        args = dict(iters=2, n_beta=1, beta_lo=1.0, beta_hi=1.0, dd_mode=oracle.DD_WINDOW, dss_radius=0,
                    early_stop_rel=0.0, arm=oracle.ARM_CJSO_ONLY)
        args.update(kw)
        with pytest.raises(ValueError):
            oracle.quantize_iter(bits, **args)


@pytest.mark.parametrize("t", [1, 2])
def test_dss_only_iteration_against_enumeration(t):
    w, bits = tensor()
    n_beta, K = 11, 2
    before, out = dss(bits, t - 1, n_beta, K), dss(bits, t, n_beta, K)
    rtn = oracle.quantize(bits, oracle.METHOD_RTN, 0)
    assert out.global_scale == rtn.global_scale                     # no closed-form step, ever
    alpha = float(out.global_scale)
    wb = w.double().numpy().reshape(-1, 16)
    centre = before.scales.reshape(-1).astype(np.int64)             # the search is centred on the stored scale
    betas = np.array([(0.5 * (n_beta - 1 - k) + 1.5 * k) / (n_beta - 1) for k in range(n_beta)])
    best = np.full(wb.shape[0], np.inf)
    for bt in betas:
        qq = nearest_grid(wb / (alpha * E4M3[centre] * bt)[:, None])
        for o in range(-K, K + 1):
            c = np.clip(centre + o, 1, 0x7E)
            best = np.minimum(best, ((wb - qq * (alpha * E4M3[c])[:, None]) ** 2).sum(axis=1))
    chosen = out.scales.reshape(-1).astype(np.int64)
    assert np.all(np.abs(chosen - centre) <= K)
    got = unpack(out.codes).reshape(-1, 16)
    e_out = ((wb - got * (alpha * E4M3[chosen])[:, None]) ** 2).sum(axis=1)
    ref = (wb * wb).sum(axis=1)
    assert np.mean(e_out <= best + 2e-6 * ref) > 0.999
    assert np.all(e_out <= best * 1.02 + 2e-6 * ref)
    assert math.isclose(out.sse, float(e_out.sum()), rel_tol=1e-5)
    if t == 1:
        # beta = 1 with the centre itself is the Eq. 1-2 state: no block can get worse than plain NVFP4
        q_prev = unpack(before.codes).reshape(-1, 16)
        e_prev = ((wb - q_prev * (alpha * E4M3[centre])[:, None]) ** 2).sum(axis=1)
        assert np.all(e_out <= e_prev * (1 + 1e-5) + 1e-30)


def test_dss_only_trace():
    _, bits = tensor(1, 1)
    d = dss(bits, 4, 101, 1)
    tr = d.trace["sse_trace"]
    assert tr[0] == oracle.quantize(bits, oracle.METHOD_RTN, 0).sse
    assert tr[1] < tr[0] and np.all(np.diff(tr) <= 1e-4 * tr[0])
    assert dss(bits, 2, 101, 1).sse == tr[2]
