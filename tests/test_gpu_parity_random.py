"""Seeded sweep of valid inputs over every entry point: random shapes (ragged against tiles and rows),
element types, leading dimensions, magnitudes, outlier structure and parameter settings, each compared
with the oracle to the bar of the dedicated parity tests."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_12245_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(rng, block):
    rows = int(rng.integers(1, 300))
    cols = block * int(rng.integers(1, 40))
    g = torch.Generator(device="cpu").manual_seed(int(rng.integers(1 << 30)))
    scale = float(2.0 ** rng.integers(-40, 30))
    w = torch.randn(rows, cols, generator=g) * scale
    kind = int(rng.integers(4))
    if kind == 1:                                   # heavy tails
        w = w * torch.exp(torch.randn(rows, cols, generator=g))
    elif kind == 2:                                 # outlier columns
        w[:, :: max(1, cols // 5)] *= 30.0
    elif kind == 3:                                 # zero blocks and rows
        w[:, : block] = 0.0
        w[rows // 2] = 0.0
    fp32 = bool(rng.integers(2))
    pad = int(rng.integers(3)) * (4 if fp32 else 8) * 4
    parent = torch.full((rows, cols + pad), float("inf"), dtype=torch.float32 if fp32 else torch.bfloat16)
    parent[:, :cols] = w.to(parent.dtype)
    dev_parent = parent.to(DEV)
    view = dev_parent[:, :cols]
    host = parent[:, :cols].contiguous()
    host = host.numpy() if fp32 else host.view(torch.int16).numpy().view(np.uint16)
    return view, host, (dev_parent, pad)


def nv_compare(out, ref, what, trace=False):
    assert int(out.status.item()) == ref.status, what
    assert np.array_equal(out.scales.cpu().numpy(), ref.scales), what
    assert np.array_equal(out.codes.cpu().numpy(), ref.codes), what
    assert np.float32(out.global_scale.item()) == ref.global_scale, what
    assert math.isclose(float(out.sse.item()), ref.sse, rel_tol=1e-6, abs_tol=0.0) or ref.sse == 0.0, what
    if trace:
        assert int(out.iters_run.item()) == ref.trace["iters_run"], what
        a, b = out.sse_trace.cpu().numpy(), ref.trace["sse_trace"]
        assert np.array_equal(np.isnan(a), np.isnan(b)) and np.array_equal(a[~np.isnan(b)], b[~np.isnan(b)]), what


@pytest.mark.parametrize("seed", range(int(os.environ.get("SOAR_RANDOM_SEEDS", "6"))))
def test_random_cases(seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(8):
        what = f"seed {seed} case {case}"
        # --- NVFP4, single step and plain, through the single-tensor entry point
        view, host, keep = make(rng, 16)
        K = int(rng.integers(0, 9))
        for method, om in ((B.SOAR_METHOD_SOAR, oracle.METHOD_SOAR), (B.SOAR_METHOD_RTN, oracle.METHOD_RTN)):
            # a forced launch shape takes the general kernels, the default one the one-workgroup kernel where it fits
            out = B.quantize(view, method, K, int(rng.integers(2)), tiles_per_wg=int(2 ** rng.integers(0, 4)))
            dflt = B.quantize(view, method, K)
            torch.cuda.synchronize()
            ref = oracle.quantize(host, om, K)
            nv_compare(out, ref, what + f" nvfp4 m{method} K{K}")
            nv_compare(dflt, ref, what + f" nvfp4 m{method} K{K}, default launch shape")
            # Eq. 3 and Eq. 4 on the stored form, one-tensor and batch calls
            packed = view.contiguous()
            sse1 = float(B.recon_error(view, dflt).item())
            sse2 = float(B.recon_error_batch([view, packed], [dflt, dflt])[1].item())
            assert math.isclose(sse1, ref.sse, rel_tol=1e-6) or ref.sse == 0.0, what
            assert math.isclose(sse2, sse1, rel_tol=1e-12) or sse1 == 0.0, what
            if not (ref.status & oracle.STATUS_NONFINITE):
                dt = torch.float32 if rng.integers(2) else torch.bfloat16
                back = B.dequantize_batch([dflt], dt)[0].cpu()
                want = oracle.dequantize(ref.codes, ref.scales, ref.global_scale, oracle.FP32 if dt == torch.float32 else oracle.BF16)
                got = back.numpy() if dt == torch.float32 else back.view(torch.int16).numpy().view(np.uint16)
                assert np.array_equal(got, want), what + " dequantize"
        # --- the iterated path and its arms
        arm = int(rng.integers(3))
        if arm == 0:
            p = B.soar_paper_params(iters=int(rng.integers(1, 5)), n_beta=int(rng.integers(1, 24)),
                                    beta_lo=float(rng.uniform(0.4, 1.0)), beta_hi=float(rng.uniform(1.0, 1.8)),
                                    dd_mode=int(rng.integers(2)), dss_radius=int(rng.integers(0, 4)),
                                    early_stop_rel=float(rng.choice([0.0, 1e-3, 5e-2])))
        elif arm == 1:
            p = B.soar_arm_params(B.SOAR_METHOD_CJSO_ONLY, iters=int(rng.integers(1, 6)),
                                  early_stop_rel=float(rng.choice([0.0, 1e-2])))
        else:
            p = B.soar_arm_params(B.SOAR_METHOD_DSS_ONLY, iters=int(rng.integers(1, 4)), early_stop_rel=0.0,
                                  n_beta=int(rng.integers(1, 16)), dss_radius=int(rng.integers(0, 3)))
        p.tiles_per_wg = int(2 ** rng.integers(0, 3))
        out = B.quantize_iter(view, p)
        torch.cuda.synchronize()
        oarm = {B.SOAR_METHOD_SOAR: 0, B.SOAR_METHOD_CJSO_ONLY: 1, B.SOAR_METHOD_DSS_ONLY: 2}[p.method]
        ref = oracle.quantize_iter(host, p.iters, p.n_beta, p.beta_lo, p.beta_hi, p.dd_mode, p.dss_radius,
                                   p.early_stop_rel, oarm)
        nv_compare(out, ref, what + f" iterated arm {arm}", trace=True)
        # --- plain NVFP4 with a supplied maximum
        amax = float(np.float32(2.0 ** rng.uniform(-45, 35)))
        out = B.quantize_rtn_amax(view, torch.tensor([amax], dtype=torch.float32, device=DEV))
        torch.cuda.synchronize()
        nv_compare(out, oracle.quantize_rtn_amax(host, amax), what + " supplied maximum")
        # padding next to the matrix is never written (and, being Inf, was never read into a maximum)
        parent, pad = keep
        if pad:
            assert torch.isinf(parent[:, -pad:]).all()
        # --- MXFP4
        view, host, keep = make(rng, 32)
        mp = B.soar_mx_default_params(dss=bool(rng.integers(2)), n_beta=int(rng.integers(1, 20)),
                                      beta_lo=float(rng.uniform(0.4, 1.0)), beta_hi=float(rng.uniform(1.0, 1.8)),
                                      radius=int(rng.integers(0, 4)), tiles_per_wg=int(2 ** rng.integers(0, 3)))
        out = B.mx_quantize(view, mp)
        torch.cuda.synchronize()
        ref = oracle.mxfp4_quantize(host, bool(mp.dss), mp.n_beta, mp.beta_lo, mp.beta_hi, mp.radius)
        assert int(out.status.item()) == ref.status == 0, what
        assert np.array_equal(out.scales.cpu().numpy(), ref.scales), what + " mxfp4"
        assert np.array_equal(out.codes.cpu().numpy(), ref.codes), what + " mxfp4"
        assert float(out.sse.item()) == ref.sse, what + " mxfp4"
