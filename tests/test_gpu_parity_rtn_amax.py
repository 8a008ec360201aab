"""GPU-vs-oracle parity of the plain NVFP4 pass with a supplied tensor maximum, through the C-ABI.
Bar: codes and scale bytes bit-exact, global scale bit-identical, error within 1e-6 relative."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2605_12245_amd import binding as B
from paper_2605_12245_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def host_of(w):
    w = w.detach().cpu().contiguous()
    return w.view(torch.int16).numpy().view(np.uint16) if w.dtype == torch.bfloat16 else w.numpy()


def check(w, amax, what):
    a = torch.tensor([amax], dtype=torch.float32, device=DEV)
    out = B.quantize_rtn_amax(w, a)
    torch.cuda.synchronize()
    ref = oracle.quantize_rtn_amax(host_of(w), float(np.float32(amax)))
    assert int(out.status.item()) == ref.status == 0, what
    assert np.array_equal(out.scales.cpu().numpy(), ref.scales), what
    assert np.array_equal(out.codes.cpu().numpy(), ref.codes), what
    assert np.float32(out.global_scale.item()) == ref.global_scale, what
    assert math.isclose(float(out.sse.item()), ref.sse, rel_tol=1e-6), what
    return out, ref


@pytest.mark.parametrize("workload,div", [(1, 1), (2, 1), (3, 2)])
@pytest.mark.parametrize("factor", [1.0, 0.3, 2.5])
def test_workloads(workload, div, factor):
    spec = synth.workload_specs(workload, div)[0]
    w = synth.make_weight(spec, DEV)
    true_max = float(w.float().abs().max().item())
    out, ref = check(w, true_max * factor, f"workload {workload} x{factor}")
    if factor == 1.0:
        # the measured-maximum path gives the same bytes
        plain = B.quantize(w, B.SOAR_METHOD_RTN, 0)
        torch.cuda.synchronize()
        assert torch.equal(plain.codes, out.codes) and torch.equal(plain.scales, out.scales)
        assert plain.global_scale.item() == out.global_scale.item()
    if factor < 1.0:
        assert (ref.scales == 0x7E).any()


@pytest.mark.parametrize("rows,cols", [(1, 16), (3, 48), (257, 272), (1000, 1040)])
def test_ragged_shapes_and_extreme_maxima(rows, cols):
    g = torch.Generator(device="cpu").manual_seed(rows * 17 + cols)
    w = (torch.randn(rows, cols, generator=g) * 0.7).to(torch.bfloat16).to(DEV)
    for amax in (1e-3, 0.5, 4.0, 3e4, 2.0 ** -100, 2.0 ** 100):
        check(w, amax, f"{rows}x{cols} amax {amax}")


def test_fp32_input_with_leading_dimension_and_batch():
    g = torch.Generator(device="cpu").manual_seed(3)
    parent = (torch.randn(300, 640, generator=g) * 2.0).to(DEV)
    views = [parent[:, 0:256], parent[:, 256:256 + 384], parent[:100, 128:128 + 512]]
    maxima = [1.0, 9.0, 3.0]
    p = B.soar_default_params(B.SOAR_METHOD_RTN, 0)
    outs = [B.new_outputs(v.shape[0], v.shape[1], DEV) for v in views]
    am = [torch.tensor([m], dtype=torch.float32, device=DEV) for m in maxima]
    descs = [B.make_desc(v, o, a) for v, o, a in zip(views, outs, am)]
    ws = B.new_batch_workspace(descs, p, DEV)
    B.quantize_batch(descs, p, ws)
    torch.cuda.synchronize()
    for v, o, m in zip(views, outs, maxima):
        ref = oracle.quantize_rtn_amax(v.cpu().contiguous().numpy(), m)
        assert np.array_equal(o.codes.cpu().numpy(), ref.codes) and np.array_equal(o.scales.cpu().numpy(), ref.scales)
        assert np.float32(o.global_scale.item()) == ref.global_scale
        assert math.isclose(float(o.sse.item()), ref.sse, rel_tol=1e-6)


def test_unusable_maximum_sets_the_status_bit():
    w = torch.ones(32, 64, dtype=torch.bfloat16, device=DEV)
    for bad in (0.0, -2.0, float("inf"), float("nan")):
        out = B.quantize_rtn_amax(w, torch.tensor([bad], dtype=torch.float32, device=DEV))
        torch.cuda.synchronize()
        assert int(out.status.item()) == B.SOAR_STATUS_BAD_AMAX


def test_full_model_workload_in_the_bench_configuration_sampled_tensors():
    """Config 4 at full size as bench.py --algorithm rtn-amax enqueues it; every 21st tensor against the oracle."""
    specs = synth.workload_specs(4)
    weights = [synth.make_weight(s, DEV) for s in specs]
    am = [w.abs().max().float().reshape(1) for w in weights]
    p = B.soar_default_params(B.SOAR_METHOD_RTN, 0)
    outs = [B.new_outputs(s.rows, s.cols, DEV) for s in specs]
    descs = [B.make_desc(w, o, a) for w, o, a in zip(weights, outs, am)]
    ws = B.new_batch_workspace(descs, p, DEV)
    B.quantize_batch(descs, p, ws)
    torch.cuda.synchronize()
    assert all(int(o.status.item()) == 0 for o in outs)
    for k in range(0, len(specs), 21):
        ref = oracle.quantize_rtn_amax(host_of(weights[k]), float(am[k].item()))
        assert np.array_equal(outs[k].codes.cpu().numpy(), ref.codes), k
        assert np.array_equal(outs[k].scales.cpu().numpy(), ref.scales), k
        assert np.float32(outs[k].global_scale.item()) == ref.global_scale, k
        assert math.isclose(float(outs[k].sse.item()), ref.sse, rel_tol=1e-6), k
