"""The single-stream entry points under HIP graph capture: every launch is an ordinary kernel on the
caller's stream (the control words are cleared by a kernel, not a memset), so a captured call can be
replayed.  Each replay runs on new input data and is checked against an eager call on the same data."""
import numpy as np
import pytest
import torch

from paper_2605_12245_amd import binding as B
from paper_2605_12245_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _same(a: B.Quantized, b: B.Quantized):
    assert torch.equal(a.codes, b.codes) and torch.equal(a.scales, b.scales)
    assert a.global_scale.item() == b.global_scale.item() and a.sse.item() == b.sse.item()
    assert a.status.item() == b.status.item()


def test_single_tensor_call_replayed_from_a_graph():
    spec = synth.workload_specs(2, 4)[0]
    w = synth.make_weight(spec, DEV)
    p = B.soar_default_params(B.SOAR_METHOD_SOAR, 4)
    ws = B.new_workspace(spec.rows, spec.cols, p, DEV)
    out = B.new_outputs(spec.rows, spec.cols, DEV)
    B.quantize(w, workspace=ws, out=out)                 # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.quantize(w, workspace=ws, out=out)
    gen = torch.Generator(device=DEV).manual_seed(3)
    for rep in range(4):
        w.copy_((torch.randn(w.shape, generator=gen, device=DEV) * (0.01 * (rep + 1))).to(torch.bfloat16))
        out.codes.zero_(); out.scales.zero_(); out.sse.zero_()
        g.replay()
        torch.cuda.synchronize()
        eager = B.quantize(w)
        torch.cuda.synchronize()
        _same(out, eager)


def test_batch_and_iterated_calls_replayed_from_a_graph():
    specs = synth.workload_specs(4, 8)[:10]
    weights = [synth.make_weight(s, DEV) for s in specs]
    for p in (B.soar_default_params(B.SOAR_METHOD_SOAR, 4, streams=1),
              B.soar_paper_params(iters=4, n_beta=9, streams=1)):
        iters = p.iters if p.iters > 1 else 0
        outs = [B.new_outputs(s.rows, s.cols, DEV, iters) for s in specs]
        descs = [B.make_desc(w, o) for w, o in zip(weights, outs)]
        ws = B.new_batch_workspace(descs, p, DEV)
        B.quantize_batch(descs, p, ws)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            B.quantize_batch(descs, p, ws)
        gen = torch.Generator(device=DEV).manual_seed(5)
        for rep in range(3):
            for w in weights:
                w.copy_((torch.randn(w.shape, generator=gen, device=DEV) * 0.02).to(torch.bfloat16))
            for o in outs:
                o.codes.zero_(); o.scales.zero_()
            g.replay()
            torch.cuda.synchronize()
            eager_outs = [B.new_outputs(s.rows, s.cols, DEV, iters) for s in specs]
            eager_descs = [B.make_desc(w, o) for w, o in zip(weights, eager_outs)]
            B.quantize_batch(eager_descs, p, B.new_batch_workspace(eager_descs, p, DEV))
            torch.cuda.synchronize()
            for a, b in zip(outs, eager_outs):
                _same(a, b)
                if iters:
                    assert a.iters_run.item() == b.iters_run.item()
