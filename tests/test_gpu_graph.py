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


def test_small_tensor_and_stored_form_calls_replayed_from_a_graph():
    """The one-workgroup kernel of a small tensor, Eq. 3 and Eq. 4 (one-tensor and batch forms, the sums
    cleared by a kernel) and the MXFP4 conversion in one captured sequence, replayed on new data."""
    gen = torch.Generator(device=DEV).manual_seed(11)
    small = (torch.randn(96, 256, generator=gen, device=DEV) * 0.05).to(torch.bfloat16)
    big = (torch.randn(700, 1024, generator=gen, device=DEV) * 0.05)
    p = B.soar_default_params(B.SOAR_METHOD_SOAR, 4)
    outs = [B.new_outputs(96, 256, DEV), B.new_outputs(700, 1024, DEV)]
    wss = [B.new_workspace(96, 256, p, DEV), B.new_workspace(700, 1024, p, DEV)]
    backs = [torch.empty(96, 256, dtype=torch.bfloat16, device=DEV), torch.empty(700, 1024, dtype=torch.float32, device=DEV)]
    sses = torch.empty(3, dtype=torch.float64, device=DEV)
    mp = B.soar_mx_default_params(n_beta=9, streams=1)
    mx_out = B.mx_new_outputs(96, 256, DEV)
    mx_ws = torch.empty(B.soar_mxfp4_workspace_bytes(96, 256, mp), dtype=torch.uint8, device=DEV)
    st = lambda: torch.cuda.current_stream().cuda_stream

    def sequence():
        for w, o, ws in zip((small, big), outs, wss):
            B.quantize(w, workspace=ws, out=o)
        descs = [B.stored_desc(o, w=w, out=b, sse=sses[k:k + 1]) for k, (w, o, b) in enumerate(zip((small, big), outs, backs))]
        assert B.soar_recon_error_batch(descs, st()) == 0
        assert B.soar_dequantize_batch(descs, st()) == 0
        assert B.soar_recon_error(small.data_ptr(), B.SOAR_BF16, 96, 256, 256, outs[0].codes.data_ptr(),
                                  outs[0].scales.data_ptr(), outs[0].global_scale.data_ptr(), sses[2:3].data_ptr(), st()) == 0
        B.mx_quantize(small, mp, mx_ws, mx_out)

    sequence()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sequence()
    for rep in range(4):
        small.copy_((torch.randn(small.shape, generator=gen, device=DEV) * (0.02 * (rep + 1))).to(torch.bfloat16))
        big.copy_(torch.randn(big.shape, generator=gen, device=DEV) * (0.03 * (rep + 1)))
        for o in outs:
            o.codes.zero_(); o.scales.zero_(); o.sse.zero_()
        sses.fill_(-1.0)
        for b in backs:
            b.zero_()
        mx_out.codes.zero_(); mx_out.scales.zero_()
        g.replay()
        torch.cuda.synchronize()
        for k, (w, o, b) in enumerate(zip((small, big), outs, backs)):
            eager = B.quantize(w)
            torch.cuda.synchronize()
            _same(o, eager)
            assert torch.equal(b, B.dequantize(eager, b.dtype))
            assert abs(sses[k].item() - eager.sse.item()) <= 1e-9 * eager.sse.item()
        assert abs(sses[2].item() - outs[0].sse.item()) <= 1e-9 * outs[0].sse.item()
        mx_eager = B.mx_quantize(small, mp)
        torch.cuda.synchronize()
        assert torch.equal(mx_out.codes, mx_eager.codes) and torch.equal(mx_out.scales, mx_eager.scales)
        assert mx_out.sse.item() == mx_eager.sse.item()


def test_two_callers_on_two_streams_share_the_internal_stream():
    """Two batches enqueued back to back on two caller streams (each with its own workspace and
    outputs) both use the library's one internal stream for their second lane: the fork / join events
    keep each ordered, and the results are those of running them one after the other."""
    specs = synth.workload_specs(4, 8)
    wa = [synth.make_weight(s, DEV) for s in specs[:21]]
    wb = [synth.make_weight(s, DEV) for s in specs[21:42]]
    p = B.soar_default_params(B.SOAR_METHOD_SOAR, 4)
    ref_a, ref_b = B.quantize_tensors(wa, p), B.quantize_tensors(wb, p)
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        with torch.cuda.stream(sa):
            out_a = B.quantize_tensors(wa, p)
            mx_a = [B.mx_quantize(w, B.soar_mx_default_params(n_beta=5)) for w in wa[:3]]
        with torch.cuda.stream(sb):
            out_b = B.quantize_tensors(wb, p)
            err_b = B.recon_error_batch(wb, out_b)
        torch.cuda.synchronize()
        for a, r in zip(out_a + out_b, ref_a + ref_b):
            _same(a, r)
        for k, r in enumerate(ref_b):
            assert abs(err_b[k].item() - r.sse.item()) <= 1e-9 * r.sse.item()
        for w, m in zip(wa[:3], mx_a):
            again = B.mx_quantize(w, B.soar_mx_default_params(n_beta=5))
            torch.cuda.synchronize()
            assert torch.equal(m.codes, again.codes) and torch.equal(m.scales, again.scales)


def test_host_threads_call_the_library_at_once():
    """Four host threads, each with its own stream, workspace and outputs, call the batch entry point (two
    launch groups: the shared internal stream and its events), the single-tensor entry point (the one-launch
    kernel, or the three-pass path when another thread's may still run), the MXFP4 one and the stored-form
    ones at the same time, several rounds.  The foreign calls run without the interpreter lock.  Every result
    equals the one computed alone."""
    import threading
    specs = synth.workload_specs(4, 8)
    p = B.soar_default_params(B.SOAR_METHOD_SOAR, 4)
    mp = B.soar_mx_default_params(n_beta=5)
    jobs = []
    for k in range(4):
        ws = [synth.make_weight(s, DEV) for s in specs[7 * k: 7 * k + 14]]
        one = synth.make_weight(specs[7 * k], DEV)
        jobs.append((ws, one))
    refs = []
    for ws, one in jobs:
        refs.append((B.quantize_tensors(ws, p), B.quantize(one), B.mx_quantize(one, mp)))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in jobs]
    results, errors = [None] * len(jobs), []
    start = threading.Barrier(len(jobs))

    def work(k):
        try:
            torch.cuda.set_device(0)
            ws, one = jobs[k]
            got = []
            start.wait()
            with torch.cuda.stream(streams[k]):
                for rep in range(5):
                    batch = B.quantize_tensors(ws, p)
                    single = B.quantize(one)
                    mx = B.mx_quantize(one, mp)
                    back = B.dequantize(single)
                    errs = B.recon_error_batch(ws, batch)
                    got.append((batch, single, mx, back, errs))
            streams[k].synchronize()
            results[k] = got
        except Exception as e:                       # noqa: BLE001 -- reported by the main thread
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(len(jobs))]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a thread did not finish"
    assert not errors, errors
    torch.cuda.synchronize()
    for k, (ref_batch, ref_single, ref_mx) in enumerate(refs):
        for batch, single, mx, back, errs in results[k]:
            for a, r in zip(batch, ref_batch):
                _same(a, r)
            # one launch or three passes, whichever the guard chose: same bytes, the error sum in another order
            assert torch.equal(single.codes, ref_single.codes) and torch.equal(single.scales, ref_single.scales)
            assert single.global_scale.item() == ref_single.global_scale.item()
            assert abs(single.sse.item() - ref_single.sse.item()) <= 1e-12 * ref_single.sse.item()
            assert torch.equal(mx.codes, ref_mx.codes) and torch.equal(mx.scales, ref_mx.scales)
            assert torch.equal(back, B.dequantize(ref_single))
            for j, r in enumerate(ref_batch):
                assert abs(errs[j].item() - r.sse.item()) <= 1e-9 * max(r.sse.item(), 1e-300)
