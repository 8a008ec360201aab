"""GPU-vs-oracle parity of the iterated path (Algorithm 1 in full), through the C-ABI.

Bar: codes and scale bytes bit-exact, the number of iterations carried out equal,
the global scale bit-identical; every entry of the error trace and the final
error within 1e-6 relative -- they are in fact expected to be bit-identical,
which the tests assert, because both sides sum the block errors with the same
binary64 adjacent-pair tree (the early-stop decision depends on it).
"""
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


def oracle_args(p):
    arm = {B.SOAR_METHOD_SOAR: oracle.ARM_SOAR, B.SOAR_METHOD_CJSO_ONLY: oracle.ARM_CJSO_ONLY,
           B.SOAR_METHOD_DSS_ONLY: oracle.ARM_DSS_ONLY}[p.method]
    return dict(arm=arm, iters=p.iters, n_beta=p.n_beta, beta_lo=p.beta_lo, beta_hi=p.beta_hi, dd_mode=p.dd_mode,
                dss_radius=p.dss_radius, early_stop_rel=p.early_stop_rel)


def compare(out, ref, what):
    assert int(out.status.item()) == ref.status, what
    assert int(out.iters_run.item()) == ref.trace["iters_run"], f"{what}: iterations {int(out.iters_run.item())} vs {ref.trace['iters_run']}"
    if ref.status & oracle.STATUS_NONFINITE:
        return
    nbad_s = int((out.scales.cpu().numpy() != ref.scales).sum())
    nbad_c = int((out.codes.cpu().numpy() != ref.codes).sum())
    assert nbad_s == 0, f"{what}: {nbad_s} scale bytes differ"
    assert nbad_c == 0, f"{what}: {nbad_c} code bytes differ"
    assert np.float32(out.global_scale.item()) == ref.global_scale, what
    if ref.status & oracle.STATUS_ALLZERO:
        assert float(out.sse.item()) == 0.0
        return
    tr = out.sse_trace.cpu().numpy()
    want = ref.trace["sse_trace"]
    assert np.array_equal(np.isnan(tr), np.isnan(want)), what
    ok = ~np.isnan(want)
    assert np.allclose(tr[ok], want[ok], rtol=1e-6, atol=0.0), what
    assert np.array_equal(tr[ok], want[ok]), f"{what}: error trace not bit-identical"
    assert float(out.sse.item()) == ref.sse, what


def run_one(w, p, what):
    out = B.quantize_iter(w, p)
    torch.cuda.synchronize()
    ref = oracle.quantize_iter(host_of(w), **oracle_args(p))
    compare(out, ref, what)
    return out, ref


def test_loop_reciprocal_equals_the_division_on_its_whole_range():
    """Every positive binary32 with biased exponent 1..252: estimate + one fused Newton step == 1/x."""
    chunk = 1 << 26
    out = torch.empty(chunk, dtype=torch.float32, device=DEV)
    base = torch.arange(chunk, dtype=torch.int64, device=DEV)
    one = np.float32(1.0)
    for c in range(1 << 23, 253 << 23, chunk):
        x = (base + c).to(torch.int32).view(torch.float32)
        assert B.soar_rcp_midrange_f32(x.data_ptr(), chunk, out.data_ptr(), 0) == 0
        got = out.cpu().numpy().view(np.uint32)
        xh = (np.arange(chunk, dtype=np.uint32) + np.uint32(c)).view(np.float32)
        with np.errstate(all="ignore"):
            want = (one / xh).view(np.uint32)
        ex = (xh.view(np.uint32) >> np.uint32(23)) & np.uint32(0xFF)
        bad = (got != want) & (ex >= 1) & (ex <= 252)          # the last chunk reaches past the range
        assert not bad.any(), f"chunk {c:#x}: {np.count_nonzero(bad)} mismatches, first at {xh[bad][:4]}"


def test_single_step_settings_match_the_single_step_path():
    """T = 1, beta = {1}, window: the iterated kernels return the bytes of the three-pass path."""
    for workload, div in ((1, 1), (2, 4)):
        spec = synth.workload_specs(workload, div)[0]
        w = synth.make_weight(spec, DEV)
        for K in (0, 1, 4):
            fast = B.quantize(w, B.SOAR_METHOD_SOAR, K)
            p = B.soar_default_params(B.SOAR_METHOD_SOAR, K)
            slow = B.quantize_iter(w, p)                      # asking for the trace selects the iterated path
            torch.cuda.synchronize()
            assert torch.equal(fast.codes, slow.codes) and torch.equal(fast.scales, slow.scales)
            assert fast.global_scale.item() == slow.global_scale.item()
            assert math.isclose(fast.sse.item(), slow.sse.item(), rel_tol=1e-6)
            assert int(slow.iters_run.item()) == 1
            ref = oracle.quantize(host_of(w), oracle.METHOD_SOAR, K)
            assert np.array_equal(slow.codes.cpu().numpy(), ref.codes) and slow.sse.item() == ref.sse


@pytest.mark.parametrize("workload,div", [(1, 1), (2, 1), (3, 2)])
def test_paper_settings_single_tensors(workload, div):
    spec = synth.workload_specs(workload, div)[0]
    w = synth.make_weight(spec, DEV)
    out, ref = run_one(w, B.soar_paper_params(), f"workload {workload}/{div}")
    rtn = oracle.quantize(host_of(w), oracle.METHOD_RTN, 0)
    assert ref.sse < rtn.sse and ref.trace["sse_trace"][0] == rtn.sse
    assert math.isclose(float(B.recon_error(w, out).item()), ref.sse, rel_tol=1e-6)


@pytest.mark.parametrize("kwargs", [
    dict(iters=3, n_beta=11, dd_mode=B.SOAR_DD_WINDOW, dss_radius=2, early_stop_rel=0.0),
    dict(iters=5, n_beta=1, beta_lo=1.0, beta_hi=1.0, early_stop_rel=0.0),
    dict(iters=15, n_beta=21, early_stop_rel=1e-2),
    dict(iters=15, n_beta=21, early_stop_rel=0.2),
    dict(iters=2, n_beta=7, beta_lo=0.8, beta_hi=1.25, dd_mode=B.SOAR_DD_WINDOW, dss_radius=0, early_stop_rel=0.0),
    dict(iters=1, n_beta=4096, early_stop_rel=0.0),
    dict(iters=64, n_beta=3, early_stop_rel=0.0),
], ids=["window-K2", "beta1-5it", "stop1e-2", "stop0.2", "narrow-grid-K0", "4096-betas", "64-iters"])
def test_parameter_variants(kwargs):
    for workload, div in ((1, 1), (5, 64)):
        spec = synth.workload_specs(workload, div)[0]
        w = synth.make_weight(spec, DEV)
        run_one(w, B.soar_paper_params(**kwargs), f"workload {workload}/{div} {kwargs}")


@pytest.mark.parametrize("rows,cols", [(1, 16), (3, 48), (257, 272), (1000, 1040), (5, 4096 * 16 + 16)])
def test_ragged_shapes(rows, cols):
    g = torch.Generator(device="cpu").manual_seed(rows * 131 + cols)
    w = (torch.randn(rows, cols, generator=g) * 0.02).to(torch.bfloat16).to(DEV)
    run_one(w, B.soar_paper_params(iters=4, n_beta=15), f"{rows}x{cols}")


def test_fp32_input_with_leading_dimension():
    g = torch.Generator(device="cpu").manual_seed(7)
    parent = (torch.randn(300, 640, generator=g) * 0.05).to(DEV)
    view = parent[:, 64:64 + 512]
    p = B.soar_paper_params(iters=3, n_beta=9)
    out = B.new_outputs(300, 512, DEV, p.iters)
    desc = B.make_desc(view, out)
    ws = B.new_batch_workspace([desc], p, DEV)
    B.quantize_batch([desc], p, ws)
    torch.cuda.synchronize()
    ref = oracle.quantize_iter(view.cpu().contiguous().numpy(), **oracle_args(p))
    compare(out, ref, "fp32 strided")


def test_outputs_do_not_depend_on_the_launch_shape():
    spec = synth.workload_specs(2, 2)[0]
    w = synth.make_weight(spec, DEV)
    base = B.quantize_iter(w, B.soar_paper_params(iters=4, n_beta=15))
    for tpw in (2, 4, 16):
        other = B.quantize_iter(w, B.soar_paper_params(iters=4, n_beta=15, tiles_per_wg=tpw))
        torch.cuda.synchronize()
        assert torch.equal(base.codes, other.codes) and torch.equal(base.scales, other.scales)
        assert torch.equal(base.sse_trace.nan_to_num(-1.0), other.sse_trace.nan_to_num(-1.0))
        assert base.global_scale.item() == other.global_scale.item()


def test_batch_with_tensors_that_stop_at_different_iterations_and_degenerate_ones():
    """One launch group: tensors of different statistics (so they stop after different numbers of
    iterations), an all-zero tensor, one with a NaN, a ragged small one; twice on the same
    workspace to show that the control words are back in their initial state."""
    g = torch.Generator(device="cpu").manual_seed(11)
    ws_list = [
        synth.make_weight(synth.workload_specs(1, 1)[0], DEV),
        synth.make_weight(synth.workload_specs(2, 8)[0], DEV),
        torch.zeros(64, 256, dtype=torch.bfloat16, device=DEV),
        (torch.randn(128, 128, generator=g) * 3.0).to(torch.bfloat16).to(DEV),
        synth.make_weight(synth.workload_specs(5, 64)[0], DEV),
        (torch.rand(33, 80, generator=g) - 0.5).to(torch.bfloat16).to(DEV),
    ]
    ws_list[2][5, 7] = -0.0
    bad = ws_list[3].clone()
    bad[17, 3] = float("nan")
    ws_list.append(bad)
    p = B.soar_paper_params(early_stop_rel=5e-3)
    outs = [B.new_outputs(w.shape[0], w.shape[1], DEV, p.iters) for w in ws_list]
    descs = [B.make_desc(w, o) for w, o in zip(ws_list, outs)]
    ws = B.new_batch_workspace(descs, p, DEV)
    refs = [oracle.quantize_iter(host_of(w), **oracle_args(p)) for w in ws_list]
    for rep in range(2):
        for o in outs:
            o.codes.zero_(); o.scales.zero_(); o.sse_trace.fill_(float("nan")); o.iters_run.zero_()
        B.quantize_batch(descs, p, ws)
        torch.cuda.synchronize()
        for k, (o, r) in enumerate(zip(outs, refs)):
            compare(o, r, f"tensor {k}, call {rep}")
    assert len({r.trace["iters_run"] for r in refs}) >= 3


def test_multi_tensor_workload_scaled_down_two_streams():
    specs = synth.workload_specs(4, 8)[:28]
    weights = [synth.make_weight(s, DEV) for s in specs]
    p = B.soar_paper_params()
    outs = [B.new_outputs(s.rows, s.cols, DEV, p.iters) for s in specs]
    descs = [B.make_desc(w, o) for w, o in zip(weights, outs)]
    ws = B.new_batch_workspace(descs, p, DEV)
    B.quantize_batch(descs, p, ws)
    torch.cuda.synchronize()
    for k, (w, o) in enumerate(zip(weights, outs)):
        compare(o, oracle.quantize_iter(host_of(w), **oracle_args(p)), f"tensor {k}")


@pytest.mark.parametrize("method", [B.SOAR_METHOD_CJSO_ONLY, B.SOAR_METHOD_DSS_ONLY], ids=["cjso-only", "dss-only"])
def test_component_study_arms(method):
    """Sec. 3.2 alone and Sec. 3.3 alone, with and without early stop, on single tensors and in one batch."""
    for workload, div in ((1, 1), (2, 2), (5, 64)):
        spec = synth.workload_specs(workload, div)[0]
        w = synth.make_weight(spec, DEV)
        for stop in (0.0, 1e-3):
            p = B.soar_arm_params(method, iters=6, early_stop_rel=stop, n_beta=21, dss_radius=2)
            out, ref = run_one(w, p, f"arm {method} workload {workload}/{div} stop {stop}")
            rtn = oracle.quantize(host_of(w), oracle.METHOD_RTN, 0)
            assert ref.sse < rtn.sse
            if method == B.SOAR_METHOD_DSS_ONLY:
                assert ref.global_scale == rtn.global_scale
    g = torch.Generator(device="cpu").manual_seed(23)
    ws_list = [synth.make_weight(synth.workload_specs(1, 1)[0], DEV),
               torch.zeros(16, 64, dtype=torch.bfloat16, device=DEV),
               (torch.randn(77, 144, generator=g) * 0.1).to(torch.bfloat16).to(DEV),
               synth.make_weight(synth.workload_specs(5, 64)[0], DEV)]
    p = B.soar_arm_params(method, iters=5, early_stop_rel=2e-3, n_beta=11, dss_radius=1)
    outs = [B.new_outputs(w.shape[0], w.shape[1], DEV, p.iters) for w in ws_list]
    descs = [B.make_desc(w, o) for w, o in zip(ws_list, outs)]
    ws = B.new_batch_workspace(descs, p, DEV)
    B.quantize_batch(descs, p, ws)
    torch.cuda.synchronize()
    for k, (w, o) in enumerate(zip(ws_list, outs)):
        compare(o, oracle.quantize_iter(host_of(w), **oracle_args(p)), f"arm {method} batch tensor {k}")


def test_arms_order_as_in_the_convergence_figure():
    """On the GPU as in the paper's figure: the closed-form steps alone end above the full method."""
    spec = synth.workload_specs(2, 2)[0]
    w = synth.make_weight(spec, DEV)
    full = B.quantize_iter(w, B.soar_paper_params(iters=8, early_stop_rel=0.0))
    cjso = B.quantize_iter(w, B.soar_arm_params(B.SOAR_METHOD_CJSO_ONLY, iters=8, early_stop_rel=0.0))
    torch.cuda.synchronize()
    assert full.sse.item() < cjso.sse.item() < full.sse_trace[0].item()
    assert cjso.sse_trace[0].item() == full.sse_trace[0].item()


def test_full_model_workload_in_the_bench_configuration_sampled_tensors():
    """Config 4 at full size, enqueued exactly as bench.py --algorithm paper does (one batch, default
    streams); the oracle checks tensors it can compute one by one: the first, one wide MLP tensor
    and the last (each tensor's result depends on that tensor alone)."""
    specs = synth.workload_specs(4)
    weights = [synth.make_weight(s, DEV) for s in specs]
    p = B.soar_paper_params()
    outs = [B.new_outputs(s.rows, s.cols, DEV, p.iters) for s in specs]
    descs = [B.make_desc(w, o) for w, o in zip(weights, outs)]
    ws = B.new_batch_workspace(descs, p, DEV)
    B.quantize_batch(descs, p, ws)
    torch.cuda.synchronize()
    assert all(int(o.status.item()) == 0 for o in outs)
    assert all(1 <= int(o.iters_run.item()) <= p.iters for o in outs)
    for k in (0, 130, len(specs) - 1):
        compare(outs[k], oracle.quantize_iter(host_of(weights[k]), **oracle_args(p)), f"tensor {k} ({specs[k].name})")
    # properties that hold for every tensor: trace falls from the plain-NVFP4 error, reported error = last entry
    for k, o in enumerate(outs):
        tr = o.sse_trace.cpu().numpy()
        n = int(o.iters_run.item())
        assert not np.isnan(tr[: n + 1]).any() and np.isnan(tr[n + 1:]).all(), k
        assert tr[n] < tr[0] and float(o.sse.item()) == tr[n], k


def test_two_pass_search_equals_the_plain_loop():
    """search_mode AUTO (codes first, errors only where a block's codes change) against FULL (every factor
    evaluated): identical bytes, trace and iteration count, for both candidate modes and a long grid."""
    spec = synth.workload_specs(2, 2)[0]
    w = synth.make_weight(spec, DEV)
    for kw in (dict(), dict(dd_mode=B.SOAR_DD_WINDOW, dss_radius=2, n_beta=31), dict(n_beta=128), dict(n_beta=4),
               dict(n_beta=129)):
        a = B.soar_paper_params(iters=3, early_stop_rel=0.0, **kw)
        f = B.soar_paper_params(iters=3, early_stop_rel=0.0, **kw)
        f.search_mode = B.SOAR_SEARCH_FULL
        oa, of = B.quantize_iter(w, a), B.quantize_iter(w, f)
        torch.cuda.synchronize()
        assert torch.equal(oa.codes, of.codes) and torch.equal(oa.scales, of.scales), kw
        assert oa.global_scale.item() == of.global_scale.item(), kw
        assert torch.equal(oa.sse_trace, of.sse_trace), kw
