"""The one-launch kernel that keeps a tensor in registers (a single tensor handed over alone, single-step
settings): against the oracle and against the three-pass path, through the C-ABI, on sizes that take every
launch shape it has (workgroups of 256 or 1024 lanes, 1, 2 or 4 blocks per lane, 1 to 256 workgroups, the last
one ragged), both element types, both methods; on workspaces holding anything; replayed on one workspace with
tensors of changing size; and its bounded wait, forced to give up from the host with a tiny limit (every
workgroup then leaves by itself: nothing hangs).
Bar: codes and scale bytes bit-exact, global scale bit-identical, error within 1e-6 relative."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2605_12245_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
REL = 1e-6


def bits(w):
    w = w.detach().cpu().contiguous()
    return w.view(torch.int16).numpy().view(np.uint16) if w.dtype == torch.bfloat16 else w.numpy()


def heavy(rows, cols, seed, dtype):
    g = torch.Generator(device="cpu").manual_seed(seed)
    w = torch.randn(rows, cols, generator=g) * torch.exp(torch.randn(rows, 1, generator=g) * 1.5) * 0.02
    w[:: max(1, rows // 7), 5 % cols] *= 37.0
    return w.to(dtype).to(DEV)


def run(w, p, ws=None, want_sse=True, want_status=True):
    rows, cols = w.shape
    o = B.new_outputs(rows, cols, DEV)
    o.codes.fill_(0x55); o.scales.fill_(0x55); o.sse.fill_(-1.0); o.status.fill_(-1); o.global_scale.fill_(-1.0)
    if ws is None:
        ws = B.new_workspace(rows, cols, p, DEV)
    rc = B.soar_quantize(w.data_ptr(), B.SOAR_BF16 if w.dtype == torch.bfloat16 else B.SOAR_FP32, rows, cols, w.stride(0),
                         p, o.codes.data_ptr(), o.scales.data_ptr(), o.global_scale.data_ptr(),
                         o.sse.data_ptr() if want_sse else 0, o.status.data_ptr() if want_status else 0,
                         ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    assert rc == B.SOAR_OK, rc
    return o


def params(method=B.SOAR_METHOD_SOAR, K=4, resident=B.SOAR_RESIDENT_AUTO, wait_us=0, mode=B.SOAR_SEARCH_AUTO):
    p = B.soar_default_params(method, K, mode)
    p.resident = resident
    p.resident_wait_us = wait_us
    return p


def same_bytes(a, b, what):
    assert torch.equal(a.scales, b.scales), f"{what}: scales"
    assert torch.equal(a.codes, b.codes), f"{what}: codes"
    assert a.global_scale.item() == b.global_scale.item(), what
    assert int(a.status.item()) == int(b.status.item()), what
    assert math.isclose(a.sse.item(), b.sse.item(), rel_tol=1e-12), what


def against_oracle(o, w, method, K, what):
    ref = oracle.quantize(bits(w), method, K)
    assert int(o.status.item()) == ref.status, what
    assert np.array_equal(o.scales.cpu().numpy(), ref.scales), f"{what}: scales differ from the oracle"
    assert np.array_equal(o.codes.cpu().numpy(), ref.codes), f"{what}: codes differ from the oracle"
    assert np.float32(o.global_scale.item()) == ref.global_scale, what
    assert math.isclose(float(o.sse.item()), ref.sse, rel_tol=REL), what


# rows x cols -> lanes per workgroup, blocks per lane, workgroups (on 256 compute units)
SHAPES = [
    (1, 16),            # 256, 1, 1
    (33, 1040),         # 256, 1, 9 (ragged)
    (255, 4096),        # 256, 1, 255
    (256, 4096),        # 256, 1, 256: the largest tensor of this shape
    (257, 4096),        # 1024, 1, 65 (ragged)
    (1023, 4096),       # 1024, 1, 256 (ragged)
    (1500, 4096),       # 1024, 2, 188 (ragged)
    (2048, 4096),       # 1024, 2, 256
    (2100, 4096),       # 1024, 4, 132 (ragged)
    (4095, 4096),       # 1024, 4, 256 (ragged)
]


@pytest.mark.parametrize("rows,cols", SHAPES)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32], ids=["bf16", "fp32"])
def test_every_launch_shape_against_the_oracle_and_the_three_pass_path(rows, cols, dtype):
    w = heavy(rows, cols, rows * 31 + cols, dtype)
    for method, K in ((B.SOAR_METHOD_SOAR, 4), (B.SOAR_METHOD_RTN, 0)):
        what = f"{rows}x{cols} {dtype} method {method}"
        one = run(w, params(method, K))
        three = run(w, params(method, K, resident=B.SOAR_RESIDENT_NEVER))
        torch.cuda.synchronize()
        same_bytes(one, three, what)
        against_oracle(one, w, method, K, what)
    # the exhaustive search and a wide window from the registers
    full = run(w, params(B.SOAR_METHOD_SOAR, 8, mode=B.SOAR_SEARCH_FULL))
    auto = run(w, params(B.SOAR_METHOD_SOAR, 8))
    torch.cuda.synchronize()
    same_bytes(full, auto, f"{rows}x{cols} {dtype} K 8, exhaustive against certified")


def test_full_size_attention_projection_is_one_launch_and_bit_exact():
    """workload 2's shape (4096 x 4096, 32 MiB of bf16): 256 workgroups of 1024 lanes, four blocks per lane"""
    from paper_2605_12245_amd import synth
    spec = synth.workload_specs(2)[0]
    w = synth.make_weight(spec, DEV)
    B.soar_kernel_timing_enable(True)
    o = run(w, params(B.SOAR_METHOD_SOAR, spec.dss_radius))
    torch.cuda.synchronize()
    launches = {k: B.soar_kernel_timing_read(k)[1] for k in (B.SOAR_KERNEL_RESIDENT, B.SOAR_KERNEL_ABSMAX, B.SOAR_KERNEL_SEARCH)}
    B.soar_kernel_timing_enable(False)
    assert launches == {B.SOAR_KERNEL_RESIDENT: 1, B.SOAR_KERNEL_ABSMAX: 0, B.SOAR_KERNEL_SEARCH: 0}
    against_oracle(o, w, oracle.METHOD_SOAR, spec.dss_radius, "workload 2")


def test_strided_rows_degenerate_tensors_and_absent_outputs():
    parent = heavy(700, 4096 + 64, 5, torch.bfloat16)
    view = parent[:, 32:32 + 4096]                                   # 179200 blocks: 1024 lanes, 175 workgroups
    p = params()
    a = run(view, p)
    b = run(view.contiguous(), p)
    torch.cuda.synchronize()
    same_bytes(a, b, "strided rows")
    against_oracle(a, view.contiguous(), oracle.METHOD_SOAR, 4, "strided rows")
    # all-zero (signed zeros keep their sign) and non-finite tensors spread over many workgroups
    z = torch.zeros(600, 4096, dtype=torch.bfloat16, device=DEV)
    z[599, 4095] = -0.0
    oz = run(z, p)
    bad = heavy(600, 4096, 6, torch.float32)
    bad[577, 123] = float("nan")
    ob = run(bad, p)
    torch.cuda.synchronize()
    assert int(oz.status.item()) == B.SOAR_STATUS_ALLZERO and oz.global_scale.item() == 1.0 and oz.sse.item() == 0.0
    assert bool((oz.scales == 1).all()) and int(oz.codes.view(-1)[-1].item()) == 0x80 and int(oz.codes.view(-1)[:-1].max().item()) == 0
    assert int(ob.status.item()) & B.SOAR_STATUS_NONFINITE
    s = ob.scales.cpu().numpy()
    assert s.min() >= 1 and s.max() <= 0x7E
    # error sum and status not asked for: the bytes and the global scale are the same
    w = heavy(1023, 4096, 7, torch.bfloat16)
    full = run(w, p)
    bare = run(w, p, want_sse=False, want_status=False)
    torch.cuda.synchronize()
    assert torch.equal(full.codes, bare.codes) and torch.equal(full.scales, bare.scales)
    assert full.global_scale.item() == bare.global_scale.item()
    assert bare.sse.item() == -1.0 and int(bare.status.item()) == -1          # untouched


def test_workspace_contents_do_not_matter_and_one_workspace_serves_changing_sizes():
    p = params()
    big = heavy(4095, 4096, 8, torch.bfloat16)
    ws = B.new_workspace(4095, 4096, p, DEV)
    ref = {}
    shapes = [(4095, 4096), (1023, 4096), (33, 1040), (2100, 4096), (1023, 4096), (4095, 4096)]
    for rows, cols in set(shapes):
        ref[(rows, cols)] = run(big[:rows, :cols].contiguous(), params(resident=B.SOAR_RESIDENT_NEVER))
    torch.cuda.synchronize()
    gen = torch.Generator(device=DEV).manual_seed(1)
    for fill in ("ones", "zeros", "random", "keep", "keep", "keep"):
        if fill == "ones":
            ws.fill_(0xFF)
        elif fill == "zeros":
            ws.zero_()
        elif fill == "random":
            ws.copy_(torch.randint(0, 256, ws.shape, generator=gen, device=DEV, dtype=torch.uint8))
        for rows, cols in shapes:                 # back to back on one workspace, nothing synchronised in between
            o = run(big[:rows, :cols].contiguous(), p, ws)
            same_bytes_later = (o, ref[(rows, cols)], f"{rows}x{cols} on a workspace filled with {fill}")
            torch.cuda.synchronize()
            same_bytes(*same_bytes_later)
    # the three-pass path in between leaves its own words in the same places
    for rows, cols in shapes[:3]:
        w = big[:rows, :cols].contiguous()
        run(w, params(resident=B.SOAR_RESIDENT_NEVER), ws)
        o = run(w, p, ws)
        torch.cuda.synchronize()
        same_bytes(o, ref[(rows, cols)], f"{rows}x{cols} after a three-pass call on the same workspace")


def test_bounded_wait_gives_up_and_the_next_call_is_unaffected():
    """A limit of one microsecond is over before the first workgroup has loaded its blocks: every workgroup
    finds its wait out of time, says so in the status word and leaves; nothing hangs.  The same workspace
    then serves an ordinary call."""
    w = heavy(4095, 4096, 9, torch.bfloat16)
    ws = B.new_workspace(4095, 4096, params(), DEV)
    ref = run(w, params(resident=B.SOAR_RESIDENT_NEVER))
    torch.cuda.synchronize()
    for rep in range(3):
        o = run(w, params(wait_us=1), ws)
        torch.cuda.synchronize()
        assert int(o.status.item()) == B.SOAR_STATUS_GAVE_UP, rep
        good = run(w, params(), ws)
        torch.cuda.synchronize()
        same_bytes(good, ref, f"after giving up, repetition {rep}")


def test_replayed_from_a_graph_on_changing_data():
    """The token of a launch must be new on every replay of a captured call (same kernel arguments): the
    workspace's epoch provides that.  Four shapes, six replays each, every replay against an eager call."""
    p = params()
    gen = torch.Generator(device=DEV).manual_seed(21)
    for rows, cols in ((1023, 4096), (4095, 4096), (300, 1040)):
        w = heavy(rows, cols, rows, torch.bfloat16)
        ws = B.new_workspace(rows, cols, p, DEV)
        out = B.new_outputs(rows, cols, DEV)
        B.quantize(w, workspace=ws, out=out)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            B.quantize(w, workspace=ws, out=out)
        for rep in range(6):
            w.copy_((torch.randn(w.shape, generator=gen, device=DEV) * (0.01 * (rep + 1))).to(torch.bfloat16))
            out.codes.zero_(); out.scales.zero_(); out.sse.zero_()
            g.replay()
            if rep % 2:
                g.replay()                       # twice in a row, nothing in between
            torch.cuda.synchronize()
            eager = run(w, params(resident=B.SOAR_RESIDENT_NEVER))
            torch.cuda.synchronize()
            same_bytes(out, eager, f"{rows}x{cols} replay {rep}")


def test_two_streams_at_once():
    """Calls that arrive on another stream while the earlier one-launch kernel may still run take the
    three-pass path (or wait their turn): both results are right whatever the interleaving."""
    p = params()
    wa, wb = heavy(4095, 4096, 31, torch.bfloat16), heavy(2048, 4096, 32, torch.float32)
    ra, rb = run(wa, params(resident=B.SOAR_RESIDENT_NEVER)), run(wb, params(resident=B.SOAR_RESIDENT_NEVER))
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(4):
        with torch.cuda.stream(sa):
            oa = [run(wa, p) for _ in range(3)]
        with torch.cuda.stream(sb):
            ob = [run(wb, p) for _ in range(3)]
        torch.cuda.synchronize()
        for o in oa:
            same_bytes(o, ra, f"stream a, repetition {rep}")
        for o in ob:
            same_bytes(o, rb, f"stream b, repetition {rep}")
