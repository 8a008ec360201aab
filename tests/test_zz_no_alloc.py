"""soar_quantize_static -- the entry point that brings its own workspace (a fixed array inside the library's
device image) and allocates nothing -- against soar_quantize on the same inputs, through the C-ABI: two calls
in a row on the shared array, the second with a smaller tensor, then a tiny one and the iterated settings.
Bar: codes and scale bytes bit-exact, global scale and error within 1e-6 relative (they are in fact equal)."""
import math

import numpy as np
import pytest
import torch

from paper_2605_12245_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
REL = 1e-6


def _outputs(rows, cols):
    return B.new_outputs(rows, cols, DEV)


def _static(w, p):
    rows, cols = w.shape
    o = _outputs(rows, cols)
    o.codes.fill_(0xAA); o.scales.fill_(0xAA)
    rc = B.soar_quantize_static(w.data_ptr(), B.SOAR_BF16 if w.dtype == torch.bfloat16 else B.SOAR_FP32, rows, cols,
                                w.stride(0), p, o.codes.data_ptr(), o.scales.data_ptr(), o.global_scale.data_ptr(),
                                o.sse.data_ptr(), o.status.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == B.SOAR_OK, rc
    return o


def _plain(w, p):
    rows, cols = w.shape
    o = _outputs(rows, cols)
    ws = B.new_workspace(rows, cols, p, DEV)
    rc = B.soar_quantize(w.data_ptr(), B.SOAR_BF16 if w.dtype == torch.bfloat16 else B.SOAR_FP32, rows, cols,
                         w.stride(0), p, o.codes.data_ptr(), o.scales.data_ptr(), o.global_scale.data_ptr(),
                         o.sse.data_ptr(), o.status.data_ptr(), ws.data_ptr(), ws.numel(),
                         torch.cuda.current_stream().cuda_stream)
    assert rc == B.SOAR_OK, rc
    torch.cuda.synchronize()
    return o


def _same(a, b, what):
    assert torch.equal(a.codes, b.codes), f"{what}: codes"
    assert torch.equal(a.scales, b.scales), f"{what}: scales"
    assert int(a.status.item()) == int(b.status.item()), what
    assert math.isclose(float(a.global_scale.item()), float(b.global_scale.item()), rel_tol=REL), what
    assert math.isclose(float(a.sse.item()), float(b.sse.item()), rel_tol=REL), what


def test_static_workspace_entry_point_equals_soar_quantize():
    g = torch.Generator(device="cpu").manual_seed(77)
    big = (torch.distributions.StudentT(4.0).sample((1024, 4096)) * 0.02).to(torch.bfloat16).to(DEV)
    big[:, 100] *= 20
    small = (torch.randn(300, 528, generator=g) * torch.exp(torch.randn(300, 1, generator=g)) * 0.02).to(DEV)   # fp32
    tiny = (torch.randn(64, 64, generator=g) * 0.1).to(torch.bfloat16).to(DEV)
    p = B.soar_default_params(B.SOAR_METHOD_SOAR, 4)
    # two calls in a row on the shared array, the second smaller; nothing is synchronised in between
    first = _static(big, p)
    second = _static(small, p)
    third = _static(tiny, p)
    torch.cuda.synchronize()
    _same(first, _plain(big, p), "1024x4096 bf16")
    _same(second, _plain(small, p), "300x528 fp32 after the larger call")
    _same(third, _plain(tiny, p), "64x64 (one-workgroup kernel)")
    # the other settings the entry point accepts: plain NVFP4, and Algorithm 1 with a grid of factors
    for q in (B.soar_default_params(B.SOAR_METHOD_RTN, 0), B.soar_paper_params(iters=3, n_beta=9)):
        a = _static(small, q)
        torch.cuda.synchronize()
        _same(a, _plain(small, q), f"method {q.method} iters {q.iters}")
    # once more the large one: what the smaller calls left in the array does not matter
    again = _static(big, p)
    torch.cuda.synchronize()
    _same(again, first, "repeat")


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    p = B.soar_default_params()
    rows, cols = 8192, 8192 + 16          # one column of blocks beyond the limit
    assert rows * (cols // 16) > B.SOAR_STATIC_MAX_BLOCKS
    rc = B.soar_quantize_static(0x1000, B.SOAR_BF16, rows, cols, cols, p, 0x2000, 0x3000, 0x4000, 0, 0, 0)
    assert rc == B.SOAR_ERR_TOO_LARGE
    assert B.lib().soar_status_string(rc).decode().startswith("tensor larger")
    assert B.soar_quantize_static(0, B.SOAR_BF16, 64, 64, 64, p, 0x2000, 0x3000, 0x4000, 0, 0, 0) == 1
    assert B.soar_quantize_static(0x1000, B.SOAR_BF16, 64, 40, 40, p, 0x2000, 0x3000, 0x4000, 0, 0, 0) == 2
