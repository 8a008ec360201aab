"""Pins for the oracle's method steps (CPU only).

The oracle's results are checked against least-squares library routines, closed
forms, theorems of the coordinate descent, exhaustive enumeration of all E4M3
block scales, and exact equivariances -- evaluated here in float64 numpy from
the oracle's *outputs*, never by calling the oracle's own arithmetic again.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2605_12245_amd import synth

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
E4M3 = torch.arange(0, 128, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)


def unpack(codes: np.ndarray) -> np.ndarray:
    """packed nibbles [rows, cols/2] -> signed float64 values [rows, cols]"""
    lo = codes & 0xF
    hi = codes >> 4
    nib = np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)
    v = E2M1[nib & 7]
    return np.where(nib & 8, -v, v)


def weights(workload, scale_down, seed_shift=0, dtype=torch.bfloat16):
    spec = synth.workload_specs(workload, scale_down)[0]
    if seed_shift:
        spec = type(spec)(**{**spec.__dict__, "index": spec.index + seed_shift})
    w = synth.make_weight(spec, "cpu", dtype)
    return spec, w


def loss(w64, q, alpha, delta_blocks):
    """Eq. 4 in float64. delta_blocks: [rows, cols/16]"""
    s = np.repeat(delta_blocks, 16, axis=1) * float(alpha)
    return float(np.sum((w64 - q * s) ** 2))


SMALL = [(1, 1), (1, 2), (2, 16), (3, 16), (4, 32), (5, 64)]


@pytest.fixture(scope="module", params=SMALL, ids=[f"wl{a}_div{b}" for a, b in SMALL])
def case(request):
    wl, div = request.param
    spec, w = weights(wl, div)
    bits = synth.bf16_bits(w)
    soar = oracle.quantize(bits, oracle.METHOD_SOAR, spec.dss_radius, want_trace=True)
    rtn = oracle.quantize(bits, oracle.METHOD_RTN, spec.dss_radius, want_trace=True)
    return dict(spec=spec, w=w, w64=w.double().numpy(), bits=bits, soar=soar, rtn=rtn)


# --------------------------------------------------------------- Eq. 1 / RTN
def test_rtn_matches_eq1_properties(case):
    w64, rtn = case["w64"], case["rtn"]
    amax = np.abs(w64).max()
    # alpha0 = max|W| / (6 * 448), one binary32 division
    assert rtn.global_scale == np.float32(np.float32(amax) / np.float32(2688.0))
    assert rtn.trace["alpha0"] == rtn.global_scale
    # the block that holds the tensor maximum gets the largest scale and code +-6
    r, c = np.unravel_index(np.argmax(np.abs(w64)), w64.shape)
    assert rtn.scales[r, c // 16] == 0x7E
    assert abs(unpack(rtn.codes)[r, c]) == 6.0
    # every block whose scale is a normal, unclipped E4M3 value maps its own
    # maximum to the largest code (E4M3 rounding moves x by at most 1/16)
    q = np.abs(unpack(rtn.codes)).reshape(w64.shape[0], -1, 16).max(axis=2)
    normal = (rtn.scales >= 0x08) & (rtn.scales < 0x7E)
    assert np.all(q[normal] == 6.0)
    # block scale = E4M3 projection of bmax/(6 alpha0): check by brute-force nearest
    bmax = np.abs(w64).reshape(w64.shape[0], -1, 16).max(axis=2)
    y = bmax / (6.0 * float(rtn.global_scale))
    d = E4M3[rtn.scales]
    nearest = np.abs(E4M3[1:0x7F][None, None, :] - np.minimum(y, 1e4)[..., None]).min(axis=2)
    assert np.all(np.abs(d - np.minimum(y, 1e4)) <= nearest * (1 + 1e-5) + 1e-12)


def test_rtn_closed_form_tensor_is_reproduced_exactly():
    """W = Q * (alpha * d) with alpha a power of two, every block holding a +-6
    and one block at scale 448: Eq. 1-2 must return Q, d, alpha and zero error."""
    rng = np.random.default_rng(7)
    rows, cols = 24, 160
    for k in (-12, -3, 0, 5):
        alpha = 2.0 ** k
        nib = rng.integers(0, 16, size=(rows, cols)).astype(np.uint8)
        # avoid "-0": a zero weight has no sign to recover
        nib[(nib & 7) == 0] = 0
        dcode = rng.integers(0x08, 0x7F, size=(rows, cols // 16)).astype(np.uint8)
        dcode[3, 2] = 0x7E
        nib[:, ::16] = 7                      # a +6 in every block
        nib[3, 32 + 5] = 15                   # and a -6 in the 448 block
        q = np.where(nib & 8, -E2M1[nib & 7], E2M1[nib & 7])
        wv = q * np.repeat(E4M3[dcode], 16, axis=1) * alpha
        wt = torch.from_numpy(wv).to(torch.float32)
        assert torch.equal(wt.to(torch.bfloat16).float(), wt)       # exactly representable
        bits = synth.bf16_bits(wt.to(torch.bfloat16))
        packed = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
        for method in (oracle.METHOD_RTN, oracle.METHOD_SOAR):
            out = oracle.quantize(bits, method, 4)
            assert out.global_scale == np.float32(alpha)
            assert np.array_equal(out.scales, dcode)
            assert np.array_equal(out.codes, packed)
            assert out.sse == 0.0
            back = oracle.dequantize(out.codes, out.scales, out.global_scale, oracle.FP32)
            assert np.array_equal(back.astype(np.float64), wv)
            back16 = oracle.dequantize(out.codes, out.scales, out.global_scale, oracle.BF16)
            assert np.array_equal(back16, bits)


# --------------------------------------------------------------- Eq. 5 / Eq. 6
def test_global_scale_is_the_least_squares_solution(case):
    w64, tr = case["w64"], case["soar"].trace
    q0 = unpack(tr["nib0"].reshape(w64.shape[0], -1))
    d0 = E4M3[tr["code0"]].reshape(w64.shape[0], -1)
    v = (q0 * np.repeat(d0, 16, axis=1)).reshape(-1)
    sol, *_ = np.linalg.lstsq(v[:, None], w64.reshape(-1), rcond=None)
    assert abs(float(tr["alpha1"]) - sol[0]) <= 2e-7 * abs(sol[0])
    # numerator / denominator of Eq. 5
    assert math.isclose(tr["N"], float(np.dot(v, w64.reshape(-1))), rel_tol=1e-6)
    assert math.isclose(tr["M"], float(np.dot(v, v)), rel_tol=1e-12)
    # alpha1 is the float32 nearest to N/M
    assert np.float32(tr["N"] / tr["M"]) == tr["alpha1"]
    assert case["soar"].global_scale == tr["alpha1"]
    # stationarity and perturbation
    base = loss(w64, q0, tr["alpha1"], d0)
    for eps in (1e-3, -1e-3, 1e-2, -1e-2):
        assert loss(w64, q0, float(tr["alpha1"]) * (1 + eps), d0) >= base


def test_block_scale_is_the_per_block_least_squares_solution(case):
    w64, tr = case["w64"], case["soar"].trace
    rows = w64.shape[0]
    q0 = unpack(tr["nib0"].reshape(rows, -1)).reshape(-1, 16)
    wb = w64.reshape(-1, 16)
    a = (wb * q0).sum(axis=1)
    b = (q0 * q0).sum(axis=1)
    assert np.allclose(tr["a"], a, rtol=1e-6, atol=0)
    assert np.array_equal(tr["b"].astype(np.float64), b)        # exact: multiples of 1/4
    nz = b > 0
    ds = tr["delta_star"].astype(np.float64)
    want = a[nz] / (float(tr["alpha1"]) * b[nz])
    assert np.allclose(ds[nz], want, rtol=5e-7, atol=0)
    assert np.all(ds > 0)
    # textbook routine on a few blocks
    for i in np.nonzero(nz)[0][:50]:
        sol, *_ = np.linalg.lstsq((q0[i] * float(tr["alpha1"]))[:, None], wb[i], rcond=None)
        assert math.isclose(ds[i], sol[0], rel_tol=1e-6)
    # blocks whose codes are all zero keep the Eq. 1 scale
    assert np.array_equal(ds[~nz], E4M3[tr["code0"]][~nz])
    # centre = E4M3 projection of Delta*: nearest representable (brute force)
    c = tr["centre"]
    dist = np.abs(E4M3[1:0x7F][None, :] - np.minimum(ds, 1e4)[:, None])
    assert np.all(np.abs(E4M3[c] - np.minimum(ds, 1e4)) <= dist.min(axis=1) * (1 + 1e-6) + 1e-12)


def test_descent_chain(case):
    """L(a0,D0,Q0) >= L(a1,D0,Q0) >= L(a1,D*,Q0) >= L(a1,D*,Q1): optimal alpha for
    the rest fixed; optimal real block scale; nearest-grid assignment for a fixed
    scale.  (Only the projection of the stored scale onto E4M3 can raise it.)"""
    w64, so, tr = case["w64"], case["soar"], case["soar"].trace
    rows = w64.shape[0]
    q0 = unpack(tr["nib0"].reshape(rows, -1))
    q1 = unpack(so.codes)
    d0 = E4M3[tr["code0"]].reshape(rows, -1)
    ds = tr["delta_star"].astype(np.float64).reshape(rows, -1)
    l0 = loss(w64, q0, tr["alpha0"], d0)
    l1 = loss(w64, q0, tr["alpha1"], d0)
    l2 = loss(w64, q0, tr["alpha1"], ds)
    l3 = loss(w64, q1, tr["alpha1"], ds)
    tol = 1e-6
    assert l0 * (1 + tol) >= l1 and l1 * (1 + tol) >= l2 and l2 * (1 + tol) >= l3
    # the RTN error the oracle reports is l0 (float32 accumulation per block)
    assert math.isclose(case["rtn"].sse, l0, rel_tol=1e-5)


def test_new_assignment_is_nearest_grid_point_under_delta_q(case):
    w64, so, tr = case["w64"], case["soar"], case["soar"].trace
    rows = w64.shape[0]
    ds = np.repeat(tr["delta_star"].astype(np.float64).reshape(rows, -1), 16, axis=1)
    x = np.abs(w64) / (float(tr["alpha1"]) * ds)
    q1 = np.abs(unpack(so.codes))
    dist = np.abs(x[..., None] - E2M1[None, None, :]).min(axis=2)
    # nearest grid point up to float32 rounding of x
    assert np.all(np.abs(x - q1) <= dist + 1e-5 * (1 + x))
    # sign bits are the signs of the weights
    nib = np.stack([so.codes & 0xF, so.codes >> 4], axis=-1).reshape(rows, -1)
    assert np.array_equal((nib & 8) != 0, np.signbit(case["w"].float().numpy()))


# --------------------------------------------------------------- Eq. 8 / DSS
def test_dss_choice_against_enumeration_of_all_e4m3_scales(case):
    spec, w64, so, tr = case["spec"], case["w64"], case["soar"], case["soar"].trace
    K = spec.dss_radius
    wb = w64.reshape(-1, 16)
    q1 = unpack(so.codes).reshape(-1, 16)
    alpha = float(tr["alpha1"])
    allc = np.arange(1, 0x7F)
    s = alpha * E4M3[allc]                                        # [126]
    # err[i, c] for every block and every E4M3 code, float64
    A = (wb * wb).sum(axis=1)[:, None]
    B = (wb * q1).sum(axis=1)[:, None]
    Cq = (q1 * q1).sum(axis=1)[:, None]
    err = A - 2 * B * s[None, :] + Cq * s[None, :] ** 2
    # direct evaluation on a subset guards the expanded form
    for i in range(0, wb.shape[0], max(1, wb.shape[0] // 64)):
        direct = ((wb[i][None, :] - q1[i][None, :] * s[:, None]) ** 2).sum(axis=1)
        assert np.allclose(direct, err[i], rtol=1e-9, atol=1e-18)
    chosen = so.scales.reshape(-1).astype(np.int64)
    centre = tr["centre"].astype(np.int64)
    assert np.all(np.abs(chosen - centre) <= K)
    assert np.all((chosen >= 1) & (chosen <= 0x7E))
    lo = np.maximum(centre - K, 1)
    hi = np.minimum(centre + K, 0x7E)
    idx = np.arange(wb.shape[0])
    e_chosen = err[idx, chosen - 1]
    inwin = (allc[None, :] >= lo[:, None]) & (allc[None, :] <= hi[:, None])
    e_win = np.where(inwin, err, np.inf).min(axis=1)
    scale_ref = np.maximum(A[:, 0], 1e-300)
    # chosen = best of its window (float32 evaluation noise only)
    assert np.all(e_chosen <= e_win + 2e-6 * scale_ref)
    # chosen is never worse than the rounded closed-form scale
    assert np.all(e_chosen <= err[idx, centre - 1] + 2e-6 * scale_ref)
    # when the best of ALL 126 scales lies in the window, the window search found it
    g = err.argmin(axis=1) + 1
    inside = (g >= lo) & (g <= hi)
    e_glob = err.min(axis=1)
    assert np.all(e_chosen[inside] <= e_glob[inside] + 2e-6 * scale_ref[inside])
    # which is nearly always, for a radius of 4 or more
    assert inside.mean() > 0.999
    # reported per-block error and total
    assert np.allclose(tr["err_best"], e_chosen, rtol=2e-5, atol=1e-6 * float(scale_ref.mean()))
    assert math.isclose(so.sse, float(e_chosen.sum()), rel_tol=1e-5)


@pytest.mark.parametrize("K", [0, 1, 2])
def test_dss_small_radius_uses_the_whole_window(K):
    """With a small radius the best code often sits on the edge of the window:
    the choice must still be the best of centre-K..centre+K, and for K = 1 both
    edges must be taken by some block."""
    spec, w = weights(2, 16)
    bits = synth.bf16_bits(w)
    out = oracle.quantize(bits, oracle.METHOD_SOAR, K, want_trace=True)
    wb = w.double().numpy().reshape(-1, 16)
    q1 = unpack(out.codes).reshape(-1, 16)
    s = float(out.trace["alpha1"]) * E4M3[1:0x7F]
    A = (wb * wb).sum(axis=1)[:, None]
    Bq = (wb * q1).sum(axis=1)[:, None]
    Cq = (q1 * q1).sum(axis=1)[:, None]
    err = A - 2 * Bq * s[None, :] + Cq * s[None, :] ** 2
    centre = out.trace["centre"].astype(np.int64)
    chosen = out.scales.reshape(-1).astype(np.int64)
    allc = np.arange(1, 0x7F)
    inwin = (allc[None, :] >= (centre - K)[:, None]) & (allc[None, :] <= (centre + K)[:, None])
    e_win = np.where(inwin, err, np.inf).min(axis=1)
    e_chosen = err[np.arange(len(chosen)), chosen - 1]
    assert np.all(np.abs(chosen - centre) <= K)
    assert np.all(e_chosen <= e_win + 2e-6 * A[:, 0])
    if K == 1:      # +-1 is chosen by about one block in ten; +-2 by one in ten thousand
        off = chosen - centre
        assert (off == -K).any() and (off == K).any()


def test_dss_exact_tie_prefers_the_centre_code():
    """A block whose codes are all zero has the same error for every candidate:
    the first in search order, the centre, must be kept."""
    w = torch.zeros(4, 64, dtype=torch.float32)
    w[0, 0] = 1.0                       # tensor maximum
    w[1, :16] = 1e-8                    # far below the global maximum: all codes 0
    w[2, 16:32] = torch.linspace(0.1, 0.5, 16)
    bits = synth.bf16_bits(w.to(torch.bfloat16))
    out = oracle.quantize(bits, oracle.METHOD_SOAR, 4, want_trace=True)
    blk = 1 * 4 + 0
    assert out.trace["b"][blk] == 0.0
    assert out.scales.reshape(-1)[blk] == out.trace["centre"][blk] == out.trace["code0"][blk]
    assert np.all((out.codes.reshape(-1, 8)[blk] & 0x77) == 0)


def test_not_worse_than_rtn_at_tensor_level():
    worse = 0
    for seed in range(40):
        wl = 1 + seed % 5
        spec, w = weights(wl, 64 if wl > 1 else 4, seed_shift=seed + 1)
        bits = synth.bf16_bits(w)
        so = oracle.quantize(bits, oracle.METHOD_SOAR, spec.dss_radius)
        rt = oracle.quantize(bits, oracle.METHOD_RTN, 0)
        worse += so.sse > rt.sse
    assert worse == 0


# --------------------------------------------------------------- whole path
def test_reported_error_equals_recon_error_and_float64(case):
    w64, so, rtn, bits = case["w64"], case["soar"], case["rtn"], case["bits"]
    for out in (so, rtn):
        assert oracle.recon_error(bits, out.codes, out.scales, out.global_scale) == out.sse
        q = unpack(out.codes)
        d = E4M3[out.scales]
        assert math.isclose(out.sse, loss(w64, q, out.global_scale, d), rel_tol=1e-5)


def test_dequantized_values_are_grid_times_scales(case):
    so = case["soar"]
    back = oracle.dequantize(so.codes, so.scales, so.global_scale, oracle.FP32)
    s = (np.float32(so.global_scale) * E4M3[so.scales].astype(np.float32)).astype(np.float32)
    want = (unpack(so.codes).astype(np.float32) * np.repeat(s, 16, axis=1)).astype(np.float32)
    assert np.array_equal(back, want)
    b16 = oracle.dequantize(so.codes, so.scales, so.global_scale, oracle.BF16)
    want16 = torch.from_numpy(want).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b16, want16)


def test_power_of_two_and_sign_equivariance(case):
    w, so, spec = case["w"], case["soar"], case["spec"]
    for k in (-7, 9):
        o2 = oracle.quantize(synth.bf16_bits((w.float() * 2.0 ** k).to(torch.bfloat16)),
                             oracle.METHOD_SOAR, spec.dss_radius)
        assert np.array_equal(o2.codes, so.codes) and np.array_equal(o2.scales, so.scales)
        assert o2.global_scale == np.float32(so.global_scale * np.float32(2.0 ** k))
        assert math.isclose(o2.sse, so.sse * 4.0 ** k, rel_tol=1e-12)
    o3 = oracle.quantize(synth.bf16_bits(-w), oracle.METHOD_SOAR, spec.dss_radius)
    assert np.array_equal(o3.codes, so.codes ^ 0x88) and np.array_equal(o3.scales, so.scales)
    assert o3.global_scale == so.global_scale and o3.sse == so.sse


def test_output_footprint_is_plain_nvfp4(case):
    w, so = case["w"], case["soar"]
    n = w.numel()
    assert so.codes.nbytes == n // 2 and so.scales.nbytes == n // 16


def test_fp32_input_and_leading_dimension(case):
    w, so, spec = case["w"], case["soar"], case["spec"]
    f = w.float().numpy()
    o32 = oracle.quantize(f, oracle.METHOD_SOAR, spec.dss_radius)
    assert np.array_equal(o32.codes, so.codes) and np.array_equal(o32.scales, so.scales)
    assert o32.global_scale == so.global_scale and o32.sse == so.sse
    wide = np.zeros((f.shape[0], f.shape[1] + 48), dtype=np.uint16)
    wide[:] = 0x7F80                    # +inf in the padding: must never be read
    wide[:, : f.shape[1]] = case["bits"]
    o_ld = oracle.quantize(wide[:, : f.shape[1]], oracle.METHOD_SOAR, spec.dss_radius)
    assert np.array_equal(o_ld.codes, so.codes) and np.array_equal(o_ld.scales, so.scales)
    assert o_ld.global_scale == so.global_scale and o_ld.sse == so.sse


def test_true_fp32_weights_follow_the_same_theorems():
    rng = np.random.default_rng(11)
    f = (rng.standard_t(4, size=(64, 256)) * 0.02).astype(np.float32)
    out = oracle.quantize(f, oracle.METHOD_SOAR, 4, want_trace=True)
    rtn = oracle.quantize(f, oracle.METHOD_RTN, 0)
    w64 = f.astype(np.float64)
    q = unpack(out.codes)
    assert math.isclose(out.sse, loss(w64, q, out.global_scale, E4M3[out.scales]), rel_tol=1e-5)
    assert out.sse <= rtn.sse
    q0 = unpack(out.trace["nib0"].reshape(64, -1))
    v = (q0 * np.repeat(E4M3[out.trace["code0"]].reshape(64, -1), 16, axis=1)).reshape(-1)
    sol, *_ = np.linalg.lstsq(v[:, None], w64.reshape(-1), rcond=None)
    assert abs(float(out.global_scale) - sol[0]) <= 2e-7 * abs(sol[0])


# --------------------------------------------------------------- tree sum
def _padded_tree(vals):
    n = 1
    while n < len(vals):
        n *= 2
    t = list(vals) + [0.0] * (n - len(vals))
    while len(t) > 1:
        t = [t[2 * k] + t[2 * k + 1] for k in range(len(t) // 2)]
    return t[0]


@pytest.mark.parametrize("rows,cols", [(1, 16), (3, 48), (5, 112), (7, 16 * 13), (16, 256)])
def test_tensor_wide_sums_follow_the_zero_padded_pair_tree(rows, cols):
    rng = np.random.default_rng(rows * 100 + cols)
    f = (rng.standard_t(3, size=(rows, cols)) * np.exp(rng.uniform(-3, 3, size=(rows, 1)))).astype(np.float32)
    out = oracle.quantize(f, oracle.METHOD_SOAR, 2, want_trace=True)
    tr = out.trace
    d0 = E4M3[tr["code0"]]
    tn = [float(a) * float(d) for a, d in zip(tr["a"], d0)]
    tm = [float(b) * float(d) * float(d) for b, d in zip(tr["b"], d0)]
    assert tr["N"] == _padded_tree(tn)
    assert tr["M"] == _padded_tree(tm)
    assert math.isclose(tr["N"], math.fsum(tn), rel_tol=1e-13)


def test_row_shards_of_aligned_power_of_two_size_reproduce_the_tree():
    """What sharding a tensor by rows would rely on: if every shard holds an aligned power-of-two range of
    blocks, the tree over the shards' own tree sums is the tree over all blocks, bit for bit; the global
    scale of the whole tensor then follows from the shards' maxima and (N, M) pairs alone."""
    rng = np.random.default_rng(11)
    f = (rng.standard_t(3, size=(64, 256)) * np.exp(rng.uniform(-2, 2, size=(64, 1))) * 0.02).astype(np.float32)
    whole = oracle.quantize(f, oracle.METHOD_SOAR, 2, want_trace=True)
    tr = whole.trace
    d0 = E4M3[tr["code0"]]
    tn = [float(a) * float(d) for a, d in zip(tr["a"], d0)]
    tm = [float(b) * float(d) * float(d) for b, d in zip(tr["b"], d0)]
    for shards in (2, 4, 8):
        n = len(tn) // shards                      # 1024 blocks: every shard an aligned power of two
        part_n = [_padded_tree(tn[k * n:(k + 1) * n]) for k in range(shards)]
        part_m = [_padded_tree(tm[k * n:(k + 1) * n]) for k in range(shards)]
        assert _padded_tree(part_n) == tr["N"] and _padded_tree(part_m) == tr["M"]
        assert np.float32(_padded_tree(part_n) / _padded_tree(part_m)) == tr["alpha1"]
    amax = max(float(np.abs(f[k * 16:(k + 1) * 16]).max()) for k in range(4))
    assert np.float32(np.float32(amax) / np.float32(2688.0)) == tr["alpha0"]


# --------------------------------------------------------------- degenerate inputs
def test_all_zero_and_non_finite_tensors():
    z = np.zeros((4, 32), dtype=np.uint16)
    z[1, 3] = 0x8000                    # -0.0
    out = oracle.quantize(z, oracle.METHOD_SOAR, 4)
    assert out.status & oracle.STATUS_ALLZERO
    assert out.global_scale == 1.0 and out.sse == 0.0
    assert np.all(out.scales == 0x01)
    assert out.codes[1, 1] == 0x80 and out.codes.sum() == 0x80
    bad = np.zeros((4, 32), dtype=np.float32)
    bad[2, 2] = np.inf
    assert oracle.quantize(bad, oracle.METHOD_SOAR, 4).status & oracle.STATUS_NONFINITE
    bad[2, 2] = np.nan
    assert oracle.quantize(bad, oracle.METHOD_RTN, 4).status & oracle.STATUS_NONFINITE


def test_bad_arguments_are_rejected():
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((4, 24), dtype=np.float32))
    with pytest.raises(TypeError):
        oracle.quantize(np.zeros((4, 32), dtype=np.float64))
