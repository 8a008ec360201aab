"""The C-ABI library loads without a GPU, exports every symbol that
include/soar.h declares, and rejects bad arguments on the host before
anything is enqueued (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

from paper_2605_12245_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "soar.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(soar_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert set(B.EXPORTS) == set(names)
    L = B.lib()
    for n in names:
        assert getattr(L, n) is not None, n


def test_version_and_status_strings():
    assert B.soar_version() >= 0x00010000
    L = B.lib()
    seen = {L.soar_status_string(k).decode() for k in range(9)}
    assert len(seen) == 9 and "ok" in seen
    assert L.soar_status_string(99).decode() == "unknown status"


def test_default_params_and_workspace_query():
    p = B.soar_default_params()
    assert (p.struct_size, p.method, p.block, p.iters, p.dss_radius, p.n_beta) == (C.sizeof(B.soar_params), 1, 16, 1, 4, 1)
    assert p.beta_lo == 1.0 and p.beta_hi == 1.0
    n = B.soar_workspace_bytes(4096, 4096, p)
    assert n > 0 and n % 256 == 0
    assert B.soar_workspace_bytes(4096, 4090, p) == 0
    assert B.soar_workspace_bytes(0, 4096, p) == 0
    p.iters = 15
    assert B.soar_workspace_bytes(4096, 4096, p) == n          # the iterated path needs no more
    p.iters = 65
    assert B.soar_workspace_bytes(4096, 4096, p) == 0
    q = B.soar_paper_params()
    assert (q.iters, q.n_beta, q.dd_mode, q.method) == (15, 101, B.SOAR_DD_BRACKET, 1)
    assert (q.beta_lo, q.beta_hi) == (0.5, 1.5) and abs(q.early_stop_rel - 1e-3) < 1e-9
    assert B.soar_workspace_bytes(4096, 4096, q) == n


def _q(p, d_w=0x1000, dtype=0, rows=64, cols=64, ld=64, codes=0x2000, scales=0x3000, gs=0x4000,
       ws=0x10000, ws_bytes=1 << 20):
    # the addresses are never dereferenced: every call below must fail validation
    return B.soar_quantize(d_w, dtype, rows, cols, ld, p, codes, scales, gs, 0, 0, ws, ws_bytes, 0)


def test_host_side_argument_validation():
    p = B.soar_default_params()
    assert _q(p, d_w=0) == 1 and _q(p, codes=0) == 1 and _q(p, scales=0) == 1 and _q(p, gs=0) == 1
    assert _q(p, cols=40, ld=40) == 2 and _q(p, rows=0) == 2 and _q(p, ld=48) != 0 and _q(p, ld=32) == 2
    assert _q(p, rows=1 << 31, cols=1 << 20, ld=1 << 20) == 2
    assert _q(p, dtype=5) == 3
    assert _q(p, d_w=0x1008) == 7 and _q(p, ld=68) == 7 and _q(p, codes=0x2004) == 7
    assert _q(p, ws=0) == 5 and _q(p, ws=0x10010) == 5 and _q(p, ws_bytes=1000) == 5
    for field, bad in (("method", 7), ("block", 32), ("iters", 0), ("iters", 65), ("dss_radius", -1),
                       ("dss_radius", 200), ("n_beta", 0), ("n_beta", 4097), ("beta_lo", 0.0), ("beta_lo", 1.5),
                       ("beta_hi", float("inf")), ("early_stop_rel", -1.0), ("early_stop_rel", float("nan")),
                       ("dd_mode", 2), ("search_mode", 9), ("tiles_per_wg", 3), ("tiles_per_wg_absmax", 70000), ("tiles_per_wg_search", -2), ("streams", 3),
                       ("struct_size", 4)):
        q = B.soar_default_params()
        setattr(q, field, bad)
        assert _q(q) == 4, field
    assert B.soar_dequantize(0, 0x10, 0x20, 4, 64, 0, 0x1000, 64, 0) == 1
    assert B.soar_dequantize(0x8, 0x10, 0x20, 4, 60, 0, 0x1000, 64, 0) == 2
    assert B.soar_recon_error(0x1000, 0, 4, 64, 64, 0x8, 0x10, 0x20, 0, 0) == 1
    assert B.soar_recon_error(0x1000, 3, 4, 64, 64, 0x8, 0x10, 0x20, 0x30, 0) == 3
    assert B.soar_e2m1_round_f32(0, 4, 0x10, 0) == 1 and B.soar_e4m3_project_f32(0x10, -1, 0x10, 0) == 2
    # the arms of the component study
    for method, field, v in ((2, "n_beta", 3), (2, "beta_lo", 0.5), (2, "dd_mode", 1), (2, "dss_radius", 1),
                             (3, "dd_mode", 1), (4, "iters", 1)):
        q = B.soar_arm_params(min(method, 3), iters=2)
        q.method = method
        setattr(q, field, v)
        if field == "beta_lo":
            q.beta_hi = v
        assert _q(q) == 4, (method, field)
    # plain NVFP4 has no iterated form
    for field, v in (("iters", 2), ("n_beta", 3), ("dd_mode", 1)):
        q = B.soar_default_params(B.SOAR_METHOD_RTN, 0)
        setattr(q, field, v)
        assert _q(q) == 4, field
    d = B.soar_tensor_desc(0x1000, 0, 64, 64, 64, 0x2000, 0x3000, 0x4000, 0, 0, 0x5000, 0)
    assert B.soar_quantize_batch([d], B.soar_default_params(B.SOAR_METHOD_RTN, 0), 0x10000, 1 << 20, 0) == 4
    # a supplied maximum: plain NVFP4 only, and for every tensor of a batch or for none
    d = B.soar_tensor_desc(0x1000, 0, 64, 64, 64, 0x2000, 0x3000, 0x4000, 0, 0, 0, 0, 0x5000)
    e = B.soar_tensor_desc(0x1000, 0, 64, 64, 64, 0x2000, 0x3000, 0x4000, 0, 0, 0, 0, 0)
    assert B.soar_quantize_batch([d], p, 0x10000, 1 << 20, 0) == 4
    assert B.soar_quantize_batch([d, e], B.soar_default_params(B.SOAR_METHOD_RTN, 0), 0x10000, 1 << 20, 0) == 4
    d = B.soar_tensor_desc(0x1000, 0, 64, 60, 64, 0x2000, 0x3000, 0x4000, 0, 0)
    assert B.soar_quantize_batch([d], p, 0x10000, 1 << 20, 0) == 2
    assert B.soar_quantize_batch([], p, 0x10000, 1 << 20, 0) == 0


def test_stored_form_batch_host_side_argument_validation():
    def desc(**kw):
        d = B.soar_stored_desc()
        d.d_codes, d.d_scales, d.d_global_scale = 0x8, 0x10, 0x20
        d.rows, d.cols, d.ld_elems, d.dtype = 4, 64, 64, 0
        d.d_w, d.d_out, d.d_sse = 0x1000, 0x2000, 0x30
        for k, v in kw.items():
            setattr(d, k, v)
        return d
    for call, own in ((B.soar_dequantize_batch, "d_out"), (B.soar_recon_error_batch, "d_w")):
        assert call([], 0) == 0
        assert call([desc(d_codes=0)], 0) == 1 and call([desc(d_global_scale=0)], 0) == 1
        assert call([desc(**{own: 0})], 0) == 1
        assert call([desc(), desc(dtype=2)], 0) == 3
        assert call([desc(cols=60)], 0) == 2 and call([desc(ld_elems=48)], 0) == 2 and call([desc(rows=0)], 0) == 2
        assert call([desc(**{own: 0x1008})], 0) == 7 and call([desc(ld_elems=68)], 0) == 7
        assert call([desc(d_codes=0x2004)], 0) == 7
    assert B.soar_recon_error_batch([desc(d_sse=0)], 0) == 1
    assert int(B.lib().soar_dequantize_batch(-1, None, None)) == 2 and int(B.lib().soar_recon_error_batch(2, None, None)) == 1
    # the MXFP4 form reads codes, scales, shape, type and output only
    assert B.soar_mxfp4_dequantize_batch([], 0) == 0
    assert B.soar_mxfp4_dequantize_batch([desc(d_codes=0x10, d_out=0)], 0) == 1
    assert B.soar_mxfp4_dequantize_batch([desc(d_codes=0x10, cols=48, ld_elems=48)], 0) == 2
    assert B.soar_mxfp4_dequantize_batch([desc(d_codes=0x8)], 0) == 7 and B.soar_mxfp4_dequantize_batch([desc(d_codes=0x10, dtype=4)], 0) == 3


def test_header_is_plain_c_and_layouts_match_the_binding(tmp_path):
    """include/soar.h through a C99 compiler in pedantic mode, linked against the library; the structure
    sizes and offsets the C side prints are those of the ctypes structures; host validation from C."""
    import subprocess
    exe = str(tmp_path / "c_abi_check")
    lib_dir = os.path.dirname(B.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", exe,
           "-L", lib_dir, "-lsoar_hip", "-Wl,-rpath," + lib_dir, "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib",
           "-Wl,--allow-shlib-undefined"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    got = {}
    for line in r.stdout.splitlines():
        key, _, val = line.rpartition(" ")
        got[key] = val
    for name in ("soar_params", "soar_tensor_desc", "soar_stored_desc", "soar_mx_params", "soar_mx_tensor_desc"):
        assert int(got["sizeof " + name]) == C.sizeof(getattr(B, name)), name
    for name, field in (("soar_params", "dss_radius"), ("soar_params", "early_stop_rel"), ("soar_params", "streams"),
                        ("soar_tensor_desc", "d_codes"), ("soar_tensor_desc", "d_amax_in"), ("soar_stored_desc", "dtype"),
                        ("soar_stored_desc", "d_sse"), ("soar_mx_params", "radius"), ("soar_mx_params", "streams"),
                        ("soar_mx_tensor_desc", "d_status")):
        assert int(got[f"{name}.{field}"]) == getattr(getattr(B, name), field).offset, (name, field)
    assert got["default iters 1 n_beta 1 block 16 struct_size"] == str(C.sizeof(B.soar_params))
    assert int(got["version"]) == B.soar_version()
    assert int(got["workspace 256x256"]) == B.soar_workspace_bytes(256, 256, B.soar_default_params())
    assert got["null weights"] == "1" and got["empty batch"] == "0" and got["bad shape"] == "2"
    assert r.stdout.splitlines()[-1].startswith("status text ") and len(r.stdout.splitlines()[-1]) > 14


def test_product_path_has_no_cpu_route():
    torch = pytest.importorskip("torch")
    w = torch.zeros(16, 16, dtype=torch.bfloat16)
    with pytest.raises(RuntimeError):
        B.quantize(w)
    src = open(os.path.join(ROOT, "paper_2605_12245_amd", "binding.py")).read()
    assert "import oracle" not in src and "from oracle" not in src


def test_mxfp4_host_side_argument_validation():
    p = B.soar_mx_default_params()
    assert (p.struct_size, p.dss, p.n_beta, p.radius) == (C.sizeof(B.soar_mx_params), 1, 101, 1)
    n = B.soar_mxfp4_workspace_bytes(4096, 4096, p)
    assert n > 0 and n % 256 == 0
    assert B.soar_mxfp4_workspace_bytes(4096, 4080, p) == 0          # cols % 32

    def q(p, d_w=0x1000, dtype=0, rows=64, cols=64, ld=64, codes=0x2000, scales=0x3000, ws=0x10000, ws_bytes=1 << 20):
        return B.soar_mxfp4_quantize(d_w, dtype, rows, cols, ld, p, codes, scales, 0, 0, ws, ws_bytes, 0)

    assert q(p, d_w=0) == 1 and q(p, codes=0) == 1 and q(p, scales=0) == 1
    assert q(p, cols=48, ld=48) == 2 and q(p, rows=0) == 2 and q(p, ld=32) == 2
    assert q(p, dtype=7) == 3
    assert q(p, d_w=0x1004) == 7 and q(p, codes=0x2008) == 7 and q(p, ld=68) == 7
    assert q(p, ws=0) == 5 and q(p, ws=0x10010) == 5 and q(p, ws_bytes=64) == 5
    for field, bad in (("dss", 2), ("n_beta", 0), ("n_beta", 5000), ("beta_lo", 0.0), ("beta_hi", 0.25),
                       ("radius", -1), ("radius", 128), ("tiles_per_wg", 3), ("single_pass", 2), ("streams", 3),
                       ("struct_size", 8)):
        r = B.soar_mx_default_params()
        setattr(r, field, bad)
        assert q(r) == 4, field
    d = B.soar_mx_tensor_desc(0x1000, 0, 64, 64, 64, 0x2000, 0x3000, 0, 0)
    bad = B.soar_mx_tensor_desc(0x1000, 0, 64, 48, 64, 0x2000, 0x3000, 0, 0)
    assert B.soar_mxfp4_batch_workspace_bytes([d] * 3, p) == 3 * n and B.soar_mxfp4_batch_workspace_bytes([d] * 20, p) == 2 * 8 * n
    assert B.soar_mxfp4_batch_workspace_bytes([d, bad], p) == 0
    assert B.soar_mxfp4_quantize_batch([d, bad], p, 0x10000, 1 << 24, 0) == 2
    assert B.soar_mxfp4_quantize_batch([d, d], p, 0x10000, n, 0) == 5
    assert B.soar_mxfp4_quantize_batch([], p, 0x10000, 1 << 20, 0) == 0
    assert B.soar_mxfp4_dequantize(0, 0x10, 4, 64, 0, 0x1000, 64, 0) == 1
    assert B.soar_mxfp4_dequantize(0x10, 0x10, 4, 48, 0, 0x1000, 48, 0) == 2
    assert B.soar_mxfp4_dequantize(0x18, 0x10, 4, 64, 0, 0x1000, 64, 0) == 7


def test_bench_refuses_more_than_one_gpu_and_a_missing_gpu():
    import subprocess
    import sys
    bench = os.path.join(ROOT, "bench.py")
    r = subprocess.run([sys.executable, bench, "--gpus", "2"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and not r.stdout.strip()
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, bench, "--steps", "1"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
        assert r.returncode == 2 and "no CPU fallback" in r.stderr and not r.stdout.strip()


def test_missing_library_raises_instead_of_falling_back(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "paper_2605_12245_amd", "no_such_library.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()
    with pytest.raises(RuntimeError):
        B.soar_default_params()


def test_arrival_counting_names_exactly_one_last_workgroup():
    """The two-level arrival counting of the kernels' hand-off ("the last workgroup of a tensor finishes the
    reduction"), modelled on the host with the library's own plan: for every number of workgroups and any
    order of arrival, every workgroup has a first-level counter, the counters' shares add up to the
    workgroups, exactly one arrival completes the top counter, and it is the last one to arrive."""
    import random
    rng = random.Random(5)
    sizes = list(range(1, 200)) + [255, 256, 257, 1000, 4095, 4096, 4097, 16383, 16384] + [rng.randrange(200, 16384) for _ in range(40)]
    for G in sizes:
        plans = [B.soar_debug_arrival_plan(G, w) for w in range(G)] if G <= 4097 else None
        if plans is None:                         # large: the plan is periodic in the workgroup number; sample it
            ns = min(G, 64)
            base = [B.soar_debug_arrival_plan(G, w) for w in range(ns)]
            plans = [base[w % ns] for w in range(G)]
            for w in rng.sample(range(G), 64):
                assert B.soar_debug_arrival_plan(G, w) == plans[w]
        ns = plans[0][0]
        assert ns == min(G, 64) and all(p[0] == ns for p in plans)
        share = {}
        for w, (_, slot, expected) in enumerate(plans):
            assert slot < ns and expected >= 1
            share.setdefault(slot, set()).add(expected)
        assert len(share) == ns and all(len(v) == 1 for v in share.values())
        assert sum(next(iter(v)) for v in share.values()) == G
        for _ in range(3 if G < 300 else 1):
            order = list(range(G))
            rng.shuffle(order)
            slots, top, last = [0] * ns, 0, []
            for w in order:
                _, slot, expected = plans[w]
                t = slots[slot]
                slots[slot] += 1
                if t != expected - 1:
                    continue
                t2 = top
                top += 1
                if t2 == ns - 1:
                    last.append(w)
            assert last == [order[-1]], (G, last)
            assert slots == [next(iter(share[k])) for k in range(ns)] and top == ns
    assert B.soar_debug_arrival_plan(0, 0) == (0xFFFFFFFF,) * 3 and B.soar_debug_arrival_plan(5, 5) == (0xFFFFFFFF,) * 3


def test_counter_table_that_bench_quotes_is_well_formed_and_points_at_committed_summaries():
    """bench.py takes roofline.traffic and the executed-instruction counts from profiles/pmc_table.json: every
    entry names a committed summary under profiles/, carries either both byte figures or an instruction count,
    and the lookup finds the headline kernel's entry (and says why when there is none)."""
    import importlib.util
    import json
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    with open(bench.PMC_TABLE) as f:
        table = json.load(f)
    assert table["calibration"]["fetch_scale"] > 0 and table["calibration"]["write_scale"] > 0
    keys = set()
    for e in table["entries"]:
        assert os.path.isfile(os.path.join(ROOT, e["source"])) and e["source"].startswith("profiles/"), e
        assert e["dtype"] in ("bf16", "fp32") and e["workload"].startswith("config") and e["kernel"].startswith("k_"), e
        has_bytes = "read_B_per_weight" in e and "written_B_per_weight" in e
        has_insts = "valu_lane_insts_per_block_factor" in e
        assert has_bytes != has_insts, e
        if has_bytes:
            assert 0 <= e["written_B_per_weight"] < 8 and 0 < e["read_B_per_weight"] < 16, e
        else:
            assert 10 < e["valu_lane_insts_per_block_factor"] < 1000, e
        key = (e["algorithm"], e["workload"], e["dtype"], e["kernel"], e.get("search", "auto"))
        assert key not in keys, key
        keys.add(key)
    e, why = bench.pmc_entry("single-step", 4, "bf16", "k_search")
    assert e is not None and why == e["source"]
    traffic, _ = bench.traffic_per_launch("single-step", 4, "bf16", "k_search", 1e6)
    assert traffic == pytest.approx((e["read_B_per_weight"] + e["written_B_per_weight"]) * 1e6)
    none, why = bench.pmc_entry("single-step", 4, "bf16", "k_search", layers=2)
    assert none is None and "subset" in why
    none, why = bench.traffic_per_launch("single-step", 9, "bf16", "k_nothing", 1.0)
    assert none is None and "no counter run" in why
