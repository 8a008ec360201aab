"""The pins must be able to fail: each mutant below plants ONE plausible mistake
in a copy of the oracle's source (on the CPU), builds it, and runs the pin tests
against it in a child process; every mutant has to be caught.  The mistakes are
planted in the oracle only -- never in the GPU path."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "soar_oracle.c")

MUTANTS = [
    ("e2m1 ties away from zero", "r = 0.5f * rintf(2.0f * a);", "r = 0.5f * roundf(2.0f * a);"),
    ("e2m1 no saturation", "        r = M_FP4;\n    return copysignf", "        r = 2.0f * rintf(a / 2.0f);\n    return copysignf"),
    ("e4m3 ties up", "rint(v / quantum) * quantum", "floor(v / quantum + 0.5) * quantum"),
    ("e4m3 subnormal spacing", "if (E < -6) E = -6;              /* below", "if (E < -7) E = -7;              /* below"),
    ("alpha0 without M_FP4", "const float alpha0 = amax / (M_FP4 * M_FP8);", "const float alpha0 = amax / M_FP8;"),
    ("block scale without M_FP4", "uint8_t c0 = soar_oracle_e4m3_project(bmax / alpha0_m);", "uint8_t c0 = soar_oracle_e4m3_project(bmax / alpha0);"),
    ("error with wrong sign", "for (int j = 0; j < BLOCK; ++j) {\n        float e = fmaf(-q[j], s, wv[j]);",
     "for (int j = 0; j < BLOCK; ++j) {\n        float e = fmaf(q[j], s, wv[j]);"),
    ("mx: error with wrong sign", "for (int j = 0; j < MX_BLOCK; ++j) {\n        float e = fmaf(-q[j], s, wv[j]);",
     "for (int j = 0; j < MX_BLOCK; ++j) {\n        float e = fmaf(q[j], s, wv[j]);"),
    ("Eq. 5 denominator with Delta instead of Delta^2",
     "termM[i] = ((double)b * (double)delta0) * (double)delta0;", "termM[i] = (double)b * (double)delta0;"),
    ("Eq. 5 numerator without Delta", "termN[i] = (double)a * (double)delta0;", "termN[i] = (double)a;"),
    ("Eq. 6 multiplied by alpha", "delta_star = (a_all[i] / b_all[i]) / alpha1;", "delta_star = (a_all[i] / b_all[i]) * alpha1;"),
    ("a = sum w^2", "sa = fmaf(wv[j], q[j], sa);", "sa = fmaf(wv[j], wv[j], sa);"),
    ("b = sum |q|", "sb = fmaf(q[j], q[j], sb);", "sb = sb + fabsf(q[j]);"),
    ("later candidate wins ties", "if (err < best_err) { best_err = err; best_code = c; }",
     "if (err <= best_err) { best_err = err; best_code = c; }"),
    ("window one code short", "for (int k = 1; k <= dss_radius; ++k) {", "for (int k = 1; k < dss_radius; ++k) {"),
    ("search only upwards", "++k) {\n            for (int sgn = -1; sgn <= 1; sgn += 2) {", "++k) {\n            for (int sgn = 1; sgn <= 1; sgn += 2) {"),
    ("nibbles swapped", "out[k] = (uint8_t)(lo | (hi << 4));", "out[k] = (uint8_t)(hi | (lo << 4));"),
    ("codes from the rounded scale (not decoupled)", "assign_codes(wv, alpha1, delta_star, q1);",
     "assign_codes(wv, alpha1, soar_oracle_e4m3_value(centre), q1);"),
    ("tree drops an odd tail", "            t[half] = t[n - 1];\n            n = half + 1;", "            n = half;"),
    ("dequantize ignores the global scale", "float s = global_scale * soar_oracle_e4m3_value(scales[i]);\n        for (int j = 0; j < BLOCK; ++j) {\n            uint8_t byte",
     "float s = soar_oracle_e4m3_value(scales[i]);\n        for (int j = 0; j < BLOCK; ++j) {\n            uint8_t byte"),
    ("bf16 rounding truncates", "u += 0x7FFFu + lsb;", "u += 0u * lsb;"),
    ("reciprocal of alpha only", "float scale = alpha * delta;\n    float r = 1.0f / scale;", "float scale = alpha * delta;\n    float r = 1.0f / alpha; (void)scale;"),
    ("block index transposed in the error sum of recon_error",
     "errs[i] = (double)block_error(wv, q, global_scale * soar_oracle_e4m3_value(scales[i]));",
     "errs[i] = (double)block_error(wv, q, global_scale * soar_oracle_e4m3_value(scales[(i % bpr) * rows + i / bpr < nblk ? (i % bpr) * rows + i / bpr : i]));"),
]

# mistakes in the iterated form of Algorithm 1 (caught by tests/test_oracle_iter.py)
MUTANTS += [
    ("iter: Eq. 5 with the search scale instead of the stored one",
     "float d = soar_oracle_e4m3_value(dd[i]);\n            termN[i]", "float d = dq[i];\n            termN[i]"),
    ("iter: codes from the previous global scale", "assign_codes(wv, alpha_new, dq_k, q);", "assign_codes(wv, alpha, dq_k, q);"),
    ("iter: beta grid one step short", "return (p->beta_lo * (float)(p->n_beta - 1 - k) + p->beta_hi * (float)k) / (float)(p->n_beta - 1);",
     "return (p->beta_lo * (float)(p->n_beta - 1 - k) + p->beta_hi * (float)k) / (float)(p->n_beta);"),
    ("iter: bracket takes the code above only", "if (lo < E4M3_CODE_MAX) cand[ncand++] = lo + 1;", "if (lo < E4M3_CODE_MAX) cand[ncand - 1] = lo + 1;"),
    ("iter: floor code off by one", "int lo = e4m3_floor_code(delta_star);", "int lo = e4m3_floor_code(delta_star) - 1; if (lo < E4M3_CODE_MIN) lo = E4M3_CODE_MIN;"),
    ("iter: search scale not kept", "dq[i] = best_dq;", "dq[i] = delta_star;"),
    ("iter: stored scale not kept", "dd[i] = (uint8_t)best_code;", "dd[i] = (uint8_t)cand[0];"),
    ("iter: early stop on the absolute drop", "(prev - cur) < (double)p->early_stop_rel * prev) break;", "(prev - cur) < (double)p->early_stop_rel) break;"),
    ("iter: early stop compares with the first error", "        prev = cur;\n    }\n    memcpy(scales, dd", "    }\n    memcpy(scales, dd"),
    ("iter: global scale not advanced", "        alpha = alpha_new;\n        cur = tree_sum(errs, nblk);", "        cur = tree_sum(errs, nblk);"),
    ("iter: Eq. 6 with the previous global scale", "delta_star = (a_all[i] / b_all[i]) / alpha_new;", "delta_star = (a_all[i] / b_all[i]) / alpha;"),
    ("iter: initial global scale without M_FP4", "    float alpha = amax / (M_FP4 * M_FP8);\n    const float alpha0_m", "    float alpha = amax / M_FP8;\n    const float alpha0_m"),
    ("iter: initial block scale without M_FP4", "dd[i] = soar_oracle_e4m3_project(bmax / alpha0_m);", "dd[i] = soar_oracle_e4m3_project(bmax / alpha);"),
    ("iter: window searched upwards only", "++k)\n                    for (int sgn = -1; sgn <= 1; sgn += 2) {", "++k)\n                    for (int sgn = 1; sgn <= 1; sgn += 2) {"),
    ("iter: trace entry of the wrong iteration", "if (sse_trace) sse_trace[t + 1] = cur;", "if (sse_trace) sse_trace[t + 1] = prev;"),
]

# mistakes in the ablation arms (caught by tests/test_oracle_arms.py)
MUTANTS += [
    ("arm: +CJSO assigns with the unrounded scale", "if (p->arm == ORACLE_ARM_CJSO_ONLY)                 /* one scale",
     "if (0)                 /* one scale"),
    ("arm: +DSS applies the closed-form global scale", "if (p->arm == ORACLE_ARM_DSS_ONLY) alpha_new = alpha;", ";"),
    ("arm: +DSS centred on Eq. 6", "if (b_all[i] == 0.0f || p->arm == ORACLE_ARM_DSS_ONLY)", "if (b_all[i] == 0.0f)"),
    ("arm: +CJSO accepts a beta grid", "(p->n_beta != 1 || p->beta_lo != 1.0f || p->dd_mode != 0 || p->dss_radius != 0))",
     "(p->beta_lo != 1.0f || p->dd_mode != 0 || p->dss_radius != 0))"),
]

# mistakes in the MXFP4 functions (caught by tests/test_oracle_mxfp4.py)
MUTANTS += [
    ("mx: element exponent 3 instead of 2", "#define MX_EMAX_ELEM 2", "#define MX_EMAX_ELEM 3"),
    ("mx: floor(log2) off by one", "int shared = (ex - 1) - MX_EMAX_ELEM;", "int shared = ex - MX_EMAX_ELEM;"),
    ("mx: E8M0 bias 128", "static float e8m0_value(int e) { return ldexpf(1.0f, e - 127); }",
     "static float e8m0_value(int e) { return ldexpf(1.0f, e - 128); }"),
    ("mx: codes assigned with the stored candidate (not decoupled)", "mx_assign(wv, x0 * beta_of(&grid, k), q);",
     "mx_assign(wv, e8m0_value(e0) , q);"),
    ("mx: search only downwards", "int code = (c & 1) ? e0 - o : e0 + o;", "int code = e0 - o;"),
    ("mx: later pair wins ties", "float err = mx_block_error(wv, q, e8m0_value(code));\n                    if (!have || err < best_err) {",
     "float err = mx_block_error(wv, q, e8m0_value(code));\n                    if (!have || err <= best_err) {"),
    ("mx: dequantize without the scale", "        float s = e8m0_value(scales[i]);", "        float s = 1.0f;"),
]

# mistakes in the supplied-maximum form (caught by tests/test_oracle_rtn_amax.py)
MUTANTS += [
    ("amax: global scale without M_FP4", "const float alpha = amax / (M_FP4 * M_FP8);", "const float alpha = amax / M_FP8;"),
    ("amax: block scale without M_FP4", "uint8_t c = soar_oracle_e4m3_project(bmax / alpha_m);", "uint8_t c = soar_oracle_e4m3_project(bmax / alpha);"),
    ("amax: block scale from the supplied maximum", "uint8_t c = soar_oracle_e4m3_project(bmax / alpha_m);", "uint8_t c = soar_oracle_e4m3_project(amax / alpha_m);"),
    ("amax: zero maximum accepted", "if (!isfinite(amax) || !(amax > 0.0f)) {", "if (!isfinite(amax)) {"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0].replace(" ", "_") for m in MUTANTS])
def test_every_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    c_file = tmp_path / "mutant.c"
    so_file = tmp_path / "libmutant.so"
    c_file.write_text(text.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-w",
                    str(c_file), "-o", str(so_file), "-lm"], check=True)
    env = dict(os.environ, SOAR_ORACLE_LIB=str(so_file))
    if name.startswith("iter:"):
        files = ["test_oracle_iter.py"]
    elif name.startswith("mx:"):
        files = ["test_oracle_mxfp4.py"]
    elif name.startswith("arm:"):
        files = ["test_oracle_arms.py"]
    elif name.startswith("amax:"):
        files = ["test_oracle_rtn_amax.py"]
    else:
        files = ["test_oracle_formats.py", "test_oracle_method.py"]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"]
                       + [os.path.join(ROOT, "tests", f) for f in files],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode != 0, f"mutant '{name}' passed every pin:\n{r.stdout[-800:]}"
    assert "failed" in r.stdout or "error" in r.stdout.lower()
