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
    ("alpha0 without M_FP4", "amax / (M_FP4 * M_FP8)", "amax / M_FP8"),
    ("block scale without M_FP4", "soar_oracle_e4m3_project(bmax / alpha0_m)", "soar_oracle_e4m3_project(bmax / alpha0)"),
    ("error with wrong sign", "float e = fmaf(-q[j], s, wv[j]);", "float e = fmaf(q[j], s, wv[j]);"),
    ("Eq. 5 denominator with Delta instead of Delta^2",
     "termM[i] = ((double)b * (double)delta0) * (double)delta0;", "termM[i] = (double)b * (double)delta0;"),
    ("Eq. 5 numerator without Delta", "termN[i] = (double)a * (double)delta0;", "termN[i] = (double)a;"),
    ("Eq. 6 multiplied by alpha", "delta_star = (a_all[i] / b_all[i]) / alpha1;", "delta_star = (a_all[i] / b_all[i]) * alpha1;"),
    ("a = sum w^2", "sa = fmaf(wv[j], q[j], sa);", "sa = fmaf(wv[j], wv[j], sa);"),
    ("b = sum |q|", "sb = fmaf(q[j], q[j], sb);", "sb = sb + fabsf(q[j]);"),
    ("later candidate wins ties", "if (err < best_err) { best_err = err; best_code = c; }",
     "if (err <= best_err) { best_err = err; best_code = c; }"),
    ("window one code short", "for (int k = 1; k <= dss_radius; ++k) {", "for (int k = 1; k < dss_radius; ++k) {"),
    ("search only upwards", "for (int sgn = -1; sgn <= 1; sgn += 2) {", "for (int sgn = 1; sgn <= 1; sgn += 2) {"),
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
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_formats.py"),
                        os.path.join(ROOT, "tests", "test_oracle_method.py")],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode != 0, f"mutant '{name}' passed every pin:\n{r.stdout[-800:]}"
    assert "failed" in r.stdout or "error" in r.stdout.lower()
