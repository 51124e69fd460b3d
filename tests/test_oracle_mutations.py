"""Do the pins bite?  Each case plants ONE plausible mistake in a temporary copy of the C oracle
(a transposed operand, a dropped term, a wrong tie, a swapped nibble, an off-by-one exponent ...),
builds it on the CPU and runs the oracle's pin tests against that build in a child process.  The
pins are worth something only if every such build fails at least one of them.  The unmodified
source must pass under the same harness.  Nothing here touches the GPU or the product library.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "torq_oracle.c")
PIN_FILES = ["tests/test_oracle_formats.py", "tests/test_oracle_rotation.py", "tests/test_oracle_gemm.py",
             "tests/test_oracle_intra.py", "tests/test_oracle_other_formats.py",
             "tests/test_oracle_butterfly.py"]

# (name, text in torq_oracle.c, replacement)
MUTATIONS = [
    ("inter_transposed", "R_inter[b * G + bp] * X[(g0 + bp) * BLK + k]", "R_inter[bp * G + b] * X[(g0 + bp) * BLK + k]"),
    ("inter_ignores_group", "R_inter[b * G + bp] * X[(g0 + bp) * BLK + k]", "R_inter[b * G + bp] * X[(bp) * BLK + k]"),
    ("intra_transposed", "Y[b * BLK + kp] * (double)R_intra[kp * BLK + k]", "Y[b * BLK + kp] * (double)R_intra[k * BLK + kp]"),
    ("intra_wrong_block", "Y[b * BLK + kp] * (double)R_intra[kp * BLK + k]", "Y[kp] * (double)R_intra[kp * BLK + k]"),
    ("inter_in_float", "acc += (double)R_inter[b * G + bp] * X[(g0 + bp) * BLK + k];",
     "acc = (float)(acc + (float)(R_inter[b * G + bp] * (float)X[(g0 + bp) * BLK + k]));"),
    ("scale_bias_1", "int byte = field - 2;", "int byte = field - 1;"),
    ("scale_bias_3", "int byte = field - 2;", "int byte = field - 3;"),
    ("scale_no_floor_clamp", "if (byte < 0) byte = 0;", ""),
    ("tie_0.25", "if      (m <= 0.25f) idx = 0;", "if      (m <  0.25f) idx = 0;"),
    ("tie_0.75", "else if (m <  0.75f) idx = 1;", "else if (m <= 0.75f) idx = 1;"),
    ("tie_1.25", "else if (m <= 1.25f) idx = 2;", "else if (m <  1.25f) idx = 2;"),
    ("tie_1.75", "else if (m <  1.75f) idx = 3;", "else if (m <= 1.75f) idx = 3;"),
    ("tie_2.5", "else if (m <= 2.5f)  idx = 4;", "else if (m <  2.5f)  idx = 4;"),
    ("tie_3.5", "else if (m <  3.5f)  idx = 5;", "else if (m <= 3.5f)  idx = 5;"),
    ("tie_5", "else if (m <= 5.0f)  idx = 6;", "else if (m <  5.0f)  idx = 6;"),
    ("codebook_top", "3.0f, 4.0f, 6.0f};", "3.0f, 4.0f, 8.0f};"),
    ("sign_dropped", "uint8_t sign = (uint8_t)((u >> 31) << 3);", "uint8_t sign = (a < 0.0f) ? 8 : 0;"),   # loses -0
    ("amax_without_abs", "float v = fabsf(zr[b * BLK + k]);", "float v = zr[b * BLK + k];"),
    ("normalise_off_by_one", "ldexpf(zr[b * BLK + k], 127 - (int)byte)", "ldexpf(zr[b * BLK + k], 126 - (int)byte)"),
    ("pack_nibbles_swapped", "(uint8_t)(c[2 * j] | (c[2 * j + 1] << 4))", "(uint8_t)(c[2 * j + 1] | (c[2 * j] << 4))"),
    ("dequant_nibbles_swapped", "uint8_t code = (j & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15u);",
     "uint8_t code = (j & 1) ? (uint8_t)(byte & 15u) : (uint8_t)(byte >> 4);"),
    ("dequant_exponent", "int e = (int)scales[m * (int64_t)B + b] - 127;", "int e = (int)scales[m * (int64_t)B + b] - 126;"),
    ("gemm_act_scale_bias", "(int)as[j / BLK] - 127", "(int)as[j / BLK] - 126"),
    ("gemm_weight_scale_index", "(int)ws[j / BLK] - 127", "(int)ws[0] - 127"),
    ("gemm_weight_nibbles_swapped", "uint8_t wc = (j & 1) ? (uint8_t)(wb >> 4) : (uint8_t)(wb & 15u);",
     "uint8_t wc = (j & 1) ? (uint8_t)(wb & 15u) : (uint8_t)(wb >> 4);"),
    ("gemm_in_float", "acc += av * wv;", "acc = (float)(acc + av * wv);"),
    ("gemm_drops_last_block", "for (int j = 0; j < d; ++j) {\n        uint8_t ab", "for (int j = 0; j < d - BLK; ++j) {\n        uint8_t ab"),
    ("bf16_truncates", "uint32_t up = (dropped > 0x8000u) || (dropped == 0x8000u && kept_lsb);", "uint32_t up = 0; (void)kept_lsb; (void)dropped;"),
    ("bf16_ties_away", "(dropped == 0x8000u && kept_lsb)", "(dropped == 0x8000u)"),
    ("gram_ignores_later_runs", "const uint16_t *X = x_bf16 + m * (int64_t)d + (int64_t)g0 * BLK;",
     "const uint16_t *X = x_bf16 + m * (int64_t)d;"),
    ("gram_sum_not_mean", "for (int i = 0; i < G * G; ++i) Sigma[i] /= (double)groups;",
     "for (int i = 0; i < G * G; ++i) Sigma[i] /= (double)M;"),
    ("gram_pos_wrong_position", "(double)torq_o_bf16_to_f32(Xg[bp * BLK + k]);", "(double)torq_o_bf16_to_f32(Xg[bp * BLK + (k ^ 1)]);"),
    ("gram_pos_layout", "Sigma_pos[((int64_t)k * G + b) * G + bp] +=", "Sigma_pos[((int64_t)b * BLK + k) * G + bp] +="),
    ("gram_pos_sum_not_mean", "Sigma_pos[i] /= (double)groups;", "Sigma_pos[i] /= (double)M;"),
    ("gram_pos_ignores_later_runs", "const uint16_t *Xg = x_bf16 + m * (int64_t)d + (int64_t)g0 * BLK;",
     "const uint16_t *Xg = x_bf16 + m * (int64_t)d;"),
    ("gram_wrong_partner", "(double)torq_o_bf16_to_f32(X[bp * BLK + k]);", "(double)torq_o_bf16_to_f32(X[bp * BLK + (k ^ 1)]);"),
    ("equalize_other_root", "const double t = -(a - c) / (g + (g >= 0.0 ? D : -D));", "const double t = -(a - c) / (g - (g >= 0.0 ? D : -D) + 1e-300);"),
    ("equalize_jacobi_angle", "const double t = -(a - c) / (g + (g >= 0.0 ? D : -D));",
     "const double t = tan(0.5 * atan2(2.0 * g, a - b)); (void)D;"),
    ("equalize_R_transposed", "R[i * B + q] = cs * ri + sn * rj;\n            R[j * B + q] = -sn * ri + cs * rj;",
     "R[i * B + q] = cs * ri - sn * rj;\n            R[j * B + q] = sn * ri + cs * rj;"),
    ("hist_counts_sign_bit", "counts[(j % BLK) * 8 + (code & 7u)] += 1;", "counts[(j % BLK) * 8 + ((code >> 1) & 7u)] += 1;"),
    ("hist_position_of_row_not_block", "counts[(j % BLK) * 8 + (code & 7u)] += 1;", "counts[(j % 16) * 8 + (code & 7u)] += 1;"),
    ("loss_not_centred", "double dev = (double)n[j] / total - 1.0 / 8.0;", "double dev = (double)n[j] / total;"),
    ("complementarity_sign", "for (int j = 0; j < 8; ++j) c -= dev[k][j] * dev[l][j];", "for (int j = 0; j < 8; ++j) c += dev[k][j] * dev[l][j];"),
    ("score_drops_partner", "H[k * BLK + l] = h[k] + h[l] + lambda * c;", "H[k * BLK + l] = h[k] + lambda * c;"),
    ("mag_tie_2.5", "if (m <= 2.5) return 4;", "if (m < 2.5) return 4;"),
    ("angle_second_axis_sign", "cnt[torq_o_mag_code(-u[b] * s + v[b] * c)] += 1;", "cnt[torq_o_mag_code(u[b] * s - v[b] * s)] += 1;"),
    ("angle_no_second_axis", "for (int axis = 0; axis < 2; ++axis) {", "for (int axis = 0; axis < 1; ++axis) {"),
    ("angle_no_plus_pi", "const double cand[4] = {base - alpha, base + alpha, base - alpha + PI, base + alpha + PI};",
     "const double cand[4] = {base - alpha, base + alpha, base - alpha, base + alpha};"),
    ("angle_drops_wrap_interval", "for (int64_t i = -1; i + 1 < uniq; ++i) {\n        double mid;", "for (int64_t i = 0; i + 1 < uniq; ++i) {\n        double mid;"),
    ("angle_ignores_rest", "for (int j = 0; j < 8; ++j) cnt[j] = rest[j];", "for (int j = 0; j < 8; ++j) cnt[j] = 0 * rest[j];"),
    ("angle_maximises", "if (!have || key < best_key || (key == best_key && mid < best_theta)) {", "if (!have || key > best_key) {"),
    ("alg2_givens_transposed", "R[i][bp] = rp * c + rq * sn;\n                R[i][bq] = -rp * sn + rq * c;",
     "R[i][bp] = rp * c - rq * sn;\n                R[i][bq] = rp * sn + rq * c;"),
    ("alg2_scale_from_unrotated", "if (fabs(acc) > amax) amax = fabs(acc);", "if (fabs(X[b * BLK + k]) > amax) amax = fabs(X[b * BLK + k]);"),
    ("alg2_pool_least_imbalanced", "if (!in_pool[k] && (arg < 0 || h[k] > h[arg])) arg = k;", "if (!in_pool[k] && (arg < 0 || h[k] < h[arg])) arg = k;"),
    ("alg2_stale_rest", "for (int j = 0; j < 8; ++j) total[j] = rest[j] + counts[bp * 8 + j] + counts[bq * 8 + j];", ""),
    ("e4m3_ties_to_odd", "if (err < best_err || (err == best_err && (c & 1) == 0)) {", "if (err < best_err || (err == best_err && (c & 1) == 1)) {"),
    ("e4m3_bias_8", "ldexpf(1.0f + (float)m / 8.0f, e - 7)", "ldexpf(1.0f + (float)m / 8.0f, e - 8)"),
    ("e4m3_allows_nan_code", "for (int c = 1; c <= 0x7E; ++c) {", "for (int c = 1; c <= 0x7F; ++c) {"),
    ("mxint4_allows_minus_8", "if (r < -7.0f) r = -7.0f;", "if (r < -8.0f) r = -8.0f;"),
    ("mxint4_truncates", "float r = rintf(ldexpf(zb[k], 127 - (int)byte));", "float r = truncf(ldexpf(zb[k], 127 - (int)byte));"),
    ("mxint4_rounds_half_away", "float r = rintf(ldexpf(zb[k], 127 - (int)byte));", "float r = roundf(ldexpf(zb[k], 127 - (int)byte));"),
    ("nvfp4_scale_to_amax", "const float D = 6.0f * global_scale;", "const float D = 1.0f * global_scale;"),
    ("nvfp4_ignores_global_scale_in_S", "const float S = torq_o_e4m3_value(q) * global_scale;", "const float S = torq_o_e4m3_value(q);"),
    ("nvfp4_dequant_block_of_32", "(torq_o_e4m3_value(scales_e4m3[j / 16]) * global_scale)", "(torq_o_e4m3_value(scales_e4m3[j / 32]) * global_scale)"),
    ("butterfly_angle_sign", "if (g != 0.0) theta = 0.5 * atan((b - a) / (2.0 * g));", "if (g != 0.0) theta = 0.5 * atan((a - b) / (2.0 * g));"),
    ("butterfly_jacobi_angle", "if (g != 0.0) theta = 0.5 * atan((b - a) / (2.0 * g));", "if (g != 0.0) theta = 0.5 * atan(2.0 * g / (a - b + 1e-300));"),
    ("butterfly_wrong_partner", "const int q = p + h;\n            const double a = Sigma[p * B + p], b = Sigma[q * B + q], g = Sigma[p * B + q];\n            double theta;",
     "const int q = p + h;\n            const double a = Sigma[p * B + p], b = Sigma[q * B + q], g = Sigma[q * B + p ^ 1];\n            double theta;"),
    ("butterfly_R_transposed", "R[p * B + k] = cs * rp + sn * rq;\n                R[q * B + k] = -sn * rp + cs * rq;",
     "R[p * B + k] = cs * rp - sn * rq;\n                R[q * B + k] = sn * rp + cs * rq;"),
    ("butterfly_skips_last_round", "for (int h = B / 2; h >= 1; h /= 2, ++round) {", "for (int h = B / 2; h >= 2; h /= 2, ++round) {"),
]


def _build(tmp_path, name, text):
    src = tmp_path / f"{name}.c"
    src.write_text(text)
    lib = tmp_path / f"lib{name}.so"
    subprocess.run(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                    f"-I{os.path.join(ROOT, 'oracle')}", "-o", str(lib), str(src), "-lm"], check=True)
    return str(lib)


def _run_pins(lib):
    env = dict(os.environ, TORQ_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                           *PIN_FILES], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Build every mutant (and the unmodified source) and run the pins against each, four child
    processes at a time: the runs are independent and mostly wait on the interpreter start-up."""
    from concurrent.futures import ThreadPoolExecutor
    tmp = tmp_path_factory.mktemp("mutants")
    text = open(SRC).read()
    jobs = [("clean", text)]
    for name, old, new in MUTATIONS:
        jobs.append((name, text.replace(old, new) if text.count(old) >= 1 else None))

    def one(job):
        name, src = job
        if src is None:
            return name, None
        return name, _run_pins(_build(tmp, name, src))

    with ThreadPoolExecutor(max_workers=4) as pool:
        return dict(pool.map(one, jobs))


def test_unmodified_oracle_passes_under_the_same_harness(outcomes):
    r = outcomes["clean"]
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(outcomes, name, old, new):
    r = outcomes[name]
    assert r is not None, f"mutation target not found in torq_oracle.c: {old!r}"
    assert r.returncode == 1, f"no pin noticed '{name}' (pytest exit {r.returncode}):\n{r.stdout[-1500:]}"
    assert " failed" in r.stdout
