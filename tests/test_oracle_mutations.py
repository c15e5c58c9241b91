"""Are the oracle's pins sharp?  Each case plants ONE plausible mistake in a copy of
the oracle's C source (a dropped term, a wrong sign or index, a transposed operand,
a shifted coordinate convention), rebuilds it and runs the CPU pins against the
broken copy in a child process: at least one pin must fail.  The unmodified copy
must pass.  Everything here runs on the CPU; the product never sees these copies."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sr_oracle.c")
PINS = ["tests/test_oracle_bicubic.py", "tests/test_oracle_assemble.py", "tests/test_oracle_fp8.py",
        "tests/test_oracle_shuffle.py", "tests/test_oracle_topk.py", "tests/test_oracle_pixel_major.py",
        "tests/test_oracle_logits.py", "tests/test_oracle_blocked.py"]

MUTATIONS = {
    "keys_inner_coefficient": ("- (a + 3.0) * t * t + 1.0", "- (a + 2.0) * t * t + 1.0"),
    "keys_outer_coefficient": ("- 5.0 * a * t * t", "- 4.0 * a * t * t"),
    "keys_outer_support": ("if (t < 2.0)", "if (t < 1.5)"),
    "no_half_pixel_centres": ("((double)Y + 0.5) / (double)s - 0.5", "(double)Y / (double)s"),
    "first_tap_off_by_one": ("*first = (long)fl - 1;", "*first = (long)fl;"),
    "inner_tap_weights_swapped": ("w[1] = orc_keys(t, a);\n    w[2] = orc_keys(1.0 - t, a);",
                                  "w[1] = orc_keys(1.0 - t, a);\n    w[2] = orc_keys(t, a);"),
    "upsampler_axes_transposed": ("acc += wy[i] * wx[j] * load_elem", "acc += wy[j] * wx[i] * load_elem"),
    "lr_column_clamped_to_height": ("clampl(fx + j, 0, w - 1)", "clampl(fx + j, 0, h - 1)"),
    "lr_border_not_replicated": ("long yy = clampl(fy + i, 0, h - 1);", "long yy = clampl(fy + i, 1, h - 1);"),
    "kept_position_instead_of_atom": ("F[j] += phi * dict[(size_t)l * kk + j];", "F[j] += phi * dict[(size_t)i * kk + j];"),
    "dictionary_rounded_to_half": (
        "F[j] += phi * dict[(size_t)l * kk + j];",
        "{ int e2; double m2 = frexp((double)dict[(size_t)l * kk + j], &e2); F[j] += phi * ldexp(nearbyint(ldexp(m2, 11)), e2 - 11); }"),
    "gamma_dropped": ("        if (gamma)\n            phi *= gamma[i];", "        (void)gamma;"),
    "filter_transposed": ("acc += F[dy * k + dx] * Uplane", "acc += F[dx * k + dy] * Uplane"),
    "filter_flipped": ("clampl(Y + dy - r, 0, H - 1)", "clampl(Y - dy + r, 0, H - 1)"),
    "patch_not_centred": ("int r = (k - 1) / 2;", "int r = k / 2 - 1;"),
    "hr_border_zero_instead_of_replicate": (
        "acc += F[dy * k + dx] * Uplane[(size_t)yy * W + xx];",
        "if (Y + dy - r == yy && X + dx - r == xx) acc += F[dy * k + dx] * Uplane[(size_t)yy * W + xx];"),
    "same_channel_for_all": ("apply_pixel(U + ((size_t)b * c + ch) * plane, H, W, Y, X, F, k);\n            }",
                             "apply_pixel(U + ((size_t)b * c) * plane, H, W, Y, X, F, k);\n            }"),
    "batch_stride_of_coefficients": ("size_t pix = (size_t)b * L * plane + (size_t)Y * W + X;\n                fold_pixel",
                                     "size_t pix = (size_t)b * plane + (size_t)Y * W + X;\n                fold_pixel"),
    "pixel_major_read_as_planar": ("size_t from = (((size_t)b * H + y) * W + x) * L + l;", "size_t from = (((size_t)b * L + l) * H + y) * W + x;"),
    "pixel_major_rows_and_columns_swapped": ("size_t from = (((size_t)b * H + y) * W + x) * L + l;", "size_t from = (((size_t)b * W + x) * H + y) * L + l;"),
    "shuffle_sub_pixels_column_major": ("size_t from = ((((size_t)b * L + l) * s + i) * s + j)", "size_t from = ((((size_t)b * L + l) * s + j) * s + i)"),
    "shuffle_atoms_interleaved": ("size_t from = ((((size_t)b * L + l) * s + i) * s + j)", "size_t from = ((((size_t)b * s + i) * s + j) * L + l)"),
    "shuffle_lands_on_lr_rows": ("((size_t)y * s + i) * W + ((size_t)x * s + j)", "((size_t)i * h + y) * W + ((size_t)x * s + j)"),
    "list_entry_stride_of_the_dense_form": ("size_t at = ((size_t)b * T + t) * plane + (size_t)Y * W + X;",
                                            "size_t at = ((size_t)b * L + t) * plane + (size_t)Y * W + X;"),
    "list_index_used_as_position": ("F[j] += v * dict[(size_t)l * kk + j];", "F[j] += v * dict[(size_t)t * kk + j];"),
    "list_keeps_last_entry_only": ("                    for (int j = 0; j < kk; ++j)\n                        F[j] += v * dict[(size_t)l * kk + j];",
                                   "                    for (int j = 0; j < kk; ++j)\n                        F[j] = v * dict[(size_t)l * kk + j];"),
    "blocked_slot_is_the_pixel_quarter": ("int unit = x / 128, j = (x % 128) / 4, q = x % 4;", "int unit = x / 128, j = (x % 128) % 32, q = (x % 128) / 32;"),
    "blocked_halves_after_the_pixels": ("within = (size_t)piece * 512 + (size_t)half * 256 + (size_t)j * 8 + e;",
                                        "within = (size_t)piece * 512 + (size_t)j * 16 + (size_t)half * 8 + e;"),
    "blocked_last_piece_as_a_full_one": ("within = (size_t)full * 512 + (size_t)half * 128 + (size_t)j * 4 + e;",
                                         "within = (size_t)full * 512 + (size_t)half * 256 + (size_t)j * 8 + e;"),
    "blocked_slots_before_units": ("size_t from = ((((size_t)b * H + y) * (W / 128) + unit) * 4 + q) * slot_elems + within;",
                                   "size_t from = ((((size_t)b * H + y) * 4 + q) * (W / 128) + unit) * slot_elems + within;"),
    "logits_maximum_not_subtracted": ("double e = exp(load_elem(in, dtype, base + (size_t)l * plane) - m);",
                                      "double e = exp(load_elem(in, dtype, base + (size_t)l * plane));"),
    "logits_exponentials_not_rounded": ("                if (round_half)\n                    e = orc_round_to_half(e);", "                (void)round_half;"),
    "logits_rounded_after_the_division": (
        "                out[base + (size_t)l * plane] /= sum;",
        "                out[base + (size_t)l * plane] = round_half ? orc_round_to_half(out[base + (size_t)l * plane] / sum) : out[base + (size_t)l * plane] / sum;"),
    "logits_sum_of_unrounded_exponentials": (
        "                out[base + (size_t)l * plane] = e;\n                sum += e;",
        "                sum += exp(load_elem(in, dtype, base + (size_t)l * plane) - m);\n                out[base + (size_t)l * plane] = e;"),
    "logits_normalised_over_the_row": ("double z = load_elem(in, dtype, base + (size_t)l * plane);\n                if (z > m)",
                                       "double z = load_elem(in, dtype, base + (size_t)l);\n                if (z > m)"),
    "logits_base_two": ("double e = exp(load_elem(in, dtype, base + (size_t)l * plane) - m);",
                        "double e = exp2(load_elem(in, dtype, base + (size_t)l * plane) - m);"),
    "half_rounding_truncates": ("return ldexp(nearbyint(ldexp(v, -ulp_exp)), ulp_exp);", "return ldexp(trunc(ldexp(v, -ulp_exp)), ulp_exp);"),
    "half_rounding_ties_away": ("return ldexp(nearbyint(ldexp(v, -ulp_exp)), ulp_exp);", "return ldexp(round(ldexp(v, -ulp_exp)), ulp_exp);"),
    "half_rounding_ten_bits": ("int ulp_exp = e - 11;                         /* 11 significant bits */", "int ulp_exp = e - 10;"),
    "half_rounding_no_subnormals": ("        ulp_exp = -24;                            /* subnormal range: fixed spacing */", "        ulp_exp = e - 11;"),
    "half_subnormal_exponent": ("v = ldexp((double)m, -24);", "v = ldexp((double)m, -25);"),
    "e4m3_bias": ("v = ldexp((double)(m + 8), e - 10);", "v = ldexp((double)(m + 8), e - 11);"),
    "e4m3_subnormals_flushed": ("v = ldexp((double)m, -9);", "v = 0.0;"),
    "e4m3_has_infinities": ("if (e == 15 && m == 7)", "if (e == 15)"),
}


def _run_pins(src_text, workdir, tag):
    src = os.path.join(workdir, f"oracle_{tag}.c")
    with open(src, "w") as f:
        f.write(src_text)
    lib = os.path.join(workdir, f"liboracle_{tag}.so")
    # the broken copy must still be valid C: a copy that does not compile proves nothing
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                           "-o", lib, src, "-lm"])
    env = dict(os.environ, SR_ORACLE_SRC=src, SR_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS],
                         cwd=ROOT, env=env, capture_output=True, text=True)
    return res.returncode, res.stdout[-1500:]


def test_every_planted_mistake_is_caught(tmp_path):
    text = open(SRC).read()
    for name, (old, new) in MUTATIONS.items():
        assert text.count(old) == 1, f"{name}: the source line to break was not found exactly once"
    rc, tail = _run_pins(text, str(tmp_path), "control")
    assert rc == 0, "the unmodified copy must pass its pins:\n" + tail

    def attempt(item):
        name, (old, new) = item
        rc, tail = _run_pins(text.replace(old, new), str(tmp_path), name)
        return name, rc

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(attempt, MUTATIONS.items()))
    survivors = [name for name, rc in results if rc == 0]
    assert not survivors, f"no pin noticed these planted mistakes: {survivors}"
    # exit status 1 = some test FAILED; anything else (collection error, crash) is not a catch
    odd = [(name, rc) for name, rc in results if rc != 1]
    assert not odd, f"these runs did not end in an ordinary test failure: {odd}"


SELECT_SRC = os.path.join(ROOT, "oracle", "select_oracle.py")
SELECT_MUTATIONS = {
    "threshold_not_halved": ("thr = 0.5 * lam * M", "thr = lam * M"),
    "soft_threshold_sign": ("(rho + thr if rho < -thr else 0.0)", "(rho - thr if rho < -thr else 0.0)"),
    "own_term_not_excluded": ("rho = b[j] - (G[j] @ beta - G[j, j] * beta[j])", "rho = b[j] - G[j] @ beta"),
    "responses_without_coefficient": ("R *= np.moveaxis(phi, 1, -1)[:, None]", "R *= 1.0"),
    "atom_transposed": ("R += tap[..., None] * D[:, dy, dx]", "R += tap[..., None] * D[:, dx, dy]"),
    "zero_padding": ('mode="edge"', 'mode="constant"'),
    "lattice_offset": ("ys, xs = np.arange(0, H, stride), np.arange(0, W, stride)",
                       "ys, xs = np.arange(stride - 1, H, stride), np.arange(stride - 1, W, stride)"),
    "target_term_abs": ("return R.T @ R, R.T @ h, float(h @ h), R.shape[0]", "return R.T @ R, R.T @ np.abs(h), float(h @ h), R.shape[0]"),
    "gamma_not_accumulated": ("        gamma_tot[S] *= gam\n", "        pass\n"),
    "right_side_not_rescaled": ("        b[S] *= gam\n", "        pass\n"),
    "keeps_fewer_than_allowed": ("        while cnt > want:\n", "        while cnt >= want:\n"),
    "regression_on_all_atoms": ("Gs, bs = np.asarray(G, dtype=np.float64)[np.ix_(S, S)], np.asarray(b, dtype=np.float64)[S]",
                                "Gs, bs = np.asarray(G, dtype=np.float64)[np.ix_(S, S)], np.asarray(b, dtype=np.float64)[S] * 0.5"),
}


def test_every_planted_mistake_in_the_selection_oracle_is_caught(tmp_path):
    text = open(SELECT_SRC).read()
    for name, (old, new) in SELECT_MUTATIONS.items():
        assert text.count(old) == 1, f"{name}: the source line to break was not found exactly once"

    def run(tag, body):
        src = os.path.join(str(tmp_path), f"select_{tag}.py")
        with open(src, "w") as f:
            f.write(body)
        compile(body, src, "exec")                       # a copy that is not valid Python proves nothing
        env = dict(os.environ, SR_SELECT_ORACLE_SRC=src, OMP_NUM_THREADS="2")
        res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                              "tests/test_oracle_select.py"], cwd=ROOT, env=env, capture_output=True, text=True)
        return tag, res.returncode

    assert run("control", text)[1] == 0, "the unmodified copy must pass its pins"
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda kv: run(kv[0], text.replace(*kv[1])), SELECT_MUTATIONS.items()))
    survivors = [name for name, rc in results if rc == 0]
    assert not survivors, f"no pin noticed these planted mistakes: {survivors}"
    odd = [(name, rc) for name, rc in results if rc != 1]
    assert not odd, f"these runs did not end in an ordinary test failure: {odd}"
