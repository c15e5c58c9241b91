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
PINS = ["tests/test_oracle_bicubic.py", "tests/test_oracle_assemble.py", "tests/test_oracle_fp8.py"]

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
