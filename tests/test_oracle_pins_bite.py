"""The oracle's pins are only worth something if a plausible mistake fails them.  Each case
plants one mistake in a COPY of the oracle's source (on the CPU, in a temp dir), builds it,
and runs the pin tests against that build in a subprocess: they must fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "dssd_oracle.cpp")

MUTATIONS = {
    "ratio_inverted": ("return (r * q < p) ? 1 : 0;", "return (r * p < q) ? 1 : 0;"),
    "residual_sign": ("const double d = P[v] - (double)Q[v];", "const double d = (double)Q[v] - P[v];"),
    "residual_uses_accept_word": ("const double r2 = dssd_oracle_u01(words[1]);",
                                  "const double r2 = dssd_oracle_u01(words[0]);"),
    "bonus_uses_residual_word": ("dssd_oracle_u01(words[2]), &res->cdf_margin);\n  }\n}",
                                 "dssd_oracle_u01(words[1]), &res->cdf_margin);\n  }\n}"),
    "edge_bonus_uses_residual_word": ("dssd_oracle_u01(words[2]), &res->cdf_margin);\n      return;",
                                      "dssd_oracle_u01(words[1]), &res->cdf_margin);\n      return;"),
    "device_uses_accept_word": ("const double r = dssd_oracle_u01(words[1]);\n  if (resid_mass)",
                                "const double r = dssd_oracle_u01(words[0]);\n  if (resid_mass)"),
    "half_truncates": ("if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) ++half;", ";"),
    "half_ties_away": ("if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) ++half;",
                       "if (rem >= 0x1000u) ++half;"),
    "edge_exports_wrong_row": ("      dssd_oracle_quantize_p_row(P.data(), V, p_dtype, p_row_out);\n      return;",
                               "      if (i > 0) dssd_oracle_softmax_row((const char*)logits, dtype, V, inv_temperature, P.data(), &m, &Z);\n"
                               "      dssd_oracle_quantize_p_row(P.data(), V, p_dtype, p_row_out);\n      return;"),
    "cdf_not_strict": ("if (upto > t) {", "if (upto >= t) {"),
    "temperature_dropped": ("const double e = std::exp(logit_at(logits_row, dtype, v) * inv_temperature - m);",
                            "const double e = std::exp(logit_at(logits_row, dtype, v) - m);"),
    "philox_multipliers_swapped": ("const uint64_t prod_a = mult_a * (uint64_t)c0;",
                                   "const uint64_t prod_a = mult_b * (uint64_t)c0;"),
    "philox_nine_rounds": ("for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {"),
    "u01_uses_low_bits": ("return (double)(w >> 8) * (1.0 / 16777216.0);",
                          "return (double)(w & 0xFFFFFF) * (1.0 / 16777216.0);"),
    "bonus_row_off_by_one": ("if (i == gamma) break;", "if (i == gamma - 1 && gamma > 1) break;"),
    "margin_sign_kept": ("const double gap = std::fabs(r * q - p);", "const double gap = r * q - p;"),
    "margin_divides_by_p": ("return q > 0.0 ? gap / q :", "return q > 0.0 ? gap / p :"),
    "margin_counts_positions_after_the_rejection": ("    if (!open) continue;\n", ""),
    "bad_token_never_reported": ("    if (!in_vocabulary) {  // malformed input met by the loop: report, emit nothing\n      open = false;",
                                 "    if (false) {\n      open = false;"),
    "stops_one_late": ("open = false;  // Flag = 0\n      res->n = i;",
                       "open = false;  // Flag = 0\n      res->n = i + 1 < gamma ? i + 1 : i;"),
}

PIN_TESTS = ["tests/test_oracle_philox.py", "tests/test_oracle_softmax.py", "tests/test_oracle_accept_cdf.py",
             "tests/test_oracle_law.py", "tests/test_oracle_split.py"]


def _run_pins(lib):
    env = dict(os.environ, DSSD_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           "-k", "not monte_carlo and not table1", *PIN_TESTS],
                          cwd=ROOT, env=env, capture_output=True, text=True)


def _build(src_text, out):
    cpp = out + ".cpp"
    with open(cpp, "w") as f:
        f.write(src_text)
    subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-o", out, cpp], check=True)
    return out


def test_unmodified_copy_passes(tmp_path):
    lib = _build(open(SRC).read(), str(tmp_path / "liborc_ok.so"))
    r = _run_pins(lib)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_fails_a_pin(tmp_path, name):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor for {name} not unique"
    lib = _build(text.replace(old, new), str(tmp_path / f"liborc_{name}.so"))
    r = _run_pins(lib)
    assert r.returncode != 0, f"no pin noticed the planted mistake '{name}'"
