"""Do the pins pin?  Each case plants one plausible mistake in a copy of the oracle's C source (a
dropped term, a wrong sign, an off-by-one window, a reversed tie rule, a swapped bit order ...),
builds it, and runs the oracle's pin tests against that copy in a child process: they must fail.
The untouched source, built the same way, must pass.  Everything here runs on the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adacomp_oracle.c")

SELECT, APPLY, WIRE = "tests/test_oracle_select.py", "tests/test_oracle_apply.py", "tests/test_oracle_wire.py"

# name, pin file, [(text in the source, replacement, occurrences)]
# (Dropping the "at least one entry" clamp of the count rule is not listed: the ceiling of a positive
# number is already >= 1, so that copy computes the same function and no pin can or should tell it apart.)
MUTANTS = [
    ("sign_not_cleared", SELECT, [("return f32_bits(x) & 0x7fffffffu;", "return f32_bits(x);", 1),
                                  ("uint64_t inv = 0x7fffffffu - mag_key(g[i]);", "uint64_t inv = 0xffffffffu - mag_key(g[i]);", 1)]),
    ("keeps_the_smallest", SELECT, [("uint64_t inv = 0x7fffffffu - mag_key(g[i]);", "uint64_t inv = mag_key(g[i]);", 1)]),
    ("ties_to_the_higher_index", SELECT, [("order[i] = (inv << 32) | i;", "order[i] = (inv << 32) | (0xffffffffull - i);", 1),
                                          ("idx_out[e] = (uint32_t)(order[e] & 0xffffffffu);",
                                           "idx_out[e] = (uint32_t)(0xffffffffull - (order[e] & 0xffffffffu));", 1)]),
    ("values_lose_their_sign", SELECT, [("val_out[e] = g[idx_out[e]];", "val_out[e] = fabsf(g[idx_out[e]]);", 1)]),
    ("output_not_sorted_by_index", SELECT, [("    qsort(idx_out, k, sizeof *idx_out, cmp_u32);\n", "", 1)]),
    ("count_rounds_down", SELECT, [("double k = ceil(y);", "double k = floor(y);", 1)]),
    ("one_domain_for_the_whole_model", SELECT,
     [("uint64_t k = k_override ? k_override[l] : adacomp_oracle_count(layer_n[l], rate);",
       "uint64_t k = k_override ? k_override[l] : adacomp_oracle_count(layer_n[0], rate); if (k > layer_n[l]) k = layer_n[l];", 1)]),
    ("window_starts_one_late", APPLY, [("for (uint64_t u = j; u < i; ++u)", "for (uint64_t u = j + 1; u < i; ++u)", 1)]),
    ("window_ends_one_early", APPLY, [("for (uint64_t u = j; u < i; ++u)", "for (uint64_t u = j; u + 1 < i; ++u)", 1)]),
    ("transmitted_zeros_count", APPLY, [("if (is_nonzero(val[e])) h->nz[w++] = idx[e];", "h->nz[w++] = idx[e];", 1),
                                        ("                if (is_nonzero(val[e])) {\n                    uint64_t b",
                                         "                {\n                    uint64_t b", 1)]),
    ("divides_by_sigma_plus_one", APPLY, [("if (sigma != 0) a = alpha / (float)sigma;", "a = alpha / (float)(sigma + 1);", 1),
                                          ("if (sigma != 0) a = alpha / (double)sigma;", "a = alpha / (double)(sigma + 1);", 1)]),
    ("step_has_the_wrong_sign", APPLY, [("return theta - p;", "return theta + p;", 2)]),
    ("learning_rate_not_divided", APPLY, [("if (sigma != 0) a = alpha / (float)sigma;", "(void)sigma;", 1),
                                          ("if (sigma != 0) a = alpha / (double)sigma;", "(void)sigma;", 1)]),
    ("global_staleness_off_by_one", APPLY, [("? (i - j)", "? (i - j + 1)", 1)]),
    ("bisection_skips_the_hit", APPLY, [("if (h->nz[mid] < k) lo = mid + 1; else hi = mid;",
                                         "if (h->nz[mid] <= k) lo = mid + 1; else hi = mid;", 1)]),
    ("history_ignores_the_tensor", APPLY, [("uint64_t lo = h->off[l], hi = h->off[l + 1];",
                                            "uint64_t lo = h->off[0], hi = h->off[ps->L];", 1),
                                           ("return lo < h->off[l + 1] && h->nz[lo] == k;",
                                            "return lo < h->off[ps->L] && h->nz[lo] == k;", 1),
                                           ("uint64_t b = ps->base[l] + k;", "uint64_t b = k; (void)l;", 1)]),
    ("update_applied_before_its_staleness_is_read", APPLY,
     [("    if (history_append(ps, layer_off, idx, val)) return -1;\n    ps->t = i + 1;\n", "    ps->t = i + 1;\n", 1),
      ("    const float lr32 = (float)lr;\n", "    if (history_append(ps, layer_off, idx, val)) return -1;\n    const float lr32 = (float)lr;\n", 1),
      ("for (uint64_t u = j; u < i; ++u)", "for (uint64_t u = j; u <= i; ++u)", 1)]),
    ("gap_without_minus_one", WIRE, [("const uint32_t d = idx[e] - idx[e - 1] - 1;", "const uint32_t d = idx[e] - idx[e - 1];", 2),
                                     ("prev += d + 1;", "prev += d;", 1)]),
    ("most_significant_bit_first", WIRE, [("out[pos + p / 32] |= 1u << (p % 32);", "out[pos + p / 32] |= 1u << (31 - p % 32);", 1),
                                          ("(in[pos + p / 32] >> (p % 32)) & 1u", "(in[pos + p / 32] >> (31 - p % 32)) & 1u", 1)]),
    ("one_bit_too_wide", WIRE, [("const uint32_t w = bit_length(largest);", "const uint32_t w = bit_length(largest) + (largest ? 1 : 0);", 1)]),
    ("blocks_of_32", WIRE, [("#define WIRE_BLOCK 64u", "#define WIRE_BLOCK 32u", 1)]),
    ("values_before_deltas_forgotten_total", WIRE, [("out[2] = (uint32_t)(total & 0xffffffffu);", "out[2] = (uint32_t)(blocks);", 1),
                                                    ("const uint64_t total = (uint64_t)in[2] | ((uint64_t)in[3] << 32);",
                                                     "const uint64_t total = layer_off ? ({uint64_t s_ = 0; for (uint32_t l_ = 0; l_ < L; ++l_) s_ += in[4 + l_]; s_;}) : 0;", 1)]),
]


def build_variant(tmp_path, name, edits):
    text = open(SRC).read()
    for old, new, count in edits:
        assert text.count(old) == count, f"{name}: {old!r} occurs {text.count(old)} times, expected {count}"
        text = text.replace(old, new)
    src = tmp_path / f"{name}.c"
    src.write_text(text)
    lib = tmp_path / f"lib{name}.so"
    subprocess.run(["gcc", "-O2", "-std=gnu11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                    str(src), "-lm", "-o", str(lib)], check=True)
    return str(lib)


def run_pins(lib, pin_file):
    env = dict(os.environ, ADACOMP_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", pin_file, "-x", "-q", "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def test_the_untouched_source_passes_its_pins(tmp_path):
    lib = build_variant(tmp_path, "control", [])
    for pin_file in (SELECT, APPLY, WIRE):
        r = run_pins(lib, pin_file)
        assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,pin_file,edits", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_the_pins(tmp_path, name, pin_file, edits):
    lib = build_variant(tmp_path, name, edits)
    r = run_pins(lib, pin_file)
    assert r.returncode != 0, f"no pin noticed the mistake '{name}'"
    assert "passed" not in r.stdout.splitlines()[-1] or "failed" in r.stdout.splitlines()[-1] or "error" in r.stdout.splitlines()[-1]
