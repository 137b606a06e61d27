"""Do the oracle's pins bite?  Each case plants one plausible mistake in a copy of the oracle's C
source (a dropped term, a wrong sign or index, a transposed layout), builds it, and runs the pin
tests against that build in a child process: the pins must fail.  Everything happens on the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adr_oracle.c")

MUTANTS = {
    "gqa_head_mapping": ("int kvh = h / G;", "int kvh = h % c->Hkv;"),
    "scale_dropped": ("s[t] = scale * dot;", "s[t] = dot;"),
    "slot_off_by_one": ("int slot = t % c->page_size;", "int slot = (t + 1) % c->page_size;"),
    "page_index_rounds_up": ("t / c->page_size]", "(t + c->page_size - 1) / c->page_size]"),
    "softmax_sign": ("s[t] = exp(s[t] - m); /* s now holds w_t */", "s[t] = exp(m - s[t]);"),
    "lse_sign": ("*lse = m + log(Z);", "*lse = m - log(Z);"),
    "not_normalised": ("out[j] /= Z;", "out[j] /= 1.0;"),
    "cache_layout_transposed": ("int64_t idx = (((int64_t)page * c->page_size + slot) * c->Hkv + head) * c->d + j;",
                                "int64_t idx = (((int64_t)page * c->Hkv + head) * c->page_size + slot) * c->d + j;"),
    "v_read_from_k": ("out[j] += s[t] * cache_elem(c->v, c->v_scale, c, page, slot, kvh, j);",
                      "out[j] += s[t] * cache_elem(c->k, c->k_scale, c, page, slot, kvh, j);"),
    "fp8_bias": ("mag = ldexp(1.0 + (double)m / 8.0, e - 7);", "mag = ldexp(1.0 + (double)m / 8.0, e - 8);"),
    "fp8_subnormal_step": ("mag = ldexp((double)m, -9);", "mag = ldexp((double)m, -10);"),
    "fp8_ties_away": ("(err == best_err && (c & 1) == 0)", "(err == best_err && (c & 1) == 1)"),
    "fp8_no_saturation": ("if (x >= 448.0)\n        return (uint8_t)(sign | 0x7E);", "if (x >= 448.0)\n        return (uint8_t)(sign | 0x7F);"),
    "append_wrong_slot": ("slot = pos % page_size;\n        if (page < 0 || page >= num_pages)",
                          "slot = (pos + 1) % page_size;\n        if (page < 0 || page >= num_pages)"),
    "append_fp8_scale_without_headroom": ("scale = amax * (2.0f / 448.0f);", "scale = amax * (1.0f / 448.0f);"),
    "append_fp8_scale_always_reset": ("if (slot == 0) {\n            float amax = 0.0f;", "if (slot >= 0) {\n            float amax = 0.0f;"),
    "merge_weights_by_lse_sign": ("double share = exp(part_lse[(int64_t)p * heads + h] - lse);",
                                  "double share = exp(lse - part_lse[(int64_t)p * heads + h]);"),
    "merge_lse_without_top": ("lse = top + log(total);", "lse = log(total);"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_fail_on_a_planted_mistake(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, "the oracle's source no longer contains the line this case edits"
    c_file = tmp_path / "mutant.c"
    c_file.write_text(text.replace(old, new))
    so = str(tmp_path / "libmutant.so")
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", so, str(c_file), "-lm"])
    env = dict(os.environ, ADR_ORACLE_MUTANT=so)
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert run.returncode != 0, "every pin passed with the mistake '%s' planted in the oracle" % name
    # a pin that failed, or a child that died outright (a mistake in an index can read outside the arrays)
    assert run.returncode < 0 or "failed" in run.stdout or "error" in run.stdout.lower(), run.stdout[-400:]
