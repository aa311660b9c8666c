"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source (a dropped term, a
wrong sign or index, a strict instead of an inclusive comparison, an update in the wrong order), builds it beside
the real one and runs the pin suite against it in a child process: at least one pin must fail.  CPU only; the
real oracle is never touched."""
import os
import subprocess
import sys

import pytest

from oracle import subgen_oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "subgen_oracle.c")

# (what is planted, text to find, replacement, pins expected to catch it: a -k expression that keeps the run short)
MUTANTS = [
    ("argmin ties go to the newer representative", "if (acc < best) { second", "if (acc <= best) { second",
     "ties_go_to_lowest_index or brute_force"),
    ("threshold test strict instead of inclusive", "if (arg >= 0 && best <= thr) {", "if (arg >= 0 && best < thr) {",
     "threshold_is_inclusive or hand_built_line"),
    ("mu bumped before the coin probability is taken", "    float p;\n    if (o->mu == 0.0)",
     "    o->mu += (double)vn;\n    float p;\n    if (o->mu == 0.0)", "second_token_probability or mu_and_first_token"),
    ("importance weight without the 1/s", "o->mu / ((double)o->s * vn)", "o->mu / (vn)", "unbiased or identical_values"),
    ("normaliser ignores the cluster counts", "den += (double)o->cnt[i] * exp", "den += exp",
     "delta_zero_denominator or identical_keys"),
    ("window terms missing from the normaliser", "        den += e;\n", "\n", "window_only_equals_textbook"),
    ("coin takes the neighbouring word of the block", "return (float)(r[slot % 4u] >> 8) * (1.0f / 16777216.0f);\n}\n\n/* Coins of",
     "return (float)(r[(slot + 1u) % 4u] >> 8) * (1.0f / 16777216.0f);\n}\n\n/* Coins of", "uniform24_counter_layout"),
    ("ring evicts the wrong slot", "const int slot = (int)(i % o->w);", "const int slot = (int)((i + 1) % o->w);",
     "lemma2_invariants or window_only or query_sees"),
    ("sampling weight from the key norm", "for (int c = 0; c < d; ++c) acc += (double)v[c] * (double)v[c];\n    const float vn",
     "for (int c = 0; c < d; ++c) acc += (double)k[c] * (double)k[c];\n    const float vn", "lemma1_sampling or mu_and_first"),
    ("sampled score uses the value row", "double e = wgt * exp(dotd(q, o->Mk", "double e = wgt * exp(dotd(q, o->Mv",
     "unbiased or identical_values or single_token"),
    ("distance is a sum of absolute differences", "acc += df * df;", "acc += fabs(df);", "brute_force or hand_built_line"),
    ("a join moves the representative", "        o->cnt[arg] += 1;\n        reservoir_update(o, arg, token, k);\n        log_decision(o, arg, 0, best, second);\n    } else if",
     "        o->cnt[arg] += 1; memcpy(o->X + (size_t)arg * d, k, d * sizeof(float));\n        reservoir_update(o, arg, token, k);\n        log_decision(o, arg, 0, best, second);\n    } else if",
     "brute_force or lemma2_invariants"),
    ("coin probability ignores mu", "p = (float)((double)vn / (o->mu + (double)vn));", "p = (float)((double)vn / (1.0 + (double)vn));",
     "lemma1_sampling or second_token_probability"),
    ("runner-up distance never recorded", "else if (acc < second) { second = acc; }", "else if (acc < second) { }",
     "hand_built_line or margins_flag"),
    ("forced decision applied one token late", "if (o->ov_token[e] != token) continue;", "if (o->ov_token[e] + 1 != token) continue;",
     "forced_decisions"),
    ("query answered before the update", "        sgo_update(o, K + (size_t)t * o->d, V + (size_t)t * o->d);\n        for (int h = 0; h < g; ++h) {\n            int rc = sgo_attend(o, Q + ((size_t)t * g + h) * o->d, out + ((size_t)t * g + h) * o->d, NULL, NULL);\n            if (rc) return rc;\n        }\n",
     "        for (int h = 0; h < g; ++h) {\n            int rc = o->n_seen ? sgo_attend(o, Q + ((size_t)t * g + h) * o->d, out + ((size_t)t * g + h) * o->d, NULL, NULL) : 0;\n            if (rc) return rc;\n        }\n        sgo_update(o, K + (size_t)t * o->d, V + (size_t)t * o->d);\n",
     "query_sees_the_token or ingest_and_decode_are_loops"),
]


@pytest.mark.parametrize("what,old,new,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, what, old, new, pins):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation anchor not unique: {old!r}"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", *subgen_oracle.GCC_FLAGS, "-o", str(lib), str(mutated), "-lm"])
    env = dict(os.environ, SUBGEN_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider", "-k", pins], env=env, cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1 and " failed" in r.stdout, f"{what}: no pin failed\n{r.stdout[-1500:]}"
