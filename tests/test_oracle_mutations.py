"""Shows that the oracle's pins have teeth: a plausible mistake planted in a *copy* of the
oracle's C source (dropped term, wrong sign or index, swapped operand) must make the pin
suite fail.  The mutants are built and exercised on the CPU only."""
import os
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SRC = (ROOT / "oracle" / "lookm_oracle.c").read_text()

PIN_FILES = ["tests/test_oracle_scores.py", "tests/test_oracle_select.py", "tests/test_oracle_nearest.py",
             "tests/test_oracle_merge.py", "tests/test_oracle_end_to_end.py", "tests/test_oracle_decode.py"]

# (name, text to find, replacement) - each must occur exactly once in the source
MUTANTS = [
    ("no_scale", "s[j] = dot / root_d;", "s[j] = dot;"),
    ("strict_causal", "for (int j = 0; j <= i; ++j) {\n            double dot = 0.0;",
     "for (int j = 0; j <= i; ++j) {\n            if (j == i && i > 0) { s[j] = -INFINITY; continue; }\n            double dot = 0.0;"),
    ("qk_swapped", "dot += (double)q[(size_t)i * d + c] * (double)k[(size_t)j * d + c];",
     "dot += (double)q[(size_t)j * d + c] * (double)k[(size_t)i * d + c];"),
    ("unnormalised_rows", "scores[j] += s[j] / z;", "scores[j] += s[j];"),
    ("lse_without_max_shift", "lse[i] = top + log(z);", "lse[i] = log(z);"),
    ("lse_without_scale", "t[j] = acc * inv_root_d;", "t[j] = acc;"),
    ("tie_to_higher_position", "return (x->pos > y->pos) - (x->pos < y->pos); /* tie", "return (x->pos < y->pos) - (x->pos > y->pos); /* tie"),
    ("lowest_scores_kept", "if (x->key > y->key) return -1;   /* higher score first */\n    if (x->key < y->key) return 1;",
     "if (x->key > y->key) return 1;\n    if (x->key < y->key) return -1;"),
    ("no_text_prior", "c[j].key = (mask[j] == 0) ? scores[j] + t_p : scores[j];", "c[j].key = scores[j];"),
    ("window_off_by_one", "const int head = L - M;             /* A_s[:-M] */", "const int head = L - M - (M > 0);"),
    ("dot_not_cosine", "return dot_seq(a, b, d) / (sqrt(na) * sqrt(nb));", "return dot_seq(a, b, d) / sqrt(na);"),
    ("argmin", "if (best < 0 || s > best_s) { best = r; best_s = s; }", "if (best < 0 || s < best_s) { best = r; best_s = s; }"),
    ("last_max_wins", "if (best < 0 || s > best_s) { best = r; best_s = s; }", "if (best < 0 || s >= best_s) { best = r; best_s = s; }"),
    ("divide_by_n", "else o[c] = ((double)xc[c] + o[c]) / (double)(n + 1);", "else o[c] = ((double)xc[c] + o[c]) / (double)(n);"),
    ("pivotal_without_half", "o[c] = ((double)xc[c] + 0.5 * o[c]) / (double)(n + 1);", "o[c] = ((double)xc[c] + o[c]) / (double)(n + 1);"),
    ("pivotal_drops_closest", "else if (mode == 2) o[c] += ((double)xe[c] + (double)xc[c]);", "else if (mode == 2) o[c] += ((double)xe[c]);"),
    ("weighted_ignores_similarity", "else o[c] += (double)xe[c] * sim[e];", "else o[c] += (double)xe[c];"),
    ("literal_rule_refuses_small_budgets", "if (rule == 0 && B < oracle_protected_count(mask, L, M)) return ORACLE_ERR_BUDGET_BELOW_PROTECTED;",
     "if (B < oracle_protected_count(mask, L, M)) return ORACLE_ERR_BUDGET_BELOW_PROTECTED;"),
    ("ratio_truncates", "const int N = (int)floor(alpha_important * (double)L + 0.5);", "const int N = (int)floor(alpha_important * (double)L);"),
    ("window_one_row_short", "scores_from_row(q, k, L, d, L - window, scores);", "scores_from_row(q, k, L, d, L - window + 1, scores);"),
    ("decode_without_scale", "p[r] = dot / root_dim;", "p[r] = dot;"),
    ("decode_unnormalised", "out[c] += (p[r] / total) * (double)v[(size_t)r * d + c];", "out[c] += p[r] * (double)v[(size_t)r * d + c];"),
    ("group_reads_wrong_key_head", "scores_from_row(q + ((size_t)kh * group + m) * L * d, k + (size_t)kh * L * d, L, d, 0, one);",
     "scores_from_row(q + ((size_t)kh * group + m) * L * d, k + (size_t)m * L * d, L, d, 0, one);"),
    ("values_not_merged", "r = oracle_merge_head(vh, d, kp, B, ev, Le, as, sm, mode, v_out", "r = oracle_merge_head(vh, d, kp, B, ev, Le, as, sm, 0, v_out"),
]


def test_every_mutation_site_exists_once():
    for name, old, _ in MUTANTS:
        assert SRC.count(old) == 1, name


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(SRC.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", str(src), "-o", str(lib), "-lm"])
    env = dict(os.environ, LOOKM_ORACLE_LIB=str(lib))
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    assert p.returncode == 1, f"mutant {name} survived the pins:\n{p.stdout[-800:]}"
