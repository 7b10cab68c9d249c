"""Do the pins notice a mistake?  Each case plants one plausible error in a COPY of the oracle's C source (a dropped
term, a flipped comparison, a transposed index, a wrong bit order, ...), builds it, and runs the pin tests against that
build in a child process: at least one pin has to fail.  A planted mistake that goes unnoticed means a pin is missing.

CPU only; the mistakes live in the oracle copy, never in the GPU code."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "plaid_oracle.c")

# name, text in plaid_oracle.c, its replacement, how often the text occurs
MISTAKES = [
    ("scq_drops_the_last_dimension",
     "for (int32_t t = 0; t < dim; ++t)\n                acc += (double)centroids",
     "for (int32_t t = 0; t < dim - 1; ++t)\n                acc += (double)centroids", 1),
    ("scq_stored_transposed", "S[c * qlen + i] = (float)acc;", "S[i * C + c] = (float)acc;", 1),
    ("ranking_prefers_the_larger_id",
     "if (x->id < y->id) return -1;\n    if (x->id > y->id) return 1;",
     "if (x->id < y->id) return 1;\n    if (x->id > y->id) return -1;", 1),
    ("ranking_ascending_in_score",
     "if (x->score > y->score) return -1;\n    if (x->score < y->score) return 1;",
     "if (x->score > y->score) return 1;\n    if (x->score < y->score) return -1;", 1),
    ("threshold_strict", "keep[c] = (m >= t_cs) ? 1 : 0;", "keep[c] = (m > t_cs) ? 1 : 0;", 1),
    ("threshold_looks_at_one_token", "for (int32_t i = 1; i < qlen; ++i)\n            if (S[c * qlen + i] > m)",
     "for (int32_t i = 1; i < 1; ++i)\n            if (S[c * qlen + i] > m)", 1),
    ("interaction_maximum_starts_at_zero", "for (int32_t i = 0; i < qlen; ++i) mx[i] = -INFINITY;",
     "for (int32_t i = 0; i < qlen; ++i) mx[i] = 0.0f;", 1),
    ("interaction_ignores_the_pruning_map", "if (keep && !keep[c]) continue;", ";", 1),
    ("interaction_empty_bag_scores_zero", "if (!any) {\n            scores[a] = -INFINITY;", "if (!any) {\n            scores[a] = 0.0f;", 1),
    ("interaction_sums_over_tokens",
     "if (S[(int64_t)c * qlen + i] > mx[i]) mx[i] = S[(int64_t)c * qlen + i];",
     "mx[i] = (mx[i] == -INFINITY ? 0.0f : mx[i]) + S[(int64_t)c * qlen + i];", 1),
    ("byte_table_least_significant_first", "(v >> (nbits * (per - 1 - t)))", "(v >> (nbits * t))", 1),
    ("decompress_subtracts_the_weight", "= cen[x] + ix->bucket_weights[b];", "= cen[x] - ix->bucket_weights[b];", 1),
    ("encode_cutoff_goes_to_the_upper_bucket", "if (cutoffs[q] < r) ++b;", "if (cutoffs[q] <= r) ++b;", 1),
    ("encode_packs_least_significant_first", "byte = (byte << nbits) | b;", "byte = byte | (b << (nbits * t));", 1),
    ("inverted_lists_keep_duplicates", "if (last[c] != p) {", "if (1) {", 2),
    ("candidates_miss_the_last_entry_of_a_list",
     "for (int64_t e = ivf_offsets[c]; e < ivf_offsets[c + 1]; ++e)",
     "for (int64_t e = ivf_offsets[c]; e < ivf_offsets[c + 1] - 1; ++e)", 1),
    ("maxsim_takes_the_minimum", "if (f > best) best = f;", "if (f < best || best == -INFINITY) best = f;", 1),
    ("maxsim_reads_the_query_transposed", "(double)Q[i * dim + t] * (double)D[j * dim + t]",
     "(double)Q[t * qlen + i] * (double)D[j * dim + t]", 1),
    ("stage2_without_pruning",
     "orc_centroid_interaction(S, qlen, cand, n_cand, ix->doc_offsets, ix->codes, keep, s2);",
     "orc_centroid_interaction(S, qlen, cand, n_cand, ix->doc_offsets, ix->codes, NULL, s2);", 1),
    ("stage3_with_pruning",
     "orc_centroid_interaction(S, qlen, sel2, n2, ix->doc_offsets, ix->codes, NULL, s3);",
     "orc_centroid_interaction(S, qlen, sel2, n2, ix->doc_offsets, ix->codes, keep, s3);", 1),
    ("stage3_keeps_half", "int64_t m3 = ndocs / 4 > 1 ? ndocs / 4 : 1;", "int64_t m3 = ndocs / 2 > 1 ? ndocs / 2 : 1;", 1),
    ("stage4_scores_the_stage2_survivors", "orc_maxsim(ix, Q, qlen, sel3, n3, s4);\n", "orc_maxsim(ix, Q, qlen, sel2, n3, s4);\n", 1),
    # vanilla ColBERTv2 retrieval
    ("vanilla_prunes_on_every_token", "if (!inE[j]) continue;", ";", 1),
    ("vanilla_prunes_at_the_cap", "int32_t pruned = n_cand > ncandidates;", "int32_t pruned = n_cand >= ncandidates;", 1),
    ("vanilla_misses_the_last_embedding_of_a_list", "for (int64_t e = eoff[c]; e < eoff[c + 1]; ++e) {",
     "for (int64_t e = eoff[c]; e < eoff[c + 1] - 1; ++e) {", 1),
    ("vanilla_embedding_lists_unsorted", "eids[fill[codes[j]]++] = j;", "eids[fill[codes[j]]++] = N - 1 - j;", 1),
    # reconstructed vectors scaled to unit length (storage variant)
    ("renormalize_divides_by_the_squared_norm", "(float)(1.0 / sqrt(n2))", "(float)(1.0 / n2)", 1),
    ("renormalize_skips_the_last_dimension", "for (int32_t x = 0; x < dim; ++x) n2 +=", "for (int32_t x = 0; x < dim - 1; ++x) n2 +=", 1),
    ("renormalize_scales_by_the_norm", "v[x] = v[x] * inv;", "v[x] = v[x] / inv;", 1),
    ("renormalize_ignores_the_flag", "if (ix->renormalize) {", "if (0) {", 1),
]


def _pins_fail(name, old, new, count, tmp):
    src = open(SRC).read()
    assert src.count(old) == count, f"{name}: the text to replace occurs {src.count(old)} times, expected {count}"
    c = os.path.join(tmp, name + ".c")
    so = os.path.join(tmp, name + ".so")
    with open(c, "w") as f:
        f.write(src.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", so, c, "-lm"])
    env = dict(os.environ, PLAID_ORACLE_LIB=so, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(HERE, "test_oracle_pins.py"), os.path.join(HERE, "test_oracle_hand_example.py"),
                        os.path.join(HERE, "test_oracle_vanilla.py"), os.path.join(HERE, "test_oracle_renormalize.py")],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    tail = "\n".join(r.stdout.strip().splitlines()[-3:])
    return name, r.returncode, tail


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda m: _pins_fail(*m, str(tmp_path)), MISTAKES))
    unnoticed = [(n, tail) for n, rc, tail in results if rc == 0]
    crashed = [(n, rc, tail) for n, rc, tail in results if rc not in (0, 1)]
    assert not crashed, f"the pin run itself broke (exit code other than 'tests failed'): {crashed}"
    assert not unnoticed, f"no pin noticed: {[n for n, _ in unnoticed]}"


def test_the_unmodified_copy_passes(tmp_path):
    """The harness above would also 'pass' if the child run always failed: an unmodified copy has to pass."""
    name, rc, tail = _pins_fail("unmodified", "/* First min(m, n) of", "/* First min(m, n) of", 1, str(tmp_path))
    assert rc == 0, tail
