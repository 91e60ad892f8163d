"""Do the oracle's pins notice a mistake?  (CPU only.)

Each case plants one plausible mistake in a COPY of the oracle's C source (a flipped sign rule, a
dropped term, a wrong index, a swapped operand ...), builds it beside the real one and runs the pin
tests of ``test_oracle_pins.py`` against it in a child process.  The pins must fail.  A mistake that
survives means a part of the oracle is tied to nothing but itself.  The real oracle is never touched:
the copy lives in a temporary folder and is selected through ``ROCKETKV_ORACLE_LIB``, which the
oracle's loader honours only together with ``ROCKETKV_ORACLE_MUTANT_RUN=1`` (set here and nowhere
else), so no other environment can swap the checker under the GPU tests.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rocketkv_oracle.c")

# (name, text in the source, replacement, which occurrence of the text)
MUTANTS = [
    ("topk_takes_the_smallest", "if (a->v > b->v) return -1;\n  if (a->v < b->v) return 1;",
     "if (a->v > b->v) return 1;\n  if (a->v < b->v) return -1;", 0),
    ("ties_go_to_the_higher_index", "return (a->i > b->i) - (a->i < b->i);", "return (a->i < b->i) - (a->i > b->i);", 0),
    ("summary_skips_the_last_token_of_a_page", "for (int j = j0 + 1; j < j1; ++j) {", "for (int j = j0 + 1; j < j1 - 1; ++j) {", 0),
    ("summary_min_follows_the_max", "if (x < mn) mn = x;", "if (x > mn) mn = x;", 0),
    ("summary_rows_transposed", "kmin[(size_t)c * P + p] = mn;", "kmin[(size_t)c * P + p] = mx;", 0),
    ("channels_ranked_by_signed_sum", "sa += fabs(x);", "sa += x;", 0),
    ("channel_weight_is_the_abs_sum", "s[c] = ss;", "s[c] = sa;", 0),
    ("sign_rule_flipped", "(s[c] >= 0.0) ? kmax[(size_t)c * P + p] : kmin[(size_t)c * P + p]",
     "(s[c] < 0.0) ? kmax[(size_t)c * P + p] : kmin[(size_t)c * P + p]", 0),
    ("score_drops_the_query_weight", "acc += s[c] * bound;", "acc += bound;", 0),
    ("pages_to_pick_rounds_up", "int kp = T / ps;", "int kp = (T + ps - 1) / ps;", 0),
    ("budget_covering_context_not_dense", "if (T >= n) return P;", "if (T > n) return P;", 0),
    ("recent_pages_forced_at_the_front", "sc[P - 1 - r] = INFINITY;", "sc[r] = INFINITY;", 0),
    ("attention_without_the_scale", "double scale = 1.0 / sqrt((double)D);", "double scale = 1.0;", 0),
    ("attention_reads_keys_for_values", "const uint16_t* vr = V + (size_t)tok[t] * D;", "const uint16_t* vr = K + (size_t)tok[t] * D;", 0),
    ("attention_weights_not_normalised", "double w = l[t] / z;", "double w = l[t];", 0),
    ("lse_without_the_sum", "lse[h] = m + log(z);", "lse[h] = m;", 0),
    ("snapkv_without_the_scale", "double scale = 1.0 / sqrt((double)D);", "double scale = 1.0;", 1),
    ("snapkv_softmax_over_the_prefix_only", "for (int j = 0; j <= t; ++j) { l[j] = exp(l[j] - m); z += l[j]; }",
     "for (int j = 0; j < L; ++j) { l[j] = exp(l[j] - m); z += l[j]; }", 0),
    ("snapkv_votes_of_the_first_head_only", "for (int h = 0; h < G; ++h)\n    for (int w = 0; w < W; ++w) {",
     "for (int h = 0; h < 1; ++h)\n    for (int w = 0; w < W; ++w) {", 0),
    ("snapkv_pool_one_wider", "int r = (ks - 1) / 2;", "int r = (ks + 1) / 2;", 0),
    ("snapkv_pool_is_an_average", "if (gv[i] > mx) mx = gv[i];", "mx += gv[i] / (double)(hi - lo + 1);", 0),
    ("snapkv_window_not_kept", "kept[keep_prefix + w] = L + w;", "kept[keep_prefix + w] = w;", 0),
    ("snapkv_budget_excludes_the_window", "int keep_prefix = N - W;", "int keep_prefix = N - W - 1;", 0),
    # the batch wrappers: offsets of a (sequence, KV head) unit, row strides, list termination
    ("attend_given_query_offset_ignores_the_group", "okv_attend_pages(q + (u * G) * D, K + u * (size_t)n_cap * D, V + u * (size_t)n_cap * D,\n                       G, D, seq_lens[b], ps, pg, kp,",
     "okv_attend_pages(q + u * D, K + u * (size_t)n_cap * D, V + u * (size_t)n_cap * D,\n                       G, D, seq_lens[b], ps, pg, kp,", 0),
    ("attend_given_values_of_the_first_unit", "K + u * (size_t)n_cap * D, V + u * (size_t)n_cap * D,\n                       G, D, seq_lens[b], ps, pg, kp,",
     "K + u * (size_t)n_cap * D, V,\n                       G, D, seq_lens[b], ps, pg, kp,", 0),
    ("attend_given_list_row_stride", "const int* pg = pages + u * pages_cap;", "const int* pg = pages + u * (pages_cap - 1);", 0),
    ("attend_given_walks_past_the_terminator", "while (kp < pages_cap && pg[kp] >= 0) ++kp;",
     "while (kp < pages_cap && pg[kp] >= 0) ++kp;\n      while (kp < pages_cap && pg[kp] < 0) ++kp;\n      while (kp < pages_cap && pg[kp] >= 0) ++kp;", 0),
    ("attend_given_length_of_the_first_sequence", "G, D, seq_lens[b], ps, pg, kp,", "G, D, seq_lens[0], ps, pg, kp,", 0),
    ("build_summaries_column_stride", "kmax[(u * D + c) * pages_cap + p] = mx[(size_t)c * P + p];", "kmax[(u * D + c) * P + p] = mx[(size_t)c * P + p];", 0),
    ("build_summaries_keys_of_the_first_unit", "okv_page_summaries(K + u * (size_t)n_cap * D, n, D, ps, mx, mn);", "okv_page_summaries(K, n, D, ps, mx, mn);", 0),
    ("build_summaries_min_from_max", "kmin[(u * D + c) * pages_cap + p] = mn[(size_t)c * P + p];", "kmin[(u * D + c) * pages_cap + p] = mx[(size_t)c * P + p];", 0),
    ("snapkv_batch_queries_of_the_first_group", "okv_snapkv_unit(qobs + u * G * (size_t)W * D,", "okv_snapkv_unit(qobs + (size_t)b * Hq * W * D,", 0),
    ("snapkv_batch_key_stride", "K + u * (size_t)S_cap * D,\n                                G, W, D, S, ks, N,", "K + u * (size_t)S * D,\n                                G, W, D, S, ks, N,", 0),
    ("snapkv_batch_length_of_the_first_sequence", "int S = seq_lens[b];\n      int* kp = kept + u * N;", "int S = seq_lens[0];\n      int* kp = kept + u * N;", 0),
]


def nth_replace(text, old, new, which):
    at = -1
    for _ in range(which + 1):
        at = text.find(old, at + 1)
        assert at >= 0, "the oracle's source no longer contains: " + old
    return text[:at] + new + text[at + len(old):]


@pytest.mark.parametrize("name,old,new,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_notice_a_planted_mistake(tmp_path, name, old, new, which):
    src = open(SRC).read()
    mutated = nth_replace(src, old, new, which)
    c_file = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    c_file.write_text(mutated)
    subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", str(c_file), "-o", str(lib), "-lm"],
                   check=True)
    env = dict(os.environ, ROCKETKV_ORACLE_LIB=str(lib), ROCKETKV_ORACLE_MUTANT_RUN="1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1, f"the pins did not notice '{name}' (pytest exit {r.returncode}):\n" + r.stdout[-1500:]
