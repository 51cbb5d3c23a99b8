"""The pins must catch plausible mistakes.  Each case below plants one mistake in
a COPY of the oracle's source (on the CPU, never in the HIP path), builds it, and
runs the pin battery against that build: at least one pin has to fail.  Mistakes
that only select another valid decomposition (a different tie-break in the
matching search) are not listed: the paper does not pin the sequence of
matchings, and neither can these tests."""
import os
import subprocess
import tempfile

import pytest

import test_oracle_bottleneck as TN
import test_oracle_bruteforce as TB
import test_oracle_build_traffic as TT
import test_oracle_pins as TP
import test_oracle_redistribution as TR
import test_oracle_spreadout as TS
import test_oracle_stage_order as TO

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "fast_oracle.cpp")

MUTATIONS = [
    ("aggregation reads the transposed tile",
     "tot += at(traffic, N, a * G + i, d * G + j);",
     "tot += at(traffic, N, d * G + j, a * G + i);"),
    ("diagonal not ignored by the sign check",
     "if (g != h && at(traffic, N, g, h) < 0) return -1;",
     "if (at(traffic, N, g, h) < 0) return -1;"),
    ("remainder bytes put on the highest lanes",
     "target[k] = q + (k < rho ? 1 : 0);",
     "target[k] = q + (k >= G - rho ? 1 : 0);"),
    ("a GPU keeps its whole load",
     "X[i * G + i] = std::min(r[i], target[i]);",
     "X[i * G + i] = r[i];"),
    ("surplus poured from the wrong end",
     "if (s[i] == 0) { ++i; continue; }",
     "if (s[i] == 0 || i == 0) { ++i; continue; }"),
    ("per-lane entry rounded down",
     "(a == d) ? 0 : (t + G - 1) / G;",
     "(a == d) ? 0 : t / G;"),
    ("embedding skips the diagonal",
     "const i64 m = std::min(dr[a], dc[a]);",
     "const i64 m = 0;"),
    ("embedding raises lines to a wrong level",
     "for (int a = 0; a < S; ++a) { dr[a] = L - dr[a]; dc[a] = L - dc[a]; }",
     "for (int a = 0; a < S; ++a) { dr[a] = L - dr[a]; dc[a] = L - dc[a] + (a == 0 && S > 1); dr[S - 1] += (a == 0 && S > 1); }"),
    ("real bytes of a cell are not consumed",
     "Rreal[(size_t)a * S + d] -= real;",
     ""),
    ("stage destination written for the column, not the row",
     "stage_row[a] = real > 0 ? d : -1;",
     "stage_row[d] = real > 0 ? a : -1;"),
    ("balance term divided by the scale-out bandwidth",
     "const double t0 = (double)bal / bw_up;",
     "const double t0 = (double)bal / bw_out;"),
    ("last redistribution without its (G-1) factor",
     "const double t3 = (double)((i64)(G - 1) * cmax) / bw_up;",
     "const double t3 = (double)cmax / bw_up;"),
    ("optimal time not divided by G",
     "out4[3] = (double)big / ((double)G * bw_out);",
     "out4[3] = (double)big / bw_out;"),
    ("exposed redistribution never added",
     "if (bw_up < (double)(G - 1) * bw_out) {",
     "if (false) {"),
    ("exposed redistribution pairs a stage with the wrong neighbour",
     "const double redis = (double)((i64)(G - 1) * c[i - 1]) / bw_up;\n            const double next = (double)c[i] / bw_out;",
     "const double redis = (double)((i64)(G - 1) * c[i]) / bw_up;\n            const double next = (double)c[i - 1] / bw_out;"),
    ("exposed redistribution evaluated in extraction order",
     "std::sort(c.begin(), c.end());\n        for (int i = 1; i < K; ++i) {",
     "for (int i = 1; i < K; ++i) {"),
    ("exposed redistribution without its (G-1) factor",
     "const double redis = (double)((i64)(G - 1) * c[i - 1]) / bw_up;",
     "const double redis = (double)c[i - 1] / bw_up;"),
    ("wake-up delay not paid per stage",
     "(K > 0 ? K : 0) +",
     "0 +"),
    ("SpreadOut mixes up the two bandwidth classes",
     "if (g / G == h / G) up = std::max(up, v); else out = std::max(out, v);",
     "if (g / G != h / G) up = std::max(up, v); else out = std::max(out, v);"),
    ("SpreadOut server stages walk the wrong diagonal",
     "m = std::max(m, at(Q.data(), S, a, (a + i) % S));",
     "m = std::max(m, at(Q.data(), S, a, (a + 1) % S));"),
    ("stage order reverses equal weights",
     "while (j >= 0 && c[order[j]] > c[x])",
     "while (j >= 0 && c[order[j]] >= c[x])"),
    ("traffic construction transposed",
     "traffic[(size_t)src * N + expert_to_gpu[e]] += c * token_bytes;",
     "traffic[(size_t)expert_to_gpu[e] * N + src] += c * token_bytes;"),
    ("a GPU hands off the head of its region instead of the tail",
     "region[k].take(std::min(r[k], target), &(*queue)[k]);   // the head stays on lane k",
     "{ Queue skip; region[k].take(r[k] - std::min(r[k], target), &skip); "
     "region[k].take(std::min(r[k], target), &(*queue)[k]); region[k] = skip; }"),
    ("redistribution matrix transposed",
     "for (const Run& run : got.runs) M[k * G + run.dest] += run.len;",
     "for (const Run& run : got.runs) M[run.dest * G + k] += run.len;"),
    ("send offset taken after the stage instead of before",
     "offsets[(size_t)s * S + a] = sent[(size_t)a * S + d];\n            sent[(size_t)a * S + d] += len;",
     "sent[(size_t)a * S + d] += len;\n            offsets[(size_t)s * S + a] = sent[(size_t)a * S + d];"),
    ("bytes that stay on the proxy GPU counted as forwarded",
     "if (o == g) continue;\n                    fwd += M[g * G + o];",
     "fwd += M[g * G + o]; if (o == g) continue;"),
    ("redistribution does not wait for the scale-up fabric",
     "const double start = std::max(out_end, up_free);",
     "const double start = out_end;"),
    ("redistribution does not wait for its own stage",
     "const double start = std::max(out_end, up_free);",
     "const double start = up_free;"),
    ("intra-server portion serialised before the first stage",
     "double out_end = t, up_free = t;\n    if (intra > 0) up_free = t + (delay + (double)intra / bw_up);",
     "if (intra > 0) t = t + (delay + (double)intra / bw_up);\n    double out_end = t, up_free = t;"),
    ("bottleneck search walks down after a success",
     "best = vals[mid];\n            lo = mid + 1;",
     "best = vals[mid];\n            hi = mid - 1;"),
    ("threshold graph drops the cells that hold exactly the threshold",
     "if (R[(size_t)a * S + d] < t || seen[d]) continue;",
     "if (R[(size_t)a * S + d] <= t || seen[d]) continue;"),
    ("fewer-stages variant matches on the support instead of the threshold graph",
     "Matcher M(S, R, t);",
     "Matcher M(S, R);"),
    ("canonical search treats its threshold as exclusive",
     "if (inF[a] && R[(size_t)a * S + d] >= thr) {",
     "if (inF[a] && R[(size_t)a * S + d] > thr) {"),
]


def battery(O):
    """A fast subset of every pin file; raises AssertionError at the first failing pin."""
    TP.test_sender_balancing_example(O)
    TP.test_three_server_example(O)
    TP.test_embedding_small_case(O)
    TP.test_uniform_all_to_all(O)
    TP.test_negative_entry_and_diagonal(O)
    TP.test_zero_and_single_cell(O)
    TP.test_theorem2_terms_on_adversarial_input(O)
    TP.test_unit_handling(O)
    TP.test_exposed_redistribution_hand_cases(O)
    TP.test_exposed_redistribution_uniform_all_to_all(O)
    TP.test_exposed_redistribution_is_the_barrier_synchronised_pipeline(O, 0)
    TP.test_exposed_redistribution_when_scale_up_is_slow(O)
    for S, G, kind in [(3, 2, "heavy"), (4, 8, "sparse"), (5, 7, "uniform")]:
        TP.test_invariants_random(O, S, G, kind)
    TB.test_total_stage_weight_is_the_brute_force_optimum(O, 3, 2, None)
    TB.test_sender_balancing_moves_the_least_possible(O)
    TS.test_four_server_example(O)
    TS.test_uniform_all_to_all_closed_forms(O)
    TS.test_single_flows(O)
    TS.test_diagonal_maxima_definition(O, 3, 4)
    TS.test_wakeup_delay_counts_executed_steps(O)
    TO.test_matches_stable_argsort_and_is_a_permutation(O)
    TT.test_identity_and_contiguous_placement(O)
    TT.test_conservation_and_permuted_placement(O)
    for args in [(3, 2, 9, 1, True), (3, 3, 5, 2, False), (2, 4, 7, 4, True)]:
        TR.test_against_byte_level_replay(O, *args)
    TR.test_closed_forms(O)
    TR.test_pipeline_hand_example(O)
    TR.test_pipeline_hides_everything_but_the_last_redistribution(O)
    TR.test_pipeline_scale_up_chain_when_nothing_hides(O)
    TN.test_bottleneck_value_is_the_best_over_all_permutations(O, 4)
    TN.test_hand_example(O)
    TN.test_stage_by_stage_replay_on_matrices_without_virtual_bytes(O, 4, 7)
    TN.test_invariants_with_virtual_bytes(O, 5, "small")


def test_battery_passes_on_the_real_oracle(oracle):
    battery(oracle)


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(oracle, what, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation target not unique in the source: {old!r}"
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "mutant.cpp")
        lib = os.path.join(tmp, "libmutant.so")
        open(src, "w").write(text.replace(old, new))
        subprocess.check_call(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", "-w", "-o", lib, src])
        with oracle.use_library(lib):
            try:
                battery(oracle)
            except AssertionError:
                return
    pytest.fail(f"no pin noticed the planted mistake: {what}")
