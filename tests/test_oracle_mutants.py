"""CPU-only: plant one plausible mistake at a time in a private copy of the
oracle's C source (a dropped term, a wrong comparison, a transposed operand)
and check that the pins notice.  The mistake lives in a temporary build of the
ORACLE on the CPU; the HIP library is not involved."""
import os
import subprocess

import pytest

import oracle
from oracle.build import SRC
from . import pins

# (name, text to replace, replacement, pins expected to fail)
MUTANTS = [
    ("router_index_transposed", "load_elem(router_w, dtype, (size_t)e * dh + i)",
     "load_elem(router_w, dtype, (size_t)i * M + e)", [pins.pin_router_logits_library]),
    ("topk_tie_high_index", "l[e] > l[best]", "l[e] >= l[best]", [pins.pin_topk_order_and_gate]),
    ("gate_not_normalised", "- top) / denom;", "- top);", [pins.pin_topk_order_and_gate]),
    ("primary_only_top1", "for (int s = 0; s < S; ++s)", "for (int s = 0; s < 1; ++s)",
     [pins.pin_reroute_against_brute]),
    ("slot_sim_transposed", "most_similar_primary(sim + (size_t)u * M, primary, M, &v, &closeness);",
     "{ float col[256]; for (int c = 0; c < M; ++c) col[c] = sim[(size_t)c * M + u];\n"
     "          most_similar_primary(col, primary, M, &v, &closeness); }",
     [pins.pin_reroute_hand_cases]),
    ("slot_tie_high_index", "if (row[v] > *value) {", "if (row[v] >= *value) {", [pins.pin_reroute_hand_cases]),
    ("slot_threshold_inclusive", "threshold_on && closeness < rho;", "threshold_on && closeness <= rho;",
     [pins.pin_reroute_hand_cases]),
    ("slot_rho0_not_disabled", "const int critical = threshold_on && closeness < rho;", "const int critical = closeness <= rho;",
     [pins.pin_reroute_against_brute]),
    ("sets_sim_transposed", "sim[(size_t)u * M + v] > sim[(size_t)u * M + v_star]",
     "sim[(size_t)v * M + u] > sim[(size_t)v_star * M + u]", [pins.pin_reroute_hand_cases]),
    ("sets_threshold_inclusive", "rho > 0.0f && sim_star[u] < rho", "rho > 0.0f && sim_star[u] <= rho",
     [pins.pin_reroute_hand_cases]),
    ("sets_critical_not_preserved", "final_set[u] = 1;           /* critical expert: preserved */",
     "final_set[u] = 0;", [pins.pin_fig2_behaviour]),
    ("slot_retained_rerouted", "if (rank < S || primary[u])", "if (rank < S)",
     [pins.pin_reroute_hand_cases]),
    ("compact_slot_major", "for (int t = 0; t < T; ++t)\n            for (int k = 0; k < K; ++k)\n                if (ids[(size_t)t * K + k] == e) {",
     "for (int k = 0; k < K; ++k)\n            for (int t = 0; t < T; ++t)\n                if (ids[(size_t)t * K + k] == e) {",
     [pins.pin_compact]),
    ("silu_sign", "return z / (1.0 + exp(-z));", "return z / (1.0 + exp(z));",
     [pins.pin_expert_closed_form]),
    ("gate_up_swapped", "scratch[j] = silu(g) * u;", "scratch[j] = silu(u) * g;",
     [pins.pin_expert_closed_form]),
    ("down_transposed", "load_elem(w_down, dtype, (size_t)r * dm + j)",
     "load_elem(w_down, dtype, (size_t)j * dh + r)", [pins.pin_expert_closed_form]),
    ("up_rows_offset", "(size_t)(dm + j) * dh + i", "(size_t)(j) * dh + i",
     [pins.pin_expert_closed_form]),
    ("gate_weight_dropped", "o[r] += w * y[r];", "o[r] += y[r];", [pins.pin_layer_dense_formulation]),
    ("shared_dropped", "for (int s = 0; s < n_sh; ++s)", "for (int s = 0; s < 0; ++s)",
     [pins.pin_shared_experts_closed_form]),
    ("frobenius_no_sqrt", "dist[(size_t)p * M + q] = sqrt(ss);", "dist[(size_t)p * M + q] = ss;",
     [pins.pin_similarity]),
    ("frobenius_not_inverted", "1.0 - dist[i] / max_dist", "dist[i] / max_dist", [pins.pin_similarity]),
    ("similarity_not_averaged", "sim[i] /= (double)N;", "sim[i] /= 1.0;", [pins.pin_similarity]),
    ("cosine_not_normalised", "total += dot / den;", "total += dot;", [pins.pin_similarity_cosine]),
    ("cosine_not_token_mean", "sim[(size_t)p * M + q] += total / (double)n;", "sim[(size_t)p * M + q] += total;",
     [pins.pin_similarity_cosine]),
    ("cosine_norm_no_sqrt", "norm[(size_t)j * n + r] = sqrt(ss);", "norm[(size_t)j * n + r] = ss;",
     [pins.pin_similarity_cosine]),
    ("cosine_not_averaged", "sim[i] = sim[i] / (double)N;", "sim[i] = sim[i];", [pins.pin_similarity_cosine]),
    ("cka_diagonal_kept", "(r == c) ? 0.0 : dot;", "dot;", [pins.pin_similarity_cka]),
    ("cka_cross_term_sign", "- 2.0 * cross / (dn - 2.0)", "+ 2.0 * cross / (dn - 2.0)", [pins.pin_similarity_cka]),
    ("cka_cross_term_weight", "- 2.0 * cross / (dn - 2.0)", "- 2.0 * cross / (dn - 1.0)", [pins.pin_similarity_cka]),
    ("cka_sum_term_weight", "sk * sl / ((dn - 1.0) * (dn - 2.0))", "sk * sl / (dn * dn)", [pins.pin_similarity_cka]),
    ("cka_sum_term_dropped", "tr + sk * sl / ((dn - 1.0) * (dn - 2.0))", "tr", [pins.pin_similarity_cka]),
    ("cka_no_sqrt", "sqrt(self[p] * self[q]);", "(self[p] * self[q]);", [pins.pin_similarity_cka]),
    ("cka_rbf_bandwidth_not_squared", "return exp(-dist2 / (2.0 * p0 * p0));", "return exp(-dist2 / (2.0 * p0));",
     [pins.pin_similarity_cka_kernels]),
    ("cka_rbf_no_factor_two", "return exp(-dist2 / (2.0 * p0 * p0));", "return exp(-dist2 / (p0 * p0));",
     [pins.pin_similarity_cka_kernels]),
    ("cka_rbf_distance_not_squared", "dist2 += (x[k] - y[k]) * (x[k] - y[k]);", "dist2 += fabs(x[k] - y[k]);",
     [pins.pin_similarity_cka_kernels]),
    ("cka_poly_offset_dropped", "return pow(dot + p0, p1);", "return pow(dot, p1);", [pins.pin_similarity_cka_kernels]),
    ("cka_poly_degree_ignored", "return pow(dot + p0, p1);", "return dot + p0;", [pins.pin_similarity_cka_kernels]),
    ("cka_not_averaged", "sim[i] = sim[i] * (1.0 / (double)N);", "sim[i] = sim[i];", [pins.pin_similarity_cka]),
]


@pytest.mark.parametrize("name,old,new,catchers", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new, catchers):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} must be unique"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / f"libmutant_{name}.so"
    subprocess.run(["gcc", "-std=c11", "-O1", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
                    str(src), "-o", str(lib), "-lm"], check=True)
    mutant = oracle.OracleLib(os.fspath(lib))
    caught = []
    for pin in catchers:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin noticed the planted mistake '{name}'"
