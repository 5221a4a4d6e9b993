"""Do the pins of the selector's reference notice a plausible mistake?

Each case plants one mistake in a copy of the reference's source (a dropped
factor, a wrong branch, a term left out), loads the copy as a module and runs
the reference's pin tests with it; at least one pin must fail for every copy.
Only the pins are run, not the comparison with the C implementation.
"""
import os
import types

import pytest

import test_strategy as TS

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "strategy_oracle.py")

PINS = [TS.test_pairwise_all_to_all_is_d_minus_one_rounds, TS.test_one_round_scatter_and_gather,
        TS.test_queue_is_textbook_mm1, TS.test_scaling_laws_of_the_latency_terms,
        TS.test_compute_term_by_hand, TS.test_memory_constraint_by_hand,
        TS.test_enumeration_on_the_papers_example_cluster,
        TS.test_select_is_the_argmax_of_the_enumeration, TS.test_hybrid_scheme_moves_less_across_nodes]

MUTANTS = [
    ("rs_not_divided", "return 0.0 if degree == 1 else size / degree / bw", "return 0.0 if degree == 1 else size / bw"),
    ("ar_of_the_whole_tensor", "return RS(size / degree, degree, bw) + AG(size / degree, degree, bw)",
     "return RS(size, degree, bw) + AG(size, degree, bw)"),
    ("a2a_d_rounds", "return size / degree * (degree - 1) / bw", "return size / degree * degree / bw"),
    ("node_boundary_off_by_one", 'cl["bw_intra"] if devices <= cl["n_proc"]', 'cl["bw_intra"] if devices < cl["n_proc"]'),
    ("psi_of_all_layers", 'psi = (mo["psi_attn"] + mo["psi_moe"]) / mo["layers"]', 'psi = (mo["psi_attn"] + mo["psi_moe"])'),
    ("tau_ignores_ep", "return psi / (d_tp * d_ep) * (b / d_dp)", "return psi / d_tp * (b / d_dp)"),
    ("tau_ignores_dp", "return psi / (d_tp * d_ep) * (b / d_dp)", "return psi / (d_tp * d_ep) * b"),
    ("one_ar_per_layer", "return 2 * ar + 2 * a2a", "return ar + 2 * a2a"),
    ("one_a2a_per_layer", "return 2 * ar + 2 * a2a", "return 2 * ar + a2a"),
    ("a2a_branches_swapped", "if d_dp >= d_ep:", "if d_dp < d_ep:"),
    ("a2a_without_top_k", 'a2a = A2A(b / d_ep * s * h * k * eb, d_dp', 'a2a = A2A(b / d_ep * s * h * eb, d_dp'),
    ("a2a_group_of_ep_when_dp_smaller", 'a2a = A2A(b / d_ep * s * h * k * eb, d_dp, _bw(cl, d_tp * d_dp))',
     'a2a = A2A(b / d_ep * s * h * k * eb, d_ep, _bw(cl, d_tp * d_dp))'),
    ("pipeline_hops", "+ (d_pp - 1) * p2p", "+ d_pp * p2p"),
    ("layers_dropped", 'return mo["layers"] * (tau(', "return 1 * (tau("),
    ("queue_is_lq_not_wq", "wq = rho / (mu * (1 - rho))", "wq = rho / (1 - rho)"),
    ("service_rate_from_prefill", 'mu = 1.0 / out["svc_dec"]', 'mu = 1.0 / out["svc_prf"]'),
    ("ttft_without_queue", 'out["ttft"] = wq + out["svc_prf"]', 'out["ttft"] = out["svc_prf"]'),
    ("throughput_one_decode_step", '+ L_out * out["svc_dec"])', '+ out["svc_dec"])'),
    ("experts_not_sliced_by_tp", '+ mo["psi_moe"] / (d_ep * d_tp)', '+ mo["psi_moe"] / d_ep'),
    ("kv_of_the_prompt_only", "+ 2 * b * (L_in + L_out) * mo", "+ 2 * b * L_in * mo"),
    ("kv_not_split_by_pp", '* mo["layers"] / d_pp', '* mo["layers"]'),
    ("memory_not_checked", 'int(out["mem_bytes"] < cl["mem_bytes"] and', "int("),
    ("dp_beyond_batch", 'while d_dp * d_tp <= n and d_dp <= rq["batch"]:', "while d_dp * d_tp <= n:"),
    ("select_smallest", 'key=lambda s: (-s["throughput"]', 'key=lambda s: (s["throughput"]'),
    ("mix_without_ag", '+ AG(sh, cl["n_proc"], cl["bw_intra"]) \\\n', "\\\n"),
    ("ep_one_a2a", 'return AR(bsh, cl["n_proc"], cl["bw_intra"]) + 2 * A2A(bsh * mo["top_k"]',
     'return AR(bsh, cl["n_proc"], cl["bw_intra"]) + A2A(bsh * mo["top_k"]'),
]


def _load(text, name):
    m = types.ModuleType(name)
    exec(compile(text, name, "exec"), m.__dict__)
    return m


def _pins_fail(monkeypatch, module):
    monkeypatch.setattr(TS, "O", module)
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            return True
    return False


def test_unchanged_copy_passes(monkeypatch):
    assert not _pins_fail(monkeypatch, _load(open(SRC).read(), "copy"))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_fails_a_pin(monkeypatch, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, "the text to replace occurs %d times" % src.count(old)
    assert _pins_fail(monkeypatch, _load(src.replace(old, new), name)), "no pin notices " + name
