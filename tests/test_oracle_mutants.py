"""Are the pins sharp?  Each case below plants one plausible mistake in a COPY of the oracle's
source (a dropped term, a missing jitter, a wrong count, a wrong overhead), builds it with g++
on the CPU and requires that at least one pin (hand-worked values, closed forms, the textbook
special case, the simulator) rejects it.  Nothing here touches the GPU library."""
import os
import subprocess
import types

import pytest

import test_oracle_continue as continue_tests
import test_oracle_des as des_tests
import test_oracle_gprio as gprio_tests
import test_oracle_pins as pin_tests
import test_oracle_sim as sim_tests

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rta_oracle.cpp")

MUTANTS = {
    "lemma10_same_core_sum_dropped": (
        "bool first_sum = tau[i].gpu() || !(options & ORACLE_OPT_LITERAL_LEMMA10);", "bool first_sum = false;"),
    "jitter_Jg_dropped": ("i64 Jg(const Task &h) const { return std::max<i64>(0, h.R - h.Ge); }",
                          "i64 Jg(const Task &h) const { (void)h; return 0; }"),
    "jitter_Jc_dropped": ("i64 Jc(const Task &h) const { return std::max<i64>(0, h.R - (h.C + h.Gm)); }",
                          "i64 Jc(const Task &h) const { (void)h; return 0; }"),
    "jitter_below_zero_when_own_demand_exceeds_the_deadline": (
        "i64 Jg(const Task &h) const { return std::max<i64>(0, h.R - h.Ge); }",
        "i64 Jg(const Task &h) const { return h.R - h.Ge; }"),
    "lemma4_tau_h_not_counted": ("    i64 nu = 1;", "    i64 nu = 0;"),
    "lemma8_blocking_dropped": ("b = add(b, mul(t.eta + 1, p.eps));", "b = add(b, 0);"),
    "lemma8_blocking_eta_only": ("b = add(b, mul(t.eta + 1, p.eps));", "b = add(b, mul(t.eta, p.eps));"),
    "own_runlist_updates_dropped": ("b = add(b, mul(2 * p.eps, t.eta));", "b = add(b, 0);"),
    "Ge_star_without_updates": ("i64 Ge_star(const Task &t) const { return add(t.Ge, mul(2 * p.eps, t.eta)); }",
                                "i64 Ge_star(const Task &t) const { return t.Ge; }"),
    "Gm_star_without_updates": ("i64 Gm_star(const Task &t) const { return add(t.Gm, mul(2 * p.eps, t.eta)); }",
                                "i64 Gm_star(const Task &t) const { return t.Gm; }"),
    "lemma1_counts_one_tsg_less": ("i64 nu = n_gpu_tasks() - (t.gpu() ? 1 : 0);",
                                   "i64 nu = n_gpu_tasks() - 1 - (t.gpu() ? 1 : 0); if (nu < 0) nu = 0;"),
    "lemma13_same_core_sum_dropped": (
        "if (same_core(h, i) && tau[h].gpu()) s = add(s, term(R + Jg(tau[h]), tau[h].T, tau[h].Ge));",
        "if (false) s = 0;"),
    "eq3_theta_dropped": ("return mul(mul(p.L + p.theta, nu), ceil_div(ge, p.L));",
                          "return mul(mul(p.L, nu), ceil_div(ge, p.L));"),
    "eq3_floor_instead_of_ceil": ("return mul(mul(p.L + p.theta, nu), ceil_div(ge, p.L));",
                                  "return mul(mul(p.L + p.theta, nu), ge / p.L);"),
    "ceil_is_floor": ("i64 ceil_div(i64 a, i64 b) { return (a + b - 1) / b; }",
                      "i64 ceil_div(i64 a, i64 b) { return a / b; }"),
    "hpp_taken_as_other_cores": ("bool same_core(size_t h, size_t i) const { return tau[h].core == tau[i].core; }",
                                 "bool same_core(size_t h, size_t i) const { return tau[h].core != tau[i].core; }"),
    "priority_order_reversed": ("return prio[a] > prio[b]; });", "return prio[a] < prio[b]; });"),
    "G_i_without_Gm": ("t.G = t.Gm + t.Ge;", "t.G = t.Ge;"),
    "gprio_jitter_Jg_dropped": ("i64 jitter_g(size_t h) const { return std::max<i64>(0, tau[h].D - tau[h].Ge); }",
                                "i64 jitter_g(size_t h) const { (void)h; return 0; }"),
    "gprio_jitter_Jg_from_deadline_only": ("i64 jitter_g(size_t h) const { return std::max<i64>(0, tau[h].D - tau[h].Ge); }",
                                           "i64 jitter_g(size_t h) const { return tau[h].D; }"),
    "gprio_jitter_Jc_from_deadline_only": (
        "i64 jitter_c(size_t h) const { return std::max<i64>(0, tau[h].D - (tau[h].C + tau[h].Gm)); }",
        "i64 jitter_c(size_t h) const { return tau[h].D; }"),
    "gprio_lemma11_dropped": ("      /* Lemma 10, second sum (eta^g_i > 0); Lemma 11 (eta^g_i = 0) */\n      for (size_t h = 0; h < n; ++h)\n        if (higher_g[h] &&",
                              "      for (size_t h = 0; h < n; ++h)\n        if (uses_gpu(i) && higher_g[h] &&"),
    "gprio_jitter_Jc_dropped": ("i64 jitter_c(size_t h) const { return std::max<i64>(0, tau[h].D - (tau[h].C + tau[h].Gm)); }",
                                "i64 jitter_c(size_t h) const { (void)h; return 0; }"),
    "gprio_Ge_star_without_updates": ("i64 ge_star(size_t h) const { return add(tau[h].Ge, updates(h)); }",
                                      "i64 ge_star(size_t h) const { return tau[h].Ge; }"),
    "gprio_lemma13_same_core_with_updates": (
        "if (on_core_of(i, h) && uses_gpu(h)) s = add(s, arrivals_times(R + jitter_g(h), h, tau[h].Ge));",
        "if (on_core_of(i, h) && uses_gpu(h)) s = add(s, arrivals_times(R + jitter_g(h), h, ge_star(h)));"),
    "gprio_lemma13_for_cpu_only_tasks_too": ("      if (uses_gpu(i)) {", "      if (true) {"),
    "gprio_blocking_dropped": (
        "return add(add(add(tau[i].C, tau[i].G), updates(i)), mul(tau[i].eta + 1, p.eps));",
        "return add(add(tau[i].C, tau[i].G), updates(i));"),
    "gprio_same_core_taken_as_other_cores": (
        "bool on_core_of(size_t i, size_t h) const { return tau[h].core == tau[i].core; }",
        "bool on_core_of(size_t i, size_t h) const { return tau[h].core != tau[i].core; }"),
    "gprio_solve_stops_early": ("      if (next == R) break;\n      R = next;", "      R = next;\n      break;"),
    "search_tries_highest_cpu_priority_first": ("for (size_t k = n_tasks; k-- > 0 && !placed;) {",
                                                "for (size_t k = 0; k < n_tasks && !placed; ++k) {"),
    "search_ignores_the_same_core_order": ("if (unassigned[m] && tau[m].core == tau[k].core) feasible = false;",
                                           "if (false) feasible = false;"),
    "search_levels_from_the_top": ("level_of[k] = (int32_t)level;", "level_of[k] = (int32_t)(n_tasks + 1 - level);"),
    "search_puts_assigned_tasks_above": ("      std::vector<char> higher_g(unassigned);\n      higher_g[k] = 0;",
                                         "      std::vector<char> higher_g(n_tasks, 1);"),
    "continue_after_miss_takes_the_period": ("      tau[k].R = tau[k].D;\n", "      tau[k].R = tau[k].T;\n"),
    "continue_after_miss_takes_zero": ("      tau[k].R = tau[k].D;\n", "      tau[k].R = 0;\n"),
    "given_priorities_batch_wrong_segment_stride": (
        "ge_us ? ge_us + so : nullptr, gprio + to,", "ge_us ? ge_us + to : nullptr, gprio + to,"),
    "given_priorities_batch_wrong_priority_stride": (
        "ge_us ? ge_us + so : nullptr, gprio + to,", "ge_us ? ge_us + so : nullptr, gprio + s,"),
    "stops_one_iteration_early": ("      } else if (next == R) {\n        break;",
                                  "      } else if (next == R || true) {\n        break;"),
}

PINS = [
    lambda o: [pin_tests.test_classic_hand_examples(o, [1, 2, 3], [4, 6, 13], [1, 3, 10], p, w)
               for p, w in pin_tests.VARIANTS],
    lambda o: [pin_tests.test_cpu_only_reduces_to_textbook_rta(o, p, w) for p, w in pin_tests.VARIANTS],
    pin_tests.test_single_core_gcaps_busy_is_classic_rta_on_inflated_wcet,
    pin_tests.test_round_robin_interleave_closed_form,
    pin_tests.test_gcaps_top_task_closed_form,
    pin_tests.test_table2_printed_verdict,
    pin_tests.test_table2_hand_worked_values,
    lambda o: [pin_tests.test_three_task_example(o, p, w, want) for p, w, want in
               [(2, 1, [26, 26, 73]), (2, 0, [26, 50, 73]), (1, 1, [26, 35, 63]), (1, 0, [26, 43, 63])]],
    pin_tests.test_carry_in_jitter_other_core,
    pin_tests.test_self_suspension_jitter_same_core,
    pin_tests.test_theta_slice_identity,
    des_tests.test_directed_carry_in_other_core,
    des_tests.test_directed_self_suspension_same_core,
    lambda o: [des_tests.test_simulated_response_never_exceeds_bound(o, p, w) for p, w in pin_tests.VARIANTS],
    continue_tests.test_hand_worked_example,
    continue_tests.test_jitter_is_not_taken_below_zero,
    continue_tests.test_every_task_missing_equals_deadline_jitters,
    lambda o: [continue_tests.test_relations_with_the_default_and_with_deadline_jitters(o, 1, w) for w in (0, 1)],
    gprio_tests.test_table2_printed_verdicts,
    gprio_tests.test_table2_hand_worked_values,
    gprio_tests.test_runlist_update_cost_hand_worked,
    gprio_tests.test_same_core_self_suspension_with_update_cost_hand_worked,
    gprio_tests.test_carry_in_jitter_is_deadline_minus_gpu_time,
    gprio_tests.test_search_prefers_the_lowest_cpu_priority_candidate,
    lambda o: [gprio_tests.test_search_finds_an_order_iff_one_exists(o, w) for w in (0, 1)],
    lambda o: [gprio_tests.test_simulated_response_never_exceeds_bound_under_separate_priorities(o, w)
               for w in (0, 1)],
    gprio_tests.test_given_priorities_batch_matches_single_calls,
]


def mutant_module(oracle, lib):
    m = types.SimpleNamespace(**{k: getattr(oracle, k) for k in dir(oracle) if k.isupper()})
    m.OracleError = oracle.OracleError
    m.rta_taskset = lambda *a, **kw: oracle.rta_taskset(*a, lib=lib, **kw)
    m.gprio_rta_taskset = lambda *a, **kw: oracle.gprio_rta_taskset(*a, lib=lib, **kw)
    m.gprio_assign_taskset = lambda *a, **kw: oracle.gprio_assign_taskset(*a, lib=lib, **kw)
    m.gprio_rta_batch = lambda *a, **kw: oracle.gprio_rta_batch(*a, lib=lib, **kw)
    return m


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_rejected_by_some_pin(oracle, tmp_path, name):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    cpp = tmp_path / "mutant.cpp"
    cpp.write_text(src.replace(old, new))
    so = tmp_path / "libmutant.so"
    subprocess.run(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", "-pthread", "-I", os.path.dirname(SRC),
                    "-o", str(so), str(cpp)], check=True)
    m = mutant_module(oracle, oracle.open_library(str(so)))
    killed_by = None
    for k, pin in enumerate(PINS):
        try:
            pin(m)
        except (AssertionError, oracle.OracleError):  # a wrong value, or an error where none is due
            killed_by = k
            break
    assert killed_by is not None, f"no pin notices the planted mistake '{name}'"


def test_unmutated_oracle_passes_the_same_pins(oracle):
    for pin in PINS:
        pin(oracle)


# ---- the simulation oracle ----------------------------------------------------------------------
SIM_SRC = os.path.join(ROOT, "oracle", "sim_oracle.cpp")

SIM_MUTANTS = {
    "no_switch_after_a_completed_segment": ("          if (!ring.empty()) switch_left = switch_into(ring.front());\n", "\n"),
    "rotation_without_switch": ("            ring.push_back(i);\n            switch_left = switch_into(ring.front());",
                                "            ring.push_back(i);\n            switch_left = 0;"),
    "free_switch_follows_the_own_slice": ("            ring.push_back(i);\n            switch_left = switch_into(ring.front());",
                                          "            ring.push_back(i);\n            switch_left = switch_into(i);"),
    "lock_waiter_spins_when_busy_waiting": ("sleep on it: the core goes to the next task */\n    if (policy == 1) {",
                                            "sleep on it: the core goes to the next task */\n    if (policy == 1 && wait == 1) {"),
    "slice_never_expires": ("        } else if (slice_used == L) {", "        } else if (false) {"),
    "remove_does_not_hand_over": ("      running = k;\n      if (k >= 0) pending[k] = 0;", "      running = -1;"),
    "add_does_not_preempt": ("    } else if (higher_g(i, running)) {\n      pending[running] = 1;",
                             "    } else if (false) {\n      pending[running] = 1;"),
    "cpu_time_dealt_last_segments_longer": ("d.c.push_back(each + (j < longer ? 1 : 0));",
                                            "d.c.push_back(each + (j >= parts - longer ? 1 : 0));"),
    "busy_waiting_leaves_the_core": ("    if (ph == PH_GPU) return wait == 0; /* busy-waiting keeps the core */",
                                     "    if (ph == PH_GPU) return false;"),
    "suspended_task_keeps_the_core": ("    if (ph == PH_GPU) return wait == 0; /* busy-waiting keeps the core */",
                                      "    if (ph == PH_GPU) return true;"),
    "priority_order_reversed": ("return a.prio > b.prio; });", "return a.prio < b.prio; });"),
    "response_measured_from_time_zero": ("s.max_resp = std::max(s.max_resp, now_end - s.release);",
                                         "s.max_resp = std::max(s.max_resp, now_end);"),
    "overrun_not_detected": ("        if (s.active) {\n          overrun = true;", "        if (false) {\n          overrun = true;"),
    "planes_swapped": ("      for (int policy = 1; policy <= 2; ++policy) {", "      for (int policy = 2; policy >= 1; --policy) {"),
    "offsets_ignored": ("        d.offset = offset ? offset[at] : 0;", "        d.offset = 0;"),
    "update_takes_twice_the_delay": ("        st[g].remaining = eps;", "        st[g].remaining = 2 * eps;"),
    "gpu_serves_a_pending_task": ("        if (s.active && !s.in_update && s.ops[s.pc].ph == PH_GPU && s.remaining > 0) s.remaining--;",
                                  "        if (s.active && !s.in_update && s.ops[s.pc].ph == PH_GPU && s.remaining > 0) s.remaining--;\n"
                                  "        for (int x = 0; x < n; ++x) if (pending[x] && st[x].remaining > 0) st[x].remaining--;"),
}

SIM_PINS = [
    sim_tests.test_gcaps_preemption_by_hand,
    sim_tests.test_round_robin_slices_by_hand,
    sim_tests.test_cpu_time_is_dealt_to_the_segments_first_segments_longer,
    sim_tests.test_single_core_cpu_only_equals_the_textbook_recurrence,
    sim_tests.test_overrun_stops_the_taskset_and_is_flagged,
    sim_tests.test_simultaneous_arrivals_take_the_gpu_in_priority_order,
    sim_tests.test_gcaps_bound_misses_a_delayed_closing_update,
    sim_tests.test_a_task_waiting_for_the_driver_lock_sleeps_in_either_mode,
    lambda: des_tests.test_own_slice_switch_outside_eq3(des_tests.des.oracle),
]


@pytest.mark.parametrize("name", sorted(SIM_MUTANTS))
def test_simulator_mutant_is_rejected_by_some_pin(oracle, tmp_path, name):
    old, new = SIM_MUTANTS[name]
    src = open(SIM_SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    cpp = tmp_path / "mutant.cpp"
    cpp.write_text(src.replace(old, new))
    so = tmp_path / "libsimmutant.so"
    subprocess.run(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", "-pthread", "-o", str(so), str(cpp)], check=True)
    genuine = oracle.sim_library()
    oracle._sim = oracle.open_sim_library(str(so))
    killed_by = None
    try:
        for k, pin in enumerate(SIM_PINS):
            try:
                pin()
            except AssertionError:
                killed_by = k
                break
    finally:
        oracle._sim = genuine
    assert killed_by is not None, f"no pin notices the planted mistake '{name}'"


def test_unmutated_simulator_passes_the_same_pins():
    for pin in SIM_PINS:
        pin()
