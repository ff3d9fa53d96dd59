"""Are the pins strong enough?  Every entry below plants one plausible mistake in a COPY of the
oracle's C source (CPU only, in a temporary directory), builds it, and runs the pin tests against
the mutated copy: at least one pin must fail.  The committed oracle itself is never modified."""
import importlib.util
import os
import shutil
import sys

import pytest

from tests import test_oracle_consistent as pins_consistent
from tests import test_oracle_pins as pins
from tests import test_oracle_priority as pins_priority
from tests import test_oracle_ranked as pins_ranked
from tests import test_oracle_reactive as pins_reactive
from tests import test_oracle_sub as pins_sub
from tests import test_oracle_window as pins_window

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in oracle/pard_oracle.c, replacement, pins that must notice)
MUTATIONS = [
    ("floor instead of ceil of a/B", "int64_t batches_ahead = (a + B - 1) / B;", "int64_t batches_ahead = a / B;", "core"),
    ("divide by W before multiplying", "((wide_t)batches_ahead * (wide_t)lat[B - 1]) / (wide_t)W;",
     "((wide_t)batches_ahead / (wide_t)W) * (wide_t)lat[B - 1];", "core"),
    ("execution at the full batch size", "int64_t b_seen = (a + 1 < B) ? a + 1 : B;", "int64_t b_seen = B;", "core"),
    ("execution at batch a instead of a+1", "int64_t b_seen = (a + 1 < B) ? a + 1 : B;",
     "int64_t b_seen = (a + 1 < B) ? (a > 0 ? a : 1) : B;", "core"),
    ("ties by descending index", "if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;",
     "if (a->idx != b->idx) return a->idx > b->idx ? -1 : 1;", "core"),
    ("HBF sorted like LBF", "if (M[s] == MODE_HBF) key = -(int64_t)deadline[r];", "if (M[s] == MODE_HBF) key = (int64_t)deadline[r];", "core"),
    ("FCFS keyed by deadline", "else if (M[s] == MODE_FCFS) key = (int64_t)arrival[r];", "else if (M[s] == MODE_FCFS) key = (int64_t)deadline[r];", "core"),
    ("minimum over paths", "                if (sum > best) best = sum;\n            }\n            wide_t cap = (wide_t)INT32_MAX;",
     "                if (best < 0 || sum < best) best = sum;\n            }\n            wide_t cap = (wide_t)INT32_MAX;", "core"),
    ("downstream stage at the request's own position", "sum += stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], ahead[i]);\n                }\n                if (sum > best) best = sum;\n            }\n            wide_t cap",
     "sum += stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], pos);\n                }\n                if (sum > best) best = sum;\n            }\n            wide_t cap", "core"),
    ("current stage counted twice", "for (int32_t t = at + 1; t < b; ++t) {\n                    int32_t i = ps.stage[t];\n                    sum += stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], ahead[i]);\n                }\n                if (sum > best) best = sum;\n            }\n            wide_t cap",
     "for (int32_t t = at; t < b; ++t) {\n                    int32_t i = ps.stage[t];\n                    sum += stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], ahead[i]);\n                }\n                if (sum > best) best = sum;\n            }\n            wide_t cap", "core"),
    ("now not added", "wide_t finish = (wide_t)now[u] + best;", "wide_t finish = best;", "core"),
    ("drop at equality", "drop[r] = (uint8_t)(finish > (wide_t)deadline[r]);", "drop[r] = (uint8_t)(finish >= (wide_t)deadline[r]);", "core"),
    ("compaction keeps the dropped", "if (!drop[r]) surv_idx[out++] = r;", "if (drop[r]) surv_idx[out++] = r;", "core"),
    ("position counts everybody in the consistent variant", "if (consistent && !drop[r]) kept[k] += 1;", "if (consistent) kept[k] += 1;", "consistent"),
    ("position counts the dropped in the consistent variant", "if (consistent && !drop[r]) kept[k] += 1;", "if (consistent && drop[r]) kept[k] += 1;", "consistent"),
    ("batch wait is the time since the last batch", "total += (uint64_t)((di - arr % di) % di);", "total += (uint64_t)(arr % di);", "sub"),
    ("quantile rank one too high", "w = (wide_t)T[rank - 1];", "w = (wide_t)T[rank < M ? rank : M - 1];", "sub"),
    ("one draw for all stages of a sample", "int64_t arr = samples[picks[j * S + i] % (uint64_t)M];", "int64_t arr = samples[picks[j * S] % (uint64_t)M];", "sub"),
    ("draws indexed stage-major", "int64_t arr = samples[picks[j * S + i] % (uint64_t)M];", "int64_t arr = samples[picks[(int64_t)i * M + j] % (uint64_t)M];", "sub"),
    ("upper variant adds the durations once", "else if (variant == 2) lsub = sum_qd + sum_d;", "else if (variant == 2) lsub = sum_qd;", "sub"),
    ("sf variant keeps the queueing delay", "else if (variant == 3) lsub = sum_d;", "else if (variant == 3) lsub = sum_qd;", "sub"),
    ("duration at the full batch size", "int64_t seen = (int64_t)nq[i] + 1 < B[i] ? (int64_t)nq[i] + 1 : B[i];\n                    wide_t d_i", "int64_t seen = B[i];\n                    wide_t d_i", "sub"),
    ("sum over paths instead of maximum (downstream latency)", "if (lsub > best) best = lsub;", "best += lsub;", "sub"),
    ("no hysteresis: LBF whenever not above the upper threshold", "else if (lhs < lo) mode = MODE_LBF;", "else mode = MODE_LBF;", "priority"),
    ("epsilon from the window sum instead of its mean", "wide_t ts = win / (t - lo + 1);", "wide_t ts = win;", "priority"),
    ("thresholds without epsilon", "hi = W * B * 1000000 * (sum + dev);\n                lo = W * B * 1000000 * (sum - dev);",
     "hi = W * B * 1000000 * sum;\n                lo = W * B * 1000000 * sum;", "priority"),
    ("throughput ignores the worker count", "hi = W * B * 1000000 * (sum + dev);", "hi = B * 1000000 * (sum + dev);", "priority"),
    ("previous priority ignored", "int32_t mode = prev_mode ? prev_mode[g] : MODE_LBF;", "int32_t mode = MODE_LBF;", "priority"),
    ("ties in a later queue go to the newcomer", "if (M[i] == MODE_HBF ? other >= deadline[r] : other <= deadline[r]) ahead[i] += 1;",
     "if (M[i] == MODE_HBF ? other > deadline[r] : other < deadline[r]) ahead[i] += 1;", "ranked"),
    ("later high-budget-first queues ranked like low-budget-first ones", "if (M[i] == MODE_HBF ? other >= deadline[r] : other <= deadline[r]) ahead[i] += 1;",
     "if (other <= deadline[r]) ahead[i] += 1;", "ranked"),
    ("later arrival-order queues ranked by deadline", "if (!ranked || M[i] == MODE_FCFS) continue;", "if (!ranked) continue;", "ranked"),
    ("ranked places ignored", "sum += stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], ahead[i]);",
     "sum += stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], qlen[i]);", "ranked"),
    ("old samples weigh most", "wide_t w = window - age;", "wide_t w = age + 1;", "window"),
    ("plain mean inside the window", "wide_t w = window - age;", "wide_t w = 1;", "window"),
    ("samples later than now counted", "if (age < 0 || age >= window) continue;", "if (age >= window) continue;", "window"),
    ("window never ends", "if (age < 0 || age >= window) continue;", "if (age < 0) continue;", "window"),
    ("negative delays kept", "wide_t x = delay[g * len + j] > 0 ? delay[g * len + j] : 0;", "wide_t x = delay[g * len + j];", "window"),
    ("every series seen from the first snapshot's clock", "wide_t age = (wide_t)now[g / S] - time[g * len + j];",
     "wide_t age = (wide_t)now[0] - time[g * len + j];", "window"),
    ("monitored delay on top of the queue-length term", "sum_qd += (q_i > 0 ? q_i : 0) + d_i;",
     "sum_qd += (q_i > 0 ? q_i : 0) + stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], nq[i]);", "window"),
    ("monitored delay without the execution duration", "sum_qd += (q_i > 0 ? q_i : 0) + d_i;", "sum_qd += (q_i > 0 ? q_i : 0);", "window"),
    ("window scan: every window takes the full batch's latency", "const wide_t batch_end = (wide_t)now[u] + (wide_t)lat[w - 1];",
     "const wide_t batch_end = (wide_t)now[u] + (wide_t)lat[B - 1];", "reactive"),
    ("window scan: a request on its deadline is late", "if (batch_end > (wide_t)deadline[order[a + p + i]]) all_meet = 0;",
     "if (batch_end >= (wide_t)deadline[order[a + p + i]]) all_meet = 0;", "reactive"),
    ("window scan: only the window's first request is looked at", "for (int64_t i = 0; i < w; ++i)\n                    if (batch_end >",
     "for (int64_t i = 0; i < 1; ++i)\n                    if (batch_end >", "reactive"),
    ("window scan: the window itself is dropped too", "drop_out[order[a + j]] = j < first ? 1 : 0;", "drop_out[order[a + j]] = j <= first ? 1 : 0;", "reactive"),
    ("window scan: the queue is read by request index", "if (batch_end > (wide_t)deadline[order[a + p + i]]) all_meet = 0;",
     "if (batch_end > (wide_t)deadline[a + p + i]) all_meet = 0;", "reactive"),
    ("window scan: now left out", "const wide_t batch_end = (wide_t)now[u] + (wide_t)lat[w - 1];", "const wide_t batch_end = (wide_t)lat[w - 1];", "reactive"),
    ("SLO split: the current module's own budget left out", "for (int32_t t = ps.ptr[q]; t <= e; ++t) {", "for (int32_t t = ps.ptr[q]; t < e; ++t) {", "reactive"),
    ("SLO split: shortest way in instead of the longest", "if (in > longest_in) longest_in = in;", "if (longest_in < 0 || in < longest_in) longest_in = in;", "reactive"),
    ("SLO split: durations at batch size one", "in += lat_us[rec * LAT_ENTRIES + batch[rec] - 1];", "in += lat_us[rec * LAT_ENTRIES];", "reactive"),
    ("SLO split: the whole SLO at every module", "else drop_out[r] = used * whole[rec] > slo * way_in[rec] ? 1 : 0;", "else drop_out[r] = used > slo ? 1 : 0;", "reactive"),
    ("SLO split: dropped already when the budget is just used up", "else drop_out[r] = used * whole[rec] > slo * way_in[rec] ? 1 : 0;",
     "else drop_out[r] = used * whole[rec] >= slo * way_in[rec] ? 1 : 0;", "reactive"),
    ("SLO split: the deadline taken for the SLO", "const wide_t slo = (wide_t)deadline[r] - (wide_t)arrival[r];", "const wide_t slo = (wide_t)deadline[r];", "reactive"),
]


def load_mutant(tmp_path, old, new):
    dst = os.path.join(tmp_path, "oracle_mutant")
    shutil.copytree(os.path.join(ROOT, "oracle"), dst, ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    src = os.path.join(dst, "pard_oracle.c")
    text = open(src).read()
    assert text.count(old) >= 1, "the mutation does not apply to the oracle source any more"
    open(src, "w").write(text.replace(old, new))
    name = "oracle_mutant_" + os.path.basename(str(tmp_path))
    spec = importlib.util.spec_from_file_location(name, os.path.join(dst, "__init__.py"), submodule_search_locations=[dst])
    mod = importlib.util.module_from_spec(spec)
    sys.modules[name] = mod
    spec.loader.exec_module(mod)
    mod.build_oracle(force=True)
    return mod


def core_pins(m):
    pins.test_hand_vector_diamond(m)
    for seed in range(24):
        pins.test_bruteforce_small_random(m, seed)
    pins.test_stage_cost_against_batch_simulation(m)
    pins.test_linear_pipeline_is_single_suffix_sum(m)
    pins.test_lone_request_sees_batch1_latencies(m)
    pins.test_single_stage_unit_batch_is_rank_times_latency(m)
    pins.test_infinite_deadline_never_dropped_and_saturation(m)
    pins.test_permutation_invariance(m)
    pins.test_compaction_invariants(m)


def consistent_pins(m):
    pins_consistent.test_hand_worked_queue(m)
    for seed in range(20):
        pins_consistent.test_brute_force(m, seed)


def sub_pins(m):
    pins_sub.test_paper_printed_quantiles(m)
    pins_sub.test_single_module_exact(m)
    for seed in range(16):
        pins_sub.test_brute_force_random_dags(m, seed)
    pins_sub.test_variant_identities_and_bounds(m)


def priority_pins(m):
    pins_priority.test_hand_worked_series(m)
    pins_priority.test_delayed_transition_holds_inside_the_band(m)
    pins_priority.test_constant_load_closed_form(m)
    for seed in range(12):
        pins_priority.test_brute_force(m, seed)


def window_pins(m):
    pins_window.test_hand_worked_windows(m)
    pins_window.test_constant_delay_is_its_own_mean(m)
    pins_window.test_equally_spaced_linear_trend_closed_form(m)
    pins_window.test_order_and_padding_do_not_matter(m)
    for seed in range(12):
        pins_window.test_brute_force(m, seed)
    pins_window.test_monitored_delay_replaces_the_queue_term(m)


def ranked_pins(m):
    pins_ranked.test_hand_worked_two_stages(m)
    for seed in range(24):
        pins_ranked.test_bruteforce_small_random(m, seed)
    pins_ranked.test_equals_the_plain_estimate_when_it_must(m)
    pins_ranked.test_never_above_the_plain_estimate_with_rising_tables(m)


def reactive_pins(m):
    pins_reactive.test_nexus_hand_worked_queues(m)
    pins_reactive.test_nexus_closed_forms(m)
    for seed in range(16):
        pins_reactive.test_nexus_brute_force(m, seed)
    pins_reactive.test_nexus_invariants(m)
    pins_reactive.test_clipper_hand_worked(m)
    pins_reactive.test_clipper_single_module_is_the_plain_rule(m)
    for seed in range(16):
        pins_reactive.test_clipper_brute_force(m, seed)


GROUPS = {"core": core_pins, "reactive": reactive_pins, "ranked": ranked_pins, "consistent": consistent_pins, "sub": sub_pins, "priority": priority_pins,
          "window": window_pins}


@pytest.mark.parametrize("name,old,new,group", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, group):
    mutant = load_mutant(str(tmp_path), old, new)
    with pytest.raises((AssertionError, ValueError)):
        GROUPS[group](mutant)


def test_unmodified_copy_passes(tmp_path):
    """The harness itself: a copy without a planted mistake passes every group."""
    clean = load_mutant(str(tmp_path), "#define LAT_ENTRIES 64", "#define LAT_ENTRIES 64 ")
    for run in GROUPS.values():
        run(clean)
