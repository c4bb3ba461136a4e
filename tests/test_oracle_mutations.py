"""The pins must notice a plausible mistake in the oracle: each case plants one in a copy of
the oracle's sources (on the CPU, in a temporary directory), builds the copy and runs the pin
file that covers the spot in a child process, which has to fail."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SOURCES = ("sailor_oracle.c", "sailor_search_oracle.c", "sailor_oracle.h")

# the pins of the search with a TP degree per stage, and of the one with two pools as well
TP_PINS = "tp_per_stage or own_tp or two_degrees or one_degree_to_choose"
BOTH_PINS = "two_pools_and_a_tp or combined_search"

MUTANTS = [
    # (pin file, text in the oracle's source, replacement[, source file if not the default[, a -k
    # expression that selects the pins of that part of the file, to keep the run short]])
    ("test_oracle_simulator.py", "(double)(Nb - 1) * max_t", "(double)(Nb) * max_t"),
    ("test_oracle_simulator.py", "2.0 * (double)(D - 1) / (double)D * grad_bytes",
     "2.0 * (double)(D) / (double)D * grad_bytes"),
    ("test_oracle_simulator.py", "if (i == P - 1) params += p->head_params;", ""),
    ("test_oracle_simulator.py", "int64_t inflight = (P - i) < Nb ? (P - i) : Nb;", "int64_t inflight = (P - i);"),
    ("test_oracle_simulator.py", "(p->egress_per_byte[(size_t)z * Z + zn] + p->egress_per_byte[(size_t)zn * Z + z])",
     "(p->egress_per_byte[(size_t)z * Z + zn])"),
    ("test_oracle_space.py", "g.pool[1] = (g.pool[0] + 1 + rel) % c->ZG;\n    if",
     "g.pool[1] = (g.pool[0] + rel) % c->ZG;\n    if"),
    ("test_oracle_selection.py", "vmin * (1.0 + SO_TIE_TOL)", "vmin"),
    ("test_oracle_per_segment_tp.py", "tp_of[i] = g->seg_tp[seg];", "tp_of[i] = g->seg_tp[0];"),
    ("test_oracle_bandwidth.py", "const double x = log2(bytes);", "const double x = log(bytes);"),
    ("test_oracle_event_schedule.py", "double start = free_at[i] > dep ? free_at[i] : dep;", "double start = dep;"),
    ("test_oracle_event_schedule.py", "int64_t w = (P - 1 - i) < M ? (P - 1 - i) : M;\n  if (pos < w)",
     "int64_t w = (P - i) < M ? (P - i) : M;\n  if (pos < w)"),
    ("test_oracle_mixed_types.py", "half_gpus_on_pool[zone_of[i] * G + type_b[i]] += tp_of[i];", ""),
    ("test_oracle_mixed_types.py", "if (f2 + b2 > f + b) { f = f2; b = b2; }\n    }\n    double x = 0.0;",
     "if (f2 + b2 < f + b) { f = f2; b = b2; }\n    }\n    double x = 0.0;"),
    # replicas of a stage over two pools: the fastest link instead of the slowest, all replicas
    # charged on one kind of pipeline, the last kind of pipeline instead of the slower
    ("test_oracle_split_replicas.py", "if (others[k] < link) link = others[k];",
     "if (others[k] > link) link = others[k];"),
    ("test_oracle_split_replicas.py", "(0.5 * (double)replicas) * msg", "((double)replicas) * msg"),
    ("test_oracle_split_replicas.py", "if (t_kind > t_pipe) t_pipe = t_kind;", "t_pipe = t_kind;"),
    # ... with a TP degree per stage: the second half's GPUs counted as one per replica, the
    # first stage's degree for every stage's activations, update time and rent
    ("test_oracle_split_replicas.py", "halves[pools_b[i]] += width;", "halves[pools_b[i]] += 1;"),
    ("test_oracle_split_replicas.py", "p->act_store_bytes[(size_t)mb_idx * p->n_tp + tp_idx[i]];",
     "p->act_store_bytes[(size_t)mb_idx * p->n_tp + tp_idx[0]];"),
    ("test_oracle_split_replicas.py", "const double u = upd_time_sum(p, gt, tp_idx[i], first_of[i], nl[i]);",
     "const double u = upd_time_sum(p, gt, tp_idx[0], first_of[i], nl[i]);"),
    ("test_oracle_split_replicas.py", "rent += (double)(replicas * (int64_t)p->tp_values[tp_idx[i]]) *",
     "rent += (double)(replicas * (int64_t)p->tp_values[tp_idx[0]]) *"),
    # a pool per replica with a TP degree per stage: one GPU per replica against the quota, the
    # first stage's degree for every stage's rent, the descriptor-less times of stage 0 everywhere
    ("test_oracle_replica_placements.py", "gpus[a] += degree;", "gpus[a] += 1;"),
    ("test_oracle_replica_placements.py", "rent += (double)p->tp_values[tp_idx[i]] * p->price_per_hour[gt];",
     "rent += (double)p->tp_values[tp_idx[0]] * p->price_per_hour[gt];"),
    ("test_oracle_replica_placements.py", "const int64_t degree = p->tp_values[tp_idx[i]];",
     "const int64_t degree = p->tp_values[tp_idx[0]];"),
    # the search: a bound that is not one, a forgotten transfer, a quota that is never full,
    # the beam's order
    ("test_oracle_search.py", "const double tsum = (st->sum + t_open) + s->Ssum[i];",
     "const double tsum = (st->sum + t_open) + 1.5 * s->Ssum[i];"),
    ("test_oracle_search.py", "st->xb_open = s->xfer[z][zp];", "st->xb_open = 0.0;"),
    ("test_oracle_search.py", "par->cnt[a] + 1 > s->cap_cnt[a]", "par->cnt[a] > s->cap_cnt[a]"),
    ("test_oracle_search.py", "if (a->key < b->key) return -1;\n  if (a->key > b->key) return 1;",
     "if (a->key < b->key) return 1;\n  if (a->key > b->key) return -1;"),
    ("test_oracle_search.py", "s->Smax[i] = fmax(s->Smax[i + 1], cmin[i + 1]);",
     "s->Smax[i] = fmax(s->Smax[i + 1], cmin[i]);", "sailor_search_oracle.c",
     "bounds_never_exceed or first_bound_is_the_value"),
    # a TP degree per stage: the quota counted in stages instead of GPUs, the rent of the first
    # degree, runs that ignore the degree, every stage evaluated at the first stage's degree
    ("test_oracle_search.py", "par->cnt[a] + s->tpv[t] > s->cap_gpus[a]", "par->cnt[a] + 1 > s->cap_gpus[a]",
     "sailor_search_oracle.c", TP_PINS),
    ("test_oracle_search.py", "st->dol = par->dol + s->dol3[g][t];", "st->dol = par->dol + s->dol3[g][0];",
     "sailor_search_oracle.c", TP_PINS),
    ("test_oracle_search.py", "(a != par->pool || t != par->tpi) ? 1 : 0", "(a != par->pool) ? 1 : 0",
     "sailor_search_oracle.c", TP_PINS),
    ("test_oracle_search.py", "tp_of[i] = p->tp_values[tp_idx[i]];", "tp_of[i] = p->tp_values[tp_idx[0]];",
     "sailor_oracle.c", TP_PINS),
    # two pools and a TP degree per stage: a stage on one pool counted once, the first pool's price
    # for both halves, runs that ignore the degree
    ("test_oracle_search.py", "if (a == b) return cnt[a] + 2 * width <= s->cap_half_gpus[a];",
     "if (a == b) return cnt[a] + width <= s->cap_half_gpus[a];", "sailor_search_oracle.c", BOTH_PINS),
    ("test_oracle_search.py", "*dol = (double)(s->D * s->tpv[t]) * (0.5 * (s->price[ga] + s->price[gb]));",
     "*dol = (double)(s->D * s->tpv[t]) * s->price[ga];", "sailor_search_oracle.c", BOTH_PINS),
    ("test_oracle_search.py", "(a != par->pool || b != par->pool_b || t != par->tpi) ? 1 : 0",
     "(a != par->pool || b != par->pool_b) ? 1 : 0", "sailor_search_oracle.c", BOTH_PINS),
    # a pool per replica: a ring that is not closed, its fastest link, the last pipeline instead of
    # the slowest, replicas counted instead of GPUs, the ring's traffic priced in the wrong direction
    ("test_oracle_replica_placements.py", "(r + 1) % D] / G;", "(r + 1 < D ? r + 1 : r)] / G;"),
    ("test_oracle_replica_placements.py", "if (w < link) link = w;", "if (w > link || link == INFINITY) link = w;"),
    ("test_oracle_replica_placements.py", "if (t_this > t_pipe) t_pipe = t_this;", "t_pipe = t_this;"),
    ("test_oracle_replica_placements.py", "traffic_cost += ring_bytes * fee[(size_t)zr * Z + zs];",
     "traffic_cost += ring_bytes * fee[(size_t)zs * Z + zr];"),
]


@pytest.mark.parametrize("mutant", MUTANTS, ids=[f"{m[0][12:-3]}-{i}" for i, m in enumerate(MUTANTS)])
def test_a_planted_mistake_fails_its_pins(tmp_path, mutant):
    pins, old, new = mutant[:3]
    for f in SOURCES:
        shutil.copy(os.path.join(ROOT, "oracle", f), tmp_path / f)
    target = mutant[3] if len(mutant) > 3 else (
        "sailor_search_oracle.c" if pins == "test_oracle_search.py" else "sailor_oracle.c")
    src = (tmp_path / target).read_text()
    assert src.count(old) == 1, "the mutation no longer matches the oracle's source"
    (tmp_path / target).write_text(src.replace(old, new))
    env = dict(os.environ, SAILOR_ORACLE_DIR=str(tmp_path))
    select = ["-k", mutant[4]] if len(mutant) > 4 else []
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pins), "-x", "-q",
                          "-p", "no:cacheprovider"] + select, cwd=ROOT, env=env, capture_output=True, text=True)
    assert run.returncode == 1, "the pins passed on a broken oracle:\n" + run.stdout[-2000:]
    assert " failed" in run.stdout


def test_the_unmodified_copy_passes(tmp_path):
    # the harness itself: the same route with nothing planted is green
    for f in SOURCES:
        shutil.copy(os.path.join(ROOT, "oracle", f), tmp_path / f)
    env = dict(os.environ, SAILOR_ORACLE_DIR=str(tmp_path))
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_bandwidth.py"),
                          "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    assert run.returncode == 0, run.stdout[-2000:]
