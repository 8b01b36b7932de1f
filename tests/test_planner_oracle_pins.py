"""Pins of the planner oracle (oracle/planner.py): hand-worked values for the memory model of appendix B, for
F(D, K) of section 3.2 and for DTM (Alg. 1); closed forms for degenerate instances of the job planner (Alg. 2);
and the invariants every packing and every schedule must satisfy (disjoint configurations, memory and GPU limits,
makespan at least work / GPUs, the tail bound of appendix D where its premise holds).  Mutations a plausible mistake
would make (a dropped base term, the rank sum replaced by a count, memory compared without the degree) fail here."""
import json
import os

import numpy as np
import pytest

from oracle import planner as pl

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "planner_hand_worked.json")))


def gold_problem(**over):
    g = dict(GOLD["pack"], **over)
    return pl.Problem(g["rank"], g["mem"], g["mem_base"], g["mem_gpu"], g["load"], g["t_base"], g["t_config"])


def test_memory_model_hand_worked():
    m = GOLD["memory"]
    model = pl.Model(**m["model"])
    args = (model, m["rank"], m["batch"], m["seq"], m["targets"])
    assert pl.lora_param_bytes(model, m["rank"], m["targets"]) == m["param_bytes"]
    assert pl.lora_act_bytes(*args) == m["act_bytes"]
    assert pl.lora_bytes(*args) == m["total"]
    assert pl.lora_bytes(*args, zero=1, d_fsdp=4) == m["zero1_fsdp4"]
    assert pl.lora_bytes(*args, zero=2, d_fsdp=4) == m["zero2_fsdp4"]
    assert pl.lora_bytes(*args, zero=3, d_fsdp=4) == m["zero3_fsdp4"]
    assert pl.lora_bytes(*args, d_tp=2) == m["tp2"]
    # one shard is no sharding; memory is linear in the rank; all seven projections of a GQA model
    for z in (1, 2, 3):
        assert pl.lora_bytes(*args, zero=z, d_fsdp=1) == m["total"]
    assert pl.lora_bytes(model, 8, 2, 8, m["targets"]) == 2 * m["total"]
    full = pl.Model(32, 4096, 1024, 14336)
    per_layer = (4096 + 4096) * 2 + (4096 + 1024) * 2 + (4096 + 14336) * 2 + (14336 + 4096)
    assert pl.lora_param_bytes(full, 16, [True] * 7) == 32 * per_layer * 16 * 2.0


def test_pack_hand_worked():
    p = gold_problem()
    for deg_idx, key in ((0, "degree1"), (1, "degree2")):
        sub, v = pl.pack(p, deg_idx, [0, 1, 2])
        assert list(sub) == GOLD["pack"][key]["configs"]
        assert v == pytest.approx(GOLD["pack"][key]["value"], rel=1e-15)
    # nothing fits: base alone fills the GPU
    assert pl.pack(gold_problem(mem_base=4.5), 0, [0, 1, 2]) == (None, 0.0)
    # only a subset is on offer
    sub, v = pl.pack(p, 0, [0, 1])
    assert list(sub) == [0, 1] and v == pytest.approx(24 / 13)


def test_dtm_hand_worked():
    for key, over in (("dtm_g2", {}), ("dtm_g2_slow_pair", {k: GOLD["pack"]["dtm_g2_slow_pair"][k] for k in ("t_base", "t_config")})):
        want = GOLD["pack"][key]
        jobs = pl.dtm(gold_problem(**over), 2, [0, 1, 2])
        assert [{"configs": list(j.configs), "gpus": j.gpus} for j in jobs] == want["jobs"]
        assert sum(j.value for j in jobs) == pytest.approx(want["throughput"], rel=1e-15)


def test_plan_hand_worked_and_closed_forms():
    s = pl.plan(gold_problem(), 1)
    assert s.makespan == GOLD["pack"]["plan_g1"]["makespan"] and pl.tail_bound(s, 1) == GOLD["pack"]["plan_g1"]["tail_bound"]
    assert [list(j.configs) for j in s.jobs] == [[1, 2], [0]] and [j.start for j in s.jobs] == [0.0, 20.0]
    # n identical configurations, q of them fit a GPU, one GPU: F grows with the pack, so every job but the last is
    # full; ceil(n / q) jobs one after the other: makespan = jobs * t_base + n * t
    n, q, t0, t = 11, 4, 7.0, 1.5
    p = pl.Problem([16] * n, [1.0] * n, 0.5, float(q) + 0.5, 1.0, [t0], [[t] * n])
    s = pl.plan(p, 1)
    assert sorted(len(j.configs) for j in s.jobs) == [3, 4, 4]
    assert s.makespan == pytest.approx(3 * t0 + n * t)
    # memory for one configuration at a time: plain sequential training
    p = pl.Problem([8, 16, 32], [1.0] * 3, 0.0, 1.0, 1.0, [5.0], [[1.0, 2.0, 3.0]])
    assert pl.plan(p, 1).makespan == pytest.approx(3 * 5.0 + 6.0)
    # G GPUs, G configurations that each fill a GPU and take the same time: all at once
    p = pl.Problem([8] * 4, [1.0] * 4, 0.0, 1.0, 1.0, [5.0], [[2.0] * 4])
    s = pl.plan(p, 4)
    assert s.makespan == pytest.approx(7.0) and all(j.start == 0.0 for j in s.jobs)
    # a configuration that fits no degree is reported, the rest is scheduled
    p = pl.Problem([8, 8], [1.0, 9.0], 0.0, 1.0, 1.0, [5.0, 3.0], [[1.0, 1.0], [0.5, 0.5]])
    s = pl.plan(p, 2)
    assert s.unscheduled == [1] and [list(j.configs) for j in s.jobs] == [[0]]


def random_problem(rng, n, n_deg):
    rank = [int(r) for r in rng.choice([8, 16, 32, 64, 128], n)]
    mem = [float(r) * rng.uniform(0.8, 1.2) for r in rank]
    t_base = [float(rng.uniform(20, 40)) / (1.7 ** i) for i in range(n_deg)]
    t_config = [[float(r) * rng.uniform(0.05, 0.15) / (1.6 ** i) for r in rank] for i in range(n_deg)]
    return pl.Problem(rank, mem, float(rng.uniform(50, 150)), float(rng.uniform(200, 500)), 0.9, t_base, t_config)


@pytest.mark.parametrize("seed", range(6))
def test_invariants_of_packings_and_schedules(seed):
    rng = np.random.default_rng(4100 + seed)
    G = int(rng.choice([1, 2, 3, 4]))
    p = random_problem(rng, int(rng.integers(3, 9)), 3)
    jobs = pl.dtm(p, G, list(range(p.n)))
    used = [k for j in jobs for k in j.configs]
    assert len(used) == len(set(used)) and sum(j.gpus for j in jobs) <= G
    for j in jobs:
        assert pl.fits(p, j.deg_idx, j.configs)
        assert j.value == pytest.approx(sum(p.rank[k] for k in j.configs) / pl.duration(p, j.deg_idx, j.configs))
    # DTM is at least as good as packing one job at the largest degree that fits on G
    top = min(G.bit_length() - 1, 2)
    one = pl.pack(p, top, list(range(p.n)))[1]
    assert sum(j.value for j in jobs) >= one - 1e-12
    s = pl.plan(p, G)
    done = [k for j in s.jobs for k in j.configs]
    assert sorted(done + list(s.unscheduled)) == list(range(p.n))
    for j in s.jobs:
        assert pl.fits(p, j.deg_idx, j.configs) and j.end == pytest.approx(j.start + pl.duration(p, j.deg_idx, j.configs))
        assert sum(o.gpus for o in s.jobs if o.start <= j.start < o.end) <= G
    if s.jobs:
        lower = pl.gpu_work(s) / G
        assert s.makespan >= lower - 1e-9
        bound = pl.tail_bound(s, G)
        assert bound >= 1.0
        # appendix D: if every GPU is busy until the job that ends last starts, W >= G F_prev + D T_last, hence
        # F / (W / G) <= F / (F - T_last (G - D) / G)
        last = max(s.jobs, key=lambda j: j.end)
        busy_before = sum(o.gpus * (min(o.end, last.start) - min(o.start, last.start)) for o in s.jobs)
        if abs(busy_before - G * last.start) < 1e-9:
            assert s.makespan / lower <= bound + 1e-9


def test_mutations_of_the_definitions_fail():
    """What the hand-worked values catch: the same cases with a mistake planted in a copy of the definition."""
    p = gold_problem()

    def pack_with(value_of, fits_of):
        best, best_v = None, 0.0
        from itertools import combinations
        for size in (1, 2, 3):
            for sub in combinations([0, 1, 2], size):
                if fits_of(sub):
                    v = value_of(sub)
                    if best is None or v > best_v:
                        best, best_v = sub, v
        return best, best_v

    right = pack_with(lambda s: sum(p.rank[k] for k in s) / pl.duration(p, 0, s), lambda s: pl.fits(p, 0, s))
    assert list(right[0]) == [1, 2]
    no_base_time = pack_with(lambda s: sum(p.rank[k] for k in s) / sum(p.t_config[0][k] for k in s), lambda s: pl.fits(p, 0, s))
    count_not_rank = pack_with(lambda s: len(s) / pl.duration(p, 0, s), lambda s: pl.fits(p, 0, s))
    no_base_mem = pack_with(lambda s: sum(p.rank[k] for k in s) / pl.duration(p, 0, s), lambda s: sum(p.mem[k] for k in s) <= 4.0)
    assert list(no_base_time[0]) != [1, 2] or no_base_time[1] != pytest.approx(2.4)
    assert list(count_not_rank[0]) != [1, 2]
    assert list(no_base_mem[0]) != [1, 2]
