"""The packing planner of the library (plora_plan_*: host code, no GPU) against the oracle: the memory model value by
value, F(D, K) against the enumeration of every subset, DTM and the job planner against the oracle's recursion and
event loop on seeded random instances with real-valued costs (no two subsets tie), plus the hand-worked cases, the
closed forms, structural validity on instances full of ties, argument checks, and a search space of the paper's size."""
import ctypes as C
import json
import os
import time

import numpy as np
import pytest

from oracle import planner as opl
from paper_2508_02932_amd import plora

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "planner_hand_worked.json")))
REL = 1e-9      # both sides work in fp64; the parametric search stops when no subset beats the ratio by rounding


def both(rank, mem, mem_base, mem_gpu, load, t_base, t_config):
    return (opl.Problem(list(rank), list(mem), mem_base, mem_gpu, load, list(t_base), [list(r) for r in t_config]),
            plora.PlanProblem(rank, mem, mem_base, mem_gpu, load, t_base, t_config))


def random_instance(rng, n, n_deg):
    rank = [int(r) for r in rng.choice([8, 16, 32, 64, 128], n)]
    mem = [float(r) * rng.uniform(0.8, 1.2) for r in rank]
    t_base = [float(rng.uniform(20, 40)) / (1.7 ** i) for i in range(n_deg)]
    t_config = [[float(r) * rng.uniform(0.05, 0.15) / (1.6 ** i) for r in rank] for i in range(n_deg)]
    return both(rank, mem, float(rng.uniform(50, 150)), float(rng.uniform(200, 500)), 0.9, t_base, t_config)


def test_memory_model_equals_oracle():
    m = GOLD["memory"]
    bits = sum(1 << i for i, on in enumerate(m["targets"]) if on)
    cfg = {"rank": m["rank"], "batch": m["batch"], "seq": m["seq"], "targets": bits}
    assert plora.plora_plan_lora_bytes(m["model"], cfg) == m["total"]
    assert plora.plora_plan_lora_bytes(m["model"], cfg, dict(zero_level=3, d_tp=1, d_pp=1, d_fsdp=4)) == m["zero3_fsdp4"]
    assert plora.plora_plan_lora_bytes(m["model"], cfg, dict(zero_level=0, d_tp=2, d_pp=1, d_fsdp=1)) == m["tp2"]
    rng = np.random.default_rng(5)
    for _ in range(200):
        model = dict(n_layers=int(rng.integers(1, 80)), hidden=int(rng.integers(1, 9000)), kv_hidden=int(rng.integers(1, 9000)),
                     inter=int(rng.integers(1, 30000)), c_prec=float(rng.choice([2.0, 4.0])), c_grad=float(rng.choice([1.0, 2.0, 3.0])))
        bits = int(rng.integers(0, 128))
        cfg = dict(rank=int(rng.integers(1, 257)), batch=int(rng.integers(1, 65)), seq=int(rng.integers(1, 4097)), targets=bits)
        sh = dict(zero_level=int(rng.integers(0, 4)), d_tp=int(rng.choice([1, 2, 4, 8])), d_pp=int(rng.choice([1, 2, 4])),
                  d_fsdp=int(rng.choice([1, 2, 4, 8])))
        want = opl.lora_bytes(opl.Model(**model), cfg["rank"], cfg["batch"], cfg["seq"], [bool(bits >> i & 1) for i in range(7)],
                              sh["zero_level"], sh["d_tp"], sh["d_pp"], sh["d_fsdp"])
        assert plora.plora_plan_lora_bytes(model, cfg, sh) == pytest.approx(want, rel=1e-14)
    assert plora.plora_plan_lora_bytes(m["model"], dict(cfg, rank=0)) < 0
    assert plora.plora_plan_lora_bytes(m["model"], cfg, dict(zero_level=4, d_tp=1, d_pp=1, d_fsdp=1)) < 0


def test_hand_worked_cases():
    g = GOLD["pack"]
    _, p = both(g["rank"], g["mem"], g["mem_base"], g["mem_gpu"], g["load"], g["t_base"], g["t_config"])
    for deg, key in ((0, "degree1"), (1, "degree2")):
        job = plora.plora_plan_pack(p, deg)
        assert job["configs"] == g[key]["configs"] and job["value"] == pytest.approx(g[key]["value"], rel=1e-15) and job["proved"]
    jobs = plora.plora_plan_dtm(p, 2)
    assert [{"configs": j["configs"], "gpus": j["gpus"]} for j in jobs] == g["dtm_g2"]["jobs"]
    s = g["dtm_g2_slow_pair"]
    _, p2 = both(g["rank"], g["mem"], g["mem_base"], g["mem_gpu"], g["load"], s["t_base"], s["t_config"])
    jobs = plora.plora_plan_dtm(p2, 2)
    assert [{"configs": j["configs"], "gpus": j["gpus"]} for j in jobs] == s["jobs"]
    assert sum(j["value"] for j in jobs) == pytest.approx(s["throughput"], rel=1e-15)
    sch = plora.plora_plan_schedule(p, 1)
    assert sch["makespan"] == g["plan_g1"]["makespan"] and sch["tail_bound"] == g["plan_g1"]["tail_bound"]
    assert [j["configs"] for j in sch["jobs"]] == [[1, 2], [0]] and [j["start"] for j in sch["jobs"]] == [0.0, 20.0]
    # nothing fits
    _, p3 = both(g["rank"], g["mem"], 4.5, g["mem_gpu"], g["load"], g["t_base"][:1], g["t_config"][:1])
    assert plora.plora_plan_pack(p3, 0)["configs"] == []
    sch = plora.plora_plan_schedule(p3, 2)
    assert sch["jobs"] == [] and sorted(sch["unscheduled"]) == [0, 1, 2] and sch["makespan"] == 0.0


@pytest.mark.parametrize("seed", range(12))
def test_pack_equals_enumeration(seed):
    rng = np.random.default_rng(9000 + seed)
    n = int(rng.integers(1, 14))
    po, pc = random_instance(rng, n, 3)
    for deg in range(3):
        avail = sorted(rng.choice(n, size=int(rng.integers(1, n + 1)), replace=False).tolist())
        sub, v = opl.pack(po, deg, avail)
        job = plora.plora_plan_pack(pc, deg, avail)
        if sub is None:
            assert job["configs"] == []
            continue
        assert job["proved"]
        assert job["value"] == pytest.approx(v, rel=REL), (job, sub, v)
        assert job["configs"] == list(sub)                  # real-valued costs: the optimum is unique
        assert opl.fits(po, deg, job["configs"])


@pytest.mark.parametrize("seed", range(8))
def test_dtm_and_schedule_equal_oracle(seed):
    rng = np.random.default_rng(9100 + seed)
    n = int(rng.integers(2, 10))
    G = int(rng.choice([1, 2, 3, 4, 5, 8]))
    po, pc = random_instance(rng, n, int(rng.choice([1, 2, 3, 4])))
    want = opl.dtm(po, G, list(range(n)))
    got = plora.plora_plan_dtm(pc, G)
    assert [(list(j.configs), j.gpus) for j in want] == [(j["configs"], j["gpus"]) for j in got]
    assert sum(j["value"] for j in got) == pytest.approx(sum(j.value for j in want), rel=REL)
    ws = opl.plan(po, G)
    gs = plora.plora_plan_schedule(pc, G)
    assert gs["makespan"] == pytest.approx(ws.makespan, rel=REL)
    assert [(list(j.configs), j.gpus) for j in ws.jobs] == [(j["configs"], j["gpus"]) for j in gs["jobs"]]
    for a, b in zip(ws.jobs, gs["jobs"]):
        assert b["start"] == pytest.approx(a.start, rel=REL) and b["end"] == pytest.approx(a.end, rel=REL)
    assert gs["gpu_work"] == pytest.approx(opl.gpu_work(ws), rel=REL)
    assert gs["tail_bound"] == pytest.approx(opl.tail_bound(ws, G), rel=REL)
    assert sorted(gs["unscheduled"]) == sorted(ws.unscheduled) and gs["all_proved"]


def test_closed_forms_and_ties():
    # n identical configurations, q fit a GPU: ceil(n / q) jobs in a row, all but the last full
    n, q, t0, t = 11, 4, 7.0, 1.5
    _, p = both([16] * n, [1.0] * n, 0.5, q + 0.5, 1.0, [t0], [[t] * n])
    s = plora.plora_plan_schedule(p, 1)
    assert sorted(len(j["configs"]) for j in s["jobs"]) == [3, 4, 4] and s["makespan"] == pytest.approx(3 * t0 + n * t)
    assert sorted(k for j in s["jobs"] for k in j["configs"]) == list(range(n)) and s["all_proved"]
    # sequential training when one configuration fills the GPU
    _, p = both([8, 16, 32], [1.0] * 3, 0.0, 1.0, 1.0, [5.0], [[1.0, 2.0, 3.0]])
    assert plora.plora_plan_schedule(p, 1)["makespan"] == pytest.approx(21.0)
    # many interchangeable configurations (the shape of a hyperparameter sweep: learning rate and alpha change neither
    # memory nor time): the value of every packing still equals the enumeration's
    rng = np.random.default_rng(77)
    rank = [int(r) for r in rng.choice([8, 16, 32], 12)]
    po, pc = both(rank, [float(r) for r in rank], 10.0, 100.0, 0.8, [30.0, 18.0], [[0.1 * r for r in rank], [0.06 * r for r in rank]])
    for deg in (0, 1):
        sub, v = opl.pack(po, deg, list(range(12)))
        job = plora.plora_plan_pack(pc, deg)
        assert job["value"] == pytest.approx(v, rel=REL) and opl.fits(po, deg, job["configs"]) and job["proved"]


def test_argument_checks():
    L = plora.lib()
    g = GOLD["pack"]
    _, p = both(g["rank"], g["mem"], g["mem_base"], g["mem_gpu"], g["load"], g["t_base"], g["t_config"])
    cfg = np.zeros(3, dtype=np.int32)
    job = plora.plora_plan_job()
    assert L.plora_plan_pack(None, 0, None, cfg.ctypes.data, C.byref(job)) == 1
    assert L.plora_plan_pack(p.ref, 0, None, None, C.byref(job)) == 1
    assert L.plora_plan_pack(p.ref, 2, None, cfg.ctypes.data, C.byref(job)) == 2
    assert L.plora_plan_pack(p.ref, -1, None, cfg.ctypes.data, C.byref(job)) == 2
    for bad in (dict(load=0.0), dict(load=1.5), dict(mem_gpu=0.0), dict(mem_base=-1.0), dict(rank=[8, 0, 32]),
                dict(t_config=[[1.0, 0.0, 8.0], [0.6, 1.2, 4.5]]), dict(t_base=[10.0, float("nan")]), dict(mem=[1.0, -2.0, 1.0])):
        gg = dict(g, **bad)
        _, pb = both(gg["rank"], gg["mem"], gg["mem_base"], gg["mem_gpu"], gg["load"], gg["t_base"], gg["t_config"])
        assert L.plora_plan_pack(pb.ref, 0, None, cfg.ctypes.data, C.byref(job)) == 2, bad
    n = C.c_int32(0)
    jobs = (plora.plora_plan_job * 4)()
    assert L.plora_plan_dtm(p.ref, 0, None, C.cast(jobs, C.c_void_p), 4, C.byref(n), cfg.ctypes.data) == 2
    s = plora.plora_plan_summary()
    assert L.plora_plan_schedule(p.ref, 1, C.cast(jobs, C.c_void_p), 1, cfg.ctypes.data, C.byref(s)) == 7     # two jobs, room for one
    assert L.plora_plan_schedule(p.ref, 1, C.cast(jobs, C.c_void_p), 4, cfg.ctypes.data, None) == 1


def test_search_space_of_the_papers_size():
    """120 configurations on 8 GPUs (the size of the paper's evaluation, whose planner ran within ten minutes): the
    schedule is valid, its makespan lies between work / GPUs and the sequential sum, and planning takes seconds."""
    rng = np.random.default_rng(120)
    n, G = 120, 8
    rank = rng.choice([8, 16, 32, 64, 128], n)
    tokens = rng.choice([1, 2, 4, 8], n) * 1024
    mem = rank * 3.0e6 * 4 + tokens * rank * 2.0 * 32 * 7
    t_config = np.array([(tokens * 6.0e-5 + rank * tokens * 2.0e-8) / (1.8 ** i) for i in range(4)])
    t_base = [4.0e-3 * (0.7 ** i) for i in range(4)]
    p = plora.PlanProblem(rank, mem, 16.0e9, 80.0e9, 0.9, t_base, t_config)
    t0 = time.time()
    s = plora.plora_plan_schedule(p, G)
    dt = time.time() - t0
    assert dt < 120.0, dt
    assert sorted(k for j in s["jobs"] for k in j["configs"]) == list(range(n)) and not s["unscheduled"]
    cap = lambda g: 0.9 * 80.0e9 * g - 16.0e9
    for j in s["jobs"]:
        assert mem[j["configs"]].sum() <= cap(j["gpus"]) and j["gpus"] in (1, 2, 4, 8)
        assert sum(o["gpus"] for o in s["jobs"] if o["start"] <= j["start"] < o["end"]) <= G
    assert s["gpu_work"] / G <= s["makespan"] * (1 + 1e-12)
    assert s["makespan"] <= float(t_base[0] * n + t_config[0].sum())
    assert s["tail_bound"] >= 1.0
