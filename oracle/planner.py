"""Packing planner: memory model, packing of one job, DTM, job planner.  Test infrastructure only.

What is computed (paper section 3.2, appendices A, B and D), written out plainly and slowly:

* the memory of one LoRA configuration (appendix B);
* F(D, K) (section 3.2, the restricted problem with the parallel degree fixed): among the
  non-empty subsets H of the configurations K that fit the memory of D GPUs, the one with the
  largest  sum_k H_k r_k / T(H, D)  - by enumerating every subset;
* DTM (Alg. 1): the recursion over parallel degrees g', g'/2, .., 1, each step packing one job
  with F and recursing on the GPUs and configurations that are left; every leaf is a candidate
  set of concurrent jobs;
* the job planner (Alg. 2): whenever GPUs are free, DTM on the free GPUs and the remaining
  configurations; then time moves to the next job completion;
* the bound of the tail effect (appendix D, the theorem on the approximation ratio).

Readings where the paper leaves a choice:

* T(): the paper's notation table defines it as a job's duration according to a cost model and does
  not print that model.  Here the caller supplies it in the form the packed execution has: for degree d = 2^i,
  T(H, d) = t_base[i] + sum_k H_k t_config[i][k]  (the base model's share grows with the packed
  tokens, every adapter adds its own low-rank work).
* Alg. 1 returns the candidate p with the least T(p); a candidate is a set of concurrent jobs, not a
  whole schedule, so the only duration it has is that of the remaining rank-work at its rate.  The
  text says DTM maximises the instantaneous throughput (the section's first expression); both say
  the same: the candidate with the largest  sum_j F_j  is returned (first one wins a tie).
* A degree at which no configuration fits the memory packs no job; the recursion skips it.
* Appendix B, gradient memory: printed as c_grad x M_param x c_prec although M_param already is in
  bytes; read as c_grad x M_param (c_grad gradient-sized buffers: gradient, momentum, velocity).
  The sharded forms name M_grad and M_opt separately: M_grad = M_param (the gradient proper),
  M_opt = (c_grad - 1) M_param, which adds up to the unsharded total.
* Appendix B gives the activation memory b x s x r x c_prec per block: counted once per layer and
  per projection that carries an adapter.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from itertools import combinations
from typing import List, Optional, Sequence, Tuple

# the seven projections LoRA can be applied to (appendix B): q, k, v, o, up, gate, down
PROJECTIONS = ("q", "k", "v", "o", "up", "gate", "down")


@dataclass
class Model:
    n_layers: int
    hidden: int          # d_model
    kv_hidden: int       # width of k and v (grouped-query attention: smaller than hidden)
    inter: int           # MLP width
    c_prec: float = 2.0  # bytes per parameter
    c_grad: float = 3.0  # gradient-sized buffers per parameter (AdamW: gradient, momentum, velocity)

    def dims(self) -> List[Tuple[int, int]]:
        """(h_in, h_out) of the seven projections."""
        h, kv, m = self.hidden, self.kv_hidden, self.inter
        return [(h, h), (h, kv), (h, kv), (h, h), (h, m), (h, m), (m, h)]


def lora_param_bytes(model: Model, rank: int, targets: Sequence[bool]) -> float:
    """Appendix B: n_layers (h_in r + h_out r) c_prec, summed over the projections with an adapter."""
    total = 0.0
    for (h_in, h_out), on in zip(model.dims(), targets):
        if on:
            total += model.n_layers * (h_in * rank + h_out * rank) * model.c_prec
    return total


def lora_act_bytes(model: Model, rank: int, batch: int, seq: int, targets: Sequence[bool]) -> float:
    """Appendix B: b s r c_prec per block."""
    n = sum(1 for on in targets if on)
    return float(model.n_layers * n * batch * seq * rank * model.c_prec)


def lora_bytes(model: Model, rank: int, batch: int, seq: int, targets: Sequence[bool], zero: int = 0,
               d_tp: int = 1, d_pp: int = 1, d_fsdp: int = 1) -> float:
    """Memory of one configuration on one device (appendix B).  zero 0: nothing sharded by FSDP; 1, 2, 3: the
    ZeRO levels.  Tensor and pipeline parallelism divide the parameter-sized terms."""
    param = lora_param_bytes(model, rank, targets) / (d_tp * d_pp)
    grad = param
    opt = (model.c_grad - 1.0) * param
    act = lora_act_bytes(model, rank, batch, seq, targets)
    if zero == 0:
        return param + grad + opt + act
    if zero == 1:
        return grad + param + opt / d_fsdp + act
    if zero == 2:
        return param + (grad + opt) / d_fsdp + act
    if zero == 3:
        return (param + grad + opt) / d_fsdp + act
    raise ValueError("zero level")


@dataclass
class Problem:
    """K with what the planner needs of every configuration; degrees are 1, 2, 4, .. 2^(n_deg-1)."""
    rank: List[int]
    mem: List[float]                 # M_lora,k
    mem_base: float
    mem_gpu: float
    load: float                      # C
    t_base: List[float]              # [n_deg]
    t_config: List[List[float]]      # [n_deg][n]

    @property
    def n(self) -> int:
        return len(self.rank)


def duration(p: Problem, deg_idx: int, chosen: Sequence[int]) -> float:
    return p.t_base[deg_idx] + sum(p.t_config[deg_idx][k] for k in chosen)


def fits(p: Problem, deg_idx: int, chosen: Sequence[int]) -> bool:
    """Section 3.2, the memory constraint: M_base + sum M_lora,k <= C M_gpu D."""
    return p.mem_base + sum(p.mem[k] for k in chosen) <= p.load * p.mem_gpu * (1 << deg_idx)


def pack(p: Problem, deg_idx: int, avail: Sequence[int]) -> Tuple[Optional[Tuple[int, ...]], float]:
    """F(D, K) by enumeration: the best non-empty feasible subset of `avail` and its value; (None, 0) if none fits.
    Ties go to the subset met first (fewer members first, then lexicographic)."""
    best, best_v = None, 0.0
    for size in range(1, len(avail) + 1):
        for sub in combinations(avail, size):
            if not fits(p, deg_idx, sub):
                continue
            v = sum(p.rank[k] for k in sub) / duration(p, deg_idx, sub)
            if best is None or v > best_v:
                best, best_v = sub, v
    return best, best_v


@dataclass
class Job:
    configs: Tuple[int, ...]
    deg_idx: int
    value: float                     # its F
    start: float = 0.0
    end: float = 0.0

    @property
    def gpus(self) -> int:
        return 1 << self.deg_idx


def dtm(p: Problem, g: int, avail: Sequence[int]) -> List[Job]:
    """Alg. 1: every leaf of the recursion is a candidate; the one with the largest total throughput is returned."""
    leaves: List[List[Job]] = []

    def helper(g_left: int, tmp: List[Job], k_left: List[int]) -> None:
        if g_left <= 0 or not k_left:
            leaves.append(list(tmp))
            return
        top = g_left.bit_length() - 1                     # g' = 2^floor(log2 g)
        went = False
        for deg_idx in range(min(top, len(p.t_base) - 1), -1, -1):
            sub, v = pack(p, deg_idx, k_left)
            if sub is None:
                continue
            went = True
            helper(g_left - (1 << deg_idx), tmp + [Job(sub, deg_idx, v)], [k for k in k_left if k not in sub])
        if not went:
            leaves.append(list(tmp))                      # nothing fits on what is left

    helper(g, [], list(avail))
    best: List[Job] = []
    best_v = -1.0
    for leaf in leaves:
        v = sum(j.value for j in leaf)
        if v > best_v:
            best, best_v = leaf, v
    return best


@dataclass
class Schedule:
    jobs: List[Job] = field(default_factory=list)
    makespan: float = 0.0
    unscheduled: List[int] = field(default_factory=list)   # configurations that fit no degree


def plan(p: Problem, G: int) -> Schedule:
    """Alg. 2: the event loop.  Jobs that end at the same time free their GPUs together."""
    left = list(range(p.n))
    running: List[Job] = []
    out = Schedule()
    now, g_avail = 0.0, G
    while left:
        if g_avail > 0:
            for j in dtm(p, g_avail, left):
                j.start = now
                j.end = now + duration(p, j.deg_idx, j.configs)
                left = [k for k in left if k not in j.configs]
                g_avail -= j.gpus
                running.append(j)
                out.jobs.append(j)
        if not left:
            break
        if not running:                                   # nothing runs and nothing could be started
            out.unscheduled = left
            break
        now = min(j.end for j in running)
        for j in [j for j in running if j.end == now]:
            g_avail += j.gpus
            running.remove(j)
    out.makespan = max((j.end for j in out.jobs), default=0.0)
    return out


def tail_bound(s: Schedule, G: int) -> float:
    """Appendix D: AR <= F / (F - T_last (G - D) / G), with the job that ends last as the last job."""
    if not s.jobs:
        return 1.0
    last = max(s.jobs, key=lambda j: j.end)
    t_last = last.end - last.start
    return s.makespan / (s.makespan - t_last * (G - last.gpus) / G)


def gpu_work(s: Schedule) -> float:
    """W = sum_j x_j t_j (appendix D)."""
    return sum(j.gpus * (j.end - j.start) for j in s.jobs)
