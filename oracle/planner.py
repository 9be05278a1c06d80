"""CPU oracle of the input-aware checkpointing planner (TEST INFRASTRUCTURE ONLY).

This file is test infrastructure: only tests, the smoke check and the bench's
cpu_baseline leg may import it.  It shares no code with the HIP library.

The planner is a heuristic, so the oracle takes the paper's steps in the
paper's order:

  * two-phase execution (Section 4.1): "sheltered" iterations run with every
    layer checkpointed and record per-layer memory; afterwards "responsive"
    iterations look a plan up in a cache keyed by input size, generating it on a
    miss;
  * lightning memory estimator (Section 4.3): per layer, a polynomial of order
    2 in the input size x (number of elements of the input tensor, Section 3.1)
    fitted by least squares to the collected samples;
  * responsive memory scheduler (Section 4.4, Algorithm 1): layers sorted by
    estimated size (descending) are grouped into buckets of sizes within 10 %
    of the bucket's first member, each bucket ordered by forward position;
    layers are then picked until the excess over the budget is covered: the
    bucket whose largest member is nearest above the excess supplies its
    earliest layer, or, when no single layer covers the excess, the earliest
    layer of the largest bucket is taken;
  * plan cache (Section 5);
  * optional use of the collected forward times (Section 4.1 has the collector
    record each layer's forward time and the scheduler work from memory and
    time; Algorithm 1 itself never reads the time): see "cost-aware" below.

Readings where the paper is silent:
  - the per-layer quantity the algorithm ranks and subtracts is the droppable
    part s_l = a_l - b_l (bytes kept when not checkpointed minus bytes kept when
    checkpointed);
  - the budget is compared with a simulated step peak (below) that includes the
    fixed bytes, the embedding stage and the head; the initial excess is
    peak(no checkpoint) - budget; after the greedy loop ends the peak of the
    chosen plan is re-evaluated and the loop continues while it still exceeds
    the budget (late layers do not lower the backward peak, Section 4.4,
    discussion of the per-encoder peak figure);
  - predictions are rounded to the nearest 256 bytes plus a fixed guard and all
    comparisons are integer;
  - ties in the descending sort are broken by forward position;
  - cost-aware selection: the bucket is chosen exactly as Algorithm 1 chooses
    it, by memory; inside that bucket, whose members free about the same
    amount, the layer taken is the earliest of those whose estimated forward
    time is within the bucket tolerance (10 %) of the bucket's cheapest
    remaining layer.  With equal times this is Algorithm 1.

Peak model of one step under plan C (LIFO activation stack):
    kept_l(C) = sum_{j<l, j not in C} a_j + sum_{j<l, j in C} b_j
    peak(C)   = F + e + max( kept_N(C) + g , max_l [ kept_l(C) + a_l + w_l ] )
F fixed bytes, e embedding stage, g head transient, w_l backward transient of
layer l.  While layer l runs backward its full activation set is live whether
or not it was dropped (it has just been rebuilt) and later layers are freed.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

Q_A, Q_B, Q_W, Q_E, Q_G, Q_F, Q_T = 0, 1, 2, 3, 4, 5, 6
GRANULE = 256


@dataclass
class Components:
    F: int
    e: int
    g: int
    a: List[int]
    b: List[int]
    w: List[int]
    t: Optional[List[int]] = None      # forward time of each layer (ns, >= 1) when collected

    @property
    def n(self) -> int:
        return len(self.a)


# ------------------------------------------------------------------ estimator
def fit_poly(xs: Sequence[float], ys: Sequence[float], order: int = 2):
    """Ordinary least squares of y on (1, x, ..., x^order), x scaled by 1/max(x)."""
    xs = np.asarray(xs, dtype=np.float64)
    ys = np.asarray(ys, dtype=np.float64)
    scale = float(xs.max()) if xs.size and xs.max() > 0 else 1.0
    V = np.vander(xs / scale, order + 1, increasing=True)
    coef, *_ = np.linalg.lstsq(V, ys, rcond=None)
    return coef, scale


def eval_poly(model, x: float) -> float:
    coef, scale = model
    t = float(x) / scale
    acc = 0.0
    for c in coef[::-1]:
        acc = acc * t + float(c)
    return acc


def to_bytes(v: float, guard: int) -> int:
    """Nearest multiple of 256 bytes, plus the guard; never negative."""
    q = int(np.floor(v / GRANULE + 0.5)) * GRANULE
    return max(q, 0) + guard


# ------------------------------------------------------------- peak simulator
def simulate_peak(c: Components, plan: int) -> int:
    kept = 0
    worst = 0
    for l in range(c.n):
        worst = max(worst, kept + c.a[l] + c.w[l])
        kept += c.b[l] if (plan >> l) & 1 else c.a[l]
    worst = max(worst, kept + c.g)
    return c.F + c.e + worst


# --------------------------------------------------------------- Algorithm 1
def make_buckets(est: Sequence[int], tol_permille: int = 100) -> List[List[int]]:
    order = sorted(range(len(est)), key=lambda l: (-est[l], l))
    buckets: List[List[int]] = []
    i = 0
    while i < len(order):
        lead = order[i]
        bucket = [lead]
        i += 1
        while i < len(order) and 1000 * est[order[i]] > (1000 - tol_permille) * est[lead]:
            bucket.append(order[i])
            i += 1
        bucket.sort()                                   # forward position, ascending
        buckets.append(bucket)
    return buckets


def greedy_select(est: Sequence[int], buckets: List[List[int]], excess: int,
                  chosen: List[int], times: Optional[Sequence[int]] = None,
                  tol_permille: int = 100) -> int:
    """Selection loop of Algorithm 1.  Mutates buckets / chosen; returns the new excess.
    times: cost-aware choice inside the selected bucket."""
    while excess > 0:
        live = [b for b in buckets if b]
        if not live:
            break
        cands = [b for b in live if max(est[l] for l in b) > excess]
        if cands:
            pick_from = min(cands, key=lambda b: max(est[l] for l in b))
        else:
            pick_from = live[0]
        if times is None:
            l = pick_from[0]
        else:
            cheapest = min(times[j] for j in pick_from)
            l = next(j for j in pick_from if 1000 * times[j] <= (1000 + tol_permille) * cheapest)
        pick_from.remove(l)
        chosen.append(l)
        excess -= est[l]
    return excess


@dataclass
class PlanResult:
    plan: int
    order: List[int]
    predicted_peak: int
    feasible: bool


def plan_from_components(c: Components, budget_eff: int, tol_permille: int = 100,
                         cost_aware: bool = False) -> PlanResult:
    if budget_eff <= 0:                                 # unlimited
        return PlanResult(0, [], simulate_peak(c, 0), True)
    s = [max(c.a[l] - c.b[l], 0) for l in range(c.n)]
    buckets = make_buckets(s, tol_permille)
    chosen: List[int] = []
    excess = simulate_peak(c, 0) - budget_eff
    times = c.t if cost_aware else None
    while True:
        greedy_select(s, buckets, excess, chosen, times, tol_permille)
        plan = 0
        for l in chosen:
            plan |= 1 << l
        pk = simulate_peak(c, plan)
        if pk <= budget_eff:
            return PlanResult(plan, chosen, pk, True)
        if len(chosen) == c.n:
            return PlanResult(plan, chosen, pk, False)
        excess = pk - budget_eff


# -------------------------------------------------------------- brute force
def brute_force_peaks(c: Components) -> np.ndarray:
    """peak(C) for every subset C, vectorised over the 2^N bitmasks."""
    n = c.n
    masks = np.arange(1 << n, dtype=np.int64)
    kept = np.zeros(1 << n, dtype=np.int64)
    worst = np.zeros(1 << n, dtype=np.int64)
    for l in range(n):
        np.maximum(worst, kept + (c.a[l] + c.w[l]), out=worst)
        bit = (masks >> l) & 1
        kept += np.where(bit == 1, c.b[l], c.a[l])
    np.maximum(worst, kept + c.g, out=worst)
    return worst + (c.F + c.e)


# ------------------------------------------------------------------- planner
class Planner:
    """Sample table + estimator + scheduler + plan cache + phase controller."""

    def __init__(self, n_layers: int, budget: int, sheltered_steps: int = 10,
                 tol_permille: int = 100, order: int = 2, quantum: int = 1,
                 reserve: int = 0, guard: int = 1024, cost_aware: bool = False):
        self.cost_aware = cost_aware
        self.n = n_layers
        self.budget = int(budget)
        self.sheltered_steps = sheltered_steps
        self.tol = tol_permille
        self.order = order
        self.quantum = max(1, quantum)
        self.reserve = int(reserve)
        self.guard = int(guard)
        self.samples: Dict[Tuple[int, int], List[Tuple[int, int]]] = {}
        self.fixed = 0
        self.steps_seen = 0
        self.xs_seen = set()
        self.models: Optional[Dict[Tuple[int, int], tuple]] = None
        self.cache: Dict[int, PlanResult] = {}
        self.hits = 0
        self.misses = 0

    # collector
    def feed(self, x: int, quantity: int, layer: int, nbytes: int) -> None:
        if quantity == Q_F:
            self.fixed = max(self.fixed, int(nbytes))
            return
        key = (quantity, layer if quantity in (Q_A, Q_B, Q_W, Q_T) else -1)
        self.samples.setdefault(key, []).append((int(x), int(nbytes)))

    def end_sheltered_step(self, x: int) -> None:
        self.steps_seen += 1
        self.xs_seen.add(int(x))

    def sheltered(self) -> bool:
        return (self.steps_seen < self.sheltered_steps
                or len(self.xs_seen) < self.order + 1)

    # estimator
    def fit(self) -> None:
        self.models = {k: fit_poly([p[0] for p in v], [p[1] for p in v], self.order)
                       for k, v in self.samples.items()}
        self.cache.clear()

    def predict(self, x: int) -> Components:
        assert self.models is not None
        def q(kind, layer=-1):
            return to_bytes(eval_poly(self.models[(kind, layer)], x), self.guard)
        t = None
        if all((Q_T, l) in self.models for l in range(self.n)):     # times: all layers or none
            t = [max(int(np.floor(eval_poly(self.models[(Q_T, l)], x) + 0.5)), 1) for l in range(self.n)]
        return Components(
            F=self.fixed, e=q(Q_E), g=q(Q_G),
            a=[q(Q_A, l) for l in range(self.n)],
            b=[q(Q_B, l) for l in range(self.n)],
            w=[q(Q_W, l) for l in range(self.n)], t=t)

    # scheduler + cache
    def key_of(self, x: int) -> int:
        q = self.quantum
        return ((int(x) + q - 1) // q) * q

    def query(self, x: int, static_x: Optional[int] = None) -> PlanResult:
        """Plan for input size x.  static_x: a static planner's behaviour (Section 3.2): the plan
        is made for that fixed, largest input size whatever x is."""
        if self.models is None:
            self.fit()
        key = self.key_of(x if static_x is None else static_x)
        if key in self.cache:
            self.hits += 1
            return self.cache[key]
        self.misses += 1
        comp = self.predict(key)
        eff = self.budget - self.reserve if self.budget > 0 else 0
        res = plan_from_components(comp, eff, self.tol, self.cost_aware)
        self.cache[key] = res
        return res


# --------------------------------------------------- analytic memory model
def analytic_layer_bytes(B: int, L: int, hidden: int, n_heads: int, ffn: int,
                         elt: int = 4, materialised_attention: bool = True) -> int:
    """Activation bytes of one transformer block following the operator classes of
    Section 4.3: tensors of linear / elementwise operators are proportional to the
    number of tokens; an unfused attention adds three seqlen x seqlen tensors per head."""
    T = B * L
    lin = T * (12 * hidden + 2 * ffn) * elt
    quad = 3 * B * n_heads * L * L * elt if materialised_attention else 0
    return lin + quad
