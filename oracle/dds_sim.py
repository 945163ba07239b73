"""Host-side parts of the framework around the iteration: the shard queue with states
(Section V-C: shard arithmetic V-C.1, states and re-queue V-C.3) and an iteration-level model of bulk-synchronous training under injected
stragglers (Section II, Eq. 1; Section VI-A; Section VII-A.2).

Test infrastructure: see the package docstring.

Shard queue.  The N samples are cut into K = ceil(N / (B*M)) shards (start, length); all start
as TODO in a queue; a worker fetches the head, which becomes DOING; when the worker has pushed
its gradients the shard becomes DONE; when a worker is lost (its gradients disregarded, or the
node killed) its DOING shards become TODO again and go to the END of the queue.

Training model.  One iteration of n workers takes max_i T_i + T_server with
T_i = F_i(B_i) + injected delay, F_i(b) = t0_i + b / v_i (the measured batch time is affine in
the batch: a latency floor plus a per-sample cost), sum_i B_i = B (Eq. 1 with the server and
communication terms lumped into T_server).  Injected delays follow Section VII-A.2: a
transient straggler adds sleep_duration * intensity to every iteration of a worker during the
first `duration` seconds of every `period` seconds, each (window, worker) pair being disturbed
with probability `prob`; a persistent straggler adds a constant delay from the start.
Policies:
  BSP             equal split B/n (Section VI-A step 1), never changed;
  ADJUST_BS       every `decide_every` seconds: short-window mean batch time per worker; when a
                  worker is lambda times slower than the mean (or, reading: lambda times faster,
                  so that a recovered worker gets its share back) the split is re-solved from the
                  short-window throughputs v_i = mean(B_i / T_i) by Eq. 3;
  BACKUP_WORKERS  the b slowest workers of every iteration are disregarded; their samples go
                  back to the queue, i.e. do not count as processed (Section VII-A.3);
  ANTDT_ND        ADJUST_BS plus: a worker whose long-window mean batch time is lambda times the
                  mean is killed and restarted: it is absent for `restart_cost` seconds (the
                  others share the fixed global batch meanwhile) and comes back without its
                  persistent delay (Section VI-A steps 2-5).
Readings (the paper gives no formulas for these): decisions are taken between iterations; on a
change of the set of present workers the batch is split equally among them; at most one
worker is killed per decision (the slowest; ties: lowest index); window means are over the
iterations that ended within the last L seconds; the pseudo-random choice of disturbed
(window, worker) pairs is MurmurHash3's 32-bit finaliser of (seed, window, worker).
"""
from __future__ import annotations

import math
from collections import deque
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

from .shard_assign import data_shards

TODO, DOING, DONE = 0, 1, 2
BSP, ADJUST_BS, BACKUP_WORKERS, ANTDT_ND = 0, 1, 2, 3


class ShardQueue:
    """Stateful dynamic data sharding (Section V-C.1 shards, Section V-C.3 states)."""

    def __init__(self, N: int, B: int, M: int):
        self.shards = data_shards(N, B, M)
        K = len(self.shards)
        self.state = [TODO] * K
        self.owner = [-1] * K
        self.queue = deque(range(K))

    def fetch(self, worker: int) -> Optional[Tuple[int, int, int]]:
        if not self.queue:
            return None
        k = self.queue.popleft()
        self.state[k], self.owner[k] = DOING, worker
        return (k,) + tuple(self.shards[k])

    def report_done(self, shard: int, worker: int) -> None:
        if not (0 <= shard < len(self.shards)) or self.state[shard] != DOING or self.owner[shard] != worker:
            raise ValueError("shard is not being worked on by this worker")
        self.state[shard], self.owner[shard] = DONE, -1

    def release_worker(self, worker: int) -> int:
        """The worker is lost: its DOING shards return to the end of the queue (ascending id)."""
        lost = [k for k in range(len(self.shards)) if self.state[k] == DOING and self.owner[k] == worker]
        for k in lost:
            self.state[k], self.owner[k] = TODO, -1
            self.queue.append(k)
        return len(lost)

    def counts(self) -> Tuple[int, int, int]:
        return tuple(sum(1 for s in self.state if s == x) for x in (TODO, DOING, DONE))


# --------------------------------------------------------------------------- training model
def fmix32(x: int) -> int:
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x85EBCA6B) & 0xFFFFFFFF
    x ^= x >> 13
    x = (x * 0xC2B2AE35) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def disturbed(seed: int, window: int, worker: int, prob: float) -> bool:
    u = fmix32(seed ^ fmix32((window * 0x9E3779B9 + worker + 1) & 0xFFFFFFFF))
    return u / 4294967296.0 < prob


def split_by_speed(B: int, speeds: Sequence[float]) -> List[int]:
    """Eq. 3 by the stated rule: floor(B v_i / sum v) - 1 each (not below 0), then one sample at
    a time to the worker whose load after the addition is smallest (ties: lowest index)."""
    tot = 0.0
    for v in speeds:
        tot += v
    out = []
    for v in speeds:
        b = int(math.floor((B * v) / tot)) - 1
        out.append(max(b, 0))
    given = sum(out)
    while given < B:
        best = 0
        for k in range(1, len(speeds)):
            if (out[k] + 1) * speeds[best] < (out[best] + 1) * speeds[k]:
                best = k
        out[best] += 1
        given += 1
    return out


def equal_sizes(B: int, n: int) -> List[int]:
    q, r = divmod(B, n)
    return [q + (1 if i < r else 0) for i in range(n)]


@dataclass
class SimConfig:
    n: int
    B: int
    N: int
    t0: Sequence[float]
    v: Sequence[float]
    t_server: float = 0.0
    period: float = 1800.0
    duration: float = 900.0
    prob: float = 0.0
    sleep_duration: float = 1.5
    intensity: float = 0.0
    seed: int = 1
    persistent_delay: Sequence[float] = ()
    policy: int = BSP
    backup_b: int = 0
    decide_every: float = 300.0
    L_trans: float = 300.0
    L_per: float = 600.0
    lam: float = 1.5
    restart_cost: float = 120.0
    max_iterations: int = 10_000_000


@dataclass
class SimResult:
    jct: float
    iterations: int
    processed: int
    adjust_actions: int
    kills: int
    max_bpt: float
    sum_bpt: float
    final_sizes: List[int] = field(default_factory=list)


def simulate_bsp(c: SimConfig) -> SimResult:
    n = c.n
    pers = list(c.persistent_delay) if len(c.persistent_delay) else [0.0] * n
    absent_until = [0.0] * n
    hist = [deque() for _ in range(n)]          # (t_end, B_i, T_i)
    present_prev: List[int] = []
    sizes = [0] * n
    t, processed, iterations = 0.0, 0, 0
    adjust_actions = kills = 0
    max_bpt = sum_bpt = 0.0
    next_decision = c.decide_every
    keep = max(c.L_trans, c.L_per)
    while processed < c.N and iterations < c.max_iterations:
        present = [i for i in range(n) if t >= absent_until[i]]
        if present != present_prev:              # membership changed: equal split among those present
            eq = equal_sizes(c.B, len(present))
            sizes = [0] * n
            for j, i in enumerate(present):
                sizes[i] = eq[j]
            present_prev = present
        window = int(math.floor(t / c.period))
        in_burst = (t - window * c.period) < c.duration
        T = {}
        for i in present:
            delay = pers[i]
            if c.prob > 0.0 and in_burst and disturbed(c.seed, window, i, c.prob):
                delay = delay + c.sleep_duration * c.intensity
            T[i] = c.t0[i] + sizes[i] / c.v[i] + delay
        if c.policy == BACKUP_WORKERS and c.backup_b > 0:
            order = sorted(present, key=lambda i: (T[i], i))
            included = order[:max(len(present) - c.backup_b, 1)]
            bpt = T[included[-1]]
            done = sum(sizes[i] for i in included)
        else:
            bpt = max(T[i] for i in present)
            done = c.B
        step = bpt + c.t_server
        t = t + step
        processed += done
        iterations += 1
        max_bpt = max(max_bpt, bpt)
        sum_bpt = sum_bpt + bpt
        for i in present:
            hist[i].append((t, sizes[i], T[i]))
            while hist[i] and hist[i][0][0] <= t - keep:
                hist[i].popleft()
        if t < next_decision:
            continue
        while next_decision <= t:
            next_decision = next_decision + c.decide_every
        if c.policy not in (ADJUST_BS, ANTDT_ND):
            continue

        def window_mean(i, L, what):
            acc, cnt = 0.0, 0
            for (te, b, ti) in hist[i]:
                if te > t - L:
                    acc = acc + (ti if what == 0 else b / ti)
                    cnt += 1
            return (acc / cnt) if cnt else None

        killed = False
        if c.policy == ANTDT_ND:
            per = {i: window_mean(i, c.L_per, 0) for i in present}
            if all(x is not None for x in per.values()) and len(present) > 1:
                mean = 0.0
                for i in present:
                    mean = mean + per[i]
                mean = mean / len(present)
                worst = max(present, key=lambda i: (per[i], -i))
                if per[worst] >= c.lam * mean:
                    absent_until[worst] = t + c.restart_cost
                    pers[worst] = 0.0
                    hist[worst].clear()
                    kills += 1
                    killed = True
        if killed:
            continue                               # the next iteration re-splits among those present
        tr = {i: window_mean(i, c.L_trans, 0) for i in present}
        if any(x is None for x in tr.values()):
            continue
        mean = 0.0
        for i in present:
            mean = mean + tr[i]
        mean = mean / len(present)
        slow = max(tr[i] for i in present) >= c.lam * mean
        fast = min(tr[i] for i in present) * c.lam <= mean
        if slow or fast:
            speeds = [window_mean(i, c.L_trans, 1) for i in present]
            if all(s is not None and s > 0.0 for s in speeds):
                new = split_by_speed(c.B, speeds)
                for j, i in enumerate(present):
                    sizes[i] = new[j]
                adjust_actions += 1
    return SimResult(t, iterations, processed, adjust_actions, kills, max_bpt, sum_bpt, list(sizes))
