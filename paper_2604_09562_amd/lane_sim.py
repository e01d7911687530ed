"""A small discrete-event simulator of the stream pairs' prefill queues, to exercise the router under load.

The paper routes every request through its router into the prefill queue of one stream pair (Section 3.1,
Algorithm 1), whose engine serves one request at a time: prefill, KV transfer, decode (Section 3.3, Algorithm 3).
The router sees, per pair, the metrics its monitor last reported (memory, load; possibly stale), the queue depth
read at selection time (Section 3.2, Algorithm 2) and, as the cache-reuse signal C_w of Eq. 1, whether the pair's
prefix cache held the request's prompt prefix at the monitor's last report.  The paper gives no service-time model;
the one below (prefill time proportional to the prompt tokens that miss the pair's prefix cache, decode time
proportional to the generated tokens) is this build's, and only serves to create queues, stale metrics and
overload episodes for the selection rule.  Host code; the selection itself is a callable, normally
``binding.ss_route_select``.
"""
from __future__ import annotations

import collections
import dataclasses
from typing import Callable, Deque, List, Optional, Sequence, Tuple

Worker = Tuple[float, float, float, float, bool]      # (cache_hit, mem, queue depth, load, stale), as ss_route_select takes it


@dataclasses.dataclass
class Request:
    arrival: float
    prompt_len: int
    gen_len: int
    group: int            # requests of one group share a prompt prefix


@dataclasses.dataclass
class Decision:
    time: float
    workers: List[Worker]   # what the router was shown
    chosen: int


class Lane:
    def __init__(self, cache_groups: int):
        self.queue: Deque[Request] = collections.deque()
        self.busy_until = 0.0
        self.cached: Deque[int] = collections.deque(maxlen=cache_groups)
        self.tokens = 0              # prompt + generated tokens of queued and running requests (memory pressure)
        self.reported = (frozenset(), 0.0, 0.0)   # (cached prefix groups, mem, load) of the last report
        self.report_time = float("-inf")
        self.running: Optional[Request] = None


class LaneSim:
    def __init__(self, n_lanes: int, select: Callable[[Sequence[Worker], float], int], *, q_max: float = 16.0,
                 mem_tokens: int = 60000, cache_groups: int = 4, report_period: float = 0.05, stale_after: float = 0.2,
                 t_prefill: float = 2e-5, t_decode: float = 2e-4, reuse: float = 0.8, silent: Sequence[Tuple[int, float, float]] = ()):
        self.lanes = [Lane(cache_groups) for _ in range(n_lanes)]
        self.select, self.q_max, self.mem_tokens = select, q_max, mem_tokens
        self.report_period, self.stale_after = report_period, stale_after
        self.t_prefill, self.t_decode, self.reuse = t_prefill, t_decode, reuse
        self.silent = list(silent)          # (lane, from, to): the lane's monitor reports nothing in that interval
        self.decisions: List[Decision] = []
        self.waits: List[float] = []
        self.hits = 0
        self.served = 0

    # -- engine side ---------------------------------------------------------------------------------
    def _start_next(self, lane: Lane, now: float) -> None:
        req = lane.queue.popleft()
        hit = req.group in lane.cached
        if hit:
            lane.cached.remove(req.group)
        lane.cached.append(req.group)
        self.hits += hit
        self.served += 1
        self.waits.append(now - req.arrival)
        prefill = self.t_prefill * req.prompt_len * ((1.0 - self.reuse) if hit else 1.0)
        lane.busy_until = now + prefill + self.t_decode * req.gen_len
        lane.running = req

    def _advance(self, now: float) -> None:
        for lane in self.lanes:
            while True:
                if lane.running is not None and lane.busy_until <= now:
                    lane.tokens -= lane.running.prompt_len + lane.running.gen_len
                    lane.running = None
                if lane.running is None and lane.queue:
                    self._start_next(lane, max(lane.busy_until, lane.queue[0].arrival))
                    continue
                break

    def _report(self, now: float) -> None:
        for i, lane in enumerate(self.lanes):
            if any(l == i and t0 <= now < t1 for l, t0, t1 in self.silent):
                continue
            if now - lane.report_time >= self.report_period:
                active = len(lane.queue) + (lane.running is not None)
                lane.reported = (frozenset(lane.cached), min(1.0, lane.tokens / self.mem_tokens), min(1.0, active / self.q_max))
                lane.report_time = now

    # -- router side ---------------------------------------------------------------------------------
    def submit(self, req: Request) -> int:
        now = req.arrival
        self._advance(now)
        self._report(now)
        workers: List[Worker] = []
        for lane in self.lanes:
            groups, m, l = lane.reported
            c = 1.0 if req.group in groups else 0.0
            workers.append((c, m, float(len(lane.queue)), l, now - lane.report_time > self.stale_after))   # depth is read now
        chosen = self.select(workers, self.q_max)
        self.decisions.append(Decision(now, workers, chosen))
        lane = self.lanes[chosen]
        lane.queue.append(req)
        lane.tokens += req.prompt_len + req.gen_len
        self._advance(now)
        return chosen

    def run(self, requests: Sequence[Request]) -> None:
        for r in sorted(requests, key=lambda r: r.arrival):
            self.submit(r)
        self._advance(float("inf"))

    @property
    def mean_wait(self) -> float:
        return sum(self.waits) / max(1, len(self.waits))

    @property
    def hit_fraction(self) -> float:
        return self.hits / max(1, self.served)
