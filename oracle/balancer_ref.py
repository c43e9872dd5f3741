"""Plain Python statement of the hierarchical load balancing of rollout requests (TEST
INFRASTRUCTURE ONLY; Section 5.2 of the paper: "Intra-Agent Load Balancing" and "Inter-Agent
Load Balancing").  Lists and linear scans, no heap: what the rollout manager's min-heap
returns is by definition the least-loaded instance, so the reference just looks for it.

Rules in the paper's order, with the readings the library header lists (the paper gives the
rules in prose only):
  * every agent has several inference instances; a new request goes to the instance of its
    agent with the lowest current load (load = unfinished requests it holds; ties: lowest id);
  * completed requests are removed;
  * the manager polls the request-queue lengths of all agents (queue = requests that wait,
    i.e. are assigned but not among the `slots` an instance runs at once), takes the disparity
    between the highest and the lowest; above the threshold delta, instances move from the
    lowest-queue agent to the highest-queue one: as many as the queue difference (in units of
    one instance's slots), but the donor keeps at least one; a moved instance hands its
    unfinished requests back to the donor's other instances (re-queued, progress kept),
    spends `migration_delay` steps receiving weights and then accepts the receiver's new
    requests.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List


@dataclass
class Req:
    id: int
    agent: int
    remaining: int
    generated: int = 0
    instance: int = -1
    done_step: int = -1


@dataclass
class BalancerRef:
    instances_per_agent: List[int]
    delta: int = 5
    slots: int = 1
    poll_interval: int = 1
    migration_delay: int = 0
    now: int = 0
    completed: int = 0
    migrations: int = 0
    reqs: Dict[int, Req] = field(default_factory=dict)

    def __post_init__(self):
        self.owner: List[int] = []
        for a, n in enumerate(self.instances_per_agent):
            self.owner += [a] * n
        self.lists: List[List[Req]] = [[] for _ in self.owner]
        self.in_transit: Dict[int, tuple] = {}          # instance -> (target agent, arrival step)

    # -- intra-agent ---------------------------------------------------------------------
    def active(self, agent: int) -> List[int]:
        return [i for i, o in enumerate(self.owner) if o == agent]

    def _dispatch(self, r: Req) -> int:
        inst = min(self.active(r.agent), key=lambda i: (len(self.lists[i]), i))
        self.lists[inst].append(r)
        r.instance = inst
        return inst

    def submit(self, agent: int, request_id: int, gen_len: int) -> int:
        assert request_id not in self.reqs and gen_len >= 1
        r = Req(request_id, agent, gen_len)
        self.reqs[request_id] = r
        return self._dispatch(r)

    # -- one decode step --------------------------------------------------------------------
    def waiting(self, agent: int) -> int:
        return sum(max(0, len(self.lists[i]) - self.slots) for i in self.active(agent))

    def step(self):
        for inst in sorted(self.in_transit):
            target, when = self.in_transit[inst]
            if when <= self.now:
                self.owner[inst] = target
                del self.in_transit[inst]
        for inst, lst in enumerate(self.lists):
            if self.owner[inst] < 0:
                continue
            for r in lst[:self.slots]:
                r.generated += 1
                r.remaining -= 1
                if r.remaining == 0:
                    r.done_step = self.now
                    r.instance = -1
                    self.completed += 1
            self.lists[inst] = [r for r in lst if r.remaining > 0]
        self.now += 1
        if self.now % self.poll_interval == 0 and len(self.instances_per_agent) > 1:
            self._inter_agent()

    # -- inter-agent --------------------------------------------------------------------------
    def _inter_agent(self):
        agents = range(len(self.instances_per_agent))
        queue = {a: self.waiting(a) for a in agents}
        receiver = min(agents, key=lambda a: (-queue[a], a))
        donor = min(agents, key=lambda a: (queue[a], -len(self.active(a)), a))
        disparity = queue[receiver] - queue[donor]
        if disparity <= self.delta:
            return
        count = min(-(-disparity // self.slots), len(self.active(donor)) - 1)
        for _ in range(count):
            inst = min(self.active(donor), key=lambda i: (len(self.lists[i]), i))
            orphans, self.lists[inst] = self.lists[inst], []
            self.owner[inst] = -1
            self.in_transit[inst] = (receiver, self.now + self.migration_delay)
            self.migrations += 1
            for r in orphans:
                self._dispatch(r)

    # -- what the decode step of an instance covers -------------------------------------------
    def instance_batch(self, inst: int):
        if self.owner[inst] < 0:
            return -1, [], []
        run = self.lists[inst][:self.slots]
        return self.owner[inst], [r.id for r in run], [r.generated for r in run]
