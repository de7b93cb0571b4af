"""CPU oracle of Expert Buffering's cache management -- TEST INFRASTRUCTURE ONLY.

Plain Python, written from the paper's description (Sec. 6, "Expert Buffering", subsections
"Cache Management" and "Cache Miss Rates").  It shares no code with the library's cache; only
tests, the smoke check and the benchmark's baseline leg may import it.

The model.  Expert parameters live in host memory; the device holds ``n_slots`` experts.  A batch
is the set of experts with a positive token count ("active").  The experts of a batch execute one
after the other in increasing id order, and the cache is consulted in that order:

* resident  -> hit;
* otherwise -> miss: the expert is copied into a free slot, or, when the cache is full, into the
  slot of a victim chosen by the policy.

Policies
  ``paper``   first the residents that are NOT active in this batch, then the active ones; inside
              each class Last In, First Out: the most recently inserted resident goes first.
              (Reading: "last in" is the order in which experts entered the cache; an active
              resident may be chosen whether or not it has already run in this batch -- the text
              names no such distinction.)
  ``fifo``    the resident that entered the cache first, active or not.
  ``lru``     the resident used least recently (an access is one expert execution).
  ``belady``  Belady's MIN on the flattened access sequence (batch by batch, ids ascending):
              the resident whose next use lies farthest in the future; needs the whole trace.

Execution stages.  A victim that already ran in the current batch must finish computing before
its slot is overwritten, so the expert that replaces it belongs to a later stage than the victim;
stages are otherwise as early as possible and never decrease along the id order.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Optional, Sequence, Tuple

POLICIES = ("paper", "fifo", "lru", "belady")


class Load:
    """One miss: ``expert`` is copied into ``slot``, replacing ``victim`` (-1: the slot was free)."""

    __slots__ = ("batch", "expert", "slot", "victim", "stage")

    def __init__(self, batch: int, expert: int, slot: int, victim: int, stage: int):
        self.batch, self.expert, self.slot, self.victim, self.stage = batch, expert, slot, victim, stage

    def astuple(self) -> Tuple[int, int, int, int, int]:
        return (self.batch, self.expert, self.slot, self.victim, self.stage)

    def __repr__(self) -> str:
        return "Load(batch=%d, expert=%d, slot=%d, victim=%d, stage=%d)" % self.astuple()


class ExpertCache:
    """Step-by-step simulator; ``step`` takes one batch's active experts."""

    def __init__(self, n_slots: int, policy: str = "paper"):
        if n_slots < 1:
            raise ValueError("n_slots must be at least 1")
        if policy not in POLICIES:
            raise ValueError("unknown policy %r" % policy)
        self.n_slots = n_slots
        self.policy = policy
        self.slot_expert: List[int] = [-1] * n_slots   # expert held by each slot
        self.where: Dict[int, int] = {}                # expert -> slot
        self.inserted: Dict[int, int] = {}             # expert -> insertion sequence number
        self.used: Dict[int, int] = {}                 # expert -> sequence number of its last execution
        self.clock = 0
        self.batch = 0
        self.hits = 0
        self.misses = 0
        self.future: Optional[List[List[int]]] = None  # belady: the remaining batches, this one first

    def _victim(self, active: Sequence[int], pos: int) -> int:
        residents = list(self.where.keys())
        if self.policy == "paper":
            active_set = set(active)
            idle = [e for e in residents if e not in active_set]
            pool = idle if idle else residents
            return max(pool, key=lambda e: self.inserted[e])
        if self.policy == "fifo":
            return min(residents, key=lambda e: self.inserted[e])
        if self.policy == "lru":
            return min(residents, key=lambda e: self.used.get(e, -1))
        # belady: distance to the next use in (rest of this batch) + (later batches)
        assert self.future is not None, "belady needs the whole trace (use simulate)"
        seq: List[int] = list(active[pos + 1:])
        for later in self.future[1:]:
            seq.extend(later)
        def next_use(e: int) -> int:
            try:
                return seq.index(e)
            except ValueError:
                return len(seq) + 1 + e  # never again: farthest; ties by id for determinism
        return max(residents, key=next_use)

    def step(self, active: Iterable[int]) -> Dict[str, object]:
        """Run one batch.  Returns slot_of (expert -> slot it executed from), stage_of, loads."""
        order = sorted(set(int(e) for e in active))
        slot_of: Dict[int, int] = {}
        stage_of: Dict[int, int] = {}
        loads: List[Load] = []
        stage = 0
        for pos, e in enumerate(order):
            self.clock += 1
            if e in self.where:
                self.hits += 1
            else:
                self.misses += 1
                victim = -1
                if len(self.where) < self.n_slots:
                    slot = self.slot_expert.index(-1)
                else:
                    victim = self._victim(order, pos)
                    slot = self.where.pop(victim)
                    del self.inserted[victim]
                    self.used.pop(victim, None)
                    if victim in stage_of:  # it already ran in this batch: its slot frees a stage later
                        stage = max(stage, stage_of[victim] + 1)
                self.slot_expert[slot] = e
                self.where[e] = slot
                self.inserted[e] = self.clock
                loads.append(Load(self.batch, e, slot, victim, stage))
            self.used[e] = self.clock
            slot_of[e] = self.where[e]
            stage_of[e] = stage
        self.batch += 1
        return dict(slot_of=slot_of, stage_of=stage_of, loads=loads, n_stages=stage + 1 if order else 0)

    def residents(self) -> List[int]:
        return sorted(self.where.keys())


def simulate(trace: Sequence[Iterable[int]], n_slots: int, policy: str = "paper") -> Dict[str, object]:
    """Whole trace (one iterable of active expert ids per batch).  Miss rate = misses / accesses,
    an access being one (batch, active expert) pair -- the paper's global cache miss rate."""
    batches = [sorted(set(int(e) for e in b)) for b in trace]
    cache = ExpertCache(n_slots, policy)
    loads: List[Load] = []
    per_batch: List[int] = []
    for i, b in enumerate(batches):
        if policy == "belady":
            cache.future = batches[i:]
        before = cache.misses
        out = cache.step(b)
        loads.extend(out["loads"])
        per_batch.append(cache.misses - before)
    accesses = cache.hits + cache.misses
    return dict(hits=cache.hits, misses=cache.misses, accesses=accesses,
                miss_rate=(cache.misses / accesses) if accesses else 0.0,
                per_batch_misses=per_batch, loads=loads, residents=cache.residents())


def optimal_misses(trace: Sequence[Iterable[int]], n_slots: int) -> int:
    """Fewest possible misses by exhaustive search over every eviction choice (tiny traces only)."""
    seq: List[int] = []
    for b in trace:
        seq.extend(sorted(set(int(e) for e in b)))
    best = [len(seq) + 1]

    def go(i: int, cache: frozenset, misses: int) -> None:
        if misses >= best[0]:
            return
        if i == len(seq):
            best[0] = misses
            return
        e = seq[i]
        if e in cache:
            go(i + 1, cache, misses)
        elif len(cache) < n_slots:
            go(i + 1, cache | {e}, misses + 1)
        else:
            for v in cache:
                go(i + 1, (cache - {v}) | {e}, misses + 1)

    go(0, frozenset(), 0)
    return best[0]
