"""CPU oracle of the static-dynamic memory construction (Section 4.1).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's CPU leg may use it; the
product path never does.  Plain Python, written from the paper's description:

  * memories are clustered into groups of segments (the clustering itself, a sentence
    encoder, is outside this build: callers say which group a segment belongs to);
  * a group is STATIC when none of its segments changed during the recent `t` steps, else
    DYNAMIC; a new group starts dynamic;
  * the KV cache of a static group is computed once for the whole group (segments
    concatenated, full attention between them); a dynamic group is cached one segment at a
    time, so an update invalidates that segment only;
  * when a group changes category its cache is recomputed the new way;
  * retrieval units: a static group as a whole, a dynamic segment on its own.

Readings where the section is silent (all listed in the design notes):
  - "changed" covers new content, a new segment and a removed segment;
  - writing back identical tokens is not a change;
  - steps are counted by `end_step`; a change made while step s is open has age 0 when s
    closes; a group is static when the age of its newest change is >= t;
  - units are listed by ascending group id, a dynamic group's segments by ascending segment
    id; a static unit's tokens are its segments' tokens in ascending segment id.

Pins (tests/test_memory_oracle.py): classification against the sentence evaluated from a
full change log, a hand-worked trace (tests/golden/memory_trace_t3.json), the invalidation
sizes the section argues with (one segment vs the whole group), unit order and contents.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

STATIC, DYNAMIC = 0, 1


@dataclass
class Segment:
    group: int
    tokens: Tuple[int, ...]
    last_change: int            # step during which the content was last written


@dataclass
class Group:
    kind: int = DYNAMIC
    segments: List[int] = field(default_factory=list)   # ascending segment ids
    last_member_change: int = 0                          # step of the last add / remove


@dataclass
class Unit:
    kind: int                   # STATIC: a whole group, DYNAMIC: one segment
    ident: int                  # group id (static) or segment id (dynamic)
    segments: Tuple[int, ...]
    n_tokens: int
    dirty: bool                 # its KV cache has to be (re)computed


@dataclass
class StepReport:
    step: int
    n_static: int
    n_dynamic: int
    to_dynamic: List[int]       # groups that left the static state at this step
    to_static: List[int]        # groups that became static at this step
    dirty_units: int
    dirty_tokens: int           # tokens whose KV has to be computed after this step


class MemoryOracle:
    def __init__(self, window_t: int):
        if window_t < 0:
            raise ValueError("window must be >= 0")
        self.t = window_t
        self.now = 0                                   # index of the open step
        self.seg: Dict[int, Segment] = {}
        self.grp: Dict[int, Group] = {}
        # caches that exist and are valid: ("S", group) or ("D", segment)
        self.clean = set()

    # -- changes inside the open step -------------------------------------------------
    def put(self, group: int, segment: int, tokens) -> bool:
        """Add a segment or replace its content.  Returns True if this was a change."""
        tokens = tuple(int(x) for x in tokens)
        if len(tokens) == 0:
            raise ValueError("empty segment")
        s = self.seg.get(segment)
        if s is not None:
            if s.group != group:
                raise ValueError("segment belongs to another group")
            if s.tokens == tokens:
                return False
            s.tokens = tokens
            s.last_change = self.now
            self.clean.discard(("D", segment))
            self.clean.discard(("S", group))
            return True
        g = self.grp.setdefault(group, Group(kind=DYNAMIC, last_member_change=self.now))
        g.segments.append(segment)
        g.segments.sort()
        g.last_member_change = self.now
        self.seg[segment] = Segment(group, tokens, self.now)
        self.clean.discard(("S", group))
        return True

    def remove(self, segment: int) -> None:
        s = self.seg.pop(segment)
        g = self.grp[s.group]
        g.segments.remove(segment)
        g.last_member_change = self.now
        self.clean.discard(("D", segment))
        self.clean.discard(("S", s.group))
        if not g.segments:
            del self.grp[s.group]

    # -- closing a step -----------------------------------------------------------------
    def newest_change(self, group: int) -> int:
        g = self.grp[group]
        return max([g.last_member_change] + [self.seg[s].last_change for s in g.segments])

    def end_step(self) -> StepReport:
        to_dyn, to_sta = [], []
        for gid in sorted(self.grp):
            g = self.grp[gid]
            age = self.now - self.newest_change(gid)    # closed steps since the newest change
            kind = STATIC if age >= self.t else DYNAMIC
            if kind != g.kind:
                (to_sta if kind == STATIC else to_dyn).append(gid)
                # the cache is recomputed the new way: nothing of the old way stays valid
                self.clean.discard(("S", gid))
                for s in g.segments:
                    self.clean.discard(("D", s))
                g.kind = kind
        units = self.units()
        rep = StepReport(self.now,
                         sum(1 for g in self.grp.values() if g.kind == STATIC),
                         sum(1 for g in self.grp.values() if g.kind == DYNAMIC),
                         to_dyn, to_sta,
                         sum(1 for u in units if u.dirty), sum(u.n_tokens for u in units if u.dirty))
        self.now += 1
        return rep

    # -- retrieval / caching units --------------------------------------------------------
    def units(self) -> List[Unit]:
        out = []
        for gid in sorted(self.grp):
            g = self.grp[gid]
            if g.kind == STATIC:
                n = sum(len(self.seg[s].tokens) for s in g.segments)
                out.append(Unit(STATIC, gid, tuple(g.segments), n, ("S", gid) not in self.clean))
            else:
                for s in g.segments:
                    out.append(Unit(DYNAMIC, s, (s,), len(self.seg[s].tokens), ("D", s) not in self.clean))
        return out

    def unit_tokens(self, u: Unit) -> List[int]:
        toks: List[int] = []
        for s in u.segments:
            toks.extend(self.seg[s].tokens)
        return toks

    def mark_computed(self, u: Unit) -> None:
        self.clean.add(("S" if u.kind == STATIC else "D", u.ident))
