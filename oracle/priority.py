"""Test oracle for the priority-ordered K,V residency of Symphony (arxiv 2412.16434), plain Python on purpose.

TEST INFRASTRUCTURE ONLY: the product never imports this module.  It states, as directly as possible, which parts of
which sessions' caches are held in HBM slots lent by the serving framework (Sec. 3.3, "priority-based K,V cache" and
"cooperative memory management"):

  * a session's cache is held layer by layer; what is moved in first and given up last are the LOWER layers, because
    the forward pass needs them first and the transfer of the later ones hides behind it;
  * when the framework needs memory, the parts it overwrites first are those of the LATER layers, and among parts of
    the same layer those of the SMALLEST caches;
  * with several announced sessions and too little memory, the lower layers of all of them are held rather than all
    layers of one.

A "unit" is one layer of one session: ceil(n_tokens / block_size) slots of one block each.  Readings where the paper is
silent: units are admitted whole or not at all; a unit that does not fit is passed over and smaller ones after it may
still be admitted (all layers of a session have one size and the room only shrinks, so once a layer of a session is
refused its later layers are too: the held layers of a session are always 0 .. r-1); equal (layer, size) are ordered
by session id, smaller id first.
"""
from __future__ import annotations


def blocks_of(n_tokens: int, block_size: int) -> int:
    return -(-n_tokens // block_size)


def units_by_priority(sessions: dict[int, int], n_layers: int, block_size: int) -> list[tuple[int, int]]:
    """All (layer, sid) units, the most important first: lower layer, then larger cache, then smaller id."""
    keyed = []
    for sid, n_tokens in sessions.items():
        for layer in range(n_layers):
            keyed.append((layer, -blocks_of(n_tokens, block_size), sid))
    keyed.sort()
    return [(layer, sid) for layer, _, sid in keyed]


def resident_layers(sessions: dict[int, int], n_layers: int, block_size: int, capacity: int) -> dict[int, int]:
    """Number of resident layers (0 .. n_layers, always layers 0 .. r-1) per session when `capacity` slots can be
    lent: walk the units in priority order and admit each one that still fits."""
    r = {sid: 0 for sid in sessions}
    used = 0
    for layer, sid in units_by_priority(sessions, n_layers, block_size):
        b = blocks_of(sessions[sid], block_size)
        if used + b <= capacity:
            r[sid] += 1
            used += b
    return r


def eviction_order(resident: dict[int, int], sessions: dict[int, int], block_size: int) -> list[tuple[int, int]]:
    """Resident units in the order in which the framework may overwrite them: later layers first, within a layer the
    smallest cache first (then the larger id: the exact reverse of the admission order)."""
    keyed = []
    for sid, r in resident.items():
        for layer in range(r):
            keyed.append((-layer, blocks_of(sessions[sid], block_size), -sid))
    keyed.sort()
    return [(-neg_layer, -neg_sid) for neg_layer, _, neg_sid in keyed]


def evicted_to_free(resident: dict[int, int], sessions: dict[int, int], block_size: int, free_now: int,
                    need: int) -> list[tuple[int, int]]:
    """The units given up so that `need` slots are free: the shortest beginning of eviction_order that is enough."""
    out = []
    for layer, sid in eviction_order(resident, sessions, block_size):
        if free_now >= need:
            break
        out.append((layer, sid))
        free_now += blocks_of(sessions[sid], block_size)
    return out


class PoolModel:
    """The same events as the library's pool object, every answer recomputed from the definitions above.  Slots have no
    identity here: only counts, resident layers and the sets of evicted / loaded units are defined uniquely."""

    def __init__(self, n_layers: int, n_slots: int, block_size: int):
        self.n_layers, self.n_slots, self.block_size = n_layers, n_slots, block_size
        self.sessions: dict[int, int] = {}
        self.resident: dict[int, int] = {}
        self.framework = 0            # slots the framework owns
        self.evicted_log: list[tuple[int, int]] = []

    def lent(self) -> int:
        return sum(r * blocks_of(self.sessions[s], self.block_size) for s, r in self.resident.items())

    def free(self) -> int:
        return self.n_slots - self.framework - self.lent()

    def advise(self, sid: int, n_tokens: int) -> bool:
        if n_tokens < 1 or (sid in self.sessions and self.sessions[sid] != n_tokens):
            return False
        self.sessions[sid] = n_tokens
        self.resident.setdefault(sid, 0)
        return True

    def drop(self, sid: int) -> bool:
        if sid not in self.sessions:
            return False
        for layer in reversed(range(self.resident[sid])):
            self.evicted_log.append((layer, sid))
        del self.sessions[sid], self.resident[sid]
        return True

    def claim(self, sid: int):
        """The request has arrived: the session's resident layers become the framework's.  Returns their number."""
        if sid not in self.sessions:
            return None
        r = self.resident[sid]
        self.framework += r * blocks_of(self.sessions[sid], self.block_size)
        del self.sessions[sid], self.resident[sid]
        return r

    def take(self, n: int):
        """The framework takes n slots; returns the units evicted for it, or None if n cannot be had at all."""
        if n < 0 or n > self.n_slots - self.framework:
            return None
        gone = evicted_to_free(self.resident, self.sessions, self.block_size, self.free(), n)
        for layer, sid in gone:
            assert self.resident[sid] == layer + 1
            self.resident[sid] = layer
        self.evicted_log += gone
        self.framework += n
        return gone

    def give(self, n: int) -> bool:
        if n < 0 or n > self.framework:
            return False
        self.framework -= n
        return True

    def settle(self):
        """Bring the resident set to what the priorities say.  Returns (evicted since the last settle, loaded now)."""
        target = resident_layers(self.sessions, self.n_layers, self.block_size, self.n_slots - self.framework)
        for sid in sorted(self.sessions):
            for layer in reversed(range(target[sid], self.resident[sid])):
                self.evicted_log.append((layer, sid))
        loaded = [(layer, sid) for sid in sorted(self.sessions) for layer in range(self.resident[sid], target[sid])]
        self.resident = dict(target)
        evicted, self.evicted_log = self.evicted_log, []
        return evicted, loaded
