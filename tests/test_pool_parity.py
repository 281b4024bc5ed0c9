"""The library's pool object (include/symph_pool.h, host code) against the residency oracle on the same seeded event
sequences: resident layers, owner counts and the sets of evicted / loaded units must agree exactly after every event;
slot numbers, where several assignments are valid, are checked for validity (in range, never owned twice, tables of
the right length, a unit that stays resident keeps its slots)."""
import numpy as np
import pytest

import paper_2412_16434_amd as S
from oracle import priority as PR


class Ledger:
    """The test's own record of who owns which slot, built only from what the library reports."""

    def __init__(self, n_slots):
        self.n_slots = n_slots
        self.framework = set()
        self.units = {}                       # (layer, sid) -> list of slots

    def lent(self):
        return {s for t in self.units.values() for s in t}

    def check_disjoint(self):
        lent = [s for t in self.units.values() for s in t]
        assert len(lent) == len(set(lent)), "a slot is lent twice"
        assert not (set(lent) & self.framework), "a slot is lent and the framework's"
        assert all(0 <= s < self.n_slots for s in lent) and all(0 <= s < self.n_slots for s in self.framework)


def run_sequence(seed, n_events, L, n_slots, bs, max_sessions, max_tokens):
    rng = np.random.default_rng(seed)
    pool = S.KvPool(L, n_slots, bs)
    model = PR.PoolModel(L, n_slots, bs)
    led = Ledger(n_slots)
    known = {}

    def compare():
        free, lent, fw = pool.counts()
        assert (free, lent, fw) == (model.free(), model.lent(), model.framework)
        assert fw == len(led.framework) and lent == len(led.lent())
        for sid in known:
            assert pool.resident_layers(sid) == model.resident[sid]
        led.check_disjoint()

    for ev in range(n_events):
        kind = rng.choice(["advise", "settle", "take", "give", "claim", "drop", "settle"])
        if kind == "advise":
            sid = int(rng.integers(0, max_sessions)) - max_sessions // 2          # negative ids too
            n = int(rng.integers(1, max_tokens + 1))
            ok = model.advise(sid, n)
            if ok:
                pool.advise(sid, n)
                known[sid] = n
            else:
                with pytest.raises(S.SymphError):
                    pool.advise(sid, n)
        elif kind == "settle":
            want_ev, want_ld = model.settle()
            got = pool.settle()
            got_ev = [(l, s) for k, s, l, _ in got if k == S.KvPool.EVICTED]
            got_ld = [(l, s) for k, s, l, _ in got if k == S.KvPool.LOAD]
            assert sorted(got_ev) == sorted(want_ev) and sorted(got_ld) == sorted(want_ld)
            kinds = [k for k, *_ in got]
            assert kinds == sorted(kinds)                                         # evictions first
            # loads come most important first
            prio = {u: i for i, u in enumerate(PR.units_by_priority(model.sessions, L, bs))}
            assert [prio[u] for u in got_ld] == sorted(prio[u] for u in got_ld)
            for u in got_ev:
                led.units.pop(u, None)                                           # (dropped sessions are gone already)
            for k, s, l, slots in got:
                if k == S.KvPool.LOAD:
                    assert len(slots) == PR.blocks_of(known[s], bs) and (l, s) not in led.units
                    led.units[(l, s)] = slots
            # what the library says it holds is what the ledger holds
            for (l, s), slots in led.units.items():
                assert pool.table(s, l) == slots
            assert set(led.units) == {(l, s) for s, r in model.resident.items() for l in range(r)}
        elif kind == "take":
            n = int(rng.integers(0, n_slots // 2 + 2))
            gone = model.take(n)
            if gone is None:
                with pytest.raises(S.SymphError) as e:
                    pool.framework_take(n)
                assert e.value.status == -4
            else:
                slots = pool.framework_take(n)
                assert len(slots) == n == len(set(slots))
                for u in gone:                     # exactly the oracle's units are gone; their slots may be reused
                    led.units.pop(u)
                assert not (set(slots) & led.lent()) and not (set(slots) & led.framework)
                led.framework |= set(slots)
        elif kind == "give":
            if led.framework:
                k = int(rng.integers(1, len(led.framework) + 1))
                slots = [int(x) for x in rng.permutation(sorted(led.framework))[:k]]
                assert model.give(k)
                pool.framework_give(slots)
                led.framework -= set(slots)
            else:
                with pytest.raises(S.SymphError):
                    pool.framework_give([0])
        elif kind == "claim" and known:
            sid = int(rng.choice(sorted(known)))
            r = model.claim(sid)
            tables = pool.claim(sid)
            assert len(tables) == r
            for l, t in enumerate(tables):
                assert led.units.pop((l, sid)) == t
                led.framework |= set(t)
            del known[sid]
            with pytest.raises(S.SymphError):
                pool.resident_layers(sid)
        elif kind == "drop" and known:
            sid = int(rng.choice(sorted(known)))
            assert model.drop(sid)
            pool.drop(sid)
            for l in range(L):
                led.units.pop((l, sid), None)
            del known[sid]
        compare()
    pool.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_event_sequences_small(seed):
    run_sequence(seed, n_events=300, L=4, n_slots=64, bs=16, max_sessions=8, max_tokens=200)


@pytest.mark.parametrize("seed", range(4))
def test_random_event_sequences_model_shapes(seed):
    # 32 layers, a pool that holds a few sessions of a few thousand tokens
    run_sequence(100 + seed, n_events=150, L=32, n_slots=20000, bs=16, max_sessions=24, max_tokens=8192)


def test_section_scenario_through_the_library():
    """Sec. 3.3: the memory holds one of two equal sessions -> after the second announcement the lower halves of both."""
    pool = S.KvPool(4, 16, 16)
    pool.advise(2, 64)
    first = pool.settle()
    assert [(k, s, l) for k, s, l, _ in first] == [(1, 2, 0), (1, 2, 1), (1, 2, 2), (1, 2, 3)]
    assert sorted(x for *_, sl in first for x in sl) == list(range(16))
    pool.advise(3, 64)
    second = pool.settle()
    assert sorted((k, s, l) for k, s, l, _ in second) == [(0, 2, 2), (0, 2, 3), (1, 3, 0), (1, 3, 1)]
    assert pool.resident_layers(2) == 2 and pool.resident_layers(3) == 2
    assert pool.table(2, 0) == first[0][3] and pool.table(2, 1) == first[1][3]      # what stays keeps its slots
    assert pool.counts() == (0, 16, 0)


def test_argument_checks_change_nothing():
    lib = S.load_library()
    import ctypes as C
    h = C.c_void_p()
    assert lib.symph_pool_create(0, 4, 16, C.byref(h)) == -1 and lib.symph_pool_create(2, 4, 16, None) == -1
    pool = S.KvPool(2, 8, 16)
    pool.advise(1, 40)                      # 3 slots per layer
    assert [x[:3] for x in pool.settle()] == [(1, 1, 0), (1, 1, 1)]
    for bad in (lambda: pool.advise(1, 41), lambda: pool.advise(5, 0), lambda: pool.drop(9), lambda: pool.claim(9),
                lambda: pool.framework_take(9), lambda: pool.framework_take(-1), lambda: pool.framework_give([0]),
                lambda: pool.table(1, 2), lambda: pool.resident_layers(9)):
        with pytest.raises(S.SymphError):
            bad()
    assert pool.counts() == (2, 6, 0) and pool.resident_layers(1) == 2
    got = pool.framework_take(2)
    assert pool.counts() == (0, 6, 2)
    with pytest.raises(S.SymphError):
        pool.framework_give([got[0], got[0]])                      # listed twice
    assert pool.counts() == (0, 6, 2)
    # settle with arrays that are too small reports the need and changes nothing
    pool.advise(7, 16)
    nc, ns = C.c_int32(), C.c_int32()
    assert lib.symph_pool_settle(pool.handle, None, 0, None, 0, C.byref(nc), C.byref(ns)) == -4
    assert (nc.value, ns.value) == (3, 2) and pool.resident_layers(7) == 0 and pool.resident_layers(1) == 2
    # capacity 6: layer 0 of session 1 (3), layer 0 of session 7 (1), layer 1: session 1 does not fit in 2, session 7 does
    got = pool.settle()
    assert sorted(x[:3] for x in got) == [(0, 1, 1), (1, 7, 0), (1, 7, 1)]
    assert pool.resident_layers(1) == 1 and pool.resident_layers(7) == 2 and pool.counts() == (1, 5, 2)


def test_extreme_lengths_and_many_sessions():
    """A session larger than the pool is never admitted (and overflows nothing); ten thousand sessions competing for
    a pool that holds part of their first layer agree with the oracle."""
    pool = S.KvPool(80, 100000, 16)
    sessions = {1: 2 ** 31 - 1, 2: 1, -9: 16000}
    for sid, n in sessions.items():
        pool.advise(sid, n)
    pool.settle()
    want = PR.resident_layers(sessions, 80, 16, 100000)
    assert {sid: pool.resident_layers(sid) for sid in sessions} == want == {1: 0, 2: 80, -9: 80}
    pool.close()
    rng = np.random.default_rng(0)
    lens = {i: int(n) for i, n in enumerate(rng.integers(1, 9000, size=10000))}
    big = S.KvPool(32, 2_000_000, 16)
    for sid, n in lens.items():
        big.advise(sid, n)
    big.settle()
    want = PR.resident_layers(lens, 32, 16, 2_000_000)
    assert all(big.resident_layers(sid) == want[sid] for sid in lens)
    free, lent, fw = big.counts()
    assert fw == 0 and lent == sum(want[s] * PR.blocks_of(lens[s], 16) for s in lens) and free == 2_000_000 - lent
    big.close()
