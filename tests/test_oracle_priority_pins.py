"""Pins of the residency oracle (oracle/priority.py) against things it did not produce itself: hand-derived cases
(tests/golden/priority_cases.txt, Sec. 3.3 of arxiv 2412.16434), a closed form for equal sessions, invariants on
seeded random inputs, and an exhaustive search on tiny inputs for the property that defines the admission walk."""
import itertools
import os

import numpy as np
import pytest

from oracle import priority as PR

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "priority_cases.txt")


def golden_cases():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, shape, sess, res, order = [f.strip() for f in line.split("|")]
        L, bs, cap = map(int, shape.split())
        sessions = {int(a): int(b) for a, b in (x.split(":") for x in sess.split())}
        resident = {int(a): int(b) for a, b in (x.split(":") for x in res.split())}
        evict = [tuple(map(int, x.split(","))) for x in order.split()]
        cases.append(pytest.param(L, bs, cap, sessions, resident, evict, id=name))
    return cases


@pytest.mark.parametrize("L,bs,cap,sessions,resident,evict", golden_cases())
def test_hand_derived_cases(L, bs, cap, sessions, resident, evict):
    got = PR.resident_layers(sessions, L, bs, cap)
    assert got == resident
    assert PR.eviction_order(got, sessions, bs) == evict


def test_framework_demand_takes_the_shortest_beginning_of_the_order():
    # three_cap36 of the golden file, nothing free: 7 slots wanted -> layer 1 of session 2 (3) and of session 3 (5)
    sessions = {1: 160, 2: 48, 3: 80}
    res = {1: 2, 2: 2, 3: 2}
    assert PR.evicted_to_free(res, sessions, 16, 0, 7) == [(1, 2), (1, 3)]
    assert PR.evicted_to_free(res, sessions, 16, 0, 8) == [(1, 2), (1, 3)]
    assert PR.evicted_to_free(res, sessions, 16, 0, 9) == [(1, 2), (1, 3), (1, 1)]
    assert PR.evicted_to_free(res, sessions, 16, 7, 7) == []          # already free
    assert PR.evicted_to_free(res, sessions, 16, 0, 36) == [(1, 2), (1, 3), (1, 1), (0, 2), (0, 3), (0, 1)]


@pytest.mark.parametrize("S,L,b,cap", [(2, 32, 128, 4096), (3, 8, 5, 61), (5, 4, 7, 7 * 20), (4, 6, 3, 1000), (4, 6, 3, 2), (1, 80, 2048, 100000)])
def test_equal_sessions_closed_form(S, L, b, cap):
    """Equal sizes: units are admitted in the order (layer, session), floor(cap / b) of them at most, so session
    number k (by id) holds q + (k < rem) layers, (q, rem) = divmod(min(floor(cap / b), S * L), S)."""
    bs = 16
    sessions = {100 + k: b * bs - 3 for k in range(S)}      # b blocks, the last one partly used
    q, rem = divmod(min(cap // b, S * L), S)
    want = {100 + k: q + (1 if k < rem else 0) for k in range(S)}
    assert PR.resident_layers(sessions, L, bs, cap) == want


def random_sessions(rng, S, bs):
    return {int(s): int(n) for s, n in zip(rng.permutation(1000)[:S], rng.integers(1, 40 * bs, size=S))}


@pytest.mark.parametrize("seed", range(40))
def test_invariants_on_random_inputs(seed):
    rng = np.random.default_rng(7000 + seed)
    bs = int(rng.choice([8, 16, 32]))
    L = int(rng.integers(1, 9))
    sessions = random_sessions(rng, int(rng.integers(1, 9)), bs)
    b = {s: PR.blocks_of(n, bs) for s, n in sessions.items()}
    total = L * sum(b.values())
    for cap in {0, 1, total // 3, total // 2, total - 1, total, total + 5}:
        cap = max(cap, 0)
        r = PR.resident_layers(sessions, L, bs, cap)
        used = sum(r[s] * b[s] for s in sessions)
        assert used <= cap and all(0 <= r[s] <= L for s in sessions)
        if cap >= total:
            assert all(r[s] == L for s in sessions)
        # nothing admissible was left out: the next layer of any session does not fit in what is left
        assert all(r[s] == L or b[s] > cap - used for s in sessions)
        # among sessions of one size, layers differ by at most one and the smaller id is the one ahead
        for s, t in itertools.combinations(sorted(sessions), 2):
            if b[s] == b[t]:
                assert r[s] - r[t] in (0, 1)
        order = PR.eviction_order(r, sessions, bs)
        assert len(order) == sum(r.values()) and len(set(order)) == len(order)
        layers = [l for l, _ in order]
        assert layers == sorted(layers, reverse=True)                       # later layers go first
        for (l0, s0), (l1, s1) in zip(order, order[1:]):
            if l0 == l1:
                assert (b[s0], -s0) < (b[s1], -s1)                          # within a layer the smallest first
        # and the order is the reverse of the order of admission
        adm = [u for u in PR.units_by_priority(sessions, L, bs) if u[0] < r[u[1]]]
        assert order == adm[::-1]


def test_admission_walk_against_exhaustive_search():
    """Tiny inputs, every capacity: the resident set is the lexicographically greatest admission vector over the
    priority order among all sets that fit and hold, for every session, layers 0..r-1 without gaps (that is what
    "walk in priority order and take what fits" means), found here by trying all vectors r."""
    rng = np.random.default_rng(99)
    for _ in range(25):
        bs, L = 16, int(rng.integers(1, 4))
        sessions = random_sessions(rng, int(rng.integers(1, 4)), bs)
        sids = sorted(sessions)
        b = {s: PR.blocks_of(sessions[s], bs) for s in sids}
        # the priority order written out independently: layer, then blocks descending, then id
        order = sorted(((l, s) for s in sids for l in range(L)), key=lambda u: (u[0], -b[u[1]], u[1]))
        for cap in range(0, L * sum(b.values()) + 2, max(1, sum(b.values()) // 3)):
            best = None
            for vec in itertools.product(range(L + 1), repeat=len(sids)):
                if sum(v * b[s] for v, s in zip(vec, sids)) > cap:
                    continue
                r = dict(zip(sids, vec))
                bits = tuple(1 if l < r[s] else 0 for l, s in order)
                if best is None or bits > best[0]:
                    best = (bits, r)
            assert PR.resident_layers(sessions, L, bs, cap) == best[1]


def test_pool_model_follows_the_section_s_scenario():
    """Sec. 3.3's scenario: session 2 is moved in and fills the memory, then session 3 is announced: the lower layers
    of both end up resident.  Then memory pressure from the framework takes the later layers first, and a request that
    arrives hands the resident layers over without a transfer."""
    m = PR.PoolModel(n_layers=4, n_slots=16, block_size=16)
    assert m.advise(2, 64)
    ev, ld = m.settle()
    assert ev == [] and ld == [(0, 2), (1, 2), (2, 2), (3, 2)] and m.free() == 0
    assert m.advise(3, 64)
    ev, ld = m.settle()
    assert sorted(ev) == [(2, 2), (3, 2)] and ld == [(0, 3), (1, 3)]
    assert m.resident == {2: 2, 3: 2}
    gone = m.take(5)                                   # pressure: 5 slots -> layer 1 of both (4 + 4)
    assert gone == [(1, 3), (1, 2)] and m.framework == 5 and m.free() == 3 and m.lent() == 8
    assert m.take(12) is None                          # only 11 are not the framework's
    assert m.claim(2) == 1 and m.framework == 9       # request for session 2: its layer 0 is simply kept
    ev, ld = m.settle()                                # 7 slots outside the framework: layer 1 of session 3 (4 + 4) stays out
    assert ev == [(1, 3), (1, 2)] and ld == [] and m.resident == {3: 1} and m.free() == 3
    assert m.give(1)                                   # one slot back: now 8 can be lent
    assert m.settle() == ([], [(1, 3)]) and m.free() == 0
    assert not m.advise(3, 65) and m.drop(3) and m.free() == 8 and not m.drop(3)
    assert m.settle() == ([(1, 3), (0, 3)], [])
    assert m.give(8) and m.free() == 16 and not m.give(1)
