"""Host-side residency manager (catalog id -> GPU slot): the outcomes the paper prints for its
cold-load control probes, and the rules of its cache-tier table.  No GPU needed."""
import numpy as np
import pytest


@pytest.fixture(scope="module")
def R():
    from paper_2605_13779_amd import binding
    binding.load_library()
    return binding.Resident


def load(r, cid):
    """Request + immediate completion; returns the slot."""
    res, slot, _ = r.request(cid)
    assert res == r.LOAD, res
    r.complete(cid)
    return slot


def test_bounded_cold_burst_loads_two_rejects_two(R):
    """Appendix cold-load table, probe A4: max in-flight 1 and queue depth 1, a burst of four cold
    requests for different adapters loads 2 and rejects 2; the rejected ones can be retried."""
    r = R(n_slots=8, max_in_flight=1, max_queue=1)
    for cid in (10, 11, 12, 13):
        r.register(cid)
    results = [r.request(cid)[0] for cid in (10, 11, 12, 13)]
    assert results == [r.LOAD, r.QUEUED, r.REJECTED, r.REJECTED]
    nxt, nslot, _ = r.complete(10)
    assert nxt == 11 and nslot >= 0                      # the queued job starts when the first ends
    assert r.complete(11) == (-1, -1, -1)
    st = r.stats()
    assert st["loads"] == 2 and st["rejects"] == 2
    assert r.lookup(10) >= 0 and r.lookup(11) >= 0 and r.lookup(12) == -1 and r.lookup(13) == -1
    assert r.request(12)[0] == r.LOAD                    # retry succeeds once there is room


def test_same_adapter_misses_share_one_load(R):
    """Probe A2: concurrent cache-miss requests for the same missing adapter share one load."""
    r = R(n_slots=4, max_in_flight=1, max_queue=4)
    r.register(77)
    first = r.request(77)
    assert first[0] == r.LOAD
    assert all(r.request(77)[0] == r.PENDING for _ in range(15))
    r.complete(77)
    st = r.stats()
    assert st["loads"] == 1 and st["shared"] == 15
    assert r.request(77)[0:2] == (r.READY, first[1])


def test_unique_adapters_are_separate_jobs_in_arrival_order(R):
    """Different missing adapters remain separate load jobs and pass through the single load path
    one after the other (the staircase of probe A2 / A3), in arrival order."""
    r = R(n_slots=16, max_in_flight=1, max_queue=16)
    ids = list(range(100, 116))
    for cid in ids:
        r.register(cid)
    assert r.request(ids[0])[0] == r.LOAD
    assert all(r.request(cid)[0] == r.QUEUED for cid in ids[1:])
    order, cur = [ids[0]], ids[0]
    while True:
        nxt, _, _ = r.complete(cur)
        if nxt < 0:
            break
        order.append(nxt)
        cur = nxt
    assert order == ids and r.stats()["loads"] == 16
    assert sorted(r.lookup(cid) for cid in ids) == list(range(16))


def test_registered_and_prewarming_are_not_visible(R):
    """A revision is exposed to traffic only when ready (registered -> prewarming -> ready)."""
    r = R(n_slots=2)
    with pytest.raises(Exception):
        r.request(5)                                     # never registered
    r.register(5)
    assert r.lookup(5) == -1                             # registered
    res, slot, _ = r.request(5)
    assert res == r.LOAD and r.lookup(5) == -1           # prewarming
    r.complete(5)
    assert r.lookup(5) == slot                           # ready
    r.register(6)
    res, slot6, _ = r.request(6)
    r.complete(6, ok=False)                              # a failed load leaves no trace
    assert r.lookup(6) == -1 and r.request(6)[0] == r.LOAD


def test_lru_eviction_and_pins(R):
    """GPU batch tier: least recently used ready adapter gives way; slots of the running batch are pinned."""
    r = R(n_slots=2, max_in_flight=1, max_queue=0)
    for cid in (1, 2, 3, 4):
        r.register(cid)
    s1, s2 = load(r, 1), load(r, 2)
    assert {s1, s2} == {0, 1}
    assert r.request(1)[0] == r.READY                    # touch 1: 2 is now the least recently used
    res, slot, ev = r.request(3)
    assert (res, slot, ev) == (r.LOAD, s2, 2)
    r.complete(3)
    assert r.lookup(2) == -1 and r.lookup(1) == s1 and r.lookup(3) == s2
    r.pin(s1), r.pin(s2)
    assert r.request(4)[0] == r.REJECTED                 # nothing evictable, no queue
    r.pin(s1, False)
    res, slot, ev = r.request(4)
    assert (res, slot, ev) == (r.LOAD, s1, 1)
    assert r.stats()["evictions"] == 2


def test_million_id_catalog_against_a_python_model(R):
    """Ids from a 10^6 catalog, Zipf-like traffic, against a dictionary model of the same rules."""
    g = np.random.default_rng(3)
    n_slots = 64
    r = R(n_slots=n_slots, max_in_flight=1, max_queue=0)
    ids = g.choice(10 ** 6, size=500, replace=False)
    for cid in ids:
        r.register(int(cid))
    order, slot_of = [], {}                              # model: LRU list (front = most recent), id -> slot
    free = list(range(n_slots))
    p = 1.0 / np.arange(1, len(ids) + 1) ** 1.1
    for cid in g.choice(ids, size=4000, p=p / p.sum()):
        cid = int(cid)
        res, slot, ev = r.request(cid)
        if cid in slot_of:
            assert (res, slot, ev) == (r.READY, slot_of[cid], -1)
            order.remove(cid)
        else:
            assert res == r.LOAD
            if free:
                want, want_ev = free.pop(0), -1
            else:
                want_ev = order.pop()
                want = slot_of.pop(want_ev)
            assert (slot, ev) == (want, want_ev)
            slot_of[cid] = slot
            r.complete(cid)
        order.insert(0, cid)
    assert r.stats()["hits"] + r.stats()["loads"] == 4000
