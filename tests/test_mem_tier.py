"""The host-memory parameter cache (paper: Appendix D, cache policy).  The oracle
(oracle/mem_tier.py) is pinned by a hand-worked trace, by its reduction to textbook LRU and LFU
caches, and by invariants under random operations; the product's implementation (through the C
ABI, host memory only: no GPU needed) must then agree with the oracle operation by operation."""
import collections
import os

import numpy as np
import pytest

from oracle.mem_tier import MemTierOracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def row(key, dim=4):
    return np.full(dim, float(key), np.float32), np.array([key + 0.5], np.float32)


def visit(t, batch, keys):
    """Visits keys: held ones are fetched, the others stored as new arrivals."""
    _, _, found = t.fetch(keys, batch)
    new = [k for k, f in zip(keys, found) if not f]
    if new:
        t.store(new, np.stack([row(k)[0] for k in new]), np.stack([row(k)[1] for k in new]), batch, True)


def run_trace(make):
    t = make(4, 1, 2, 2)
    out = []
    for line in open(os.path.join(ROOT, "tests", "golden", "mem_tier_trace.txt")):
        parts = line.split()
        if not parts or parts[0].startswith("#"):
            continue
        if parts[0] == "visit":
            visit(t, int(parts[1]), [int(k) for k in parts[2:]])
        elif parts[0] == "complete":
            t.complete_batch(int(parts[1]))
            out += [k for k, _, _ in t.take_evicted()]
        else:
            want = dict(p.split("=") for p in parts[1:])
            lst = lambda s: [int(k) for k in s.split(",")] if s else []
            assert t.lru_keys() == lst(want["lru"]), line
            assert t.lfu_keys() == lst(want["lfu"]), line
            assert out == lst(want["out"]), line


class OracleView(MemTierOracle):
    def lru_keys(self):
        return list(self.lru)

    def lfu_keys(self):
        return list(self.lfu)


def test_oracle_follows_the_hand_worked_trace():
    run_trace(OracleView)


def test_oracle_without_an_lfu_cache_is_a_textbook_lru_cache():
    """One key per batch, LFU capacity 0: what is collected, and when, is what a plain LRU cache
    of the same capacity evicts (simulated with an ordered dictionary)."""
    rng = np.random.default_rng(0)
    t = OracleView(4, 1, 3, 0)
    ref = collections.OrderedDict()
    for b, k in enumerate(rng.integers(0, 8, size=400).tolist()):
        visit(t, b, [k])
        t.complete_batch(b)
        got = [e[0] for e in t.take_evicted()]
        ref[k] = True
        ref.move_to_end(k)
        want = []
        while len(ref) > 3:
            want.append(ref.popitem(last=False)[0])
        assert got == want
        assert t.lru_keys() == list(reversed(ref))


def test_oracle_without_an_lru_cache_is_a_textbook_lfu_cache():
    """One key per batch, LRU capacity 0: every completed key drops into the LFU cache at once;
    the key collected is always one of least frequency among those held."""
    rng = np.random.default_rng(1)
    t = OracleView(4, 1, 0, 3)
    counts = collections.Counter()
    for b, k in enumerate(rng.integers(0, 8, size=400).tolist()):
        held_before = set(t.lfu_keys())
        visit(t, b, [k])
        counts[k] += 1
        t.complete_batch(b)
        gone = [e[0] for e in t.take_evicted()]
        assert len(gone) <= 1 and t.lru_keys() == []
        if gone:
            candidates = held_before | {k}
            assert counts[gone[0]] == min(counts[c] for c in candidates)
            del counts[gone[0]]               # its frequency starts over when it comes back
        assert len(t.lfu_keys()) <= 3


def random_ops(make, seed, n_ops=300):
    """Random visits by overlapping batches (up to three open at a time), value updates and
    completions; returns every observable after every operation."""
    rng = np.random.default_rng(seed)
    t = make(4, 1, int(rng.integers(0, 6)), int(rng.integers(0, 6)))
    open_batches, next_batch, log = [], 0, []
    truth = {}
    for _ in range(n_ops):
        r = rng.random()
        if r < 0.5 or not open_batches:
            if len(open_batches) < 3 and (rng.random() < 0.5 or not open_batches):
                open_batches.append(next_batch)
                next_batch += 1
            b = int(rng.choice(open_batches))
            keys = rng.integers(0, 24, size=int(rng.integers(1, 6))).tolist()
            w, a, found = t.fetch(keys, b)
            for i, k in enumerate(keys):
                if found[i]:
                    assert np.array_equal(w[i], truth[k][0]) and np.array_equal(a[i], truth[k][1])
            new = sorted(set(k for k, f in zip(keys, found) if not f))
            if new:
                vals = {k: (rng.normal(size=4).astype(np.float32), rng.normal(size=1).astype(np.float32)) for k in new}
                t.store(new, np.stack([vals[k][0] for k in new]), np.stack([vals[k][1] for k in new]), b, True)
                truth.update(vals)
            log.append(("fetch", tuple(found.tolist())))
        elif r < 0.7:
            held = t.lru_keys()
            if held:                                    # the collect step: new values, no visit
                k = int(rng.choice(held))
                truth[k] = (rng.normal(size=4).astype(np.float32), rng.normal(size=1).astype(np.float32))
                t.store([k], truth[k][0][None], truth[k][1][None], open_batches[0], False)
        else:
            b = open_batches.pop(int(rng.integers(0, len(open_batches))))
            t.complete_batch(b)
            gone = t.take_evicted()
            for k, w, a in gone:
                assert np.array_equal(w, truth[k][0]) and np.array_equal(a, truth[k][1])
                del truth[k]
            log.append(("evicted", tuple(k for k, _, _ in gone)))
        log.append(("state", tuple(t.lru_keys()), tuple(t.lfu_keys())))
        # every held key is in exactly one of the two caches
        assert sorted(t.lru_keys() + t.lfu_keys()) == sorted(truth)
    return log, t


@pytest.mark.parametrize("seed", range(20))
def test_oracle_invariants_under_random_operations(seed):
    log, t = random_ops(OracleView, seed)
    for b in list(t.batch_keys):
        t.complete_batch(b)
    # nothing pinned any more: both caches within their capacities
    assert len(t.lru_keys()) <= t.lru_capacity and len(t.lfu_keys()) <= t.lfu_capacity


# ---- the product's implementation against the oracle (host memory only) ------------------

def native(dim, acc_len, lru_capacity, lfu_capacity):
    import paper_2003_05622_amd as hps
    return hps.MemTier(dim, acc_len, lru_capacity, lfu_capacity)


def test_native_follows_the_hand_worked_trace():
    run_trace(native)


@pytest.mark.parametrize("seed", range(20))
def test_native_agrees_with_the_oracle_operation_by_operation(seed):
    want, _ = random_ops(OracleView, seed)
    got, _ = random_ops(native, seed)
    assert got == want


def test_native_rejects_bad_arguments():
    import ctypes
    import paper_2003_05622_amd as hps
    L = hps.lib()
    h = ctypes.c_void_p()
    assert L.hps_mem_create(None, 4, 1, 2, 2) == hps.EINVAL
    assert L.hps_mem_create(ctypes.byref(h), 0, 1, 2, 2) == hps.EINVAL
    assert L.hps_mem_fetch(None, None, 0, 0, None, None, None) == hps.EINVAL
    assert L.hps_mem_destroy(None) == hps.EINVAL
