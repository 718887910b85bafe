"""GPU parity at the full sizes of the five workloads, in the launch configuration
bench.py times (same binding calls, same table shapes).

The oracle cannot hold 10^8..10^9 rows, so it keeps only touched rows: resident keys are
"declared" and materialised from the deterministic initialiser on first use (an untouched
row is a pure function of its key).  Compared per step: unique keys and inverse ranks
(bit-exact, whole arrays), unique/inserted counts, pooled sums (whole array, tolerance);
after the steps: every touched row through hps_get (tolerance; rows that were only
initialised bit-exact), a sample of untouched resident rows against the initialiser
(bit-exact), absent keys reported absent, and the table size.
"""
import time

import numpy as np
import pytest
import torch

import paper_2003_05622_amd as hps
import synth
from oracle import OracleTable

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-6, 1e-5


def dev_keys(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).cuda()


def excess(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float((np.abs(got - want) - (ATOL + RTOL * np.abs(want))).max(initial=-1.0))


def run_full(name, steps, pipelined=False):
    cfg = synth.CONFIGS[name]
    t0 = time.time()
    stream = synth.BatchStream(cfg)
    batches = [stream.next() for _ in range(steps)]
    n_max = max(b.n_keys for b in batches)
    kw = dict(lr=cfg.lr, eps=cfg.eps, init_acc=cfg.init_acc, init_range=cfg.init_range,
              init_seed=cfg.init_seed)
    gt = hps.HpsTable(cfg.capacity, cfg.dim, n_max, cfg.n_bags, **kw)
    chunk = 1 << 23
    for lo in range(0, cfg.n_prefill, chunk):
        gt.insert(dev_keys(synth.prefill_keys(lo, min(lo + chunk, cfg.n_prefill))))
        if (lo // chunk) % 16 == 0:
            print("prefill", lo, "of", cfg.n_prefill, "%.0fs" % (time.time() - t0), flush=True)
    st = gt.stats()
    assert st.error == 0 and st.size == cfg.n_prefill
    ot = OracleTable(cfg.capacity, cfg.dim, **kw)
    ot.declare_resident(cfg.n_prefill)
    touched = []
    # pipelined: the schedule bench.py times by default -- the dedup of mini-batch i+1 is
    # enqueued on a second stream between the pull and the push of mini-batch i
    side = torch.cuda.Stream()
    dev = [(dev_keys(b.keys), torch.from_numpy(b.offsets).cuda()) for b in batches] if pipelined else None
    if pipelined:
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            gt.prepare(dev[0][0], dev[0][1], cfg.n_examples, cfg.n_slots)
    for step, b in enumerate(batches):
        res, fresh = synth.resident_split(cfg, b)
        ot.materialize(res)
        touched.append(np.unique(b.keys))
        if pipelined:
            pooled = gt.pull_prepared()
            if step + 1 < len(batches):
                with torch.cuda.stream(side):
                    gt.prepare(dev[step + 1][0], dev[step + 1][1], cfg.n_examples, cfg.n_slots)
        else:
            pooled = gt.pull(dev_keys(b.keys), torch.from_numpy(b.offsets).cuda(), cfg.n_examples,
                             cfg.n_slots)
        want = ot.pull(b.keys, b.offsets)
        uniq, inv = gt.last_unique()
        ou, oi = ot.last_unique()
        st = gt.stats()
        assert st.error == 0
        assert st.last_n_unique == ot.n_unique and st.last_n_inserted == ot.n_inserted
        assert np.array_equal(uniq.cpu().numpy().view(np.uint64), ou), "unique keys"
        assert np.array_equal(inv.cpu().numpy(), oi), "inverse"
        assert excess(pooled.cpu().numpy(), want) <= 0, "pooled"
        gt.push(torch.from_numpy(b.grads).cuda())
        ot.push(b.grads)
        print("step", step, "N", b.n_keys, "U", ot.n_unique, "inserted", ot.n_inserted,
              "%.0fs" % (time.time() - t0), flush=True)
    assert gt.stats().size == ot.size
    # every touched row
    keys = np.unique(np.concatenate(touched))
    w, a, f = gt.get(dev_keys(keys))
    ow, oa, of = ot.get(keys)
    assert f.all().item() and of.all()
    w, a = w.cpu().numpy(), a.cpu().numpy()
    assert excess(w, ow) <= 0 and excess(a, oa) <= 0
    init_only = (oa == np.float32(cfg.init_acc)).all(axis=1)
    assert np.array_equal(w[init_only].view(np.uint32), ow[init_only].view(np.uint32))
    # untouched resident rows equal the initialiser; keys never seen are absent
    rng = np.random.default_rng(123)
    ids = rng.integers(0, cfg.n_prefill, size=4096, dtype=np.uint64)
    sample = np.setdiff1d(synth.mix64(ids), keys)
    w, a, f = gt.get(dev_keys(sample))
    assert f.all().item()
    want_rows = np.stack([ot.init_row(int(k)) for k in sample])
    assert np.array_equal(w.cpu().numpy().view(np.uint32), want_rows.view(np.uint32))
    assert (a.cpu().numpy() == np.float32(cfg.init_acc)).all()
    absent = synth.mix64(np.arange(2**62, 2**62 + 512, dtype=np.uint64))
    assert not gt.get(dev_keys(absent))[2].any().item()
    return gt


# A table's first two dedups take the plain radix passes, later ones of this size the
# bucket path (it learns the heavy keys from the lookups): four steps cover both.

def test_mid_full_size(monkeypatch):
    monkeypatch.delenv("HPS_DEDUP", raising=False)
    run_full("mid", steps=4)


def test_mid_full_size_default_schedule_of_the_benchmark(monkeypatch):
    monkeypatch.delenv("HPS_DEDUP", raising=False)
    run_full("mid", steps=5, pipelined=True)


def test_insert_heavy_full_size(monkeypatch):
    monkeypatch.delenv("HPS_DEDUP", raising=False)
    run_full("insert_heavy", steps=4)


def test_skewed_full_size(monkeypatch):
    monkeypatch.delenv("HPS_DEDUP", raising=False)
    run_full("skewed", steps=4)


def test_skewed_full_size_bucket_path_without_a_hint(monkeypatch):
    # pinned to the bucket path from the first batch on: the hottest key (a quarter of all
    # occurrences) is not known to be heavy yet, its region is ordered through global memory
    monkeypatch.setenv("HPS_DEDUP", "bucket")
    run_full("skewed", steps=2)


def test_skewed_shifted_full_size(monkeypatch):
    # the "top 1000 keys are about 40 % of the lookups" reading of the skewed workload
    monkeypatch.delenv("HPS_DEDUP", raising=False)
    run_full("skewed_shifted", steps=3)


def test_insert_heavy_all_fifty_steps(monkeypatch):
    """The insert-heavy workload as it is defined: 50 consecutive steps, 0.8 M new keys each,
    the table going from 24 % to 67 % of its slots.  Unique keys, inverse ranks, counts and pooled
    sums every step; every touched row and the size at the end."""
    monkeypatch.delenv("HPS_DEDUP", raising=False)
    run_full("insert_heavy", steps=50)


def test_large_full_size(monkeypatch):
    monkeypatch.delenv("HPS_DEDUP", raising=False)
    run_full("large", steps=4)


def test_dedup_two_million_keys_that_do_not_suit_the_buckets():
    """The dedup at the mid workload's size (2 M occurrences) on key sets the bucket form is
    not made for, in the order that is hardest for its hints: hashed keys first (so the table
    is past its first two dedups), then unhashed consecutive ids, then a key that makes up a
    third of the batch without having been frequent before (one workgroup orders its 7*10^5
    pairs through global memory while a thousand others wait for its count), the same again
    (now announced), long-tailed raw ids (most keys in one part of the range: the library goes
    back to the plain form for a long while), and hashed keys again.  Unique keys and inverse ranks must be the
    oracle's, bit for bit, every time, and no wait may give up."""
    import oracle
    rng = np.random.default_rng(77)
    n, dim, n_bags = 2_000_000, 8, 4096
    gt = hps.HpsTable(12_000_000, dim, n, n_bags)
    offsets = np.minimum(np.arange(n_bags + 1, dtype=np.int64) * ((n + n_bags - 1) // n_bags), n).astype(np.int32)
    d_off = torch.from_numpy(offsets).cuda()
    zero = torch.zeros((n_bags, dim), device="cuda")

    def hashed():
        return synth.mix64(rng.integers(0, 1_500_000, size=n).astype(np.uint64))

    def hot(keys):
        keys = keys.copy()
        keys[rng.random(n) < 0.35] = np.uint64(0x123456789ABCDEF)
        return keys

    cases = [
        ("hashed", hashed()), ("hashed", hashed()), ("hashed", hashed()),
        ("raw consecutive ids", np.uint64(1 << 40) + rng.integers(0, 1_500_000, size=n).astype(np.uint64)),
        ("hashed, one key suddenly a third of the batch", hot(hashed())),
        ("the same key again", hot(hashed())),
        ("long-tailed raw ids", np.minimum(rng.pareto(1.0, size=n) * 1000.0, 5e7).astype(np.uint64)),
        ("long-tailed raw ids", np.minimum(rng.pareto(1.0, size=n) * 1000.0, 5e7).astype(np.uint64)),
        ("hashed", hashed()), ("hashed", hashed()), ("hashed", hashed()),
        ("long-tailed raw ids", np.minimum(rng.pareto(1.0, size=n) * 1000.0, 5e7).astype(np.uint64)),
        ("long-tailed raw ids", np.minimum(rng.pareto(1.0, size=n) * 1000.0, 5e7).astype(np.uint64)),
        ("hashed", hashed()),
    ]
    # two id spaces 2^50 apart, a million ids each: no 40 leading bits tell a space's ids apart
    # (the plain form repairs everything once, then sorts by all 64 bits)
    for _ in range(3):
        low = rng.integers(0, 1_000_000, size=n).astype(np.uint64)
        cases.append(("two id spaces far apart", np.where(rng.random(n) < 0.5, low, np.uint64(1 << 50) + low)))
    cases.append(("hashed", hashed()))
    for what, keys in cases:
        t0 = time.time()
        gt.pull(dev_keys(keys), d_off, n_bags, 1)
        st = gt.stats()
        print(what, "pull %.1f ms" % ((time.time() - t0) * 1e3), "unique", st.last_n_unique,
              "fallbacks", st.n_plain_fallbacks, st.n_full_fallbacks, flush=True)
        ou, oi = oracle.dedup(keys)
        assert st.error == 0 and st.last_n_unique == ou.size, what
        uniq, inv = gt.last_unique()
        assert np.array_equal(uniq.cpu().numpy().view(np.uint64), ou), what + ": unique keys"
        assert np.array_equal(inv.cpu().numpy(), oi), what + ": inverse"
        gt.push(zero)
    # once for the key that turned frequent (a short stay in the plain form: the next hint lists
    # it), once for the long-tailed ids that met the bucket form (a long stay)
    assert gt.stats().n_plain_fallbacks == 2 and gt.stats().n_full_fallbacks == 1


def test_first_pull_creates_three_million_rows():
    """A pull whose keys are nearly all new, so many that the blocks of the lookup cannot
    note all their missing keys and the insert falls back to scanning for them: 3 M distinct
    keys into an empty table.  Unique keys, inverse, the inserted count, pooled rows and a
    sample of the created rows against the oracle."""
    rng = np.random.default_rng(5)
    n, dim, n_bags = 3_000_000, 4, 65536
    keys = synth.mix64(rng.permutation(4_000_000)[:n].astype(np.uint64) + np.uint64(10**12))
    offsets = np.minimum(np.arange(n_bags + 1, dtype=np.int64) * ((n + n_bags - 1) // n_bags), n).astype(np.int32)
    kw = dict(lr=0.05, eps=1e-8, init_acc=0.1, init_range=0.01, init_seed=3)
    gt = hps.HpsTable(4_000_000, dim, n, n_bags, **kw)
    ot = OracleTable(4_000_000, dim, **kw)
    pooled = gt.pull(dev_keys(keys), torch.from_numpy(offsets).cuda(), n_bags, 1)
    want = ot.pull(keys, offsets)
    st = gt.stats()
    assert st.error == 0 and st.last_n_unique == n and st.last_n_inserted == n and st.size == n
    uniq, inv = gt.last_unique()
    ou, oi = ot.last_unique()
    assert np.array_equal(uniq.cpu().numpy().view(np.uint64), ou) and np.array_equal(inv.cpu().numpy(), oi)
    assert excess(pooled.cpu().numpy(), want) <= 0, "pooled"
    gt.push(torch.zeros((n_bags, dim), device="cuda"))
    probe = keys[:: 997]
    w, a, f = gt.get(dev_keys(probe))
    ow, oa, of = ot.get(probe)
    assert f.all() and np.array_equal(w.cpu().numpy(), ow)          # initial rows: bit-exact


def test_dedup_thirteen_million_occurrences():
    """More occurrences than the bucket form takes (1.2 * 10^7): the plain form with six
    passes at a size no workload has.  Unique keys and inverse ranks against the oracle."""
    import oracle
    rng = np.random.default_rng(13)
    n, dim, n_bags = 13_000_000, 4, 4096
    keys = synth.mix64(rng.integers(0, 6_000_000, size=n).astype(np.uint64))
    keys[rng.random(n) < 0.05] = synth.mix64(np.uint64(42))          # and one frequent key
    offsets = np.minimum(np.arange(n_bags + 1, dtype=np.int64) * ((n + n_bags - 1) // n_bags), n).astype(np.int32)
    gt = hps.HpsTable(8_000_000, dim, n, n_bags)
    d_keys, d_off = dev_keys(keys), torch.from_numpy(offsets).cuda()
    zero = torch.zeros((n_bags, dim), device="cuda")
    ou, oi = oracle.dedup(keys)
    for rounds in range(3):       # the third would take the bucket form if the size allowed it
        gt.pull(d_keys, d_off, n_bags, 1)
        st = gt.stats()
        assert st.error == 0 and st.last_n_unique == ou.size
        uniq, inv = gt.last_unique()
        assert np.array_equal(uniq.cpu().numpy().view(np.uint64), ou), "unique keys"
        assert np.array_equal(inv.cpu().numpy(), oi), "inverse"
        gt.push(zero)
