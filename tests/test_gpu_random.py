"""Randomised parity on the GPU: seeded random shapes (dim 4..260, 0..300 000 occurrences,
ragged bags, empty batches), key mixes (hashed Zipf, raw consecutive ids, a handful of
distinct keys, all distinct, one heavy key, long-tailed raw ids), options (both optimizers,
sum / mean pooling, float32 / bfloat16 rows, pooling with the frequent keys' rows in LDS, interleaved accumulates, the serial and the
pipelined schedule) and dedup forms; each case is a few pull+push steps checked against the
oracle step by step and by a final dump."""
import numpy as np
import pytest
import torch

import paper_2003_05622_amd as hps
import oracle
import synth
from oracle import OracleTable

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-6, 1e-5


def dev_keys(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).cuda()


def close(got, want, what, atol=ATOL, rtol=RTOL):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    err = np.abs(got - want) - (atol + rtol * np.abs(want))
    assert err.max(initial=-1) <= 0, "%s: excess %g" % (what, err.max())


def make_keys(rng, n, kind, universe):
    if kind == 0:       # hashed, Zipf-distributed
        ranks = np.minimum(rng.zipf(1.2, size=n), universe) - 1
        return synth.mix64(ranks.astype(np.uint64))
    if kind == 1:       # raw consecutive ids at some offset
        return np.uint64(rng.integers(0, 2**40)) + rng.integers(0, universe, size=n).astype(np.uint64)
    if kind == 2:       # a handful of distinct keys
        pool = synth.mix64(rng.integers(0, 2**30, size=int(rng.integers(1, 9))).astype(np.uint64))
        return pool[rng.integers(0, pool.size, size=n)]
    if kind == 3:       # all distinct
        return synth.mix64(np.uint64(rng.integers(0, 2**40)) + np.arange(n, dtype=np.uint64))
    if kind == 4:       # one heavy key among uniform hashed ones
        keys = synth.mix64(rng.integers(0, universe, size=n).astype(np.uint64))
        keys[rng.random(n) < rng.random() * 0.9] = np.uint64(rng.integers(0, 2**63))
        return keys
    return np.minimum(rng.pareto(1.0, size=n) * 100.0, 1e9).astype(np.uint64)   # long-tailed raw ids


def pooled_from_rows(rows, inverse, offsets, n_bags, dim, mean):
    """The definition of the pooling in float64: the sum (or mean) over each bag's occurrences of
    the row of its key; rows[u] is the row of unique key u, inverse[i] the unique index of
    occurrence i."""
    out = np.zeros((n_bags, dim))
    lengths = np.diff(offsets)
    if inverse.size:
        np.add.at(out, np.repeat(np.arange(n_bags), lengths), rows[inverse].astype(np.float64))
    if mean:
        out /= np.maximum(lengths, 1)[:, None]
    return out


def run_case(seed, monkeypatch, sizes=(1, 50, 3000, 70000, 300000)):
    rng = np.random.default_rng(seed)
    dim = int(rng.choice([4, 8, 12, 16, 32, 64, 100, 128, 256, 260]))
    n_bags_max = int(rng.choice([1, 7, 64, 1000, 20000]))
    n_max = int(rng.choice(sizes))
    if dim >= 128:
        n_max = min(n_max, 70000)
    # bags of thousands of rows are outside the float32 tolerance: mean bag length <= 32
    n_bags_max = max(n_bags_max, n_max // 16 + 1)
    opt = int(rng.integers(0, 2))
    mean = bool(rng.integers(0, 2))
    bf16 = bool(rng.integers(0, 4) == 0)
    form = ["auto", "bucket", "radix"][int(rng.integers(0, 3))]
    if form == "auto":
        monkeypatch.delenv("HPS_DEDUP", raising=False)
    else:
        monkeypatch.setenv("HPS_DEDUP", form)       # read when the table is created
    universe = int(rng.choice([10, 1000, 100000, 10**7]))
    # one case in four pools with the most frequent keys' rows held in LDS (off by default)
    lds_rows = bool(rng.integers(0, 4) == 0)
    if lds_rows:
        monkeypatch.setenv("HPS_POOL", "lds")       # read when the table is created
    else:
        monkeypatch.delenv("HPS_POOL", raising=False)
    kw = dict(opt=opt, lr=0.05, eps=1e-8, init_acc=0.1, init_range=0.01,
              init_seed=int(rng.integers(0, 2**32)))
    print("seed", seed, "dim", dim, "max bags", n_bags_max, "max n", n_max, "opt", opt, "mean", mean,
          "bf16", bf16, "form", form, "universe", universe, "lds rows", lds_rows, flush=True)
    capacity = max(2_000_000, 6 * n_max)
    gt = hps.HpsTable(capacity, dim, n_max, n_bags_max,
                      row_format=hps.ROWS_BF16 if bf16 else hps.ROWS_F32, **kw)
    ot = OracleTable(capacity, dim, row_format=oracle.ROWS_BF16 if bf16 else oracle.ROWS_F32, **kw)
    if mean:
        gt.set_pooling(True)
        ot.set_pooling(True)
    steps = int(rng.integers(1, 6))
    # the default schedule of the benchmark: the dedup of the next mini-batch is enqueued on a
    # second stream between the current pull and its push
    pipelined = bool(rng.integers(0, 2))
    batches = []
    for step in range(steps):
        n = int(rng.integers(0, n_max + 1)) if rng.random() < 0.8 else n_max
        n_bags = int(rng.integers(max(1, n // 32), n_bags_max + 1))
        # ragged bags (some empty) of at most about 2 * n / n_bags occurrences
        grid = (np.arange(1, n_bags, dtype=np.int64) * n) // n_bags
        half = max(1, n // n_bags // 2)
        cuts = np.sort(np.clip(grid + rng.integers(-half, half + 1, size=n_bags - 1), 0, n))
        offsets = np.concatenate([[0], cuts, [n]]).astype(np.int32)
        keys = make_keys(rng, n, int(rng.integers(0, 6)), universe) if n else np.zeros(0, np.uint64)
        grads = rng.normal(0, 1e-3, size=(n_bags, dim)).astype(np.float32)
        batches.append((keys, offsets, grads, dev_keys(keys), torch.from_numpy(offsets).cuda()))
    side = torch.cuda.Stream()

    def prepare(i):
        keys, offsets, _, dk, do = batches[i]
        side.wait_stream(torch.cuda.current_stream())      # the inputs were copied on this stream
        with torch.cuda.stream(side):
            gt.prepare(dk, do, offsets.size - 1, 1)

    if pipelined:
        prepare(0)
    for step in range(steps):
        keys, offsets, grads, dk, do = batches[step]
        n, n_bags = keys.size, offsets.size - 1
        if pipelined:
            pooled = gt.pull_prepared()
            if step + 1 < steps:
                prepare(step + 1)
        else:
            pooled = gt.pull(dk, do, n_bags, 1)
        want = ot.pull(keys, offsets)
        st = gt.stats()
        assert st.error == 0
        assert st.last_n_unique == ot.n_unique and st.last_n_inserted == ot.n_inserted
        uniq, inv = gt.last_unique()
        ou, oi = ot.last_unique()
        assert np.array_equal(uniq.cpu().numpy().view(np.uint64), ou), "unique keys"
        assert np.array_equal(inv.cpu().numpy(), oi), "inverse"
        # Pooled sums at the stated tolerance, in two parts.  Against the pooling (written out in
        # float64) of the rows the GPU table itself holds: that isolates the pooling kernel from
        # whatever the two sides' weights have drifted apart by.  And against the oracle: at step
        # 0 both tables hold bit-identical rows; later the weights differ in their last bits (each
        # side within the tolerance of the exact update), and a bag of rows of both signs can
        # cancel to a sum much smaller than those differences, so the oracle comparison then
        # allows the weights' tolerance per summed row.
        gpu = pooled.cpu().numpy().astype(np.float64)
        if n:
            w_gpu = gt.get(dev_keys(ou))[0].cpu().numpy()
            close(gpu, pooled_from_rows(w_gpu, oi, offsets, n_bags, dim, mean), "pooled against the table's own rows")
        if step == 0:
            close(gpu, want, "pooled at step 0")
        elif not bf16 and n:
            mag = pooled_from_rows(np.abs(ot.get(ou)[0]), oi, offsets, n_bags, dim, mean)
            err = np.abs(gpu - want) - (ATOL + RTOL * np.abs(want) + RTOL * mag)
            assert err.max(initial=-1) <= 0, "pooled: excess %g" % err.max()
        gt.push(torch.from_numpy(grads).cuda())
        ot.push(grads)
        if rng.random() < 0.3 and n and not pipelined:     # (not between a prepare and its pull)
            k2 = keys[: max(1, n // 3)]
            v2 = rng.normal(0, 1e-3, size=(k2.size, dim)).astype(np.float32)
            gt.accumulate(dev_keys(k2), torch.from_numpy(v2).cuda())
            ot.accumulate(k2, v2)
    torch.cuda.synchronize()
    k, w, a = gt.dump()
    k = k.cpu().numpy().view(np.uint64)
    order = np.argsort(k, kind="stable")
    ok, ow, oa = ot.dump()
    assert np.array_equal(k[order], ok), "key sets"
    if bf16:    # a few bfloat16 steps of the size the weights have had
        close(w.cpu().numpy()[order], ow, "weights", atol=ATOL + 2e-4 * steps, rtol=RTOL + 4 * 2.0 ** -7)
    else:
        close(w.cpu().numpy()[order], ow, "weights")
    close(a.cpu().numpy()[order], oa, "accumulators")
    assert gt.stats().size == ot.size


@pytest.mark.parametrize("seed0", [11, 12, 13])
def test_random_cases_against_the_oracle(seed0, monkeypatch):
    for case in range(40):
        run_case(seed0 * 100000 + case, monkeypatch)
