"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Integer results (unique keys, inverse indices, key sets, sizes,
rows that were only initialised) are bit-exact; float32 results (pooled sums,
updated weights and accumulators) within |gpu - oracle| <= 1e-6 + 1e-5 * |oracle|."""
import numpy as np
import pytest
import torch

import oracle
import paper_2003_05622_amd as hps
import synth
from oracle import OracleTable

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["auto", "bucket", "radix"], autouse=True)
def dedup_form(request, monkeypatch):
    """Every test runs with the dedup chosen by size and history (small batches and a table's
    first two take the plain radix passes), pinned to the bucket path (so that tiny and odd
    inputs, and batches without a hint about heavy keys, go through it too) and pinned to the
    plain passes.  The library reads the variable when a table is created."""
    if request.param == "auto":
        monkeypatch.delenv("HPS_DEDUP", raising=False)
    else:
        monkeypatch.setenv("HPS_DEDUP", request.param)
    return request.param

ATOL, RTOL = 1e-6, 1e-5


def dev_keys(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).cuda()


def host_keys(t):
    return t.cpu().numpy().view(np.uint64)


def assert_close(got, want, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, what
    err = np.abs(got - want) - (ATOL + RTOL * np.abs(want))
    assert err.max(initial=-1.0) <= 0, "%s: worst excess %g at %s" % (
        what, err.max(), np.unravel_index(err.argmax(), err.shape))


def compare_tables(gt, ot, what, touched_keys=None):
    """touched_keys: keys whose rows may differ in the last bits (default: the rows whose
    accumulator has moved; an accumulate leaves no such trace, so its tests pass the keys)."""
    k, w, a = gt.dump()
    k, w, a = host_keys(k), w.cpu().numpy(), a.cpu().numpy()
    order = np.argsort(k, kind="stable")
    k, w, a = k[order], w[order], a[order]
    ok, ow, oa = ot.dump()
    assert np.array_equal(k, ok), what + ": key sets differ"
    assert_close(w, ow, what + " weights")
    assert_close(a, oa, what + " accumulators")
    untouched = (oa == np.float32(ot_init_acc(ot))).all(axis=1)
    if touched_keys is not None:
        untouched &= ~np.isin(ok, touched_keys)
    assert np.array_equal(w[untouched].view(np.uint32), ow[untouched].view(np.uint32)), \
        what + ": rows that were only initialised must be bit-identical"
    assert gt.stats().size == ot.size


def ot_init_acc(ot):
    return ot._init_acc


def make_pair(cfg, max_keys, opt=hps.ADAGRAD_ROWWISE, row_format=hps.ROWS_F32):
    kw = dict(lr=cfg.lr, eps=cfg.eps, init_acc=cfg.init_acc, init_range=cfg.init_range,
              init_seed=cfg.init_seed)
    gt = hps.HpsTable(cfg.capacity, cfg.dim, max_keys, cfg.n_bags, opt=opt, row_format=row_format, **kw)
    # (the wide format is a layout of float32 rows: the same values)
    ot = OracleTable(cfg.capacity, cfg.dim, opt=opt, **kw,
                     row_format=oracle.ROWS_BF16 if row_format == hps.ROWS_BF16 else oracle.ROWS_F32)
    ot._init_acc = cfg.init_acc
    return gt, ot


def run_steps(cfg, steps, opt=hps.ADAGRAD_ROWWISE, check_every=1, mean=False, row_format=hps.ROWS_F32):
    stream = synth.BatchStream(cfg)
    mean_bag = cfg.bag_mean if cfg.bag_kind == "poisson" else cfg.bag_hi
    max_keys = int(cfg.n_bags * mean_bag * 1.5) + 4096
    gt, ot = make_pair(cfg, max_keys, opt, row_format)
    pre = synth.prefill_keys(0, cfg.n_prefill)
    gt.insert(dev_keys(pre))
    ot.insert(pre)
    if mean:
        gt.set_pooling(True)
        ot.set_pooling(True)
    touched = []
    for step in range(steps):
        b = stream.next()
        touched.append(np.unique(b.keys))
        print("step", step, "N", b.n_keys, flush=True)
        dk, do = dev_keys(b.keys), torch.from_numpy(b.offsets).cuda()
        pooled = gt.pull(dk, do, cfg.n_examples, cfg.n_slots)
        want = ot.pull(b.keys, b.offsets)
        if step % check_every == 0:
            uniq, inv = gt.last_unique()
            ou, oi = ot.last_unique()
            st = gt.stats()
            assert st.error == 0
            assert st.last_n_unique == ot.n_unique and st.last_n_inserted == ot.n_inserted
            assert np.array_equal(host_keys(uniq), ou), "unique keys"
            assert np.array_equal(inv.cpu().numpy(), oi), "inverse"
            assert_close(pooled.cpu().numpy(), want, "pooled step %d" % step)
        gt.push(torch.from_numpy(b.grads).cuda())
        ot.push(b.grads)
    # (a touched row's accumulator can round back to its initial value when the gradients
    # are tiny, so the touched keys are named rather than inferred from the accumulators)
    compare_tables(gt, ot, cfg.name, np.concatenate(touched))
    return gt, ot


def test_tiny_config_full_size():
    run_steps(synth.CONFIGS["tiny"], steps=3)


@pytest.mark.parametrize("opt", [hps.ADAGRAD_ROWWISE, hps.ADAGRAD_ELEMENTWISE])
@pytest.mark.parametrize("name,n_prefill,n_examples,n_slots", [
    ("mid", 60_000, 96, 50),               # dim 16: a row and its accumulator(s) in one or two lines
    ("skewed", 40_000, 128, 32),           # dim 64: records of three (row-wise) or four lines
    ("tiny", 20_000, 64, 20),              # dim 8
])
def test_wide_rows(name, n_prefill, n_examples, n_slots, opt):
    """HPS_ROWS_F32_WIDE: every row's accumulators behind its weights, records padded to whole
    128-byte lines.  A layout only: the same results as with plain float32 rows, to the same
    bar; get / dump / dump_dirty / accumulate / clear go through the same row accessors."""
    cfg = synth.scaled(synth.CONFIGS[name], n_prefill=n_prefill, n_examples=n_examples,
                       n_slots=n_slots, steps=4)
    gt, ot = run_steps(cfg, steps=4, opt=opt, row_format=hps.ROWS_F32_WIDE)
    rng = np.random.default_rng(5)
    k, w, a = gt.dump()
    k = host_keys(k)
    pick = k[rng.integers(0, k.size, size=min(k.size, 2000))]
    v = rng.normal(0, 1e-3, size=(pick.size, cfg.dim)).astype(np.float32)
    gt.accumulate(dev_keys(pick), torch.from_numpy(v).cuda())
    ot.accumulate(pick, v)
    compare_tables(gt, ot, "wide rows after accumulate", pick)
    gw, ga, found = gt.get(dev_keys(pick[:100]))
    ow, oa, of = ot.get(pick[:100])
    assert found.cpu().numpy().all() and of.all()
    assert_close(gw.cpu().numpy(), ow, "get weights")
    assert_close(ga.cpu().numpy(), oa, "get accumulators")
    dk, dw, da = gt.dump(dirty=True)
    assert np.array_equal(np.sort(host_keys(dk)), ot.dump_dirty()[0])
    gt.clear()
    assert gt.stats().size == 0


@pytest.mark.parametrize("room", ["0", "5"])
def test_lookup_with_its_list_of_created_keys_full(room, monkeypatch):
    """The pull's lookup notes the keys it creates in a list per block and writes their initial
    rows at its end, all lanes together.  With room for only a few entries (or none) the keys
    that find the list full get their rows on the spot: same results."""
    monkeypatch.setenv("HPS_LOOKUP_NEW_LIST", room)          # read when the table is created
    cfg = synth.scaled(synth.CONFIGS["insert_heavy"], n_prefill=40_000, n_examples=128, n_slots=40, steps=4)
    run_steps(cfg, steps=4)
    cfg = synth.scaled(synth.CONFIGS["mid"], n_prefill=3000, n_examples=64, n_slots=20, steps=3)
    run_steps(cfg, steps=3, opt=hps.ADAGRAD_ELEMENTWISE)


@pytest.mark.parametrize("name,n_prefill,n_examples,n_slots", [
    ("mid", 200_000, 128, 100),            # ~64k occurrences: several sort tiles, ragged tail
    ("insert_heavy", 50_000, 64, 100),
    ("large", 300_000, 96, 200),
    ("skewed", 100_000, 256, 64),          # dim 64, hot keys with long segments
])
def test_scaled_configs(name, n_prefill, n_examples, n_slots):
    cfg = synth.scaled(synth.CONFIGS[name], n_prefill=n_prefill, n_examples=n_examples,
                       n_slots=n_slots, steps=4)
    run_steps(cfg, steps=4)


@pytest.mark.parametrize("opt", [hps.ADAGRAD_ROWWISE, hps.ADAGRAD_ELEMENTWISE])
@pytest.mark.parametrize("name,n_prefill,n_examples,n_slots", [
    ("mid", 60_000, 96, 50),               # dim 16: 8-byte accesses per lane
    ("skewed", 40_000, 128, 32),           # dim 64, hot keys with long segments
])
def test_bf16_rows(name, n_prefill, n_examples, n_slots, opt):
    """Weights stored as bfloat16.  What is exact stays exact: key sets, sizes, unique keys,
    rows that were only initialised (the float32 initial row rounded to nearest even), and
    the first pull's pooled rows to the float32 tolerance.  A stored weight is the float32
    result rounded, and the two sides' float32 results differ in their last bits, so now and
    then one lands on the other side of a rounding boundary: after the first push nearly all
    weights are bit-identical and the rest are one bfloat16 step apart (2^-7 relative at
    most); a step does not depend on the weight it is applied to, so over a few more steps
    such differences neither heal nor grow beyond a step or two."""
    cfg = synth.scaled(synth.CONFIGS[name], n_prefill=n_prefill, n_examples=n_examples,
                       n_slots=n_slots, steps=4)
    stream = synth.BatchStream(cfg)
    mean_bag = cfg.bag_mean if cfg.bag_kind == "poisson" else cfg.bag_hi
    gt, ot = make_pair(cfg, int(cfg.n_bags * mean_bag * 1.5) + 4096, opt, hps.ROWS_BF16)
    pre = synth.prefill_keys(0, cfg.n_prefill)
    gt.insert(dev_keys(pre))
    ot.insert(pre)

    def dumps():
        k, w, a = gt.dump()
        k, w, a = host_keys(k), w.cpu().numpy(), a.cpu().numpy()
        order = np.argsort(k, kind="stable")
        ok, ow, oa = ot.dump()
        assert np.array_equal(k[order], ok), "key sets differ"
        assert not (w.view(np.uint32) & 0xFFFF).any(), "a stored weight is not a bfloat16 value"
        return ok, w[order], a[order], ow, oa

    _, w, a, ow, oa = dumps()
    assert np.array_equal(w.view(np.uint32), ow.view(np.uint32)), "initial rows"
    touched = np.zeros(0, dtype=np.uint64)
    for step in range(4):
        b = stream.next()
        touched = np.union1d(touched, b.keys)
        pooled = gt.pull(dev_keys(b.keys), torch.from_numpy(b.offsets).cuda(), cfg.n_examples, cfg.n_slots)
        want = ot.pull(b.keys, b.offsets)
        uniq, inv = gt.last_unique()
        ou, oi = ot.last_unique()
        assert np.array_equal(host_keys(uniq), ou) and np.array_equal(inv.cpu().numpy(), oi)
        assert gt.stats().last_n_inserted == ot.n_inserted
        if step == 0:
            assert_close(pooled.cpu().numpy(), want, "pooled, first pull")
        gt.push(torch.from_numpy(b.grads).cuda())
        ot.push(b.grads)
        k, w, a, ow, oa = dumps()
        assert_close(a, oa, "accumulators step %d" % step)
        same = w.view(np.uint32) == ow.view(np.uint32)
        steps_apart = 1 if step == 0 else 2
        # bfloat16 steps of the size the weight had when the difference arose (at least the
        # initial range), on top of the float32 tolerance: where a step nearly cancels a weight,
        # the two float32 results differ by far more than a bfloat16 step of what is left
        size = np.maximum(np.abs(ow), cfg.init_range)
        err = np.abs(w.astype(np.float64) - ow) - steps_apart * 2.0 ** -7 * size - (ATOL + RTOL * np.abs(ow))
        assert err.max() <= 0, "weights more than %d bfloat16 step(s) apart" % steps_apart
        assert same.mean() > 0.999, "too many weights differ: %g" % (1 - same.mean())
        rows_untouched = ~np.isin(k, touched)
        assert same[rows_untouched].all(), "rows that were only initialised must be bit-identical"
    assert gt.stats().size == ot.size and gt.stats().error == 0
    # get returns what is stored; dump -> insert into a fresh table is the identity
    probe = k[:: max(1, k.size // 500)]
    gw, ga, gf = gt.get(dev_keys(probe))
    assert gf.all() and np.array_equal(gw.cpu().numpy(), w[:: max(1, k.size // 500)])
    g2, _ = make_pair(cfg, 1024, opt, hps.ROWS_BF16)
    kk, ww, aa = gt.dump()
    g2.insert(kk, ww, aa)
    k2, w2, a2 = g2.dump()
    o1, o2 = np.argsort(host_keys(kk), kind="stable"), np.argsort(host_keys(k2), kind="stable")
    assert np.array_equal(host_keys(kk)[o1], host_keys(k2)[o2])
    assert torch.equal(ww[torch.from_numpy(o1).cuda()], w2[torch.from_numpy(o2).cuda()])
    assert torch.equal(aa[torch.from_numpy(o1).cuda()], a2[torch.from_numpy(o2).cuda()])


def test_elementwise_adagrad():
    cfg = synth.scaled(synth.CONFIGS["mid"], n_prefill=20_000, n_examples=64, n_slots=20, steps=3)
    run_steps(cfg, steps=3, opt=hps.ADAGRAD_ELEMENTWISE)


@pytest.mark.parametrize("opt", [hps.ADAGRAD_ROWWISE, hps.ADAGRAD_ELEMENTWISE])
def test_mean_pooling(opt):
    # bags averaged instead of summed; in the push an occurrence gets 1/len of its bag's gradient
    cfg = synth.scaled(synth.CONFIGS["skewed"], n_prefill=30_000, n_examples=96, n_slots=32, steps=4)
    gt, ot = run_steps(cfg, steps=4, opt=opt, mean=True)
    b = synth.BatchStream(cfg).next()
    with pytest.raises(hps.HpsError):                      # the mode cannot change inside a step
        gt.pull(dev_keys(b.keys), torch.from_numpy(b.offsets).cuda(), cfg.n_examples, cfg.n_slots)
        gt.set_pooling(False)
    gt.push(torch.from_numpy(b.grads).cuda())
    gt.set_pooling(False)


def test_long_run_insert_heavy_50_steps_and_determinism():
    cfg = synth.scaled(synth.CONFIGS["insert_heavy"], n_prefill=23_000, n_examples=8,
                       n_slots=100, steps=50)
    g1, _ = run_steps(cfg, steps=50, check_every=7)
    k1, w1, a1 = g1.dump()
    o1 = torch.argsort(k1)
    del _
    g2, _ = run_steps(cfg, steps=50, check_every=50)
    k2, w2, a2 = g2.dump()
    o2 = torch.argsort(k2)
    assert torch.equal(k1[o1], k2[o2]) and torch.equal(w1[o1], w2[o2]) and torch.equal(a1[o1], a2[o2])


def mixed_run_keys():
    """Keys that agree in their high bits in groups: two-key groups, a 40-key group, and a
    frequent key (600 occurrences) that shares its top 56 bits with two rare ones."""
    rng = np.random.default_rng(9)
    base = synth.mix64(np.arange(300, dtype=np.uint64)) & np.uint64(0xFFFFFFFFFFFFFF00)
    pairs = np.concatenate([base[:100], base[:100] | np.uint64(1)])
    group40 = base[100] | np.arange(40, dtype=np.uint64)
    hot = np.concatenate([np.full(600, base[101] | np.uint64(7)), np.full(2, base[101] | np.uint64(3)),
                          np.full(3, base[101] | np.uint64(200))])
    filler = synth.mix64(rng.integers(0, 500, size=1500, dtype=np.uint64))
    keys = np.concatenate([pairs, group40, group40[:10], hot, filler])
    return keys[rng.permutation(keys.shape[0])]


def test_prepare_overlapping_the_previous_push():
    """hps_prepare of mini-batch i+1 on a second stream between pull and push of mini-batch i
    gives the same results as plain pulls (the oracle knows nothing of the schedule)."""
    cfg = synth.scaled(synth.CONFIGS["insert_heavy"], n_prefill=60_000, n_examples=64,
                       n_slots=100, steps=8)
    stream = synth.BatchStream(cfg)
    batches = [stream.next() for _ in range(8)]
    gt, ot = make_pair(cfg, max(b.n_keys for b in batches))
    pre = synth.prefill_keys(0, cfg.n_prefill)
    gt.insert(dev_keys(pre))
    ot.insert(pre)
    dev = [(dev_keys(b.keys), torch.from_numpy(b.offsets).cuda(), torch.from_numpy(b.grads).cuda())
           for b in batches]
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        gt.prepare(dev[0][0], dev[0][1], cfg.n_examples, cfg.n_slots)
    for i, b in enumerate(batches):
        pooled = gt.pull_prepared()
        if i + 1 < len(batches):
            with torch.cuda.stream(side):
                gt.prepare(dev[i + 1][0], dev[i + 1][1], cfg.n_examples, cfg.n_slots)
        want = ot.pull(b.keys, b.offsets)
        uniq, inv = gt.last_unique()
        ou, oi = ot.last_unique()
        assert np.array_equal(host_keys(uniq), ou) and np.array_equal(inv.cpu().numpy(), oi)
        assert gt.stats().last_n_inserted == ot.n_inserted
        assert_close(pooled.cpu().numpy(), want, "pooled step %d" % i)
        gt.push(dev[i][2])
        ot.push(b.grads)
    compare_tables(gt, ot, "pipelined")
    with pytest.raises(hps.HpsError) as e:
        gt.pull_prepared()                      # nothing prepared
    assert e.value.status == hps.ESTATE


def test_edge_cases():
    cfg = synth.scaled(synth.CONFIGS["tiny"], n_prefill=1000, n_examples=4, n_slots=4,
                       capacity=8000, steps=1)
    gt, ot = make_pair(cfg, 5000)
    pre = synth.prefill_keys(0, 1000)
    gt.insert(dev_keys(pre))
    ot.insert(pre)
    zero_grads = torch.zeros((16, cfg.dim), device="cuda")
    # empty batch: every bag empty
    offs = torch.zeros(17, dtype=torch.int32, device="cuda")
    pooled = gt.pull(torch.zeros(0, dtype=torch.int64, device="cuda"), offs, 4, 4)
    assert torch.equal(pooled, torch.zeros_like(pooled))
    assert gt.stats().last_n_unique == 0
    gt.push(zero_grads)
    # keys without a single bag to hold them: refused on the host
    with pytest.raises(hps.HpsError) as e:
        gt.pull(dev_keys(pre[:8]), torch.zeros(1, dtype=torch.int32, device="cuda"), 0, 4)
    assert e.value.status == hps.EINVAL
    # one key; all-equal keys; keys around 2^32 and 2^63; raw sequential (unmixed) keys
    cases = [
        np.array([pre[5]], dtype=np.uint64),
        np.full(3000, pre[7], dtype=np.uint64),
        np.array([2**32 - 1, 2**32, 2**32 + 1, 2**63 - 1, 2**63, 2**63 + 1, 0, 1, 2**64 - 2] * 7,
                 dtype=np.uint64),
        np.arange(4097, dtype=np.uint64)[::-1].copy(),
        mixed_run_keys(),
    ]
    rng = np.random.default_rng(0)
    for keys in cases:
        n = keys.shape[0]
        cuts = np.sort(rng.integers(0, n + 1, size=15))
        offsets = np.concatenate([[0], cuts, [n]]).astype(np.int32)     # ragged, some empty bags
        grads = rng.normal(0, 1e-3, size=(16, cfg.dim)).astype(np.float32)
        pooled = gt.pull(dev_keys(keys), torch.from_numpy(offsets).cuda(), 4, 4)
        want = ot.pull(keys, offsets)
        uniq, inv = gt.last_unique()
        ou, oi = ot.last_unique()
        assert np.array_equal(host_keys(uniq), ou) and np.array_equal(inv.cpu().numpy(), oi)
        assert_close(pooled.cpu().numpy(), want, "pooled")
        gt.push(torch.from_numpy(grads).cuda())
        ot.push(grads)
    compare_tables(gt, ot, "edge")
    # push without pull
    with pytest.raises(hps.HpsError) as e:
        gt.push(zero_grads)
    assert e.value.status == hps.ESTATE
    # a second pull while the first still waits for its push
    k2 = dev_keys(pre[:8])
    o2 = torch.from_numpy(np.arange(0, 9, dtype=np.int32)).cuda()
    gt.pull(k2, o2, 2, 4)
    with pytest.raises(hps.HpsError) as e:
        gt.pull(k2, o2, 2, 4)
    assert e.value.status == hps.ESTATE
    gt.push(torch.zeros((8, cfg.dim), device="cuda"))
    ot.pull(pre[:8], np.arange(0, 9, dtype=np.int32))
    ot.push(np.zeros((8, cfg.dim), dtype=np.float32))
    # get: present and absent keys
    probe = np.concatenate([pre[:10], synth.mix64(np.arange(10**9, 10**9 + 10, dtype=np.uint64))])
    w, a, f = gt.get(dev_keys(probe))
    ow, oa, of = ot.get(probe)
    assert np.array_equal(f.cpu().numpy(), of)
    assert_close(w.cpu().numpy()[of], ow[of], "get weights")
    assert_close(a.cpu().numpy()[of], oa[of], "get acc")


def test_reserved_key_and_table_full_are_reported():
    gt = hps.HpsTable(100, 8, 1000, 4)
    gt.insert(dev_keys(np.arange(100, dtype=np.uint64)))
    assert gt.stats().size == 100 and gt.stats().error == 0
    offs = torch.tensor([0, 1, 2, 2, 2], dtype=torch.int32, device="cuda")
    gt.pull(dev_keys(np.array([5, 2**64 - 1], dtype=np.uint64)), offs, 2, 2)
    assert gt.stats().error == hps.ERESERVED
    gt.clear_error()
    gt.pull(dev_keys(np.array([5, 1000], dtype=np.uint64)), offs, 2, 2)       # key 1000 does not fit
    st = gt.stats()
    assert st.error == hps.EFULL and st.size == 100
    gt.clear_error()
    # clearing the status abandons the failed mini-batch: there is nothing valid to push
    with pytest.raises(hps.HpsError) as e:
        gt.push(torch.zeros((4, 8), device="cuda"))
    assert e.value.status == hps.ESTATE
    pooled = gt.pull(dev_keys(np.array([5, 6], dtype=np.uint64)), offs, 2, 2)   # present keys: fine
    assert gt.stats().error == 0
    w, _, f = gt.get(dev_keys(np.array([5, 6], dtype=np.uint64)))
    assert f.all() and torch.equal(pooled[:2], w)
    with pytest.raises(hps.HpsError) as e:
        gt.pull(dev_keys(np.arange(2000, dtype=np.uint64)), offs, 2, 2)         # n_keys > max_keys
    assert e.value.status == hps.EINVAL


def test_dump_insert_roundtrip():
    cfg = synth.scaled(synth.CONFIGS["mid"], n_prefill=5000, n_examples=16, n_slots=20, steps=2)
    gt, _ = run_steps(cfg, steps=2)
    k, w, a = gt.dump()
    g2 = hps.HpsTable(cfg.capacity, cfg.dim, 1000, 10)
    g2.insert(k, w, a)
    k2, w2, a2 = g2.dump()
    o1, o2 = torch.argsort(k), torch.argsort(k2)
    assert torch.equal(k[o1], k2[o2]) and torch.equal(w[o1], w2[o2]) and torch.equal(a[o1], a2[o2])
    assert g2.stats().size == k.numel()


def zipf_pairs(rng, keys, n, dim, s=1.2):
    """n (key, value row) pairs whose keys repeat with a Zipf-like skew: a few keys come
    thousands of times (long / chunked reductions), most once or twice."""
    w = 1.0 / np.arange(1, keys.size + 1) ** s
    pick = rng.choice(keys.size, size=n, p=w / w.sum())
    return keys[pick], rng.normal(0, 1e-3, size=(n, dim)).astype(np.float32)


@pytest.mark.parametrize("opt", [hps.ADAGRAD_ROWWISE, hps.ADAGRAD_ELEMENTWISE])
def test_accumulate_literal_form(opt):
    # Section 4.1 accumulate: value rows are added onto the rows of their keys
    rng = np.random.default_rng(9)
    cfg = synth.scaled(synth.CONFIGS["mid"], n_prefill=50_000, n_examples=64, n_slots=8)
    gt, ot = make_pair(cfg, 300_000, opt)
    pre = synth.prefill_keys(0, cfg.n_prefill)
    gt.insert(dev_keys(pre))
    ot.insert(pre)
    touched = []
    for n in (250_000, 0, 1, 70_001):
        k, v = zipf_pairs(rng, pre, n, cfg.dim)
        touched.append(k)
        if n > 1:      # some keys the table does not hold: skipped, counted, nothing created
            k = k.copy()
            k[:: 997] = synth.mix64(np.arange(2**50, 2**50 + k[::997].size, dtype=np.uint64))
        print("accumulate", n, flush=True)
        gt.accumulate(dev_keys(k), torch.from_numpy(v).cuda())
        absent = ot.accumulate(k, v)
        st = gt.stats()
        assert st.error == 0 and st.last_n_absent == absent and st.size == ot.size
    touched = np.concatenate(touched)
    compare_tables(gt, ot, "after accumulate", touched)
    # works between training steps, and not inside one
    b = synth.BatchStream(cfg).next()
    dk, do = dev_keys(b.keys), torch.from_numpy(b.offsets).cuda()
    pooled = gt.pull(dk, do, cfg.n_examples, cfg.n_slots)
    assert_close(pooled.cpu().numpy(), ot.pull(b.keys, b.offsets), "pooled after accumulate")
    with pytest.raises(hps.HpsError):
        gt.accumulate(dk[:4], torch.zeros((4, cfg.dim), device="cuda"))
    gt.push(torch.from_numpy(b.grads).cuda())
    ot.push(b.grads)
    compare_tables(gt, ot, "step after accumulate", touched)


def test_accumulate_is_deterministic_and_rejects_the_reserved_key():
    rng = np.random.default_rng(10)
    pre = synth.prefill_keys(0, 20_000)
    k, v = zipf_pairs(rng, pre, 200_000, 16, s=1.4)
    dumps = []
    for _ in range(2):
        gt = hps.HpsTable(40_000, 16, 200_000, 16)
        gt.insert(dev_keys(pre))
        gt.accumulate(dev_keys(k), torch.from_numpy(v).cuda())
        kk, w, a = gt.dump()
        order = np.argsort(host_keys(kk), kind="stable")
        dumps.append((host_keys(kk)[order], w.cpu().numpy()[order], a.cpu().numpy()[order]))
    for x, y in zip(*dumps):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))
    bad = k[:100].copy()
    bad[50] = np.uint64(2**64 - 1)
    gt.accumulate(dev_keys(bad), torch.ones((100, 16), device="cuda"))
    assert gt.stats().error == hps.ERESERVED
    gt.clear_error()
    kk, w, _ = gt.dump()
    order = np.argsort(host_keys(kk), kind="stable")
    assert np.array_equal(w.cpu().numpy()[order], dumps[1][1])      # nothing was added


@pytest.mark.parametrize("opt", [hps.ADAGRAD_ROWWISE, hps.ADAGRAD_ELEMENTWISE])
def test_dump_dirty_rows(opt):
    cfg = synth.scaled(synth.CONFIGS["insert_heavy"], n_prefill=40_000, n_examples=128, n_slots=10)
    gt, ot = make_pair(cfg, 20_000, opt)
    pre = synth.prefill_keys(0, cfg.n_prefill)
    gt.insert(dev_keys(pre))
    ot.insert(pre)

    def compare_dirty(what):
        k, w, a = gt.dump(dirty=True)
        k, w, a = host_keys(k), w.cpu().numpy(), a.cpu().numpy()
        order = np.argsort(k, kind="stable")
        ok, ow, oa = ot.dump_dirty()
        assert np.array_equal(k[order], ok), what + ": dirty key sets differ"
        assert_close(w[order], ow, what + " weights")
        assert_close(a[order], oa, what + " accumulators")
        return ok

    assert compare_dirty("after insert").size == 0
    stream = synth.BatchStream(cfg)
    for step in range(3):
        b = stream.next()
        dk, do = dev_keys(b.keys), torch.from_numpy(b.offsets).cuda()
        gt.pull(dk, do, cfg.n_examples, cfg.n_slots)
        ot.pull(b.keys, b.offsets)
        if step == 2:
            with pytest.raises(hps.HpsError):                   # not inside a step
                gt.dump(dirty=True)
        gt.push(torch.from_numpy(b.grads).cuda())
        ot.push(b.grads)
        if step == 0:
            assert compare_dirty("after step 0").size == np.unique(b.keys).size
    assert compare_dirty("after steps 1-2").size > 0
    assert compare_dirty("nothing since").size == 0
    rng = np.random.default_rng(3)
    k, v = zipf_pairs(rng, pre, 5000, cfg.dim)
    gt.accumulate(dev_keys(k), torch.from_numpy(v).cuda())
    ot.accumulate(k, v)
    assert compare_dirty("after accumulate").size == np.unique(k).size
    # too small a buffer: what fits is handed over, the rest stays marked
    b = stream.next()
    gt.pull(dev_keys(b.keys), torch.from_numpy(b.offsets).cuda(), cfg.n_examples, cfg.n_slots)
    gt.push(torch.from_numpy(b.grads).cuda())
    want = np.unique(b.keys)
    with pytest.raises(hps.HpsError):
        gt.dump(max_rows=want.size // 2, dirty=True)
    rest, _, _ = gt.dump(dirty=True)
    assert rest.numel() == want.size - want.size // 2
    assert np.isin(host_keys(rest), want).all()
    compare_tables_keys_only = gt.dump()[0]
    assert compare_tables_keys_only.numel() == gt.stats().size
    # accumulators read back without the mark
    _, a, f = gt.get(dev_keys(want))
    assert f.all().item() and (a >= 0).all().item()


def test_dedup_only_batches_with_shifting_hot_keys(dedup_form):
    """The dedup alone (unique keys and inverse ranks, bit-exact) on mid-sized batches whose
    heavy keys change from batch to batch: the bucket form learns heavy keys from earlier
    lookups, so a key that turns hot without warning makes a region too large for LDS and
    takes the route through global memory; unhashed, consecutive keys share all their leading
    bits (the dedup places keys inside the range a sample of them spans), also together with a
    hashed key far outside that range.  Each case must give the oracle's result whichever
    form runs."""
    rng = np.random.default_rng(21)
    dim, n_bags = 8, 4096
    gt = hps.HpsTable(1_000_000, dim, 400_000, n_bags, lr=0.05)
    ids = synth.mix64(np.arange(500_000, dtype=np.uint64))
    offsets = None

    def batch(n, hot, share, plain_ids=False):
        cold = rng.integers(0, 400_000, size=n)
        keys = ids[cold]
        if plain_ids:
            keys = (np.uint64(1) << np.uint64(40)) + cold.astype(np.uint64)   # unhashed
        for h, s in zip(hot, share):
            keys[rng.random(n) < s] = ids[400_000 + h]
        return keys

    cases = [
        (300_000, [], []),
        (300_000, [1, 2, 3], [0.2, 0.05, 0.01]),       # first hot keys: no hint yet
        (300_000, [1, 2, 3], [0.2, 0.05, 0.01]),
        (300_000, [1, 2, 3], [0.2, 0.05, 0.01]),       # hinted from here on
        (350_000, [7, 8], [0.3, 0.02]),                # new hot keys without warning
        (350_000, [7, 8, 1], [0.1, 0.1, 0.1]),
        (200_000, [7], [0.9]),                         # one key nearly everything
        (150_000, [], [], True),                       # consecutive integers
        (150_000, [], [], True),
        (200_000, [], [], True),
        (200_000, [3], [0.3], True),                   # with a hashed hot key far outside their range
        (300_000, [9], [0.001]),                       # back to ordinary
        (300_000, [9], [0.001]),
        (390_000, list(range(100, 2100)), [0.0004] * 2000),   # 2000 keys of ~150 occurrences: more
        (390_000, list(range(100, 2100)), [0.0004] * 2000),   # frequent keys than the hint can list
        (390_000, list(range(100, 2100)), [0.0004] * 2000),
    ]
    def batch_many(n, n_hot, per_key):
        """n_hot keys of per_key occurrences each among cold ones."""
        keys = ids[rng.integers(0, 400_000, size=n)]
        at = rng.choice(n, size=n_hot * per_key, replace=False)
        keys[at] = np.repeat(ids[400_000 + np.arange(n_hot)], per_key)
        return keys

    # 3000 frequent keys: the list of frequent keys is put in order as two halves and merged,
    # and the kernels that consult it read it from global memory; 5000: more than it can hold
    many = [(390_000, 3000, 100)] * 3 + [(390_000, 5000, 70)] * 3 + [(300_000, 2047, 100), (300_000, 2048, 100),
                                                                      (300_000, 2049, 100), (300_000, 2049, 100)]
    for case in cases + many:
        keys = batch_many(*case) if case in many else batch(*case)
        n = keys.size
        offsets = np.minimum(np.arange(n_bags + 1, dtype=np.int64) * ((n + n_bags - 1) // n_bags), n).astype(np.int32)
        print("dedup case", case[:3] if case not in many else ("many",) + case, "n", n, flush=True)
        gt.pull(dev_keys(keys), torch.from_numpy(offsets).cuda(), n_bags, 1)
        ou, oi = oracle.dedup(keys)
        uniq, inv = gt.last_unique()
        st = gt.stats()
        assert st.error == 0 and st.last_n_unique == ou.size
        assert np.array_equal(host_keys(uniq)[: ou.size], ou), "unique keys"
        assert np.array_equal(inv.cpu().numpy(), oi), "inverse"
        gt.push(torch.zeros((n_bags, dim), device="cuda"))


def test_dedup_keys_bunched_inside_their_range(dedup_form):
    """Raw ids with a long-tailed distribution: nearly all keys lie in a tiny part of the range
    the keys span, so equal parts of that range are no use as buckets and the bucket form
    orders most of the batch through global memory.  Results must be the oracle's in every
    form; left to itself the library must notice (the lookups report it) and go back to the
    plain form for a while."""
    rng = np.random.default_rng(33)
    dim, n_bags, n = 8, 2048, 200_000
    gt = hps.HpsTable(1_000_000, dim, n, n_bags, lr=0.05)
    offsets = np.minimum(np.arange(n_bags + 1, dtype=np.int64) * ((n + n_bags - 1) // n_bags), n).astype(np.int32)
    for step in range(8):
        keys = np.minimum(rng.pareto(1.0, size=n) * 1000.0, 5e7).astype(np.uint64) + np.uint64(17)
        print("bunched keys, step", step, flush=True)
        gt.pull(dev_keys(keys), torch.from_numpy(offsets).cuda(), n_bags, 1)
        ou, oi = oracle.dedup(keys)
        uniq, inv = gt.last_unique()
        st = gt.stats()
        assert st.error == 0 and st.last_n_unique == ou.size
        assert np.array_equal(host_keys(uniq)[: ou.size], ou), "unique keys"
        assert np.array_equal(inv.cpu().numpy(), oi), "inverse"
        gt.push(torch.zeros((n_bags, dim), device="cuda"))
    torch.cuda.synchronize()
    fallbacks = gt.stats().n_plain_fallbacks
    if dedup_form == "auto":
        assert fallbacks >= 1, "the bucket form was never given up"
    else:
        assert fallbacks == 0


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 2047, 2048, 2049, 4096, 4097, 6143, 6144, 6145,
                               65535, 65536, 65537, 131072])
def test_dedup_sizes_around_tile_and_region_borders(n, dedup_form):
    """Unique keys and inverse ranks (bit-exact) for batch sizes at and next to the sizes where
    the dedup changes shape: a wave, a sort tile (3072), a region span (2048) and capacity
    (4096), one pass or two (65536).  Three key mixes per size: all distinct, few distinct
    (long runs of equal keys across region borders), and one heavy key among distinct ones."""
    rng = np.random.default_rng(n)
    dim = 4
    gt = hps.HpsTable(400_000, dim, 140_000, 64, lr=0.05)
    pool = synth.mix64(np.arange(300_000, dtype=np.uint64))
    mixes = [
        pool[rng.permutation(300_000)[:n]],
        pool[rng.integers(0, 7, size=n)],
        np.where(rng.random(n) < 0.6, pool[5], pool[rng.integers(0, 300_000, size=n)]),
    ]
    for rounds in range(2):            # the second round runs with a hint about heavy keys
        for keys in mixes:
            offsets = np.minimum(np.arange(65, dtype=np.int64) * ((n + 63) // 64), n).astype(np.int32)
            gt.pull(dev_keys(keys), torch.from_numpy(offsets).cuda(), 64, 1)
            ou, oi = oracle.dedup(keys)
            uniq, inv = gt.last_unique()
            st = gt.stats()
            assert st.error == 0 and st.last_n_unique == ou.size
            assert np.array_equal(host_keys(uniq), ou), "unique keys"
            assert np.array_equal(inv.cpu().numpy(), oi), "inverse"
            gt.push(torch.zeros((64, dim), device="cuda"))


def test_many_dedups_status_words_start_over(dedup_form):
    """The cross-workgroup status words of the dedup carry the dedup's number modulo 4095, and
    the library clears them whenever the numbers start over.  4300 small mini-batches of
    varying size go past that point; the results around it (and every 97th before) must be
    the oracle's."""
    rng = np.random.default_rng(4095)
    dim, n_bags, n_max = 4, 64, 9000
    gt = hps.HpsTable(300_000, dim, n_max, n_bags)
    pool = synth.mix64(np.arange(200_000, dtype=np.uint64))
    zero = torch.zeros((n_bags, dim), device="cuda")
    for step in range(4300):
        n = int(rng.integers(1, n_max + 1))
        keys = pool[rng.integers(0, pool.size, size=n)]
        offsets = np.minimum(np.arange(n_bags + 1, dtype=np.int64) * ((n + n_bags - 1) // n_bags), n).astype(np.int32)
        gt.pull(dev_keys(keys), torch.from_numpy(offsets).cuda(), n_bags, 1)
        if step % 97 == 0 or 4085 <= step <= 4105:
            ou, oi = oracle.dedup(keys)
            uniq, inv = gt.last_unique()
            st = gt.stats()
            assert st.error == 0 and st.last_n_unique == ou.size, "step %d" % step
            assert np.array_equal(host_keys(uniq), ou), "unique keys, step %d" % step
            assert np.array_equal(inv.cpu().numpy(), oi), "inverse, step %d" % step
        gt.push(zero)
    assert gt.stats().error == 0


def test_dedup_two_clusters_far_apart(dedup_form):
    """Unhashed ids in two small clusters at opposite ends of the 64-bit range: whatever leading
    bits (of the key, or of its place in the key range) the passes sort by, the keys of a
    cluster agree in all of them, so the plain form has to repair nearly everything and the
    bucket form gets two oversized regions.  Results must still be exact, and left to itself
    the library must end up sorting by all 64 bits."""
    rng = np.random.default_rng(8)
    dim, n_bags, n = 4, 256, 120_000
    gt = hps.HpsTable(400_000, dim, n, n_bags)
    offsets = np.minimum(np.arange(n_bags + 1, dtype=np.int64) * ((n + n_bags - 1) // n_bags), n).astype(np.int32)
    for step in range(6):
        low = rng.integers(0, 60_000, size=n).astype(np.uint64)
        keys = np.where(rng.random(n) < 0.5, low, np.uint64(2**63) + low)
        gt.pull(dev_keys(keys), torch.from_numpy(offsets).cuda(), n_bags, 1)
        ou, oi = oracle.dedup(keys)
        uniq, inv = gt.last_unique()
        st = gt.stats()
        assert st.error == 0 and st.last_n_unique == ou.size
        assert np.array_equal(host_keys(uniq), ou), "unique keys"
        assert np.array_equal(inv.cpu().numpy(), oi), "inverse"
        gt.push(torch.zeros((n_bags, dim), device="cuda"))
    st = gt.stats()
    if dedup_form == "auto":
        assert st.n_full_fallbacks >= 1 and st.n_plain_fallbacks >= 1
    else:
        assert st.n_full_fallbacks == 0 and st.n_plain_fallbacks == 0


def test_load_factor_and_probe_lengths():
    """The table's occupancy figures: load factor = stored keys / slots; every stored key is found
    within a few buckets of the one its hash names (buckets of sixteen slots, one 128-byte memory
    line; load at most 0.7)."""
    gt = hps.HpsTable(1_000_000, 8, 1000, 10)
    assert gt.probe_lengths() == (0.0, 0)
    keys = synth.mix64(np.arange(700_000, dtype=np.uint64))
    gt.insert(dev_keys(keys))
    st = gt.stats()
    assert st.size == 700_000 and abs(st.load_factor - 700_000 / st.n_slots) < 1e-12
    assert 0.45 < st.load_factor < 0.5            # slots = capacity / 0.7
    mean, most = gt.probe_lengths()
    assert 1.0 <= mean < 1.02 and 1 <= most <= 4, (mean, most)
    # raw consecutive ids must spread as well as hashed ones (the table hashes its keys itself)
    gt.clear()
    gt.insert(dev_keys(np.arange(700_000, dtype=np.uint64)))
    mean, most = gt.probe_lengths()
    assert 1.0 <= mean < 1.02 and 1 <= most <= 4, (mean, most)


def test_clear_and_rebuild_for_the_next_batch():
    """Algorithm 1's outer loop: per batch the table is filled with that batch's working
    parameters, its mini-batches are run, the updates are handed over and the table is
    emptied.  Two such batches; the second starts from the rows the first handed over (for
    the keys they share) and the table must again hold exactly what the oracle holds."""
    cfg = synth.scaled(synth.CONFIGS["mid"], n_prefill=30_000, n_examples=64, n_slots=40, steps=6)
    stream = synth.BatchStream(cfg)
    gt, ot = make_pair(cfg, 40_000)
    host = {}                                     # the host tier: key -> (weights, accumulator)
    for outer in range(2):
        batches = [stream.next() for _ in range(3)]
        working = np.unique(np.concatenate([b.keys for b in batches]))
        known = np.array([k for k in working if int(k) in host], dtype=np.uint64)
        new = np.setdiff1d(working, known)
        for table, to_dev in ((gt, True), (ot, False)):
            if known.size:
                w = np.stack([host[int(k)][0] for k in known])
                a = np.stack([host[int(k)][1] for k in known])
                if to_dev:
                    table.insert(dev_keys(known), torch.from_numpy(w).cuda(), torch.from_numpy(a).cuda())
                else:
                    table.insert(known, w, a)
            table.insert(dev_keys(new) if to_dev else new)
        assert gt.stats().size == working.size == ot.size
        for b in batches:
            pooled = gt.pull(dev_keys(b.keys), torch.from_numpy(b.offsets).cuda(), cfg.n_examples, cfg.n_slots)
            want = ot.pull(b.keys, b.offsets)
            assert gt.stats().last_n_inserted == 0 == ot.n_inserted     # the working set was there
            assert_close(pooled.cpu().numpy(), want, "pooled")
            gt.push(torch.from_numpy(b.grads).cuda())
            ot.push(b.grads)
        compare_tables(gt, ot, "outer batch %d" % outer, working)
        k, w, a = ot.dump_dirty()                 # the updates go to the host tier ...
        gk, gw, ga = gt.dump(dirty=True)
        assert np.array_equal(np.sort(host_keys(gk)), k)
        for key, wr, ar in zip(k, w, a):
            host[int(key)] = (wr.copy(), ar.copy())
        gt.clear()                                # ... and the table is emptied
        ot.clear()
        st = gt.stats()
        assert st.size == 0 and st.error == 0
        assert not gt.get(dev_keys(working[:100]))[2].any()
        kk, _, _ = gt.dump()
        assert kk.numel() == 0


def test_outer_batches_through_the_memory_tier():
    """Algorithm 1 with all three roles: an SSD stand-in (a dictionary), the host-memory cache
    (hps_mem_*: LRU -> LFU with pinned batches) and the HBM table, rebuilt for every batch of the
    outer loop from exactly its working parameters.  Three outer batches of three mini-batches
    each with overlapping working sets, against ONE flat oracle table that never forgets
    anything: pooled sums every mini-batch, and at the end every parameter ever touched,
    wherever it has ended up (cache or dictionary)."""
    dim, n_bags = 8, 64
    kw = dict(lr=0.05, eps=1e-8, init_acc=0.1, init_range=0.01, init_seed=11)
    gt = hps.HpsTable(8000, dim, 4096, n_bags, **kw)
    ot = OracleTable(100000, dim, **kw)
    mem = hps.MemTier(dim, 1, 1500, 1000)
    ssd = {}
    rng = np.random.default_rng(21)
    seen = set()
    for outer in range(3):
        batches = []
        for _ in range(3):
            n = int(rng.integers(1500, 2500))
            ids = np.minimum(rng.zipf(1.2, size=n), 6000) - 1 + 1500 * outer     # the hot ids move on
            offsets = np.sort(np.concatenate([[0, n], rng.integers(0, n + 1, size=n_bags - 1)])).astype(np.int32)
            batches.append((synth.mix64(ids.astype(np.uint64)), offsets,
                            rng.normal(0, 1e-3, size=(n_bags, dim)).astype(np.float32)))
        working = np.unique(np.concatenate([b[0] for b in batches]))
        # pull the working parameters: cache, then the SSD stand-in, then (never seen) a new row
        w, a, found = mem.fetch(working, outer)
        miss = working[~found]
        if miss.size:
            mw = np.stack([ssd[int(k)][0] if int(k) in ssd else ot.init_row(int(k)) for k in miss])
            ma = np.stack([ssd[int(k)][1] if int(k) in ssd else np.array([kw["init_acc"]], np.float32) for k in miss])
            for k in miss:
                ssd.pop(int(k), None)
            mem.store(miss, mw, ma, outer, True)
            w[~found], a[~found] = mw, ma
        fresh = np.array([k for k in working if int(k) not in seen], dtype=np.uint64)
        if fresh.size:
            ot.insert(fresh)                      # the flat table creates them with their initial rows
        seen.update(int(k) for k in working)
        gt.insert(dev_keys(working), torch.from_numpy(w).cuda(), torch.from_numpy(a).cuda())
        assert gt.stats().size == working.size
        for keys, offsets, grads in batches:
            pooled = gt.pull(dev_keys(keys), torch.from_numpy(offsets).cuda(), n_bags, 1)
            want = ot.pull(keys, offsets)
            assert gt.stats().last_n_inserted == 0 and ot.n_inserted == 0     # the working set was complete
            assert_close(pooled.cpu().numpy(), want, "pooled, outer batch %d" % outer)
            gt.push(torch.from_numpy(grads).cuda())
            ot.push(grads)
        # collect the updates, update the cache, dump what it evicts
        k, uw, ua = gt.dump(dirty=True)
        mem.store(k.cpu().numpy().view(np.uint64), uw.cpu().numpy(), ua.cpu().numpy(), outer, False)
        mem.complete_batch(outer)
        st = mem.stats()
        assert st.pinned == 0 and st.lru_size <= 1500 and st.lfu_size <= 1000
        ek, ew, ea = mem.take_evicted_arrays()
        for i in range(ek.size):
            ssd[int(ek[i])] = (ew[i].copy(), ea[i].copy())
        gt.clear()
    # every parameter is in exactly one place, with the values of the flat table
    everything = np.array(sorted(seen), dtype=np.uint64)
    w, a, found = mem.fetch(everything, 99)
    assert (st.lru_size + st.lfu_size) == int(found.sum()) and len(ssd) == int((~found).sum())
    for i in np.nonzero(~found)[0]:
        w[i], a[i] = ssd[int(everything[i])]
    ow, oa, of = ot.get(everything)
    assert of.all()
    assert_close(w, ow, "weights through the tiers")
    assert_close(a, oa, "accumulators through the tiers")
    assert len(ssd) > 0 and st.lfu_size > 0            # all three places were in use
