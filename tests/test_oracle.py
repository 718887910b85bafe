"""Pins for the CPU oracle: everything here checks oracle/ against something that
is not the oracle -- published known answers, the paper's worked example, closed
forms evaluated with exact/decimal arithmetic, library routines (torch
EmbeddingBag / Adagrad), brute force on tiny inputs, and invariants.

The paper prints no numeric value for the pull/push path, so no pin is a
"paper value"; Appendix A's key-set example is the only fixture it provides.
"""
import math
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import OracleTable, OracleError
import synth
from conftest import read_golden

TOL_ABS, TOL_REL = 1e-6, 1e-5


def close(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.all(np.abs(a - b) <= TOL_ABS + TOL_REL * np.abs(b))


# ----------------------------------------------------------------------------- mix

def test_mix_known_answers():
    for state, out in read_golden("splitmix64_known_answers.txt"):
        assert oracle.mix(int(state, 16)) == int(out, 16)


def test_mix_is_injective_and_matches_generator_module():
    x = np.arange(1 << 20, dtype=np.uint64)
    y = synth.mix64(x)
    assert np.unique(y).shape[0] == x.shape[0]
    # two independently written implementations (numpy there, C++ here)
    rng = np.random.default_rng(7)
    probe = rng.integers(0, 2**64, size=4096, dtype=np.uint64)
    want = synth.mix64(probe)
    got = np.array([oracle.mix(int(v)) for v in probe], dtype=np.uint64)
    assert np.array_equal(got, want)


# ----------------------------------------------------------------------------- init

def _init_by_exact_arithmetic(key, dim, seed, a):
    """Row initialiser re-derived with Python ints and exactly rounded float32 steps."""
    M = (1 << 64) - 1

    def mix(x):
        z = (x + 0x9E3779B97F4A7C15) & M
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        return z ^ (z >> 31)

    a32 = np.float32(a)
    two_a = np.float32(Fraction(float(a32)) * 2)         # exact doubling
    base = mix(key ^ seed)
    out = []
    for j in range(dim):
        t = mix((base + j) & M) >> 40
        u = Fraction(t, 1 << 24)
        prod = np.float32(float(u * Fraction(float(two_a))))       # 48-bit product fits a double
        out.append(np.float32(float(Fraction(float(prod)) - Fraction(float(a32)))))
    return np.array(out, dtype=np.float32)


def test_init_bits_range_and_moments():
    t = OracleTable(1 << 20, 8, init_range=0.01, init_seed=0)
    for key in (0, 1, 0xDEADBEEF, 2**63, 2**64 - 2, int(synth.mix64(np.uint64(5)))):
        want = _init_by_exact_arithmetic(key, 8, 0, 0.01)
        assert np.array_equal(t.init_row(key).view(np.uint32), want.view(np.uint32))
    t2 = OracleTable(16, 4, init_range=0.25, init_seed=0x1234)
    assert np.array_equal(t2.init_row(99).view(np.uint32),
                          _init_by_exact_arithmetic(99, 4, 0x1234, 0.25).view(np.uint32))
    rows = np.stack([t.init_row(int(k)) for k in synth.prefill_keys(0, 20000)])
    assert rows.min() >= -0.01 and rows.max() < 0.01
    assert abs(rows.mean()) < 3 * 0.02 / math.sqrt(12 * rows.size) * 1.5
    assert abs(rows.var() - 0.02**2 / 12) < 0.02 * 0.02**2 / 12
    # columns are not copies of each other, rows are not copies of each other
    assert np.unique(rows[:, 0]).shape[0] > 19000
    assert not np.array_equal(rows[:, 0], rows[:, 1])


# ----------------------------------------------------------------------------- dedup

def _dedup_brute(keys):
    uniq = []
    for k in keys:
        if all(k != u for u in uniq):
            uniq.append(k)
    # selection sort, no library ordering
    for i in range(len(uniq)):
        m = i
        for j in range(i + 1, len(uniq)):
            if uniq[j] < uniq[m]:
                m = j
        uniq[i], uniq[m] = uniq[m], uniq[i]
    inv = []
    for k in keys:
        inv.append(next(r for r, u in enumerate(uniq) if u == k))
    return uniq, inv


@pytest.mark.parametrize("case", ["random", "all_equal", "all_distinct", "empty", "one",
                                  "straddle"])
def test_dedup_vs_brute_force(case):
    rng = np.random.default_rng(3)
    if case == "random":
        keys = synth.mix64(rng.integers(0, 300, size=1500, dtype=np.uint64))
    elif case == "all_equal":
        keys = np.full(700, 0x1234567890ABCDEF, dtype=np.uint64)
    elif case == "all_distinct":
        keys = synth.mix64(np.arange(900, dtype=np.uint64))
    elif case == "empty":
        keys = np.zeros(0, dtype=np.uint64)
    elif case == "one":
        keys = np.array([42], dtype=np.uint64)
    else:
        base = np.array([2**32 - 1, 2**32, 2**32 + 1, 2**63 - 1, 2**63, 2**63 + 1, 0, 1,
                         2**64 - 2], dtype=np.uint64)
        keys = base[rng.integers(0, base.shape[0], size=200)]
    uniq, inv = oracle.dedup(keys)
    bu, bi = _dedup_brute([int(k) for k in keys])
    assert [int(u) for u in uniq] == bu
    assert [int(i) for i in inv] == bi
    assert all(int(uniq[i]) < int(uniq[i + 1]) for i in range(len(uniq) - 1))
    assert np.array_equal(uniq[inv], keys) if len(keys) else True


# ----------------------------------------------------------------------------- table

def test_appendix_a_key_sets():
    rows = {r[0]: np.array([int(v) for v in r[1:]], dtype=np.uint64)
            for r in read_golden("appendix_a_example.txt")}
    assert sorted(set(rows["gpu1"]) | set(rows["gpu2"])) == sorted(rows["working"])
    assert all(k <= 50 for k in rows["gpu1"]) and all(k > 50 for k in rows["gpu2"])
    t = OracleTable(len(rows["working"]), 4)
    t.insert(rows["working"])                       # insert_into_hashtable
    before = t.dump()
    offsets = np.array([0, 3], dtype=np.int32)
    pooled = t.pull(rows["worker1"], offsets)       # pull touches exactly worker 1's keys
    uniq, inv = t.last_unique()
    assert list(uniq) == [11, 87, 98] and list(inv) == [0, 1, 2]
    assert t.n_inserted == 0 and t.size == 9
    w, _, found = t.get(rows["worker1"])
    assert found.all() and close(pooled[0], w.astype(np.float64).sum(0))
    t.push(np.ones((1, 4), dtype=np.float32))
    after = t.dump()
    assert np.array_equal(before[0], after[0]) and list(after[0]) == sorted(rows["working"])
    touched = np.isin(after[0], rows["worker1"])
    assert np.array_equal(before[1][~touched], after[1][~touched])     # others bit-identical
    assert np.array_equal(before[2][~touched], after[2][~touched])
    assert (before[1][touched] != after[1][touched]).all()


def test_key_set_is_union_capacity_and_reserved():
    rng = np.random.default_rng(11)
    t = OracleTable(1000, 4)
    seen = set()
    pre = synth.prefill_keys(0, 300)
    t.insert(pre)
    seen |= set(int(k) for k in pre)
    for _ in range(5):
        keys = synth.mix64(rng.integers(0, 600, size=200, dtype=np.uint64))
        offsets = np.arange(0, 201, 4, dtype=np.int32)
        new = len(set(int(k) for k in keys) - seen)
        t.pull(keys, offsets)
        assert t.n_inserted == new
        seen |= set(int(k) for k in keys)
        t.push(np.zeros((50, 4), dtype=np.float32))
        assert set(int(k) for k in t.dump()[0]) == seen and t.size == len(seen)
    # zero key is an ordinary key, all-ones is reserved
    t.insert(np.array([0], dtype=np.uint64))
    assert t.get(np.array([0], dtype=np.uint64))[2][0]
    with pytest.raises(OracleError) as e:
        t.insert(np.array([2**64 - 1], dtype=np.uint64))
    assert e.value.status == oracle.ERESERVED
    with pytest.raises(OracleError) as e:
        t.pull(np.array([5, 2**64 - 1], dtype=np.uint64), np.array([0, 2], dtype=np.int32))
    assert e.value.status == oracle.ERESERVED
    # capacity is a hard bound on the number of keys
    small = OracleTable(10, 2)
    small.insert(np.arange(10, dtype=np.uint64))
    with pytest.raises(OracleError) as e:
        small.insert(np.array([77], dtype=np.uint64))
    assert e.value.status == oracle.EFULL and small.size == 10
    with pytest.raises(OracleError) as e:
        small.pull(np.array([3, 78], dtype=np.uint64), np.array([0, 2], dtype=np.int32))
    assert e.value.status == oracle.EFULL
    small.pull(np.array([3, 4], dtype=np.uint64), np.array([0, 2], dtype=np.int32))   # present: fine
    with pytest.raises(OracleError) as e:
        OracleTable(10, 2).push(np.zeros((1, 2), dtype=np.float32))                   # no pull
    assert e.value.status == oracle.ESTATE


def test_dump_insert_roundtrip_is_identity():
    rng = np.random.default_rng(5)
    t = OracleTable(5000, 8)
    t.insert(synth.prefill_keys(0, 2000))
    for _ in range(3):
        keys = synth.mix64(rng.integers(0, 3000, size=1000, dtype=np.uint64))
        t.pull(keys, np.arange(0, 1001, 5, dtype=np.int32))
        t.push(rng.normal(0, 1e-2, size=(200, 8)).astype(np.float32))
    k, w, a = t.dump()
    t2 = OracleTable(5000, 8)
    perm = rng.permutation(k.shape[0])
    t2.insert(k[perm], w[perm], a[perm])
    k2, w2, a2 = t2.dump()
    assert np.array_equal(k, k2)
    assert np.array_equal(w.view(np.uint32), w2.view(np.uint32))
    assert np.array_equal(a.view(np.uint32), a2.view(np.uint32))


def test_implicit_residency_equals_explicit_prefill():
    cfg = synth.scaled(synth.CONFIGS["mid"], n_prefill=4000, n_examples=16, n_slots=10, steps=3)
    ex = OracleTable(cfg.capacity, cfg.dim)
    ex.insert(synth.prefill_keys(0, cfg.n_prefill))
    im = OracleTable(cfg.capacity, cfg.dim)
    im.declare_resident(cfg.n_prefill)
    s1, s2 = synth.BatchStream(cfg), synth.BatchStream(cfg)
    for _ in range(3):
        b = s1.next()
        b2 = s2.next()
        res, _ = synth.ctr.resident_split(cfg, b2)
        im.materialize(res)
        p1, p2 = ex.pull(b.keys, b.offsets), im.pull(b2.keys, b2.offsets)
        assert np.array_equal(p1, p2) and ex.n_inserted == im.n_inserted and ex.size == im.size
        ex.push(b.grads)
        im.push(b2.grads)
    k, w, a = im.dump()
    w1, a1, f = ex.get(k)
    assert f.all() and np.array_equal(w, w1) and np.array_equal(a, a1)


# ----------------------------------------------------------------------------- pooling

def _table_with_values(rng, n_keys, dim, **kw):
    t = OracleTable(4 * n_keys, dim, **kw)
    keys = synth.prefill_keys(0, n_keys)
    w = rng.uniform(-1, 1, size=(n_keys, dim)).astype(np.float32)
    t.insert(keys, w)
    return t, keys, w


def test_pool_vs_torch_embedding_bag():
    rng = np.random.default_rng(21)
    t, keys, w = _table_with_values(rng, 200, 8)
    sizes = rng.integers(0, 6, size=64)               # includes empty bags
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    idx = rng.integers(0, 200, size=int(offsets[-1]))
    pooled = t.pull(keys[idx], offsets)
    want = torch.nn.functional.embedding_bag(
        torch.from_numpy(idx), torch.from_numpy(w.astype(np.float64)),
        torch.from_numpy(offsets[:-1].astype(np.int64)), mode="sum").numpy()
    assert pooled.shape == (64, 8) and close(pooled, want)
    assert np.array_equal(pooled[sizes == 0], np.zeros((int((sizes == 0).sum()), 8), np.float32))
    assert t.n_inserted == 0


def test_pool_properties():
    rng = np.random.default_rng(22)
    t, keys, w = _table_with_values(rng, 50, 4)
    # a bag of one key returns that row exactly; a repeated key counts twice
    p = t.pull(keys[[7, 9, 9]], np.array([0, 1, 3], dtype=np.int32))
    assert np.array_equal(p[0], w[7])
    assert np.array_equal(p[1], (2.0 * w[9].astype(np.float64)).astype(np.float32))
    # permuting inside a bag / concatenating bags
    idx = rng.integers(0, 50, size=12)
    a = t.pull(keys[idx], np.array([0, 12], dtype=np.int32))[0]
    b = t.pull(keys[idx[::-1]], np.array([0, 12], dtype=np.int32))[0]
    c = t.pull(keys[idx], np.array([0, 5, 12], dtype=np.int32))
    assert close(a, b) and close(a, c.astype(np.float64).sum(0))
    # transposed-operand check: row r column j is w[r, j], not w[j, r]
    t4, k4, w4 = _table_with_values(rng, 4, 4)
    assert np.array_equal(t4.pull(k4[[2]], np.array([0, 1], dtype=np.int32))[0], w4[2])


# ----------------------------------------------------------------------------- push

def _dec_adagrad(w, G, g, lr, eps, rowwise):
    getcontext().prec = 60
    w = [Decimal(float(x)) for x in w]
    g = [Decimal(float(x)) for x in g]
    lr, eps = Decimal(float(np.float32(lr))), Decimal(float(np.float32(eps)))
    if rowwise:
        Gn = Decimal(float(G[0])) + sum(x * x for x in g) / Decimal(len(g))
        return [float(wi - lr * gi / (Gn.sqrt() + eps)) for wi, gi in zip(w, g)], [float(Gn)]
    Gn = [Decimal(float(Gj)) + gi * gi for Gj, gi in zip(G, g)]
    return ([float(wi - lr * gi / (Gj.sqrt() + eps)) for wi, gi, Gj in zip(w, g, Gn)],
            [float(x) for x in Gn])


@pytest.mark.parametrize("opt", [oracle.ADAGRAD_ROWWISE, oracle.ADAGRAD_ELEMENTWISE])
def test_adagrad_closed_form_single_key(opt):
    # hand example with exactly representable inputs:
    #   w = (0.5, -0.25), G = 0.125, g = (0.5, 0.25), lr = 1/16, eps = 0
    #   row-wise:  G' = 0.125 + (0.25 + 0.0625)/2 = 0.28125, sqrt = 0.5303300858899106...
    #              w' = (0.5 - 0.03125/0.53033..., -0.25 - 0.015625/0.53033...)
    #   element-wise: G' = (0.375, 0.1875)
    t = OracleTable(4, 2, opt=opt, lr=0.0625, eps=0.0, init_acc=0.125)
    t.insert(np.array([10], dtype=np.uint64), np.array([[0.5, -0.25]], dtype=np.float32))
    t.pull(np.array([10], dtype=np.uint64), np.array([0, 1], dtype=np.int32))
    t.push(np.array([[0.5, 0.25]], dtype=np.float32))
    w, a, _ = t.get(np.array([10], dtype=np.uint64))
    if opt == oracle.ADAGRAD_ROWWISE:
        want_w = [0.5 - 0.03125 / math.sqrt(0.28125), -0.25 - 0.015625 / math.sqrt(0.28125)]
        want_a = [0.28125]
        assert abs(want_w[0] - 0.44107443490112104) < 1e-15     # digits worked out by hand
    else:
        want_w = [0.5 - 0.03125 / math.sqrt(0.375), -0.25 - 0.015625 / math.sqrt(0.1875)]
        want_a = [0.375, 0.1875]
        assert abs(want_w[1] + 0.28608439182435161) < 1e-15
    assert np.array_equal(w[0], np.array(want_w, dtype=np.float32))
    assert np.array_equal(a[0], np.array(want_a, dtype=np.float32))


@pytest.mark.parametrize("opt", [oracle.ADAGRAD_ROWWISE, oracle.ADAGRAD_ELEMENTWISE])
def test_adagrad_decimal_random_rows_and_eps_placement(opt):
    rng = np.random.default_rng(31)
    rowwise = opt == oracle.ADAGRAD_ROWWISE
    for trial in range(20):
        d = int(rng.integers(1, 9))
        lr, eps, acc0 = 0.05, [1e-8, 0.5][trial % 2], 0.1     # big eps exposes a misplaced eps
        t = OracleTable(4, d, opt=opt, lr=lr, eps=eps, init_acc=acc0)
        w0 = rng.uniform(-1, 1, size=(1, d)).astype(np.float32)
        g = rng.normal(0, 0.3, size=(1, d)).astype(np.float32)
        t.insert(np.array([3], dtype=np.uint64), w0)
        t.pull(np.array([3], dtype=np.uint64), np.array([0, 1], dtype=np.int32))
        t.push(g)
        w, a, _ = t.get(np.array([3], dtype=np.uint64))
        G0 = [np.float32(acc0)] * (1 if rowwise else d)
        ww, aa = _dec_adagrad(w0[0], G0, g[0], lr, eps, rowwise)
        assert np.array_equal(w[0], np.array(ww, dtype=np.float32))
        assert np.array_equal(a[0], np.array(aa, dtype=np.float32))


def test_reduce_then_single_step_not_per_occurrence():
    # key 5 occurs three times, in three bags with different gradients: the row must
    # take ONE step with the summed gradient (0.5, 0.25), as in the closed form above.
    t = OracleTable(4, 2, lr=0.0625, eps=0.0, init_acc=0.125)
    t.insert(np.array([5, 6], dtype=np.uint64),
             np.array([[0.5, -0.25], [1.0, 1.0]], dtype=np.float32))
    keys = np.array([5, 6, 5, 5], dtype=np.uint64)
    t.pull(keys, np.array([0, 2, 3, 4], dtype=np.int32))
    grads = np.array([[0.25, 0.125], [0.125, 0.0625], [0.125, 0.0625]], dtype=np.float32)
    t.push(grads)
    w, a, _ = t.get(np.array([5, 6], dtype=np.uint64))
    assert np.array_equal(w[0], np.array([0.5 - 0.03125 / math.sqrt(0.28125),
                                          -0.25 - 0.015625 / math.sqrt(0.28125)], np.float32))
    assert a[0, 0] == np.float32(0.28125)
    # key 6 saw only bag 0's gradient
    G6 = 0.125 + (0.25**2 + 0.125**2) / 2
    assert np.array_equal(w[1], np.array([1 - 0.0625 * 0.25 / math.sqrt(G6),
                                          1 - 0.0625 * 0.125 / math.sqrt(G6)], np.float32))


def test_elementwise_push_vs_torch_sparse_adagrad():
    rng = np.random.default_rng(41)
    n_keys, d, nb = 60, 6, 40
    t, keys, w = _table_with_values(rng, n_keys, d, opt=oracle.ADAGRAD_ELEMENTWISE, lr=0.05,
                                    eps=1e-8, init_acc=0.1)
    emb = torch.nn.EmbeddingBag(n_keys, d, mode="sum", sparse=True).double()
    with torch.no_grad():
        emb.weight.copy_(torch.from_numpy(w.astype(np.float64)))
    opt = torch.optim.Adagrad(emb.parameters(), lr=float(np.float32(0.05)),
                              initial_accumulator_value=float(np.float32(0.1)),
                              eps=float(np.float32(1e-8)))
    for step in range(4):
        sizes = rng.integers(0, 5, size=nb)
        offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        idx = rng.integers(0, n_keys, size=int(offsets[-1]))
        grads = rng.normal(0, 0.1, size=(nb, d)).astype(np.float32)
        pooled = t.pull(keys[idx], offsets)
        opt.zero_grad()
        out = emb(torch.from_numpy(idx), torch.from_numpy(offsets[:-1].astype(np.int64)))
        assert close(pooled, out.detach().numpy())
        out.backward(torch.from_numpy(grads.astype(np.float64)))
        opt.step()
        t.push(grads)
        wo, ao, f = t.get(keys)
        assert f.all() and close(wo, emb.weight.detach().numpy())
    # the accumulators too: torch keeps them in the optimizer state
    state_sum = opt.state[emb.weight]["sum"].numpy()
    assert close(ao, state_sum)


def test_rowwise_equals_elementwise_when_they_must():
    # dim 1, and rows whose gradient components are all equal: mean(g^2) = g_j^2
    rng = np.random.default_rng(43)
    for d, equal in ((1, False), (4, True)):
        a = OracleTable(64, d, opt=oracle.ADAGRAD_ROWWISE)
        b = OracleTable(64, d, opt=oracle.ADAGRAD_ELEMENTWISE)
        keys = synth.prefill_keys(0, 20)
        w = rng.uniform(-1, 1, size=(20, d)).astype(np.float32)
        a.insert(keys, w)
        b.insert(keys, w)
        for _ in range(3):
            idx = rng.integers(0, 20, size=30)
            offsets = np.arange(0, 31, 3, dtype=np.int32)
            g = rng.normal(0, 0.2, size=(10, 1)).astype(np.float32)
            g = np.repeat(g, d, axis=1) if equal else g
            a.pull(keys[idx], offsets)
            b.pull(keys[idx], offsets)
            a.push(g)
            b.push(g)
        wa, aa, _ = a.get(keys)
        wb, ab, _ = b.get(keys)
        assert np.array_equal(wa, wb) and np.array_equal(aa[:, 0], ab[:, 0])
    # ... and differ otherwise (mean, not sum, not per element)
    a = OracleTable(4, 2, opt=oracle.ADAGRAD_ROWWISE)
    a.insert(np.array([1], dtype=np.uint64), np.zeros((1, 2), np.float32))
    a.pull(np.array([1], dtype=np.uint64), np.array([0, 1], np.int32))
    a.push(np.array([[3.0, 4.0]], np.float32))
    assert a.get(np.array([1], dtype=np.uint64))[1][0, 0] == np.float32(0.1 + 12.5)


def test_push_invariants():
    rng = np.random.default_rng(51)
    cfg = synth.scaled(synth.CONFIGS["tiny"], n_prefill=3000, n_examples=32, n_slots=4, steps=6)
    t = OracleTable(cfg.capacity, cfg.dim)
    t.insert(synth.prefill_keys(0, cfg.n_prefill))
    stream = synth.BatchStream(cfg)
    k0, w0, a0 = t.dump()
    prev_a = a0.copy()
    for step in range(6):
        b = stream.next()
        t.pull(b.keys, b.offsets)
        grads = b.grads if step != 2 else np.zeros_like(b.grads)
        t.push(grads)
        k, w, a = t.dump()
        assert np.array_equal(k, k0)
        assert (a >= prev_a).all()                                  # accumulators never decrease
        touched = np.isin(k, b.keys)
        assert np.array_equal(w[~touched], w0[~touched]) and np.array_equal(a[~touched], prev_a[~touched])
        if step == 2:                                               # zero gradient: nothing moves
            assert np.array_equal(w, w0) and np.array_equal(a, prev_a)
        else:
            assert (a[touched] > prev_a[touched]).all()
        w0, prev_a = w, a
    # mass conservation of the reduction: sum over unique rows of g equals the sum over
    # occurrences; visible through a table with lr so small that only G moves ... checked
    # through the brute-force model below instead.


# ----------------------------------------------------------------------------- whole step

class _BruteModel:
    """Independent model of the whole path: python dict, lists, float64, no sorting library."""

    def __init__(self, dim, lr, eps, acc0, init_fn):
        self.dim, self.lr, self.eps, self.acc0, self.init_fn = dim, lr, eps, acc0, init_fn
        self.rows = {}

    def row(self, key):
        if key not in self.rows:
            self.rows[key] = [[float(x) for x in self.init_fn(key)], float(np.float32(self.acc0))]
        return self.rows[key]

    def pull(self, keys, offsets):
        self.keys, self.offsets = keys, offsets
        out = []
        for b in range(len(offsets) - 1):
            acc = [0.0] * self.dim
            for i in range(offsets[b], offsets[b + 1]):
                r = self.row(keys[i])[0]
                acc = [x + y for x, y in zip(acc, r)]
            out.append(acc)
        return out

    def push(self, grads):
        gsum = {}
        for b in range(len(self.offsets) - 1):
            for i in range(self.offsets[b], self.offsets[b + 1]):
                g = gsum.setdefault(self.keys[i], [0.0] * self.dim)
                for j in range(self.dim):
                    g[j] += float(grads[b][j])
        for key, g in gsum.items():
            w, G = self.rows[key]
            G = G + sum(x * x for x in g) / self.dim
            den = math.sqrt(G) + self.eps
            neww = [float(np.float32(wj - self.lr * gj / den)) for wj, gj in zip(w, g)]
            self.rows[key] = [neww, float(np.float32(G))]


def test_whole_step_vs_brute_force_model():
    cfg = synth.scaled(synth.CONFIGS["insert_heavy"], n_prefill=150, n_examples=6, n_slots=5,
                       steps=5)
    t = OracleTable(cfg.capacity, cfg.dim, lr=cfg.lr, eps=cfg.eps, init_acc=cfg.init_acc)
    t.insert(synth.prefill_keys(0, cfg.n_prefill))
    m = _BruteModel(cfg.dim, float(np.float32(cfg.lr)), float(np.float32(cfg.eps)), cfg.init_acc,
                    lambda k: _init_by_exact_arithmetic(k, cfg.dim, 0, 0.01))
    for k in synth.prefill_keys(0, cfg.n_prefill):
        m.row(int(k))
    stream = synth.BatchStream(cfg)
    total_g_occ = 0.0
    for _ in range(5):
        b = stream.next()
        p = t.pull(b.keys, b.offsets)
        pm = m.pull([int(k) for k in b.keys], [int(o) for o in b.offsets])
        assert close(p, np.array(pm))
        t.push(b.grads)
        m.push(b.grads)
        total_g_occ += float(np.sum(b.grads.astype(np.float64)
                                    * np.diff(b.offsets)[:, None]))
    k, w, a = t.dump()
    assert set(int(x) for x in k) == set(m.rows)
    wm = np.array([m.rows[int(x)][0] for x in k])
    am = np.array([m.rows[int(x)][1] for x in k])
    assert close(w, wm) and close(a[:, 0], am)
    assert t.size == len(m.rows)
    assert np.isfinite(total_g_occ)


def test_reduction_conserves_gradient_mass():
    # With w = 0, eps = 0, lr = 1 and a huge initial accumulator G0 the step is
    # w' = -g / sqrt(G0 + tiny), so sum over rows of w' * sqrt(G0) recovers -sum of all
    # occurrence gradients.
    rng = np.random.default_rng(61)
    G0 = 2.0**40
    t = OracleTable(256, 3, lr=1.0, eps=0.0, init_acc=G0)
    keys = synth.prefill_keys(0, 100)
    t.insert(keys, np.zeros((100, 3), np.float32))
    sizes = rng.integers(0, 7, size=50)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    idx = rng.integers(0, 100, size=int(offsets[-1]))
    grads = rng.normal(0, 1, size=(50, 3)).astype(np.float32)
    t.pull(keys[idx], offsets)
    t.push(grads)
    w, _, _ = t.get(keys)
    got = -(w.astype(np.float64) * math.sqrt(G0)).sum(0)
    want = (grads.astype(np.float64) * sizes[:, None]).sum(0)
    assert np.allclose(got, want, rtol=1e-5, atol=1e-4)


# ----------------------------------------------------------------------------- inputs

def test_workload_shapes_and_zipf_mass():
    cfg = synth.CONFIGS["tiny"]
    s = synth.BatchStream(cfg)
    b = s.next()
    assert b.offsets.shape[0] == 512 * 16 + 1 and b.offsets[0] == 0 and b.offsets[-1] == b.n_keys
    assert 1 <= np.diff(b.offsets).min() and np.diff(b.offsets).max() <= 4
    assert b.grads.shape == (8192, 8) and b.grads.dtype == np.float32
    assert (b.ids < cfg.n_prefill).all()
    # exact bounded Zipf(1.1) over 2^20 ranks: most frequent key carries ~12.4 % of lookups
    p1 = s.zipf.top_mass(1)
    assert abs(p1 - 0.124) < 0.003
    top = (b.ids == 0).mean()
    assert abs(top - p1) < 0.02
    # determinism
    b2 = synth.BatchStream(cfg).next()
    assert np.array_equal(b.keys, b2.keys) and np.array_equal(b.grads, b2.grads)
    mid = synth.scaled(synth.CONFIGS["mid"], n_prefill=50000, n_examples=64, n_slots=20)
    bm = synth.BatchStream(mid).next()
    frac_fresh = (bm.ids >= mid.n_prefill).mean()
    assert abs(frac_fresh - 0.05) < 0.01
    assert abs(np.diff(bm.offsets).mean() - 5.0) < 0.2


# ----------------------------------------------------------------------------- accumulate

def test_accumulate_exact_small_binary_fractions():
    # Section 4.1 accumulate: values add onto the rows their keys reference.  All numbers are
    # small binary fractions, so every sum is exact and the expected rows are written out.
    t = OracleTable(16, 4)
    keys = np.array([10, 20, 30], dtype=np.uint64)
    w0 = np.array([[1.0, 2.0, -3.0, 0.5], [0.25, 0.0, 8.0, -1.0], [4.0, 4.0, 4.0, 4.0]], dtype=np.float32)
    t.insert(keys, weights=w0)
    _, a0, _ = t.get(keys)
    absent = t.accumulate(np.array([20, 10, 20, 99, 20], dtype=np.uint64),
                          np.array([[0.5, 0.5, 0.5, 0.5],
                                    [-1.0, 0.25, 0.0, 2.0],
                                    [0.125, 0.0, -8.0, 1.0],
                                    [7.0, 7.0, 7.0, 7.0],        # key 99 is not stored: skipped
                                    [0.25, 1.0, 0.0, 0.0]], dtype=np.float32))
    assert absent == 1 and t.size == 3
    w, a, f = t.get(np.array([10, 20, 30, 99], dtype=np.uint64))
    assert f.tolist() == [True, True, True, False]
    assert w[0].tolist() == [0.0, 2.25, -3.0, 2.5]
    assert w[1].tolist() == [1.125, 1.5, 0.5, 0.5]             # three value rows summed, one step
    assert w[2].tolist() == [4.0, 4.0, 4.0, 4.0]
    assert np.array_equal(a[:3], a0)                            # optimizer state untouched


def test_accumulate_vs_torch_index_add():
    rng = np.random.default_rng(77)
    dim, n_rows, n = 8, 500, 4000
    keys = synth.mix64(np.arange(n_rows, dtype=np.uint64))
    t = OracleTable(1000, dim)
    t.insert(keys)
    w0, a0, _ = t.get(keys)
    pick = rng.integers(0, n_rows, size=n)
    vals = rng.normal(0, 1e-2, size=(n, dim)).astype(np.float32)
    assert t.accumulate(keys[pick], vals) == 0
    want = torch.from_numpy(w0.astype(np.float64)).index_add_(
        0, torch.from_numpy(pick), torch.from_numpy(vals.astype(np.float64))).numpy()
    w, a, _ = t.get(keys)
    # one rounding of an exactly (double) accumulated sum: at most half an ulp from torch's
    assert np.array_equal(w, want.astype(np.float32))
    assert np.array_equal(a, a0)
    untouched = ~np.isin(np.arange(n_rows), pick)
    assert np.array_equal(w[untouched], w0[untouched])


def test_accumulate_state_and_reserved_key():
    t = OracleTable(8, 4)
    t.insert(np.array([1, 2], dtype=np.uint64))
    with pytest.raises(OracleError):
        t.accumulate(np.array([2**64 - 1], dtype=np.uint64), np.zeros((1, 4), np.float32))
    t.pull(np.array([1], dtype=np.uint64), np.array([0, 1], dtype=np.int32))
    with pytest.raises(OracleError):                            # between a pull and its push
        t.accumulate(np.array([1], dtype=np.uint64), np.zeros((1, 4), np.float32))
    t.push(np.zeros((1, 4), np.float32))
    assert t.accumulate(np.zeros(0, np.uint64), np.zeros((0, 4), np.float32)) == 0


def test_push_equals_accumulate_of_the_closed_form_step():
    # Section 4.1: the paper's push hands the table a worker-computed delta.  With one key per
    # bag and no repeats, delta = -lr * g / (sqrt(G + mean g^2) + eps) written out here must
    # move the weights as push(g) does.
    rng = np.random.default_rng(5)
    dim, n = 8, 64
    keys = synth.mix64(np.arange(n, dtype=np.uint64))
    g = rng.normal(0, 1e-1, size=(n, dim)).astype(np.float32)
    a = OracleTable(100, dim, lr=0.05, eps=1e-8, init_acc=0.1)
    b = OracleTable(100, dim, lr=0.05, eps=1e-8, init_acc=0.1)
    a.insert(keys); b.insert(keys)
    a.pull(keys, np.arange(n + 1, dtype=np.int32))
    a.push(g)
    G = float(np.float32(0.1)) + (g.astype(np.float64) ** 2).mean(axis=1, keepdims=True)
    delta = -float(np.float32(0.05)) * g.astype(np.float64) / (np.sqrt(G) + float(np.float32(1e-8)))
    b.accumulate(keys, delta.astype(np.float32))
    wa, _, _ = a.get(keys)
    wb, _, _ = b.get(keys)
    assert np.abs(wa.astype(np.float64) - wb.astype(np.float64)).max() <= 2.0 ** -24 * np.abs(wa).max() * 2


# ----------------------------------------------------------------------------- dirty rows

def test_dump_dirty_hands_over_exactly_the_updated_rows_once():
    cfg = synth.scaled(synth.CONFIGS["tiny"], n_prefill=3000, n_examples=32, n_slots=4, steps=3)
    t = OracleTable(cfg.capacity, cfg.dim)
    t.insert(synth.prefill_keys(0, cfg.n_prefill))
    k, _, _ = t.dump_dirty()
    assert k.size == 0                                          # inserted rows are not updates
    stream = synth.BatchStream(cfg)
    seen = []
    for _ in range(2):
        b = stream.next()
        t.pull(b.keys, b.offsets)
        t.push(b.grads)
        seen.append(b.keys)
    want = np.unique(np.concatenate(seen))                      # includes keys created by the pulls
    k, w, a = t.dump_dirty()
    assert np.array_equal(k, want)
    gw, ga, f = t.get(want)
    assert f.all() and np.array_equal(w, gw) and np.array_equal(a, ga)
    assert t.dump_dirty()[0].size == 0                          # marks are forgotten
    some = want[::7]
    assert t.accumulate(np.concatenate([some, [np.uint64(12345)]]),
                        np.ones((some.size + 1, cfg.dim), np.float32)) == 1
    k, w, _ = t.dump_dirty()
    assert np.array_equal(k, some) and np.array_equal(w, gw[::7] + np.float32(1.0))
    assert np.array_equal(t.dump()[0], np.unique(np.concatenate([synth.prefill_keys(0, cfg.n_prefill), want])))


# ----------------------------------------------------------------------------- mean pooling

def test_mean_pooling_whole_step_vs_torch_autograd():
    # EmbeddingBag(mode="mean") forward, torch autograd for the routing of the bag gradients
    # (each occurrence gets 1/len of it), torch's sparse Adagrad for the step: three library
    # routines the oracle's mean pooling has to agree with over several steps.
    rng = np.random.default_rng(43)
    n_keys, d, nb = 50, 6, 48
    t, keys, w = _table_with_values(rng, n_keys, d, opt=oracle.ADAGRAD_ELEMENTWISE, lr=0.05,
                                    eps=1e-8, init_acc=0.1)
    t.set_pooling(True)
    emb = torch.nn.EmbeddingBag(n_keys, d, mode="mean", sparse=True).double()
    with torch.no_grad():
        emb.weight.copy_(torch.from_numpy(w.astype(np.float64)))
    opt = torch.optim.Adagrad(emb.parameters(), lr=float(np.float32(0.05)),
                              initial_accumulator_value=float(np.float32(0.1)),
                              eps=float(np.float32(1e-8)))
    for step in range(4):
        sizes = rng.integers(0, 6, size=nb)               # includes empty bags
        offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        idx = rng.integers(0, n_keys, size=int(offsets[-1]))
        grads = rng.normal(0, 0.1, size=(nb, d)).astype(np.float32)
        pooled = t.pull(keys[idx], offsets)
        opt.zero_grad()
        out = emb(torch.from_numpy(idx), torch.from_numpy(offsets[:-1].astype(np.int64)))
        assert close(pooled, out.detach().numpy())
        assert not pooled[sizes == 0].any()
        out.backward(torch.from_numpy(grads.astype(np.float64)))
        opt.step()
        t.push(grads)
        wo, ao, f = t.get(keys)
        assert f.all() and close(wo, emb.weight.detach().numpy())
    assert close(ao, opt.state[emb.weight]["sum"].numpy())


def test_mean_pooling_closed_forms_and_state():
    t = OracleTable(16, 4, lr=0.5, eps=0.0, init_acc=0.0)
    keys = np.array([3, 4], dtype=np.uint64)
    t.insert(keys, weights=np.array([[1, 2, 3, 4], [3, 2, 1, 0]], np.float32))
    t.set_pooling(True)
    # bag 0 = {3, 3, 4, 4}: mean = (2, 2, 2, 2); bag 1 = {4}: the row itself
    pooled = t.pull(np.array([3, 3, 4, 4, 4], dtype=np.uint64), np.array([0, 4, 5], np.int32))
    assert pooled.tolist() == [[2.0, 2.0, 2.0, 2.0], [3.0, 2.0, 1.0, 0.0]]
    with pytest.raises(OracleError):
        t.set_pooling(False)                               # not inside a step
    # key 3: two occurrences in a bag of four -> 2 * g0 / 4; key 4: 2 * g0 / 4 + g1
    g = np.array([[4, 0, -4, 8], [1, 1, 1, 1]], np.float32)
    t.push(g)
    w, a, _ = t.get(keys)
    g3 = np.array([2, 0, -2, 4], np.float64)
    g4 = np.array([3, 1, -1, 5], np.float64)
    for row, acc, w0, gk in ((w[0], a[0], [1, 2, 3, 4], g3), (w[1], a[1], [3, 2, 1, 0], g4)):
        G = (gk ** 2).mean()
        assert acc[0] == np.float32(G)
        assert np.array_equal(row, (np.array(w0, np.float64) - 0.5 * gk / np.sqrt(G)).astype(np.float32))
    t.set_pooling(False)                                   # back to sums
    pooled = t.pull(np.array([3, 3], dtype=np.uint64), np.array([0, 2], np.int32))
    assert np.array_equal(pooled[0], (w[0].astype(np.float64) * 2).astype(np.float32))


# ---- rows stored as bfloat16 -------------------------------------------------------------

def _torch_bf16(a):
    """Round float32 values to bfloat16 and back with torch's conversion (nearest, ties to even)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def test_nearest_bf16_ties_and_against_torch():
    # bfloat16 keeps 8 significant bits: next to 1.0 the values are 1, 1 + 2^-7, 1 + 2^-6, ...
    assert oracle.nearest_bf16(1.0) == 1.0
    assert oracle.nearest_bf16(1.0 + 2.0 ** -8) == 1.0                       # tie -> even (fraction 0)
    assert oracle.nearest_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6       # tie -> even (fraction 2)
    assert oracle.nearest_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7   # just above the tie
    assert oracle.nearest_bf16(-(1.0 + 2.0 ** -8)) == -1.0
    assert oracle.nearest_bf16(0.0) == 0.0 and oracle.nearest_bf16(2.0 ** -130) == 2.0 ** -130   # subnormal kept
    assert oracle.nearest_bf16(float(np.float32(1.99999988))) == 2.0         # carry into the exponent
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 1, 50_000), rng.uniform(-0.01, 0.01, 50_000),
                        rng.normal(0, 1, 20_000) * 10.0 ** rng.integers(-30, 30, 20_000)]).astype(np.float32)
    bits = rng.integers(0, 2 ** 32, 50_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    x = np.concatenate([x, bits[np.isfinite(bits)]])
    got = np.array([oracle.nearest_bf16(float(v)) for v in x], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), _torch_bf16(x).view(np.uint32))


@pytest.mark.parametrize("opt", [oracle.ADAGRAD_ROWWISE, oracle.ADAGRAD_ELEMENTWISE])
def test_bf16_rows_whole_step_closed_form(opt):
    """A table that stores weights as bfloat16: every stored weight is a bfloat16 value; a new
    row is the float32 initial row rounded; pooling sums the rounded rows; a push computes the
    float32 table's step from the rounded weights and rounds the result.  All of it written out
    here with numpy float64 and torch's conversion."""
    rng = np.random.default_rng(12)
    d, lr, eps, acc0 = 8, 0.05, 1e-8, 0.1
    tb = OracleTable(64, d, opt=opt, lr=lr, eps=eps, init_acc=acc0, row_format=oracle.ROWS_BF16)
    tf = OracleTable(64, d, opt=opt, lr=lr, eps=eps, init_acc=acc0)
    keys = np.array([7, 9, 7, 11, 9, 7], dtype=np.uint64)
    offsets = np.array([0, 2, 3, 6], dtype=np.int32)
    uniq = np.array([7, 9, 11], dtype=np.uint64)
    w0 = _torch_bf16(np.stack([tf.init_row(int(k)) for k in uniq]))          # rounded float32 init rows
    assert np.array_equal(np.stack([tb.init_row(int(k)) for k in uniq]), w0)
    pooled = tb.pull(keys, offsets)
    inv = np.array([0, 1, 0, 2, 1, 0])
    want = np.stack([w0[inv[a:b]].astype(np.float64).sum(0) for a, b in zip(offsets[:-1], offsets[1:])])
    assert np.array_equal(pooled, want.astype(np.float32))
    grads = rng.normal(0, 0.05, size=(3, d)).astype(np.float32)
    tb.push(grads)
    bag = np.array([0, 0, 1, 2, 2, 2])
    g = np.stack([grads[bag[inv == u]].astype(np.float64).sum(0) for u in range(3)])
    if opt == oracle.ADAGRAD_ROWWISE:
        G = np.float64(np.float32(acc0)) + (g ** 2).mean(1, keepdims=True)
    else:
        G = np.float64(np.float32(acc0)) + g ** 2
    step = w0.astype(np.float64) - np.float64(np.float32(lr)) * g / (np.sqrt(G) + np.float64(np.float32(eps)))
    w, a, f = tb.get(uniq)
    assert f.all()
    assert np.array_equal(w, _torch_bf16(step.astype(np.float32)))
    assert np.array_equal(a, G.astype(np.float32))
    assert not (w.view(np.uint32) & 0xFFFF).any()                            # bfloat16 values only
    # accumulate and insert store rounded values too; dump -> insert is the identity
    tb.accumulate(uniq[:2], np.full((2, d), 1e-3, np.float32))
    w2, _, _ = tb.get(uniq[:2])
    assert np.array_equal(w2, _torch_bf16((w[:2].astype(np.float64) + np.float64(np.float32(1e-3))).astype(np.float32)))
    tb.insert(np.array([100], dtype=np.uint64), np.full((1, d), 0.3, np.float32))
    assert np.array_equal(tb.get(np.array([100], dtype=np.uint64))[0][0], _torch_bf16(np.full(d, 0.3, np.float32)))
    k, ww, aa = tb.dump()
    t2 = OracleTable(64, d, opt=opt, lr=lr, eps=eps, init_acc=acc0, row_format=oracle.ROWS_BF16)
    t2.insert(k, ww, aa)
    k2, ww2, aa2 = t2.dump()
    assert np.array_equal(k, k2) and np.array_equal(ww, ww2) and np.array_equal(aa, aa2)
    with pytest.raises(OracleError):
        lib_table = OracleTable(4, 2)
        lib_table.insert(np.array([1], dtype=np.uint64))
        oracle._check(oracle.lib().hpo_set_row_format(lib_table._h, oracle.ROWS_BF16), "set_row_format")


def test_clear_empties_the_table_and_keeps_the_settings():
    # Algorithm 1: one table per batch of the outer loop.  After a clear the table behaves
    # like a new one with the same settings: nothing is found, rows are created from the
    # initialiser again (whatever they had become), and nothing counts as updated.
    t = OracleTable(8, 4, opt=oracle.ADAGRAD_ELEMENTWISE, lr=0.5, eps=0.0, init_acc=0.25, init_seed=9)
    fresh = OracleTable(8, 4, opt=oracle.ADAGRAD_ELEMENTWISE, lr=0.5, eps=0.0, init_acc=0.25, init_seed=9)
    keys = np.array([5, 6, 7], dtype=np.uint64)
    offsets = np.array([0, 2, 3], dtype=np.int32)
    t.set_pooling(True)
    fresh.set_pooling(True)
    t.pull(keys, offsets)
    with pytest.raises(OracleError) as e:
        t.clear()                                           # not between a pull and its push
    assert e.value.status == oracle.ESTATE
    t.push(np.ones((2, 4), dtype=np.float32))
    assert t.size == 3 and not np.array_equal(t.get(keys)[0][0], t.init_row(5))
    t.clear()
    assert t.size == 0 and not t.get(keys)[2].any()
    assert t.dump()[0].size == 0 and t.dump_dirty()[0].size == 0
    for table in (t, fresh):                                # same steps on the cleared and on a new table
        table.insert(np.arange(8, dtype=np.uint64))         # capacity 8 is available again
        table.pull(keys, offsets)
        table.push(np.full((2, 4), 0.5, dtype=np.float32))
    for a, b in zip(t.dump(), fresh.dump()):
        assert np.array_equal(a, b)
    for a, b in zip(t.dump_dirty(), fresh.dump_dirty()):
        assert np.array_equal(a, b)
