"""The entry point that allocates nothing: hps_accumulate_static, called through the C ABI,
against hps_accumulate on a table of the same content.  Two calls in a row, the second with
a smaller input (the static array keeps the first call's contents).  Both entry points sum a
key's value rows in occurrence order with the same fixed-shape sums, so the tables must end
bit-identical; the count of absent keys must agree too."""
import numpy as np
import pytest
import torch

import paper_2003_05622_amd as hps
import synth

pytestmark = pytest.mark.gpu


def dev_keys(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).cuda()


def sorted_dump(t):
    k, w, a = t.dump()
    k = k.cpu().numpy().view(np.uint64)
    order = np.argsort(k, kind="stable")
    return k[order], w.cpu().numpy()[order], a.cpu().numpy()[order]


@pytest.mark.parametrize("dim", [16, 64])
def test_accumulate_static_matches_accumulate(dim, monkeypatch):
    monkeypatch.delenv("HPS_DEDUP", raising=False)
    rng = np.random.default_rng(dim)
    resident = synth.mix64(np.arange(200_000, dtype=np.uint64))
    kw = dict(lr=0.05, eps=1e-8, init_acc=0.1, init_range=0.01, init_seed=9)
    tables = [hps.HpsTable(400_000, dim, 65536, 65536, **kw) for _ in range(2)]
    for t in tables:
        t.insert(dev_keys(resident))
    for n in (60_000, 65_536, 700, 0, 1):          # two full-size calls, then smaller ones
        ranks = np.minimum(rng.zipf(1.2, size=n), resident.size) - 1
        keys = resident[ranks]
        if n > 10:
            keys[rng.random(n) < 0.05] = synth.mix64(np.uint64(10**12) + rng.integers(0, 1000, dtype=np.uint64))  # absent
        values = rng.normal(0, 1e-3, size=(n, dim)).astype(np.float32)
        dk, dv = dev_keys(keys), torch.from_numpy(values).cuda()
        tables[0].accumulate(dk, dv)
        tables[1].accumulate_static(dk, dv)
        s0, s1 = tables[0].stats(), tables[1].stats()
        assert s0.error == 0 and s1.error == 0
        assert s0.last_n_absent == s1.last_n_absent
        k0, w0, a0 = sorted_dump(tables[0])
        k1, w1, a1 = sorted_dump(tables[1])
        assert np.array_equal(k0, k1)
        assert np.array_equal(w0.view(np.uint32), w1.view(np.uint32)), "n = %d" % n
        assert np.array_equal(a0.view(np.uint32), a1.view(np.uint32))


def test_accumulate_static_rejects_what_does_not_fit():
    t = hps.HpsTable(1000, 8, 100_000, 100_000)
    keys = dev_keys(synth.mix64(np.arange(65_537, dtype=np.uint64)))
    values = torch.zeros((65_537, 8), device="cuda")
    with pytest.raises(hps.HpsError) as e:
        t.accumulate_static(keys, values)
    assert e.value.status == hps.EINVAL
