"""Pins for the oracle's key packing (Eq. 4) and set membership (Eq. 5)."""
import itertools
import os

import numpy as np
import pytest

import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "eq4_worked_example.txt")


def test_eq4_printed_example(oracle):
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    for r in rows:
        v = list(map(int, r))
        keys, ok = oracle.pack([v[0:3]], v[3:6])
        assert ok.all() and int(keys[0]) == v[6]


@pytest.mark.parametrize("radices", [[3, 5, 4], [7, 2, 9, 4], [2], [16, 16], [5, 1, 3]])
def test_eq4_is_a_bijection_onto_the_range(oracle, radices):
    tuples = np.array(list(itertools.product(*[range(r) for r in radices])), dtype=np.int32)
    keys, ok = oracle.pack(tuples, radices)
    total = int(np.prod(radices))
    assert ok.all()
    assert len(set(keys.tolist())) == total
    assert int(keys.min()) == 0 and int(keys.max()) == total - 1
    assert (oracle.unpack(keys, radices) == tuples).all()


def test_eq4_level_one_is_least_significant(oracle):
    radices = [3, 5, 7]
    unit = np.eye(3, dtype=np.int32)
    keys, _ = oracle.pack(unit, radices)
    assert keys.tolist() == [1, 3, 15]          # empty product = 1, then T1, then T1*T2
    keys, _ = oracle.pack([[2, 4, 6]], radices)
    assert int(keys[0]) == 2 + 4 * 3 + 6 * 15 == 104


def test_eq4_matches_python_integers_on_wide_radices(oracle):
    radices = [4096, 4096, 4096, 1 << 20]
    rng = np.random.default_rng(0)
    t = np.stack([rng.integers(0, r, 1000) for r in radices], 1).astype(np.int32)
    keys, ok = oracle.pack(t, radices)
    for row, k in zip(t.tolist(), keys.tolist()):
        want, mul = 0, 1
        for c, r in zip(row, radices):
            want += c * mul
            mul *= r
        assert k == want
    assert ok.all()


def test_out_of_range_codes_are_flagged(oracle):
    keys, ok = oracle.pack([[0, 0, 0], [3, 0, 0], [0, -1, 0], [2, 4, 3]], [3, 5, 4])
    assert ok.tolist() == [True, False, False, True]
    assert int(keys[1]) == 2**64 - 1


def test_radix_product_must_fit(oracle):
    with pytest.raises(OverflowError):
        oracle.pack([[0, 0, 0]], [1 << 30, 1 << 30, 1 << 4])
    keys, ok = oracle.pack([[(1 << 30) - 1, (1 << 30) - 1, 7]], [1 << 30, 1 << 30, 1 << 3])
    assert ok.all() and int(keys[0]) == 2**63 - 1


def _python_keys(tuples, radices):
    mul, out = 1, np.zeros(len(tuples), dtype=object)
    for l, r in enumerate(radices):
        out = out + tuples[:, l].astype(object) * mul
        mul *= r
    return np.array([int(x) for x in out], dtype=np.uint64)


def test_membership_against_sorted_array(oracle):
    radices = [64, 32, 16]
    cat, pi = synth.uniform_catalog(radices, 5000, 7)
    cat = np.concatenate([cat, cat[:100]])               # duplicates are stored once
    s = oracle.ItemSet(cat, radices)
    assert len(s) == 5000
    ref = np.sort(_python_keys(cat[:5000], radices))
    q = np.array(list(itertools.product(range(64), range(32), range(16))), dtype=np.int32)
    qk = _python_keys(q, radices)
    pos = np.searchsorted(ref, qk).clip(0, ref.size - 1)
    want = ref[pos] == qk
    mask, idx = s.verify_tuples(q)
    assert (mask.astype(bool) == want).all()
    assert (idx == np.nonzero(want)[0]).all()            # ascending, stable
    assert int(want.sum()) == 5000
    assert (s.contains_keys(qk) == want).all()


def test_membership_rejects_out_of_range_queries(oracle):
    radices = [4, 4]
    s = oracle.ItemSet([[0, 0], [3, 3]], radices)
    mask, idx = s.verify_tuples([[0, 0], [4, -1], [3, 3], [-1, 0], [1, 1]])
    assert mask.tolist() == [1, 0, 1, 0, 0] and idx.tolist() == [0, 2]
    with pytest.raises(ValueError):
        oracle.ItemSet([[0, 4]], radices)


def test_membership_tiny_config_against_bitmap(oracle):
    cfg = synth.get_config("tiny")
    cat, pi = synth.uniform_catalog(cfg.radices, cfg.N, 42)
    s = oracle.ItemSet(cat, cfg.radices)
    V = cfg.V
    bitmap = np.zeros((V, V, V), dtype=bool)             # indexed [t1, t2, t3]
    bitmap[cat[:, 0], cat[:, 1], cat[:, 2]] = True
    t3, t2, t1 = np.meshgrid(np.arange(V), np.arange(V), np.arange(V), indexing="ij")
    q = np.stack([t1.ravel(), t2.ravel(), t3.ravel()], 1).astype(np.int32)
    mask, idx = s.verify_tuples(q)
    assert (mask.astype(bool) == bitmap[q[:, 0], q[:, 1], q[:, 2]]).all()
    assert idx.size == cfg.N
    absent = synth.absent_tuples(cfg.radices, cfg.N, pi, 42, 20000)
    assert not s.verify_tuples(absent)[0].any()
