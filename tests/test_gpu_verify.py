"""GPU parity of the hash-set verifier (nezha_build_itemset, nezha_verify_tuples) against the
CPU oracle: masks, accepted-index lists and counts must be bit-exact."""
import numpy as np
import pytest
import torch

import synth
import paper_2511_18793_amd as nz
from _gpu_common import device
from _parity import to_np

pytestmark = pytest.mark.gpu


def run_verify(gset, q):
    mask, idx, cnt = nz.verify_tuples(gset, torch.from_numpy(np.ascontiguousarray(q)).to(device()))
    torch.cuda.synchronize()
    c = int(cnt.item())
    return to_np(mask), to_np(idx)[:c], c


@pytest.mark.parametrize("radices,N,lf", [
    ([256, 256, 256], 10_000, 0.5), ([7, 300, 11, 5], 20_000, 0.9), ([1000], 400, 0.5),
    ([4, 3, 5, 2, 6, 3, 4, 2], 9_000, 0.3), ([4096, 4096, 4096], 300_000, 0.75),
    ([1024] * 4, 250_000, 0.5),
])
def test_verify_matches_oracle(oracle, radices, N, lf):
    cat, pi = synth.uniform_catalog(radices, N, 11)
    cat_dup = np.concatenate([cat, cat[: N // 7]])
    oset = oracle.ItemSet(cat_dup, radices)
    gset = nz.build_itemset(cat_dup, radices, lf)
    info = gset.info()
    assert info["n_distinct"] == N == len(oset) and info["radices"] == radices
    assert info["n_slots"] >= N / lf and info["n_slots"] % 8 == 0
    size = int(np.prod(radices, dtype=object))
    nq = 50_003
    absent = synth.absent_tuples(radices, N, pi, 5, nq // 2) if size > N else cat[:0]
    q = np.concatenate([cat[: nq // 2], absent])
    q = q[np.argsort(synth.mix64(np.arange(len(q), dtype=np.uint64)), kind="stable")]
    q[::97, 0] = radices[0]            # out-of-range codes are rejected, not errors
    q[5::101, -1] = -1
    want_mask, want_idx = oset.verify_tuples(q)
    mask, idx, c = run_verify(gset, q)
    assert (mask == want_mask).all()
    assert c == len(want_idx) and (idx == want_idx).all()
    gset.close()


@pytest.mark.parametrize("n", [0, 1, 63, 1024, 1025, 4099])
def test_verify_ragged_and_empty_batches(oracle, n):
    radices = [64, 64, 64]
    cat, pi = synth.uniform_catalog(radices, 50_000, 3)
    oset, gset = oracle.ItemSet(cat, radices), nz.build_itemset(cat, radices)
    q, _ = synth.stress_queries(radices, 50_000, pi, 9, max(n, 1))
    q = q[:n]
    mask, idx, c = run_verify(gset, q.reshape(n, 3))
    want_mask, want_idx = oset.verify_tuples(q.reshape(n, 3))
    assert (mask == want_mask).all() and c == len(want_idx) and (idx == want_idx).all()


def test_empty_catalog_and_device_resident_codes(oracle):
    radices = [16, 16]
    gset = nz.build_itemset(np.zeros((0, 2), np.int32), radices)
    assert gset.info()["n_distinct"] == 0
    q = np.array([[0, 0], [15, 15]], dtype=np.int32)
    mask, idx, c = run_verify(gset, q)
    assert c == 0 and not mask.any()
    cat, _ = synth.uniform_catalog(radices, 100, 1)
    g2 = nz.build_itemset(torch.from_numpy(cat).to(device()), radices)
    assert g2.info()["n_distinct"] == 100
    mask, idx, c = run_verify(g2, cat)
    assert c == 100 and mask.all()


def test_build_rejects_out_of_range_catalog_codes():
    with pytest.raises(nz.NezhaError) as ei:
        nz.build_itemset(np.array([[0, 0], [4, 0]], dtype=np.int32), [4, 4])
    assert ei.value.code == -4


def test_mask_only_call(oracle):
    radices = [64, 64, 64]
    cat, pi = synth.uniform_catalog(radices, 10_000, 3)
    gset = nz.build_itemset(cat, radices)
    q, present = synth.stress_queries(radices, 10_000, pi, 9, 3000)
    mask, idx, cnt = nz.verify_tuples(gset, torch.from_numpy(q).to(device()), want_index=False)
    torch.cuda.synchronize()
    assert idx is None and cnt is None and (to_np(mask).astype(bool) == present).all()


def test_serving_catalog_zipf_first_level(oracle):
    cfg = synth.get_config("serving")
    cat = synth.zipf_catalog(cfg.radices, cfg.N, 42, cfg.zipf_s)
    oset, gset = oracle.ItemSet(cat, cfg.radices), nz.build_itemset(cat, cfg.radices)
    assert gset.info()["n_distinct"] == cfg.N
    rng = np.random.default_rng(0)
    q = np.concatenate([cat[rng.integers(0, cfg.N, 200_000)],
                        rng.integers(0, 256, (200_000, 3)).astype(np.int32)])
    q = q[rng.permutation(len(q))]
    want_mask, want_idx = oset.verify_tuples(q)
    mask, idx, c = run_verify(gset, q)
    assert (mask == want_mask).all() and (idx == want_idx).all()


def test_stress_shape_full_size_by_construction():
    """100,000,000 items at load factor 0.5 and 4,000,000 queries: membership is known from
    how the generator built catalog and queries, so no 10^8-element CPU set is needed."""
    cfg = synth.get_config("stress")
    cat, pi = synth.uniform_catalog(cfg.radices, cfg.N, 42)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    del cat
    info = gset.info()
    assert info["n_distinct"] == cfg.N and info["n_slots"] == 2 * cfg.N
    q, present = synth.stress_queries(cfg.radices, cfg.N, pi, 42, cfg.queries)
    mask, idx, c = run_verify(gset, q)
    assert (mask.astype(bool) == present).all()
    assert c == int(present.sum()) and (idx == np.nonzero(present)[0]).all()
    gset.close()


def test_double_free_is_refused():
    radices = [16, 16]
    cat, _ = synth.uniform_catalog(radices, 50, 2)
    gset = nz.build_itemset(cat, radices)
    h = gset._h
    lib = nz.load_library()
    assert lib.nezha_free_itemset(h) == 0
    assert lib.nezha_free_itemset(h) == -1              # not read again: the registry answers
    assert lib.nezha_itemset_info(h, None, None, None, None) == -1
    gset._h = None


def test_self_check_finds_every_item_of_the_catalog():
    """After a build every tuple of the catalog must be found through prefilter and table
    (a filter bit that was not set would silently drop a valid item in the draft step)."""
    cfg = synth.get_config("serving")
    cat = synth.zipf_catalog(cfg.radices, cfg.N, 42, cfg.zipf_s)
    gset = nz.build_itemset(cat, cfg.radices)
    assert gset.check(cat) == 0                                       # host catalog, staged
    assert gset.check(torch.from_numpy(cat[:70_001]).to(device())) == 0
    absent = cat[:1000].copy()
    absent[:, 0] = (absent[:, 0] + 1) % 256
    own = set(map(tuple, cat.tolist()))
    want = sum(tuple(t) not in own for t in absent.tolist())
    assert want > 0 and gset.check(absent) == want
    bad = cat[:10].copy()
    bad[3, 1] = 256                                                   # out of range: never found
    assert gset.check(bad) == 1


def test_allocation_failures_during_build_leak_nothing(monkeypatch):
    """Each allocation of a build is made to fail in turn (host catalog: handle, table, status
    words, staging buffer, prefilter).  Failures 1-4 give NEZHA_ENOMEM and return the device
    memory they held; without its prefilter (5) the set is still exact."""
    radices = [256, 256, 256]
    N = 3_000_000                                     # a 48 MB table: a leak would show
    cat, pi = synth.uniform_catalog(radices, N, 8)
    torch.cuda.synchronize()
    nz.build_itemset(cat[:10], radices).close()       # anything lazy in the runtime is paid now
    free0 = torch.cuda.mem_get_info()[0]
    for nth in (1, 2, 3, 4):
        monkeypatch.setenv("NEZHA_TEST_FAIL_ALLOC", str(nth))
        with pytest.raises(nz.NezhaError) as ei:
            nz.build_itemset(cat, radices)
        assert ei.value.code == -2
        assert abs(torch.cuda.mem_get_info()[0] - free0) < (4 << 20), nth
    monkeypatch.setenv("NEZHA_TEST_FAIL_ALLOC", "5")
    gset = nz.build_itemset(cat, radices)
    monkeypatch.delenv("NEZHA_TEST_FAIL_ALLOC")
    assert gset.info()["n_distinct"] == N and gset.check(cat) == 0
    q, present = synth.stress_queries(radices, N, pi, 8, 100_000)
    mask, idx, c = run_verify(gset, q)
    assert (mask.astype(bool) == present).all() and c == int(present.sum())
    # the draft step consults the set without a prefilter: same answer as with one
    cfg = synth.StepConfig("nofilter", B=8, d=64, e=32, L=3, V=256, K=8, N=N, dtype="bf16",
                           catalog="uniform")
    x = synth.draft_inputs(cfg, 8)
    H = torch.from_numpy(x["H"]).to(device()).to(torch.bfloat16)
    W = [torch.from_numpy(w).to(device()).to(torch.bfloat16) for w in x["W"]]
    E = [torch.from_numpy(w).to(device()).to(torch.bfloat16) for w in x["E"]]
    full = nz.build_itemset(cat, radices)
    a = nz.decode(H, W, E, cfg.radices, cfg.K, gset)
    a = [{k: v.clone() for k, v in o.items()} for o in a]
    b = nz.decode(H, W, E, cfg.radices, cfg.K, full)
    torch.cuda.synchronize()
    for k in a[-1]:
        assert torch.equal(a[-1][k], b[-1][k]), k
    before_close = torch.cuda.mem_get_info()[0]
    gset.close()
    full.close()
    # both tables (48 MB each) and the one prefilter go back to the device
    assert torch.cuda.mem_get_info()[0] - before_close > (90 << 20)
