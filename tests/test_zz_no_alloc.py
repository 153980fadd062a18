"""The verifier entry point that allocates nothing (nezha_verify_tuples_static: scratch in a fixed
device array of the library) against nezha_verify_tuples on the same queries: masks, ascending
index lists and counts bit-exact, on two calls in a row, the second with a smaller input (the
shared array keeps the first call's contents), then across the multi-block scan, and the size
limit."""
import numpy as np
import pytest
import torch

import synth
import paper_2511_18793_amd as nz

pytestmark = pytest.mark.gpu


def _both(gset, qd, outs):
    """Runs both entry points on qd; `outs` are preallocated (mask, index, count) for the static
    call.  Returns the two result triples as numpy (index lists cut to the count)."""
    n = qd.shape[0]
    mask, idx, cnt = nz.verify_tuples(gset, qd)
    m2, i2, c2 = outs
    m2[:n].fill_(7)
    i2[:n].fill_(-1)
    c2.fill_(-1)
    torch.cuda.synchronize()
    mv, iv = m2[:n], i2[:n]
    before = torch.cuda.memory_stats()["allocation.all.allocated"]      # allocation events so far
    nz.verify_tuples_static(gset, qd, mv, iv, c2)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    torch.cuda.synchronize()
    c = int(cnt.item())
    return ((mask.cpu().numpy(), idx.cpu().numpy()[:c], c),
            (m2[:n].cpu().numpy(), i2[:c].cpu().numpy(), int(c2.item())))


def test_static_verifier_equals_the_workspace_verifier():
    dev = torch.device("cuda:0")
    radices = [4096, 4096, 4096]
    N = 1_000_000
    cat, pi = synth.uniform_catalog(radices, N, 3)
    gset = nz.build_itemset(cat, radices, 0.5)
    n1, n2 = 3_000_011, 70_001
    cap = 16384 * 1024 + 300_000
    outs = (torch.empty(cap, dtype=torch.uint8, device=dev),
            torch.empty(cap, dtype=torch.int64, device=dev),
            torch.empty(1, dtype=torch.int64, device=dev))
    q1, p1 = synth.stress_queries(radices, N, pi, 3, n1)
    q2, p2 = synth.stress_queries(radices, N, pi, 4, n2)
    for q, present in ((q1, p1), (q2, p2)):          # two calls in a row, the second smaller
        qd = torch.from_numpy(q).to(dev)
        (m, i, c), (ms, is_, cs) = _both(gset, qd, outs)
        assert c == cs == int(present.sum())
        assert (m == ms).all() and (m.astype(bool) == present).all()
        assert (i == is_).all() and (is_ == np.nonzero(present)[0]).all()
    # more than 16384 blocks: the scan kernel's offsets live in the same array
    q3, p3 = synth.stress_queries(radices, N, pi, 5, cap)
    qd = torch.from_numpy(q3).to(dev)
    del q3
    (m, i, c), (ms, is_, cs) = _both(gset, qd, outs)
    assert c == cs == int(p3.sum()) and (m == ms).all() and (i == is_).all()
    # ... and a small call after the largest one, mask only / count only / empty
    qd = torch.from_numpy(q2[:1000]).to(dev)
    m2 = torch.empty(1000, dtype=torch.uint8, device=dev)
    nz.verify_tuples_static(gset, qd, m2)
    torch.cuda.synchronize()
    assert (m2.cpu().numpy().astype(bool) == p2[:1000]).all()
    c2 = torch.full((1,), -1, dtype=torch.int64, device=dev)
    nz.verify_tuples_static(gset, qd, m2, None, c2)
    torch.cuda.synchronize()
    assert int(c2.item()) == int(p2[:1000].sum())
    nz.verify_tuples_static(gset, qd[:0], m2[:0], None, c2)
    torch.cuda.synchronize()
    assert int(c2.item()) == 0
    gset.close()


def test_static_verifier_refuses_sizes_beyond_its_array():
    dev = torch.device("cuda:0")
    gset = nz.build_itemset(np.zeros((1, 2), np.int32), [16, 16])

    class Fake:                                        # a query batch that is only a size
        shape = (nz.VERIFY_STATIC_MAX + 1, 2)

        @staticmethod
        def data_ptr():
            return 0x1000

    m = torch.empty(16, dtype=torch.uint8, device=dev)
    with pytest.raises(nz.NezhaError) as ei:
        nz.verify_tuples_static(gset, Fake, m)
    assert ei.value.code == -1 and "NEZHA_VERIFY_STATIC_MAX" in str(ei.value)
    gset.close()
