"""GPU parity of the code paths that only the full-size workloads take: resident workgroups that
walk the batch (more requests than workgroups, so every workgroup reuses its LDS and its list
scratch for a second and third request), the hand-back of flagged beams and requests to the
general kernels in the middle of such a batch, the multi-block scan of the stand-alone verifier
(more than 16384 blocks of queries), and the Large workload at its full batch in the launch form
the benchmark times, checked on sampled requests."""
import numpy as np
import pytest
import torch

import synth
import paper_2511_18793_amd as nz
from _gpu_common import (check_decode, device, planted_workload, to_device, tolerance)
from _parity import to_np

pytestmark = pytest.mark.gpu


def _per_request_config(B, e, K, V=1104, d=64, L=3):
    # bf16, K_in >= 16 and a codebook too large for the small-codebook kernels: levels 2.. take
    # the one-workgroup-per-request kernel (level 2 without a set: the whole-level form; level L
    # with the item set: per-beam lists + merge)
    return synth.StepConfig("walk", B=B, d=d, e=e, L=L, V=V, K=K, N=200_000, dtype="bf16",
                            catalog="uniform", w_std=0.05)


def _resident_groups():
    return min(2 * torch.cuda.get_device_properties(0).multi_processor_count, 1024)


@pytest.mark.parametrize("B,e,K", [
    (1100, 32, 17),      # two waves per workgroup, one MFMA step over the state
    (1040, 128, 20),     # the Large workload's state width (four MFMA steps)
    (600, 128, 70),      # five waves per workgroup; some workgroups take two requests, some one
])
def test_resident_workgroups_walk_the_batch(oracle, B, e, K):
    cfg = _per_request_config(B, e, K)
    assert cfg.B > _resident_groups()                 # at least one workgroup takes two requests
    x, cat = planted_workload(oracle, cfg, 23)
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    Wp = [nz.pack_weights(l + 1, cfg.L, cfg.radices, W[l], cfg.d) for l in range(cfg.L)]
    plan = nz.DecodePlan(H, Wp, E, cfg.radices, cfg.K, gset)
    first = [{k: v.clone() for k, v in o.items()} for o in plan.run()]
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, first, oset, tolerance(cfg))
    assert soft <= cfg.B // 50 + 8                     # beams swapped inside the score tolerance
    counts = to_np(first[-1]["count"])
    assert counts.max() <= cfg.K and 0.3 * cfg.K < counts.mean() < cfg.K
    # the same bits on every run: list places come from atomic counters, the order from sorts
    for _ in range(2):
        again = plan.run()
        torch.cuda.synchronize()
        for a, b in zip(first, again):
            for k in a:
                assert torch.equal(a[k], b[k]), k


def test_flagged_requests_inside_a_walked_batch(oracle):
    """Requests that the per-request kernel cannot finish (a logit spread of several hundred; many
    large logits crowded into few code groups) scattered over a batch larger than the number of
    resident workgroups: the workgroup that flags one goes on to its next request with clean
    counters, and the general kernels redo exactly the flagged ones."""
    cfg = _per_request_config(1040, 64, 24, V=2048)
    x, cat = planted_workload(oracle, cfg, 29, plant=False)
    groups = _resident_groups()
    spread = np.array([0, 3, groups - 1, groups, groups + 3, 2 * groups + 1, cfg.B - 1])
    spread = spread[spread < cfg.B]
    crowded = np.array([1, 7, groups + 1, groups + 7, cfg.B - 2])
    for lvl in (1, 2):                                  # levels 2 and 3
        x["H"][spread, lvl] = synth.round_to_bf16(x["H"][spread, lvl] * 400.0)
    # crowding: a constant input component lifts 480 codes, all in 30 of the 128 code groups;
    # only the crowded requests carry that component
    lifted = (np.arange(cfg.V) % 128) < 30
    for lvl in (1, 2):
        x["H"][:, lvl, 0] = 0.0
        x["H"][crowded, lvl, 0] = 1.0
        x["W"][lvl][0, :] = np.where(lifted, 30.0, 0.0).astype(np.float32)
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K, round_state_bf16=True)
    tuples = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(tuples, cfg.radices, 29)
    cat = synth.planted_catalog(cfg.radices, cat, tuples[keep], tuples[~keep], 29)
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    # logits of the order of 1000 from float32 sums of 64 products: a few 1e-3 of rounding
    soft = check_decode(oracle, nz, cfg, x, outs, oset, 4e-3)
    assert soft <= cfg.B // 50 + 8


def test_one_beam_far_ahead_of_the_others(oracle):
    """Requests whose first-level distribution is sharply peaked: the best beam's children take
    all K places of level 2, while the request's threshold is taken from 16 candidates per beam,
    most of them from the other beams.  The list of candidates at or above it overflows, and the
    kernel tightens the threshold from the listed candidates and sweeps again (also at level 3,
    where the same beams arrive with the same gaps).  Lists of more than 256 entries per beam at
    the verified level are covered by the crowded requests of the test above."""
    cfg = _per_request_config(300, 64, 24, V=2048)
    x, cat = planted_workload(oracle, cfg, 31, plant=False)
    peaked = np.array([0, 5, 17, 150, 299])
    x["H"][peaked, 0] = synth.round_to_bf16(x["H"][peaked, 0] * 400.0)
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K, round_state_bf16=True)
    gap = free[0]["score"][peaked, 0] - free[0]["score"][peaked, 1]
    assert (gap > 6.0).all()                            # the best first-level code is far ahead
    tuples = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(tuples, cfg.radices, 31)
    cat = synth.planted_catalog(cfg.radices, cat, tuples[keep], tuples[~keep], 31)
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, 4e-3)
    assert soft <= cfg.B // 50 + 8


def test_verifier_scan_over_more_than_16384_blocks():
    """17.3 million queries: the accepted positions of a block are offset by a scan over the block
    counts (above 16384 blocks of 1024 queries a kernel of its own).  Membership and therefore the
    whole ascending index list are known from how catalog and queries were generated."""
    radices = [4096, 4096, 4096]
    N = 2_000_000
    n = 16384 * 1024 + 517_123
    cat, pi = synth.uniform_catalog(radices, N, 5)
    gset = nz.build_itemset(cat, radices, 0.5)
    del cat
    q, present = synth.stress_queries(radices, N, pi, 5, n)
    qd = torch.from_numpy(q).to(device())
    del q
    mask, idx, cnt = nz.verify_tuples(gset, qd)
    torch.cuda.synchronize()
    c = int(cnt.item())
    assert c == int(present.sum())
    assert (to_np(mask).astype(bool) == present).all()
    assert (to_np(idx)[:c] == np.nonzero(present)[0]).all()
    gset.close()


def test_large_workload_full_batch_sampled_requests(oracle):
    """The Large workload as the benchmark launches it (B = 4096, d = 2048, T_l = 4096, K = 100,
    packed weights, one nezha_decode call): every resident workgroup takes eight requests.  The
    oracle checks sampled requests level by level (requests are independent, so a request's
    outputs depend on its own inputs only); the catalog has the full 5 * 10^7 items, planted from
    the oracle's unverified beams of the sampled requests."""
    cfg = synth.get_config("large")
    x = synth.draft_inputs(cfg, 42)
    groups = _resident_groups()
    sample = np.array([0, groups + 5, 3 * groups + 2, cfg.B - 1])
    xs = {"H": x["H"][sample], "W": x["W"], "E": x["E"]}
    free = oracle.decode(xs["H"], xs["W"], xs["E"], cfg.radices, cfg.K, round_state_bf16=True)
    tuples = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(tuples, cfg.radices, 42)
    background = synth.zipf_catalog(cfg.radices, cfg.N, 42, cfg.zipf_s)
    cat = synth.planted_catalog(cfg.radices, background, tuples[keep], tuples[~keep], 42)
    del background
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    assert gset.info()["n_distinct"] == cfg.N
    del cat
    H, W, E = to_device(x, cfg)
    Wp = [nz.pack_weights(l + 1, cfg.L, cfg.radices, W[l], cfg.d) for l in range(cfg.L)]
    del W
    plan = nz.DecodePlan(H, Wp, E, cfg.radices, cfg.K, gset)
    outs = plan.run()
    torch.cuda.synchronize()
    idx = torch.from_numpy(sample).to(device())
    outs_s = [{k: v[idx] for k, v in o.items()} for o in outs]
    soft = check_decode(oracle, nz, cfg.scaled(B=len(sample)), xs, outs_s, oset, tolerance(cfg))
    assert soft <= 8
    assert int(outs_s[-1]["count"].sum()) > 0
    # structure of every request's answer (holds at any size): counts in range, scores
    # non-increasing, keys distinct, padding beyond the count, every emitted key in the catalog
    cnt = to_np(outs[-1]["count"])
    keys = to_np(outs[-1]["key"]).view(np.uint64)
    score = to_np(outs[-1]["score"])
    assert cnt.min() >= 0 and cnt.max() <= cfg.K
    live = np.arange(cfg.K)[None, :] < cnt[:, None]
    assert (keys[~live] == np.uint64(2**64 - 1)).all() and np.isneginf(score[~live]).all()
    assert oset.contains_keys(keys[live]).all()
    for b in range(0, cfg.B, 61):
        n = int(cnt[b])
        assert (np.diff(score[b, :n]) <= 0).all() and len(set(keys[b, :n].tolist())) == n
    # levels below the last keep K distinct beams per request
    for o in outs[:-1]:
        assert (to_np(o["count"]) == cfg.K).all()
        kk = to_np(o["key"]).view(np.uint64)
        assert all(len(set(kk[b].tolist())) == cfg.K for b in range(0, cfg.B, 61))
    # a second run gives the same bits
    first = [{k: v.clone() for k, v in o.items()} for o in outs]
    again = plan.run()
    torch.cuda.synchronize()
    for a, b in zip(first, again):
        for k in a:
            assert torch.equal(a[k], b[k]), k
