"""GPU parity of beams wider than 128 (the recall setting: beam 512 to 1000) against the CPU
oracle, level by level on identical inputs, through the same C-ABI calls as every other shape."""
import numpy as np
import pytest
import torch

import synth
import paper_2511_18793_amd as nz
from _gpu_common import (check_decode, device, planted_workload, to_device, tolerance, torch_dtype)
from _parity import to_np

pytestmark = pytest.mark.gpu


def _run(oracle, cfg, seed, N, verify=True, **kw):
    x, cat = planted_workload(oracle, cfg, seed, N)
    oset = oracle.ItemSet(cat, cfg.radices) if verify else None
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor) if verify else None
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset, **kw)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, tolerance(cfg))
    return outs, soft


@pytest.mark.parametrize("B,d,e,V,K,L,dtype", [
    (3, 64, 128, 1024, 512, 3, "bf16"),     # beam 512: every beam is cut to 512 of 1024 codes, then probed
    (2, 64, 64, 1024, 1000, 2, "bf16"),     # beam 1000
    (2, 32, 32, 256, 256, 3, "bf16"),       # beam = codebook: no per-beam cut, all 65536 candidates probed
    (2, 64, 96, 2048, 130, 2, "bf16"),      # state width that is not a power of two; just above 128
    (2, 24, 12, 320, 200, 3, "f32"),        # float32 path
    (5, 64, 128, 4096, 129, 2, "bf16"),     # large codebook
    (2, 64, 64, 8192, 140, 2, "bf16"),      # a codebook too large for a beam's logits to stay in registers
    (256, 32, 32, 256, 130, 3, "bf16"),     # a batch large enough for one workgroup per request
    (1, 32, 32, 1024, 1024, 2, "bf16"),     # the widest beam there is (= the codebook: no per-beam cut)
    (1, 32, 64, 2048, 1024, 2, "f32"),      # the widest beam, cut from 2048 codes, float32
])
def test_wide_beam_shapes(oracle, B, d, e, V, K, L, dtype):
    cfg = synth.StepConfig("widebeam", B=B, d=d, e=e, L=L, V=V, K=K, N=min(V ** L // 4, 200_000),
                           dtype=dtype, catalog="uniform", w_std=0.05)
    outs, soft = _run(oracle, cfg, 23, cfg.N)
    assert soft <= 16
    counts = to_np(outs[-1]["count"])
    assert counts.max() > 128               # more survivors than the narrow kernels can hold


def test_recall_config_request_subsample(oracle):
    cfg = synth.get_config("recall").scaled(B=2)
    outs, soft = _run(oracle, cfg, 42, 200_000)
    assert soft <= 16
    assert to_np(outs[-1]["count"]).min() > 128


def test_wide_beam_without_verification_keeps_k_beams(oracle):
    cfg = synth.StepConfig("widebeam", B=3, d=64, e=64, L=3, V=512, K=400, N=1000, dtype="bf16",
                           catalog="uniform", w_std=0.05)
    outs, soft = _run(oracle, cfg, 24, cfg.N, verify=False)
    assert soft <= 16
    assert (to_np(outs[-1]["count"]) == cfg.K).all()


@pytest.mark.parametrize("dtype,B", [("bf16", 2), ("f32", 2), ("bf16", 256)])
def test_wide_beam_zero_weights_follow_the_tie_rule(oracle, dtype, B):
    """All logits equal: every selection is decided by the tie rule alone (lower parent, then
    lower code), both in the per-beam cut and in the request's K best; the lists that would hold
    everything at or above the bound overflow, so the exact radix selection runs."""
    cfg = synth.StepConfig("ties", B=B, d=32, e=32, L=3, V=256, K=200, N=1, dtype=dtype,
                           catalog="uniform")
    x = synth.draft_inputs(cfg, 3)
    x["W"] = [np.zeros_like(w) for w in x["W"]]
    V, K = cfg.V, cfg.K
    # every tuple (t1, t2, t3) with t3 even is an item
    t = np.array([(a, b, c) for a in range(2) for b in range(V) for c in range(0, V, 2)], dtype=np.int32)
    oset = oracle.ItemSet(t, cfg.radices)
    gset = nz.build_itemset(t, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, K, gset)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, tolerance(cfg))
    assert soft == 0
    o1, o2, o3 = (dict((k, to_np(v)) for k, v in o.items() if k != "state") for o in outs)
    assert (o1["code"] == np.arange(K)).all()
    assert (o2["parent"] == 0).all() and (o2["code"] == np.arange(K)).all()
    # level 3: parent 0 = (0, 0): its K lowest codes are candidates, the even ones are items
    assert (o3["parent"][:, :100] == 0).all() and (o3["code"][:, :100] == np.arange(0, K, 2)).all()
    assert (o3["parent"][:, 100:] == 1).all() and (o3["code"][:, 100:] == np.arange(0, K, 2)).all()


def test_wide_beam_recurrent_transition_and_prefix_sets(oracle):
    cfg = synth.StepConfig("widebeam", B=2, d=64, e=64, L=3, V=512, K=300, N=60_000, dtype="bf16",
                           catalog="uniform", w_std=0.05)
    seed = 29
    x = synth.draft_inputs(cfg, seed)
    x["E"] = [synth.round_to_bf16(em * 25.0) for em in x["E"]]
    rng = np.random.default_rng(seed)
    U = [synth.round_to_bf16((rng.standard_normal((cfg.e, cfg.e)) / np.sqrt(cfg.e)).astype(np.float32))
         for _ in range(cfg.L - 1)]
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K, round_state_bf16=True, U=U)
    tuples = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(tuples, cfg.radices, seed)
    cat = synth.planted_catalog(cfg.radices, synth.uniform_catalog(cfg.radices, cfg.N, seed)[0],
                                tuples[keep], tuples[~keep], seed)
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    opre, gpre = [], []
    for l in range(1, cfg.L):
        pre = np.unique(cat[:, :l], axis=0)
        opre.append(oracle.ItemSet(pre, cfg.radices[:l]))
        gpre.append(nz.build_itemset(pre, cfg.radices[:l], cfg.load_factor))
    H, W, E = to_device(x, cfg)
    Ud = [torch.from_numpy(u).to(device()).to(torch.bfloat16) for u in U]
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset, U=Ud, prefix_sets=gpre)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, tolerance(cfg), U=U, prefix_sets=opre)
    assert soft <= 16
    assert int(outs[-1]["count"].sum()) > 0


def test_wide_beam_with_empty_beam_slots(oracle):
    """A catalog with few first-level codes and prefix sets: level 1 keeps fewer than K beams, so
    levels 2 and 3 see empty slots (index 2^64-1, score -inf) among their parents."""
    cfg = synth.StepConfig("widebeam", B=3, d=64, e=64, L=3, V=512, K=200, N=40_000, dtype="bf16",
                           catalog="uniform", w_std=0.05)
    x, cat = planted_workload(oracle, cfg, 31, cfg.N)
    first = np.unique(cat[:, 0])
    cat = cat[np.isin(cat[:, 0], first[:150])]
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    opre, gpre = [], []
    for l in range(1, cfg.L):
        pre = np.unique(cat[:, :l], axis=0)
        opre.append(oracle.ItemSet(pre, cfg.radices[:l]))
        gpre.append(nz.build_itemset(pre, cfg.radices[:l], cfg.load_factor))
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset, prefix_sets=gpre)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, tolerance(cfg), prefix_sets=opre)
    assert soft <= 16
    c1 = to_np(outs[0]["count"])                        # of a beam's 200 best codes only the valid stay
    assert c1.max() < cfg.K and c1.min() > 0
    assert int(outs[-1]["count"].sum()) > 0


def test_wide_beam_limits():
    cfg = synth.StepConfig("widebeam", B=1, d=32, e=32, L=2, V=2048, K=1025, N=1, dtype="bf16",
                           catalog="uniform")
    x = synth.draft_inputs(cfg, 1)
    H, W, E = to_device(x, cfg)
    with pytest.raises(nz.NezhaError):
        nz.draft_step(1, cfg.L, cfg.radices, 1025, H[:, 0], W[0], E[0])
