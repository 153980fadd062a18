"""GPU parity of nezha_draft_step against the CPU oracle, level by level on identical inputs."""
import numpy as np
import pytest
import torch

import synth
import paper_2511_18793_amd as nz
from _gpu_common import (check_decode, device, outputs_to_numpy, planted_workload, to_device,
                         tolerance, torch_dtype)
from _parity import to_np

pytestmark = pytest.mark.gpu


def run_config(oracle, cfg, seed, N=None, plant=True, verify=True):
    x, cat = planted_workload(oracle, cfg, seed, N, plant)
    oset = oracle.ItemSet(cat, cfg.radices) if verify else None
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor) if verify else None
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, tolerance(cfg))
    return outs, soft


def test_tiny_config(oracle):
    cfg = synth.get_config("tiny")
    for seed in (42, 43, 44):
        outs, soft = run_config(oracle, cfg, seed)
        assert soft == 0
        assert int(outs[-1]["count"].sum()) > 0


def test_tiny_config_unplanted_catalog_gives_short_or_empty_results(oracle):
    cfg = synth.get_config("tiny")
    outs, _ = run_config(oracle, cfg, 42, plant=False)
    assert int(outs[-1]["count"].min()) < cfg.K


def test_serving_config_full_size(oracle):
    cfg = synth.get_config("serving")
    outs, soft = run_config(oracle, cfg, 42)
    assert soft <= 8                       # beams swapped inside the score tolerance
    counts = to_np(outs[-1]["count"])
    assert counts.max() == cfg.K and counts.mean() > 0.5 * cfg.K


def test_no_verification_keeps_k_beams(oracle):
    cfg = synth.get_config("serving").scaled(B=16)
    outs, _ = run_config(oracle, cfg, 43, verify=False)
    assert (to_np(outs[-1]["count"]) == cfg.K).all()


@pytest.mark.parametrize("name", ["paper_yelp", "paper_games"])
def test_paper_public_shape(oracle, name):
    cfg = synth.get_config(name).scaled(B=24)
    run_config(oracle, cfg, 44)


def test_wide_config_request_subsample(oracle):
    # full d, V, K and L = 4 of the wide shape on 12 requests; catalog cut to 10^6 items
    cfg = synth.get_config("wide").scaled(B=12)
    run_config(oracle, cfg, 42, N=1_000_000)


def test_large_config_request_subsample(oracle):
    # full d = 2048, V = 4096, K = 100 of the large shape on 3 requests
    cfg = synth.get_config("large").scaled(B=3)
    run_config(oracle, cfg, 42, N=1_000_000)


@pytest.mark.parametrize("B,d,e,V,K,L,dtype", [
    (5, 64, 32, 48, 7, 3, "bf16"),        # partial last block of codes, ragged rows
    (3, 3, 4, 16, 16, 2, "f32"),          # K = V: every code is taken
    (2, 64, 32, 128, 1, 3, "bf16"),       # K = 1: greedy
    (2, 64, 64, 256, 128, 2, "bf16"),     # the largest beam
    (17, 96, 96, 80, 33, 3, "f32"),       # 256-entry buffers in float32
    (33, 64, 256, 64, 5, 4, "bf16"),      # widest state
])
def test_odd_shapes(oracle, B, d, e, V, K, L, dtype):
    cfg = synth.StepConfig("odd", B=B, d=d, e=e, L=L, V=V, K=K, N=min(V ** L // 4, 100_000),
                           dtype=dtype, catalog="uniform", w_std=0.05)
    run_config(oracle, cfg, 7)


def test_zero_weights_follow_the_tie_rule(oracle):
    cfg = synth.StepConfig("ties", B=3, d=64, e=32, L=3, V=64, K=6, N=1000, dtype="bf16",
                           catalog="uniform")
    x = synth.draft_inputs(cfg, 1)
    x["W"] = [np.zeros_like(w) for w in x["W"]]
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, None)
    torch.cuda.synchronize()
    for l, o in enumerate(outs):
        g = outputs_to_numpy(o)
        assert (g["code"] == np.arange(cfg.K)).all() and (g["parent"] == 0).all()
        assert np.allclose(g["score"], -(l + 1) * np.log(64), atol=1e-5)
    want = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K, round_state_bf16=True)
    assert (want[-1]["key"] == to_np(outs[-1]["key"]).view(np.uint64)).all()


def test_zero_weights_with_a_large_codebook(oracle):
    """All 2048 logits of every row tie: the bound of the two-sweep kernel lets every code
    through, the lists overflow and the streaming fallback has to give codes 0..K-1."""
    cfg = synth.StepConfig("ties_large", B=2, d=64, e=32, L=2, V=2048, K=100, N=1000,
                           dtype="bf16", catalog="uniform")
    x = synth.draft_inputs(cfg, 1)
    x["W"] = [np.zeros_like(w) for w in x["W"]]
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, None)
    torch.cuda.synchronize()
    for l, o in enumerate(outs):
        g = outputs_to_numpy(o)
        assert (g["code"] == np.arange(cfg.K)).all() and (g["parent"] == 0).all()
        assert np.allclose(g["score"], -(l + 1) * np.log(2048), atol=1e-5)


def test_large_codebook_odd_sizes(oracle):
    # T_l not a multiple of the chunk of 256 codes, K between 65 and 128, ragged rows
    cfg = synth.StepConfig("odd_large", B=3, d=64, e=64, L=2, V=1104, K=70, N=50_000,
                           dtype="bf16", catalog="uniform", w_std=0.05)
    run_config(oracle, cfg, 11)


def test_results_are_deterministic(oracle):
    cfg = synth.get_config("serving").scaled(B=64)
    x, cat = planted_workload(oracle, cfg, 42, N=200_000)
    gset = nz.build_itemset(cat, cfg.radices)
    H, W, E = to_device(x, cfg)
    first = [{k: v.clone() for k, v in o.items()} for o in nz.decode(H, W, E, cfg.radices, cfg.K, gset)]
    for _ in range(2):
        again = nz.decode(H, W, E, cfg.radices, cfg.K, gset)
        torch.cuda.synchronize()
        for a, b in zip(first, again):
            for k in a:
                assert torch.equal(a[k], b[k]), k


def test_decode_replays_correctly_from_a_hip_graph(oracle):
    cfg = synth.get_config("serving").scaled(B=32)
    x, cat = planted_workload(oracle, cfg, 43, N=200_000)
    gset = nz.build_itemset(cat, cfg.radices)
    H, W, E = to_device(x, cfg)
    bufs = nz.DraftBuffers(cfg.B, cfg.L, cfg.K, cfg.d, cfg.e, cfg.radices, torch_dtype(cfg), device())
    eager = [{k: v.clone() for k, v in o.items()}
             for o in nz.decode(H, W, E, cfg.radices, cfg.K, gset, buffers=bufs)]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        nz.decode(H, W, E, cfg.radices, cfg.K, gset, buffers=bufs)
    for rep in range(3):
        for o in bufs.outs:
            for v in o.values():
                v.zero_()
        junk = torch.randn(256, 256, device=device()) @ torch.randn(256, 256, device=device())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, bufs.outs):
            for k in a:
                assert torch.equal(a[k], b[k]), (rep, k)
        del junk


def test_weights_packed_once_give_identical_results(oracle):
    cfg = synth.get_config("serving").scaled(B=48)
    x, cat = planted_workload(oracle, cfg, 44, N=100_000)
    gset = nz.build_itemset(cat, cfg.radices)
    H, W, E = to_device(x, cfg)
    ref = [{k: v.clone() for k, v in o.items()} for o in nz.decode(H, W, E, cfg.radices, cfg.K, gset)]
    Wp = [nz.pack_weights(l + 1, cfg.L, cfg.radices, W[l], cfg.d) for l in range(cfg.L)]
    got = nz.decode(H, Wp, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    for a, b in zip(ref, got):
        for k in a:
            assert torch.equal(a[k], b[k]), k


def test_user_projection_is_the_level_one_logits(oracle):
    """A_l = H_l W_l[0:d]: the logits of Eq. 2 at zero state, against a float64 product."""
    for name, tol in (("tiny", 1e-5), ("serving", 2e-2)):
        cfg = synth.get_config(name).scaled(B=37)
        x = synth.draft_inputs(cfg, 42)
        H, W, E = to_device(x, cfg)
        A = nz.user_projection(1, cfg.L, cfg.radices, H[:, 0, :], W[0], h_row_stride=H.stride(0))
        torch.cuda.synchronize()
        want = x["H"][:, 0].astype(np.float64) @ x["W"][0][:cfg.d].astype(np.float64)
        err = np.abs(to_np(A) - want).max()
        assert err < min(tol, 1e-4), (name, err)


@pytest.mark.parametrize("B,d,V", [
    (2100, 96, 4112),     # 256 x 256 tiles (both operands through LDS), ragged in rows and columns, a k loop shorter than the pipeline
    (2304, 1024, 3840),   # the same tiles, a long k loop
    (700, 256, 2000),     # 32 x 64 tiles with the k loop in four parts, ragged
    (1500, 160, 4000),    # 128 x 128 tiles
])
def test_user_projection_tile_forms(B, d, V):
    """Every tile form of the bf16 user-part product against the float64 product of the same
    (bf16-rounded) inputs: float32 accumulation of d products of magnitude <= ~0.1."""
    rng = np.random.default_rng(B + d + V)
    Hn = synth.round_to_bf16(rng.standard_normal((B, d)).astype(np.float32))
    Wn = synth.round_to_bf16((rng.standard_normal((d + 32, V)) * 0.02).astype(np.float32))
    H = torch.from_numpy(Hn).to(device()).to(torch.bfloat16)
    W = torch.from_numpy(Wn).to(device()).to(torch.bfloat16)
    A = nz.user_projection(1, 2, [V, V], H, W)
    torch.cuda.synchronize()
    want = (torch.from_numpy(Hn).double() @ torch.from_numpy(Wn[:d]).double()).numpy()
    err = np.abs(to_np(A) - want).max()
    assert err < 1e-4, err


def test_zero_requests_is_a_no_op():
    dev = device()
    H = torch.zeros((0, 64), dtype=torch.bfloat16, device=dev)
    W = torch.zeros((96, 64), dtype=torch.bfloat16, device=dev)
    E = torch.zeros((64, 32), dtype=torch.bfloat16, device=dev)
    o = nz.draft_step(1, 2, [64, 64], 4, H, W, E, h_row_stride=64)
    torch.cuda.synchronize()
    assert o["key"].shape == (0, 4)


# ---- recurrent Transition (c' = tanh(U c + e_l)) ------------------------------------------------
def _rnn_inputs(cfg, seed):
    """U_l with entries of order 1/sqrt(e) and code embeddings scaled up so that tanh bends:
    values rounded to the working type, as float32 numpy (for the oracle)."""
    rng = np.random.default_rng(seed + 1000)
    U = [(rng.standard_normal((cfg.e, cfg.e)) / np.sqrt(cfg.e)).astype(np.float32)
         for _ in range(cfg.L - 1)]
    if cfg.dtype == "bf16":
        U = [synth.round_to_bf16(u) for u in U]
    return U


@pytest.mark.parametrize("name,B", [("tiny", 64), ("serving", 64), ("wide", 6), ("large", 2)])
def test_recurrent_transition(oracle, name, B):
    cfg = synth.get_config(name).scaled(B=B)
    seed = 61
    x = synth.draft_inputs(cfg, seed)
    scale = 25.0                                   # code embeddings of order 0.5: tanh is not linear there
    x["E"] = [synth.round_to_bf16(em * scale) if cfg.dtype == "bf16" else (em * scale).astype(np.float32)
              for em in x["E"]]
    U = _rnn_inputs(cfg, seed)
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K,
                         round_state_bf16=cfg.dtype == "bf16", U=U)
    tuples = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(tuples, cfg.radices, seed)
    cat = synth.planted_catalog(cfg.radices, synth.uniform_catalog(cfg.radices, 20000, seed)[0],
                                tuples[keep], tuples[~keep], seed)
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    Ud = [torch.from_numpy(u).to(device()).to(torch_dtype(cfg)) for u in U]
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset, U=Ud)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, tolerance(cfg), U=U)
    assert soft <= 8
    assert int(outs[-1]["count"].sum()) > 0
    # the cell changes the answer: the additive Transition on the same inputs gives other beams
    plain = nz.decode(H, W, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    assert not torch.equal(plain[-1]["key"], outs[-1]["key"])


def test_recurrent_transition_needs_its_matrix():
    cfg = synth.get_config("serving").scaled(B=2)
    x = synth.draft_inputs(cfg, 1)
    H, W, E = to_device(x, cfg)
    U = torch.zeros((cfg.e, cfg.e), dtype=torch.bfloat16, device=device())
    with pytest.raises(nz.NezhaError):
        # misaligned matrix (offset by one element)
        nz.draft_step(1, cfg.L, cfg.radices, cfg.K, H[:, 0], W[0], E[0],
                      U_l=torch.zeros(cfg.e * cfg.e + 8, dtype=torch.bfloat16, device=device())[1:1 + cfg.e * cfg.e].view(cfg.e, cfg.e))
    out = nz.draft_step(1, cfg.L, cfg.radices, cfg.K, H[:, 0], W[0], E[0], U_l=U)
    torch.cuda.synchronize()
    # zero U and zero initial state: c' = tanh(E[code])
    want = torch.tanh(E[0].float()[out["code"].long()]).to(torch.bfloat16)
    assert torch.equal(out["state"], want)


# ---- verification below the last level against sets of valid prefixes ---------------------------
@pytest.mark.parametrize("name,B", [("tiny", 64), ("serving", 64), ("wide", 6), ("large", 2)])
def test_prefix_verification(oracle, name, B):
    cfg = synth.get_config(name).scaled(B=B)
    seed = 71
    x, cat = planted_workload(oracle, cfg, seed, N=20000)
    # a catalog whose first-level codes are few, so that level 1 already loses beams
    first = np.unique(cat[:, 0])
    cat = cat[np.isin(cat[:, 0], first[: max(2, len(first) // 8)])]
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
    assert soft <= 8
    c1 = to_np(outs[0]["count"])
    assert c1.min() < cfg.K                        # empty beam slots did enter level 2
    # every beam of every level is a prefix of an item
    for l in range(1, cfg.L + 1):
        n = to_np(outs[l - 1]["count"])
        keys = to_np(outs[l - 1]["key"]).view(np.uint64)
        live = np.concatenate([keys[b, :n[b]] for b in range(cfg.B)])
        ref = oset if l == cfg.L else opre[l - 1]
        assert ref.contains_keys(live).all()
    # a set of the wrong length is refused
    if cfg.L >= 3:
        with pytest.raises(nz.NezhaError):
            nz.draft_step(1, cfg.L, cfg.radices, cfg.K, H[:, 0], W[0], E[0], itemset=gpre[1])


# ---- the head without its autoregressive state (ablation / parallel multi-token heads) ----------
@pytest.mark.parametrize("name,B,shared_hidden", [("serving", 32, False), ("serving", 32, True),
                                                  ("wide", 4, False), ("tiny", 16, True)])
def test_head_without_state(oracle, name, B, shared_hidden):
    cfg = synth.get_config(name).scaled(B=B)
    x, cat = planted_workload(oracle, cfg, 81, N=20000, plant=False)
    if shared_hidden:                               # one hidden state for all levels
        x["H"] = np.repeat(x["H"][:, :1], cfg.L, axis=1).copy()
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K, use_state=False,
                         round_state_bf16=cfg.dtype == "bf16")
    tuples = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(tuples, cfg.radices, 81)
    cat = synth.planted_catalog(cfg.radices, cat, tuples[keep], tuples[~keep], 81)
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset, use_state=False)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, tolerance(cfg), use_state=False)
    assert soft <= 8
    assert int(outs[-1]["count"].sum()) > 0
    # without a state every beam of a request sees the same distribution: all parents of a
    # level pick the same K codes
    lvl2 = outputs_to_numpy(outs[1])
    with_state = nz.decode(H, W, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    assert not torch.equal(with_state[-1]["key"], outs[-1]["key"])
    assert lvl2["count"].min() > 0


@pytest.mark.parametrize("name,B", [("serving", 48), ("wide", 4), ("large", 2), ("tiny", 16)])
def test_head_without_placeholder_hidden_states(oracle, name, B):
    """Ablation "without h_l": one hidden vector (h_1) serves every level, the autoregressive
    state is kept.  A caller-side combination of the same kernels: every H_l is the same [B, d]
    view (the row stride of H lets one tensor serve all levels)."""
    cfg = synth.get_config(name).scaled(B=B)
    x, cat = planted_workload(oracle, cfg, 83, N=20000, plant=False)
    x["H"] = np.repeat(x["H"][:, :1], cfg.L, axis=1).copy()
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K,
                         round_state_bf16=cfg.dtype == "bf16")
    tuples = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(tuples, cfg.radices, 83)
    cat = synth.planted_catalog(cfg.radices, cat, tuples[keep], tuples[~keep], 83)
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    # the device tensor holds h_1 only: [B, 1, d] expanded over the levels without a copy
    H1 = H[:, :1, :].contiguous().expand(cfg.B, cfg.L, cfg.d)
    outs = nz.decode(H1, W, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    soft = check_decode(oracle, nz, cfg, x, outs, oset, tolerance(cfg))
    assert soft <= 8
    assert int(outs[-1]["count"].sum()) > 0
    full = synth.draft_inputs(cfg, 83)
    Hf = torch.from_numpy(full["H"]).to(device()).to(torch_dtype(cfg))
    with_h = nz.decode(Hf, W, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    assert not torch.equal(with_h[-1]["key"], outs[-1]["key"])


def test_initial_state_of_level_one(oracle):
    """Eq. 1: the head may start from a given context state instead of zeros.  nezha_draft_step
    takes it as state_in at level 1; nezha_draft_levels / nezha_decode through desc.state_init:
    same bits, and parity with the oracle fed the same state."""
    for name, B in (("serving", 40), ("large", 2), ("tiny", 8)):
        cfg = synth.get_config(name).scaled(B=B)
        x, cat = planted_workload(oracle, cfg, 85, N=20000, plant=False)
        rng = np.random.default_rng(85)
        s0 = (rng.standard_normal((cfg.B, 1, cfg.e)) * 0.5).astype(np.float32)
        if cfg.dtype == "bf16":
            s0 = synth.round_to_bf16(s0)
        H, W, E = to_device(x, cfg)
        S0 = torch.from_numpy(s0).to(device()).to(torch_dtype(cfg))
        # level by level through nezha_draft_step
        outs = nz.decode(H, W, E, cfg.radices, cfg.K, None, state_init=S0)
        torch.cuda.synchronize()
        g1 = outputs_to_numpy(outs[0])
        o1 = oracle.draft_level(1, cfg.L, cfg.radices, cfg.K, x["H"][:, 0], x["W"][0], x["E"][0],
                                s0, None, None, None, round_state_bf16=cfg.dtype == "bf16")
        zero = oracle.draft_level(1, cfg.L, cfg.radices, cfg.K, x["H"][:, 0], x["W"][0], x["E"][0],
                                  None, None, None, None, round_state_bf16=cfg.dtype == "bf16")
        assert (o1["code"] != zero["code"]).any()           # the state changes the answer
        same = (o1["code"] == g1["code"]).all(axis=1)
        assert same.mean() > 0.9
        assert np.abs(o1["score"][same] - g1["score"][same]).max() <= tolerance(cfg)
        assert (o1["state"][same] == g1["state"][same]).all()
        if cfg.dtype != "bf16":
            continue
        # all levels in one call (one launch at the serving shape): the same bits
        Wp = [nz.pack_weights(l + 1, cfg.L, cfg.radices, W[l], cfg.d) for l in range(cfg.L)]
        first = [{k: v.clone() for k, v in o.items()}
                 for o in nz.decode(H, Wp, E, cfg.radices, cfg.K, None, state_init=S0)]
        plan = nz.DecodePlan(H, Wp, E, cfg.radices, cfg.K, None, state_init=S0)
        got = plan.run()
        torch.cuda.synchronize()
        for a, b, c in zip(outs, first, got):
            for k in a:
                assert torch.equal(a[k], b[k]) and torch.equal(a[k], c[k]), k


# ---- all levels in one call ---------------------------------------------------------------------
@pytest.mark.parametrize("name,B,variant", [("serving", 256, "plain"), ("serving", 40, "rnn"),
                                            ("serving", 40, "prefix"), ("paper_yelp", 64, "plain"),
                                            ("wide", 8, "plain")])
def test_draft_levels_equals_the_level_loop(oracle, name, B, variant):
    """nezha_draft_levels (one launch for all levels where the shapes allow) against L calls of
    nezha_draft_step on the same inputs: identical outputs, and parity with the oracle."""
    cfg = synth.get_config(name).scaled(B=B)
    x, cat = planted_workload(oracle, cfg, 91, N=20000)
    if variant == "prefix":
        first = np.unique(cat[:, 0])
        cat = cat[np.isin(cat[:, 0], first[: max(2, len(first) // 8)])]
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    U = Ud = opre = gpre = None
    if variant == "rnn":
        U = _rnn_inputs(cfg, 91)
        Ud = [torch.from_numpy(u).to(device()).to(torch_dtype(cfg)) for u in U]
    if variant == "prefix":
        opre, gpre = [], []
        for l in range(1, cfg.L):
            pre = np.unique(cat[:, :l], axis=0)
            opre.append(oracle.ItemSet(pre, cfg.radices[:l]))
            gpre.append(nz.build_itemset(pre, cfg.radices[:l], cfg.load_factor))
    Wp = [nz.pack_weights(l + 1, cfg.L, cfg.radices, W[l], cfg.d) for l in range(cfg.L)]
    b1 = nz.DraftBuffers(cfg.B, cfg.L, cfg.K, cfg.d, cfg.e, cfg.radices, H.dtype, H.device)
    b2 = nz.DraftBuffers(cfg.B, cfg.L, cfg.K, cfg.d, cfg.e, cfg.radices, H.dtype, H.device)
    parts = nz.user_projection_levels(H, Wp, cfg.radices, b1.user_parts)
    one = nz.draft_levels(H, Wp, E, cfg.radices, cfg.K, gset, b1, U=Ud, prefix_sets=gpre,
                          user_parts=parts)
    torch.cuda.synchronize()
    state = key = score = None
    for level in range(1, cfg.L + 1):
        s = gset if level == cfg.L else (gpre[level - 1] if gpre else None)
        o = nz.draft_step(level, cfg.L, cfg.radices, cfg.K, H[:, level - 1, :], Wp[level - 1],
                          E[level - 1] if level < cfg.L else None, state, key, score, s,
                          out=b2.outs[level - 1], workspace=b2.workspace,
                          h_row_stride=H.stride(0), user_part=parts[level - 1],
                          U_l=Ud[level - 1] if (Ud and level < cfg.L) else None)
        state, key, score = o.get("state"), o["key"], o["score"]
    torch.cuda.synchronize()
    for l in range(cfg.L):
        for k in b2.outs[l]:
            assert torch.equal(one[l][k], b2.outs[l][k]), (l, k)
    soft = check_decode(oracle, nz, cfg, x, one, oset, tolerance(cfg), U=U, prefix_sets=opre)
    assert soft <= 8
    # without the user parts the call falls back to the level loop and still agrees
    b3 = nz.DraftBuffers(cfg.B, cfg.L, cfg.K, cfg.d, cfg.e, cfg.radices, H.dtype, H.device)
    loop = nz.draft_levels(H, Wp, E, cfg.radices, cfg.K, gset, b3, U=Ud, prefix_sets=gpre)
    torch.cuda.synchronize()
    for l in range(cfg.L):
        for k in ("key", "score", "parent", "code", "count"):
            assert torch.equal(loop[l][k], one[l][k]), (l, k)


# ---- the one-workgroup-per-request expansion (bf16, K_in >= 16, large codebooks) -----------------
@pytest.mark.parametrize("B,d,e,V,K,L", [
    (3, 64, 32, 1104, 70, 2),      # one MFMA step over the state, ragged last chunk
    (2, 64, 64, 2048, 17, 3),      # the smallest beam that takes this path (two waves, one nearly empty)
    (2, 64, 256, 1536, 100, 2),    # widest state
    (2, 128, 128, 4096, 128, 2),   # the largest beam, eight full waves
    (5, 64, 128, 80, 70, 2),       # fewer codes than one chunk: most code groups are empty
    (1, 32, 32, 32768, 16, 2),     # the largest codebook this kernel takes (16-bit list counts)
    (1, 32, 32, 32784, 16, 2),     # one tile more: the general kernel takes the level
])
def test_request_kernel_shapes(oracle, B, d, e, V, K, L):
    cfg = synth.StepConfig("req", B=B, d=d, e=e, L=L, V=V, K=K, N=min(V ** L // 4, 50_000),
                           dtype="bf16", catalog="uniform", w_std=0.05)
    outs, soft = run_config(oracle, cfg, 13)
    assert soft <= 8


def test_request_kernel_hands_hard_rows_to_the_general_kernel(oracle):
    """Logits with a spread of several hundred (a lane's first logit can lie far below the rest,
    so the fixed reference of the sum of exponentials is unusable) and logits crowded into one
    code group (the group-maxima bound lets too many through): both must end in the flagged
    beams being redone, with the same results as everywhere else."""
    cfg = synth.StepConfig("hard", B=4, d=64, e=64, L=2, V=2048, K=40, N=50_000, dtype="bf16",
                           catalog="uniform", w_std=0.05)
    x, cat = planted_workload(oracle, cfg, 17, plant=False)
    # (1) requests 0, 1: huge spread (the hidden state of level 2 scaled up)
    x["H"][:2, 1] = synth.round_to_bf16(x["H"][:2, 1] * 400.0)
    # (2) requests 2, 3: 480 codes lifted far above the rest, all of them in 30 of the 128 code
    #     groups (a code's group is its value modulo 128), through a constant input component
    x["H"][2:, 1, 0] = 1.0
    lifted = (np.arange(cfg.V) % 128) < 30
    x["W"][1][0, :] = np.where(lifted, 30.0, 0.0).astype(np.float32)
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K, round_state_bf16=True)
    tuples = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(tuples, cfg.radices, 17)
    cat = synth.planted_catalog(cfg.radices, cat, tuples[keep], tuples[~keep], 17)
    oset = oracle.ItemSet(cat, cfg.radices)
    gset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    H, W, E = to_device(x, cfg)
    outs = nz.decode(H, W, E, cfg.radices, cfg.K, gset)
    torch.cuda.synchronize()
    # logits of the order of 1000 formed by float32 sums of 64 products: a few 1e-3 of rounding
    # (the bf16 allowance is 2e-2)
    soft = check_decode(oracle, nz, cfg, x, outs, oset, 4e-3)
    assert soft <= 8


@pytest.mark.parametrize("name,B,variant", [("serving", 64, "plain"), ("serving", 24, "rnn"),
                                            ("wide", 5, "prefix"), ("large", 2, "plain")])
def test_decode_in_one_call_equals_the_level_loop(oracle, name, B, variant):
    """nezha_decode (projections of all levels + the level loop in one host call, arguments
    marshalled once) against L calls of nezha_draft_step: the same bits, also on a second run."""
    cfg = synth.get_config(name).scaled(B=B)
    x, cat = planted_workload(oracle, cfg, 45, N=50_000)
    gset = nz.build_itemset(cat, cfg.radices)
    H, W, E = to_device(x, cfg)
    U = gpre = None
    if variant == "rnn":
        U = [torch.from_numpy(u).to(device()).to(torch_dtype(cfg)) for u in _rnn_inputs(cfg, 45)]
    if variant == "prefix":
        gpre = [nz.build_itemset(np.unique(cat[:, :l], axis=0), cfg.radices[:l], cfg.load_factor)
                for l in range(1, cfg.L)]
    Wp = [nz.pack_weights(l + 1, cfg.L, cfg.radices, W[l], cfg.d) for l in range(cfg.L)]
    ref = []
    state = key = score = None
    for l in range(1, cfg.L + 1):
        o = nz.draft_step(l, cfg.L, cfg.radices, cfg.K, H[:, l - 1, :], Wp[l - 1],
                          E[l - 1] if l < cfg.L else None, state, key, score,
                          gset if l == cfg.L else (gpre[l - 1] if gpre else None),
                          h_row_stride=H.stride(0),
                          U_l=U[l - 1] if (U is not None and l < cfg.L) else None)
        ref.append({k: v.clone() for k, v in o.items()})
        state, key, score = o.get("state"), o["key"], o["score"]
    plan = nz.DecodePlan(H, Wp, E, cfg.radices, cfg.K, gset, U=U, prefix_sets=gpre)
    for _ in range(2):
        got = plan.run()
        torch.cuda.synchronize()
        for a, b in zip(ref, got):
            for k in a:
                assert torch.equal(a[k], b[k]), k
    with pytest.raises(ValueError):
        nz.DecodePlan(H, W, E, cfg.radices, cfg.K, gset)       # weights not packed
