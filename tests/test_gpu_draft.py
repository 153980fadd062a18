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


def test_zero_requests_is_a_no_op():
    dev = device()
    H = torch.zeros((0, 64), dtype=torch.bfloat16, device=dev)
    W = torch.zeros((96, 64), dtype=torch.bfloat16, device=dev)
    E = torch.zeros((64, 32), dtype=torch.bfloat16, device=dev)
    o = nz.draft_step(1, 2, [64, 64], 4, H, W, E, h_row_stride=64)
    torch.cuda.synchronize()
    assert o["key"].shape == (0, 4)
