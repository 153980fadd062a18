"""Shared pieces of the GPU parity tests: build a workload, run it through the C ABI, and
compare every level with the oracle on identical inputs."""
import numpy as np
import torch

import synth
from _parity import compare_level, to_np


def device():
    return torch.device("cuda:0")


def torch_dtype(cfg):
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


def background_catalog(cfg, seed, N=None):
    N = cfg.N if N is None else N
    if cfg.catalog == "uniform":
        return synth.uniform_catalog(cfg.radices, N, seed)[0]
    depth = 2 if cfg.catalog == "zipf12" else 1
    return synth.zipf_catalog(cfg.radices, N, seed, cfg.zipf_s, depth=depth)


def planted_workload(orc, cfg, seed, N=None, plant=True):
    """Inputs plus a catalog in which about 70 % of the unverified top-K beams (computed by
    the oracle, never by the GPU path) are valid items."""
    x = synth.draft_inputs(cfg, seed)
    cat = background_catalog(cfg, seed, N)
    if plant:
        free = orc.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K,
                          round_state_bf16=cfg.dtype == "bf16")
        tuples = orc.unpack(free[-1]["key"].ravel(), cfg.radices)
        keep = synth.plant_mask(tuples, cfg.radices, seed)
        cat = synth.planted_catalog(cfg.radices, cat, tuples[keep], tuples[~keep], seed)
    return x, cat


def to_device(x, cfg):
    dev, dt = device(), torch_dtype(cfg)
    H = torch.from_numpy(x["H"]).to(dev).to(dt)
    W = [torch.from_numpy(w).to(dev).to(dt) for w in x["W"]]
    E = [torch.from_numpy(w).to(dev).to(dt) for w in x["E"]]
    return H, W, E


def outputs_to_numpy(o):
    return {k: to_np(v.float() if v.dtype == torch.bfloat16 else v) for k, v in o.items()}


def check_decode(orc, nz, cfg, x, outs, oset, tol, U=None, prefix_sets=None, use_state=True):
    """Level by level: the oracle is fed what the GPU produced at the level before.  U: per-level
    [e, e] matrices of the recurrent Transition (numpy, the values the GPU read); prefix_sets:
    oracle sets of the valid prefixes of length 1..L-1."""
    state = key = score = None
    soft_total = 0
    for l in range(1, cfg.L + 1):
        g = outputs_to_numpy(outs[l - 1])
        inp = {"H": x["H"][:, l - 1], "W": x["W"][l - 1],
               "E": x["E"][l - 1] if l < cfg.L else None,
               "state": state if use_state else None, "key": key, "score": score,
               "U": U[l - 1] if (U is not None and l < cfg.L) else None}
        lset = oset if l == cfg.L else (prefix_sets[l - 1] if prefix_sets else None)
        soft_total += compare_level(orc, l, cfg.L, cfg.radices, cfg.K, inp, g, lset, tol,
                                    cfg.dtype == "bf16")
        state, key, score = g.get("state"), g["key"].view(np.uint64), g["score"]
    return soft_total


def tolerance(cfg):
    # float32 workloads: 1e-5 absolute on log-probabilities and scores.  bf16 workloads read
    # bf16 inputs exactly and accumulate in float32, so they are held to 1e-4, far inside the
    # 2e-2 allowed for bf16.
    return 1e-5 if cfg.dtype == "f32" else 1e-4
