"""Dense inputs of the draft head: hidden states, per-level weights and code
embeddings.  Values are returned as float32 numpy arrays; for bf16 workloads
they are rounded once to bf16 (round-to-nearest-even) so that every consumer
reads exactly the same numbers."""
import numpy as np
from .rng import normal


def round_to_bf16(x):
    """float32 array -> float32 array holding the nearest bf16 values (RNE)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def draft_inputs(cfg, seed):
    """dict with H [B,L,d] ~ N(0,1); W[l] [(d+e),V] ~ N(0,w_std); E[l] [V,e] ~
    N(0,w_std) for l < L (levels are 0-based list positions here)."""
    B, L, d, e, V = cfg.B, cfg.L, cfg.d, cfg.e, cfg.V
    cast = round_to_bf16 if cfg.dtype == "bf16" else (lambda a: a.astype(np.float32))
    H = cast(normal(seed, 1, B * L * d).astype(np.float32).reshape(B, L, d))
    W = [cast(normal(seed, 10 + l, (d + e) * V, cfg.w_std).astype(np.float32)
              .reshape(d + e, V)) for l in range(L)]
    E = [cast(normal(seed, 40 + l, V * e, cfg.w_std).astype(np.float32)
              .reshape(V, e)) for l in range(L - 1)]
    return {"H": H, "W": W, "E": E}
