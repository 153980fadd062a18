"""Independent float64 restatements of what the draft head computes, used only
to pin the CPU oracle.  Nothing here is shared with the oracle or the GPU
library: the chain score of a full tuple is written from its definition
(Eq. 1-3 with the additive or the recurrent Transition, softmax over the level's codes)."""
import itertools

import numpy as np


def log_softmax(z):
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def chain_scores_by_definition(h, W, E, U=None):
    """All V^L tuples of one request, one at a time, straight from the
    definition.  h [L,d]; W[l] [(d+e),V]; E[l] [V,e]; U[l] [e,e] or None (additive
    Transition).  Returns dict tuple->score."""
    L = len(W)
    V = W[0].shape[1]
    d = h.shape[1]
    e = W[0].shape[0] - d
    out = {}
    for t in itertools.product(range(V), repeat=L):
        c = np.zeros(e)
        s = 0.0
        for l in range(L):
            x = np.concatenate([h[l].astype(np.float64), c])
            lp = log_softmax(x @ W[l].astype(np.float64))
            s += lp[t[l]]
            if l < L - 1:
                emb = E[l][t[l]].astype(np.float64)
                c = c + emb if U is None else np.tanh(U[l].astype(np.float64) @ c + emb)
        out[t] = s
    return out


def chain_scores_grid_L3(h, W, E):
    """All V^3 chain scores of one request as an array [t1,t2,t3] (float64),
    using the linearity of the head: logits = user part + sum of per-code parts."""
    d = h.shape[1]
    W = [w.astype(np.float64) for w in W]
    E = [x.astype(np.float64) for x in E]
    h = h.astype(np.float64)
    A = [h[l] @ W[l][:d] for l in range(3)]
    lp1 = log_softmax(A[0])                                     # [V]
    lp2 = log_softmax(A[1][None, :] + E[0] @ W[1][d:])          # [t1, v]
    P31 = E[0] @ W[2][d:]
    P32 = E[1] @ W[2][d:]
    lp3 = log_softmax(A[2][None, None, :] + P31[:, None, :] + P32[None, :, :])
    return lp1[:, None, None] + lp2[:, :, None] + lp3, lp1
