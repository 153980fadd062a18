"""Comparison of one level of the GPU draft step with the CPU oracle run on the same inputs.

Integer work (indices of Eq. 4, parents, codes, counts, membership) must agree exactly.
Scores must agree within `tol`.  Where the two sides pick different beams the difference
has to be explained by a gap smaller than `tol` between the scores involved (floating point
decides an order there); anything else is an error."""
import numpy as np


def to_np(t):
    return t.detach().cpu().numpy()


def compare_level(orc, level, L, radices, K, inp, gpu, oset, tol, bf16_state):
    """inp: dict of numpy inputs H, W, E, state, key, score, U (float32 / uint64, the values the
    GPU read).  gpu: dict of numpy outputs.  oset: the set this level is verified against (the
    items at level L, valid prefixes below it) or None.  Returns the number of beams that differ
    from the oracle's list for tolerance reasons."""
    if level < L and oset is not None:
        assert oset.L == level
    elif level == L and oset is not None:
        assert oset.L == L
    o = orc.draft_level(level, L, radices, K, inp["H"], inp["W"], inp.get("E"),
                        inp.get("state"), inp.get("key"), inp.get("score"),
                        oset, round_state_bf16=bf16_state, want_logp=True, U_l=inp.get("U"))
    logp = o["logp"]
    B, K_in, V = logp.shape
    mult = np.uint64(int(np.prod([int(r) for r in radices[:level - 1]], dtype=object)))
    key_in = inp["key"] if inp.get("key") is not None else np.zeros((B, K_in), np.uint64)
    score_in = inp["score"] if inp.get("score") is not None else np.zeros((B, K_in), np.float32)
    gk = gpu["key"].view(np.uint64)
    soft = 0
    for b in range(B):
        n = int(gpu["count"][b])
        assert 0 <= n <= K
        par, code, sc = gpu["parent"][b, :n], gpu["code"][b, :n], gpu["score"][b, :n]
        assert ((par >= 0) & (par < K_in) & (code >= 0) & (code < V)).all()
        assert len({(int(p), int(c)) for p, c in zip(par, code)}) == n
        assert (gk[b, :n] == key_in[b, par] + code.astype(np.uint64) * mult).all()
        assert (gk[b, n:] == np.uint64(2**64 - 1)).all()
        assert np.isneginf(gpu["score"][b, n:]).all()
        assert (gpu["parent"][b, n:] == -1).all() and (gpu["code"][b, n:] == -1).all()
        want = score_in[b, par].astype(np.float64) + logp[b, par, code]
        assert np.abs(sc - want).max(initial=0) <= tol, (b, np.abs(sc - want).max())
        assert (np.diff(sc) <= 0).all()
        assert (key_in[b, par] != np.uint64(2**64 - 1)).all()              # no child of an empty slot
        valid_g = oset.contains_keys(gk[b, :n]) if oset is not None else None
        if valid_g is not None:
            assert valid_g.all()
        # fast path: identical to the oracle's list
        on = int(o["count"][b])
        same = (n == on and (o["key"][b] == gk[b]).all() and (o["parent"][b] == gpu["parent"][b]).all()
                and (o["code"][b] == gpu["code"][b]).all())
        if same:
            if "state" in gpu and "state" in o:
                if inp.get("U") is None:
                    assert (gpu["state"][b] == o["state"][b]).all()
                else:
                    # tanh of a float32 (GPU) or float64 (oracle) sum of e products.  float32
                    # states: equal within the float32 tolerance of the path; bf16 states: the
                    # rounding to bf16 hides that difference except where it straddles a rounding
                    # boundary, so a few elements may differ by one bf16 unit in the last place
                    gs, os_ = gpu["state"][b].astype(np.float64), o["state"][b].astype(np.float64)
                    if bf16_state:
                        assert (np.abs(gs - os_) <= 2.0 ** -7 * np.maximum(np.abs(os_), 2.0 ** -10)).all()
                        assert (gs != os_).mean() < 0.02
                    else:
                        assert np.abs(gs - os_).max() <= 1e-5
            continue
        # explain the difference by tolerance
        kth = np.sort(logp[b], axis=-1)[:, V - min(K, V)]                  # per-beam K-th largest logp
        assert (logp[b, par, code] >= kth[par] - tol).all()                 # eligible in its beam
        elig = logp[b] > (kth[:, None] + tol)                               # robustly eligible
        pp, vv = np.nonzero(elig)
        ckey = key_in[b, pp] + vv.astype(np.uint64) * mult
        cscore = score_in[b, pp].astype(np.float64) + logp[b, pp, vv]
        if oset is not None:
            ok = oset.contains_keys(ckey)
            pp, vv, ckey, cscore = pp[ok], vv[ok], ckey[ok], cscore[ok]
        have = set(gk[b, :n].tolist())
        missing = np.array([k not in have for k in ckey.tolist()], dtype=bool)
        if n < K:
            assert not missing.any(), "a valid, clearly eligible candidate was dropped"
        else:
            assert (cscore[missing] <= sc[-1] + tol).all(), "a better candidate was left out"
        gset, oset_k = set(gk[b, :n].tolist()), set(o["key"][b, :on].tolist())
        soft += len(gset ^ oset_k) + (0 if gset != oset_k else 1)
    return soft
