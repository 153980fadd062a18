"""Pins for the oracle's draft head and beam search (Eq. 1-3, Alg. 3 inference)."""
import numpy as np
import pytest
import torch

import synth
from _definitions import chain_scores_by_definition, chain_scores_grid_L3, log_softmax


def _small(seed, B=3, d=8, e=4, V=6, L=3, w_std=0.7):
    cfg = synth.StepConfig("t", B=B, d=d, e=e, L=L, V=V, K=1, N=1, dtype="f32",
                           catalog="uniform", w_std=w_std)
    return cfg, synth.draft_inputs(cfg, seed)


def test_level1_logp_is_a_library_matvec_and_log_softmax(oracle):
    cfg, x = _small(1, B=5, d=33, e=7, V=19)
    o = oracle.draft_level(1, cfg.L, cfg.radices, 4, x["H"][:, 0], x["W"][0], x["E"][0],
                           want_logp=True)
    z = torch.from_numpy(x["H"][:, 0]).double() @ torch.from_numpy(x["W"][0][:33]).double()
    want = torch.log_softmax(z, dim=-1).numpy()
    assert np.abs(o["logp"][:, 0, :] - want).max() < 1e-12
    assert np.abs(np.exp(o["logp"]).sum(-1) - 1).max() < 1e-12


def test_level2_logits_use_the_concatenated_input(oracle):
    cfg, x = _small(2, B=4, d=16, e=5, V=11)
    rng = np.random.default_rng(3)
    state = rng.normal(size=(4, 3, 5)).astype(np.float32)
    key = np.arange(12, dtype=np.uint64).reshape(4, 3)
    score = -rng.random((4, 3)).astype(np.float32)
    o = oracle.draft_level(2, 3, cfg.radices, 3, x["H"][:, 1], x["W"][1], x["E"][1],
                           state, key, score, want_logp=True)
    Hc = torch.cat([torch.from_numpy(x["H"][:, 1]).double()[:, None, :].expand(4, 3, 16),
                    torch.from_numpy(state).double()], dim=-1)
    want = torch.log_softmax(Hc @ torch.from_numpy(x["W"][1]).double(), dim=-1).numpy()
    assert np.abs(o["logp"] - want).max() < 1e-12
    # swapping the two blocks of W (a transposed-operand style mistake) must be visible
    Wsw = np.concatenate([x["W"][1][16:], x["W"][1][:16]])
    bad = torch.log_softmax(Hc @ torch.from_numpy(Wsw).double(), dim=-1).numpy()
    assert np.abs(o["logp"] - bad).max() > 1e-3
    # candidate bookkeeping: score = parent score + logp, key = parent key + code * T_1
    for b in range(4):
        for j in range(3):
            p, c = o["parent"][b, j], o["code"][b, j]
            assert o["key"][b, j] == key[b, p] + np.uint64(c * 11)
            assert abs(o["score"][b, j] - (score[b, p] + want[b, p, c])) < 1e-6
            assert np.allclose(o["state"][b, j], state[b, p] + x["E"][1][c], atol=1e-7)


def test_zero_weights_give_uniform_probabilities_and_the_tie_rule(oracle):
    cfg, x = _small(3, B=2, d=8, e=4, V=9)
    W0 = [np.zeros_like(w) for w in x["W"]]
    outs = oracle.decode(x["H"], W0, x["E"], cfg.radices, 4)
    o1, o2, o3 = outs
    assert (o1["code"] == np.arange(4)).all() and (o1["parent"] == 0).all()
    assert np.allclose(o1["score"], -np.log(9))
    # level 2: all 16 candidates tie; parent rank 0 wins, lower codes first
    assert (o2["parent"] == 0).all() and (o2["code"] == np.arange(4)).all()
    assert np.allclose(o2["score"], -2 * np.log(9))
    assert (o3["parent"] == 0).all() and (o3["code"] == np.arange(4)).all()
    assert (o3["key"][0] == np.array([0, 81, 162, 243], dtype=np.uint64)).all()
    assert (o3["count"] == 4).all()


def test_per_beam_topk_then_merge_equals_global_topk_below_last_level(oracle):
    cfg, x = _small(4, B=6, d=12, e=6, V=13)
    K = 5
    o1 = oracle.draft_level(1, 3, cfg.radices, K, x["H"][:, 0], x["W"][0], x["E"][0],
                            want_logp=True)
    order = np.argsort(-o1["logp"][:, 0, :], axis=-1, kind="stable")[:, :K]
    assert (o1["code"] == order).all()                      # level 1 = full sort of V values
    o2 = oracle.draft_level(2, 3, cfg.radices, K, x["H"][:, 1], x["W"][1], x["E"][1],
                            o1["state"], o1["key"], o1["score"], want_logp=True)
    for b in range(6):
        allc = [(-(np.float32(np.float64(o1["score"][b, p]) + o2["logp"][b, p, v])), p, v)
                for p in range(K) for v in range(13)]
        allc.sort()
        want = allc[:K]
        got = [(-o2["score"][b, j], o2["parent"][b, j], o2["code"][b, j]) for j in range(K)]
        assert got == want


@pytest.mark.parametrize("seed,V,L", [(5, 4, 3), (6, 7, 2), (7, 3, 3)])
def test_exhaustive_beam_equals_brute_force_over_all_tuples(oracle, seed, V, L):
    cfg, x = _small(seed, B=2, d=6, e=3, V=V, L=L)
    total = V ** L
    rng = np.random.default_rng(seed)
    valid = rng.random(total) < 0.4
    tuples = np.array([t for t in np.ndindex(*([V] * L))], dtype=np.int32)
    cat = tuples[valid]
    s = oracle.ItemSet(cat, cfg.radices)
    K = total                                   # no pruning can bite: beam search is exhaustive
    outs = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, K, itemset=s)
    last = outs[-1]
    for b in range(2):
        truth = chain_scores_by_definition(x["H"][b], x["W"], x["E"])
        assert abs(sum(np.exp(v) for v in truth.values()) - 1) < 1e-12
        vt = sorted(((-truth[tuple(t)], i) for i, t in enumerate(cat.tolist())))
        assert last["count"][b] == len(cat)
        got = oracle.unpack(last["key"][b, :len(cat)], cfg.radices)
        got_scores = last["score"][b, :len(cat)]
        want_scores = np.array([-v for v, _ in vt])
        assert np.abs(got_scores - want_scores).max() < 2e-6
        assert (np.diff(got_scores) <= 0).all()
        assert sorted(map(tuple, got.tolist())) == sorted(map(tuple, cat.tolist()))
        for t, sc in zip(got.tolist(), got_scores):
            assert abs(truth[tuple(t)] - sc) < 2e-6
        assert (last["key"][b, len(cat):] == np.uint64(2**64 - 1)).all()
        assert np.isneginf(last["score"][b, len(cat):]).all()


def test_beam_search_invariants_with_real_pruning(oracle):
    cfg, x = _small(8, B=5, d=10, e=5, V=12)
    K = 4
    tuples = np.array([t for t in np.ndindex(12, 12, 12)], dtype=np.int32)
    rng = np.random.default_rng(8)
    cat = tuples[rng.random(len(tuples)) < 0.3]
    s = oracle.ItemSet(cat, cfg.radices)
    outs = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, K, itemset=s)
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, K, itemset=None)
    assert (free[-1]["count"] == K).all()
    o2, o3 = outs[1], outs[2]
    chk = oracle.draft_level(3, 3, cfg.radices, K, x["H"][:, 2], x["W"][2], None,
                             o2["state"], o2["key"], o2["score"], None, want_logp=True)
    catset = set(map(tuple, cat.tolist()))
    for b in range(5):
        truth = chain_scores_by_definition(x["H"][b], x["W"], x["E"])
        # the K x K candidates of the last level: per-beam top-K codes
        cands = []
        for p in range(K):
            top = np.argsort(-chk["logp"][b, p], kind="stable")[:K]
            prefix = tuple(oracle.unpack(o2["key"][b, p:p + 1], cfg.radices)[0][:2])
            cands += [prefix + (int(v),) for v in top]
        assert len(set(cands)) == K * K
        valid = [t for t in cands if t in catset]
        n = int(o3["count"][b])
        assert n == min(K, len(valid))
        got = [tuple(t) for t in oracle.unpack(o3["key"][b, :n], cfg.radices).tolist()]
        assert len(set(got)) == n and set(got) <= set(valid)
        sc = o3["score"][b, :n]
        assert (np.diff(sc) <= 0).all()
        for t, v in zip(got, sc):
            assert abs(truth[t] - v) < 2e-6                 # carries its brute-force chain score
        worst = sc[-1] if n else np.inf
        for t in valid:
            if t not in got:
                assert truth[t] <= worst + 2e-6             # nothing better was left out


def test_tiny_config_against_all_256_cubed_tuples(oracle):
    cfg = synth.get_config("tiny")
    x = synth.draft_inputs(cfg, 42)
    cat, _ = synth.uniform_catalog(cfg.radices, cfg.N, 42)
    # the tiny catalog has density 0.06 %, so plant the unverified beams' tuples too
    free = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K)
    plant = oracle.unpack(free[-1]["key"].ravel(), cfg.radices)
    keep = synth.plant_mask(plant, cfg.radices, 42)
    cat2 = synth.planted_catalog(cfg.radices, cat, plant[keep], plant[~keep], 42)
    assert cat2.shape == cat.shape
    s = oracle.ItemSet(cat2, cfg.radices)
    outs = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K, itemset=s)
    bitmap = np.zeros((256,) * 3, dtype=bool)
    bitmap[cat2[:, 0], cat2[:, 1], cat2[:, 2]] = True
    emitted = 0
    for b in range(cfg.B):
        grid, lp1 = chain_scores_grid_L3(x["H"][b], x["W"], x["E"])
        assert abs(np.exp(grid).sum() - 1) < 1e-9
        top1 = np.argsort(-lp1, kind="stable")[:cfg.K]
        assert (outs[0]["code"][b] == top1).all()
        assert np.abs(outs[0]["score"][b] - lp1[top1]).max() < 1e-6
        n = int(outs[2]["count"][b])
        emitted += n
        t = oracle.unpack(outs[2]["key"][b, :n], cfg.radices)
        assert bitmap[t[:, 0], t[:, 1], t[:, 2]].all()
        assert np.abs(grid[t[:, 0], t[:, 1], t[:, 2]] - outs[2]["score"][b, :n]).max() < 2e-6
        tf = oracle.unpack(free[2]["key"][b], cfg.radices)
        assert np.abs(grid[tf[:, 0], tf[:, 1], tf[:, 2]] - free[2]["score"][b]).max() < 2e-6
    assert emitted > 0
    # un-planted: almost surely nothing survives; counts may be zero and must pad correctly
    s0 = oracle.ItemSet(cat, cfg.radices)
    o0 = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, cfg.K, itemset=s0)[-1]
    for b in range(cfg.B):
        n = int(o0["count"][b])
        assert (o0["parent"][b, n:] == -1).all() and (o0["code"][b, n:] == -1).all()


def test_state_rounding_to_bf16(oracle):
    cfg, x = _small(9, B=2, d=8, e=16, V=10, w_std=0.3)
    o = oracle.draft_level(1, 3, cfg.radices, 3, x["H"][:, 0], x["W"][0], x["E"][0],
                           round_state_bf16=True)
    want = torch.from_numpy(x["E"][0][o["code"]]).to(torch.bfloat16).float().numpy()
    assert (o["state"] == want).all()
    assert (synth.round_to_bf16(x["E"][0]) == torch.from_numpy(x["E"][0]).to(torch.bfloat16).float().numpy()).all()


# ---- recurrent Transition: c' = tanh(U c + e_l) -------------------------------------------------
def _rnn_weights(seed, L, e, scale=0.6):
    rng = np.random.default_rng(seed)
    return [(rng.standard_normal((e, e)) * scale).astype(np.float32) for _ in range(L - 1)]


@pytest.mark.parametrize("seed,V,L", [(15, 4, 3), (16, 6, 2)])
def test_rnn_exhaustive_beam_equals_brute_force(oracle, seed, V, L):
    cfg, x = _small(seed, B=2, d=6, e=3, V=V, L=L)
    U = _rnn_weights(seed, L, 3)
    x["E"] = [em * 20 for em in x["E"]]             # large enough for tanh to bend
    total = V ** L
    outs = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, total, U=U)
    last = outs[-1]
    for b in range(2):
        truth = chain_scores_by_definition(x["H"][b], x["W"], x["E"], U=U)
        plain = chain_scores_by_definition(x["H"][b], x["W"], x["E"])
        assert abs(sum(np.exp(v) for v in truth.values()) - 1) < 1e-12
        assert max(abs(truth[t] - plain[t]) for t in truth) > 1e-3   # the cell is not the sum
        assert last["count"][b] == total
        got = oracle.unpack(last["key"][b], cfg.radices)
        for t, sc in zip(got.tolist(), last["score"][b]):
            assert abs(truth[tuple(t)] - sc) < 2e-6
        assert (np.diff(last["score"][b]) <= 0).all()


def test_rnn_state_closed_forms(oracle):
    cfg, x = _small(17, B=3, d=8, e=4, V=16)
    K = 5
    E1 = x["E"][0] * 30
    zero = np.zeros((4, 4), np.float32)
    o1 = oracle.draft_level(1, 3, cfg.radices, K, x["H"][:, 0], x["W"][0], E1, U_l=zero)
    # level 1 starts from the zero state: c' = tanh(e_l) whatever U is
    assert np.allclose(o1["state"], np.tanh(E1[o1["code"]].astype(np.float64)), atol=1e-7)
    U = (np.random.default_rng(17).standard_normal((4, 4)) * 0.7).astype(np.float32)
    o1u = oracle.draft_level(1, 3, cfg.radices, K, x["H"][:, 0], x["W"][0], E1, U_l=U)
    assert (o1u["state"] == o1["state"]).all()
    # level 2: row j of U meets the parent state (a transposed U must be visible)
    E2 = x["E"][1] * 30
    o2 = oracle.draft_level(2, 3, cfg.radices, K, x["H"][:, 1], x["W"][1], E2, o1["state"],
                            o1["key"], o1["score"], U_l=U)
    par = o1["state"][np.arange(3)[:, None], o2["parent"]].astype(np.float64)      # [B,K,e]
    want = np.tanh(np.einsum("ji,bki->bkj", U.astype(np.float64), par) + E2[o2["code"]])
    wrong = np.tanh(np.einsum("ij,bki->bkj", U.astype(np.float64), par) + E2[o2["code"]])
    assert np.allclose(o2["state"], want, atol=1e-6)
    assert np.abs(want - wrong).max() > 1e-2
    # the beams themselves do not depend on the Transition of the same level
    o2a = oracle.draft_level(2, 3, cfg.radices, K, x["H"][:, 1], x["W"][1], E2, o1["state"],
                             o1["key"], o1["score"])
    assert (o2a["key"] == o2["key"]).all() and (o2a["score"] == o2["score"]).all()
    assert np.allclose(o2a["state"], par + E2[o2["code"]], atol=1e-6)
    # bf16 rounding of the state applies to the cell's output too
    o2r = oracle.draft_level(2, 3, cfg.radices, K, x["H"][:, 1], x["W"][1], E2, o1["state"],
                             o1["key"], o1["score"], U_l=U, round_state_bf16=True)
    assert (o2r["state"] == synth.round_to_bf16(o2["state"])).all()


# ---- verification below the last level against sets of valid prefixes ---------------------------
def test_prefix_verification_by_definition(oracle):
    cfg, x = _small(18, B=6, d=10, e=5, V=12)
    K = 4
    rng = np.random.default_rng(18)
    tuples = np.array([t for t in np.ndindex(12, 12, 12)], dtype=np.int32)
    first_ok = np.isin(tuples[:, 0], [0, 3, 4, 7, 9])             # most first codes start no item
    cat = tuples[first_ok & (rng.random(len(tuples)) < 0.12)]
    full = oracle.ItemSet(cat, cfg.radices)
    p1 = oracle.ItemSet(np.unique(cat[:, :1], axis=0), cfg.radices[:1])
    p2 = oracle.ItemSet(np.unique(cat[:, :2], axis=0), cfg.radices[:2])
    outs = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, K, itemset=full,
                         prefix_sets=[p1, p2])
    ok1 = set(map(tuple, np.unique(cat[:, :1], axis=0).tolist()))
    ok2 = set(map(tuple, np.unique(cat[:, :2], axis=0).tolist()))
    catset = set(map(tuple, cat.tolist()))
    # level 1 from its definition: the K most probable codes, then those that start an item
    lp1 = log_softmax(x["H"][:, 0].astype(np.float64) @ x["W"][0][:10].astype(np.float64))
    for b in range(6):
        top = np.argsort(-lp1[b], kind="stable")[:K]
        want = [int(v) for v in top if (int(v),) in ok1]
        n = int(outs[0]["count"][b])
        assert outs[0]["code"][b, :n].tolist() == want
        assert (outs[0]["key"][b, n:] == np.uint64(2**64 - 1)).all()
    assert (outs[0]["count"] < K).any()                # some slots are empty at level 2's input
    # level 2 and 3 from their definition, on what the level before handed over
    for lvl, okset in ((2, ok2), (3, catset)):
        prev, cur = outs[lvl - 2], outs[lvl - 1]
        live = int(prev["count"].max())
        chk = oracle.draft_level(lvl, 3, cfg.radices, K, x["H"][:, lvl - 1], x["W"][lvl - 1], None,
                                 prev["state"][:, :live], prev["key"][:, :live],
                                 prev["score"][:, :live], None, want_logp=True)
        for b in range(6):
            cands = []
            for p in range(int(prev["count"][b])):
                prefix = tuple(oracle.unpack(prev["key"][b, p:p + 1], cfg.radices)[0][:lvl - 1])
                for v in np.argsort(-chk["logp"][b, p], kind="stable")[:K]:
                    t = prefix + (int(v),)
                    if t in okset:
                        sc = np.float32(np.float64(prev["score"][b, p]) + chk["logp"][b, p, v])
                        cands.append((-float(sc), p, int(v), t))
            cands.sort(key=lambda c: (c[0], c[1]))     # stable in (parent, within-beam rank)
            want = cands[:K]
            n = int(cur["count"][b])
            assert n == len(want)
            got = [tuple(t[:lvl]) for t in oracle.unpack(cur["key"][b, :n], cfg.radices).tolist()]
            assert got == [c[3] for c in want]
            assert np.allclose(cur["score"][b, :n], [-c[0] for c in want], atol=1e-6)
    # prefixes of items only: every emitted item is in the catalog, and an exhaustive search with
    # the prefix filter returns exactly what it returns without it
    K_all = 12 ** 3
    cfg2, y = _small(19, B=1, d=6, e=3, V=12)
    a = oracle.decode(y["H"], y["W"], y["E"], cfg2.radices, K_all, itemset=full)
    bb = oracle.decode(y["H"], y["W"], y["E"], cfg2.radices, K_all, itemset=full,
                       prefix_sets=[p1, p2])
    n = int(a[-1]["count"][0])
    assert n == len(cat) == int(bb[-1]["count"][0])
    assert (a[-1]["key"][0, :n] == bb[-1]["key"][0, :n]).all()


# ---- the head without its state: the chain probability is a product of per-level marginals ------
def test_without_state_the_score_factorizes(oracle):
    cfg, x = _small(21, B=3, d=7, e=3, V=5, L=3)
    K = 5 ** 3
    outs = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, K, use_state=False)
    last = outs[-1]
    lp = [log_softmax(x["H"][:, l].astype(np.float64) @ x["W"][l][:7].astype(np.float64))
          for l in range(3)]
    for b in range(3):
        assert last["count"][b] == K
        got = oracle.unpack(last["key"][b], cfg.radices)
        want = lp[0][b][got[:, 0]] + lp[1][b][got[:, 1]] + lp[2][b][got[:, 2]]
        assert np.abs(last["score"][b] - want).max() < 2e-6
        assert len(set(map(tuple, got.tolist()))) == K
    with_state = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, K)
    assert np.abs(with_state[-1]["score"] - last["score"]).max() > 1e-4


def test_head_without_placeholder_hidden_states(oracle):
    """Ablation "without h_l" (Sec. 4.3): the head sees one hidden vector at every level (the
    caller passes h_1 as every H_l) and keeps its autoregressive state.  With an exhaustive beam
    the scores must be the chain scores written from the definition with that single vector, for
    all tuples, and they must differ from the full model's."""
    cfg, x = _small(27, B=2, d=6, e=3, V=4, L=3)
    K = 4 ** 3
    H2 = np.repeat(x["H"][:, :1], 3, axis=1).copy()
    last = oracle.decode(H2, x["W"], x["E"], cfg.radices, K)[-1]
    full = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, K)[-1]
    for b in range(2):
        one_vector = np.tile(x["H"][b, 0], (3, 1))
        truth = chain_scores_by_definition(one_vector, x["W"], x["E"])
        assert abs(sum(np.exp(v) for v in truth.values()) - 1) < 1e-12
        assert last["count"][b] == K
        got = oracle.unpack(last["key"][b], cfg.radices)
        assert len(set(map(tuple, got.tolist()))) == K
        for t, sc in zip(got.tolist(), last["score"][b]):
            assert abs(truth[tuple(t)] - sc) < 2e-6
        # the state still matters (unlike the head without state, scores do not factorize) ...
        lp = [log_softmax(one_vector[l].astype(np.float64) @ x["W"][l][:6].astype(np.float64))
              for l in range(3)]
        fact = lp[0][got[:, 0]] + lp[1][got[:, 1]] + lp[2][got[:, 2]]
        assert np.abs(fact - last["score"][b]).max() > 1e-4
    # ... and the placeholder hidden states matter too
    assert np.abs(np.sort(full["score"], axis=1) - np.sort(last["score"], axis=1)).max() > 1e-4


def test_wide_beam_against_the_grid_of_all_tuples(oracle):
    """A beam wider than 128 (the recall setting of the paper: beam 512 to 1000), checked against
    beam search restated on the array of all V^3 chain scores: level 1 keeps the K most probable
    codes, level 2 the K best (t1, t2) pairs among the kept t1, level 3 cuts every beam to its K
    most probable codes, drops what is not in the catalog and keeps the K best."""
    V, K = 144, 136
    cfg, x = _small(21, B=2, d=10, e=6, V=V, w_std=0.5)
    rng = np.random.default_rng(21)
    bitmap = rng.random((V, V, V)) < 0.05
    cat = np.argwhere(bitmap).astype(np.int32)
    s = oracle.ItemSet(cat, cfg.radices)
    outs = oracle.decode(x["H"], x["W"], x["E"], cfg.radices, K, itemset=s)
    for b in range(2):
        grid, lp1 = chain_scores_grid_L3(x["H"][b], x["W"], x["E"])
        t1 = np.argsort(-lp1, kind="stable")[:K]
        assert (outs[0]["code"][b] == t1).all()
        # level 2: all K*V pairs, order (score, parent rank, code)
        d = cfg.d
        lp2 = log_softmax((x["H"][b, 1].astype(np.float64) @ x["W"][1][:d].astype(np.float64))[None, :]
                          + x["E"][0][t1].astype(np.float64) @ x["W"][1][d:].astype(np.float64))
        s2 = (lp1[t1][:, None] + lp2).ravel()
        pick = np.argsort(-s2, kind="stable")[:K]
        assert (outs[1]["parent"][b] == pick // V).all() and (outs[1]["code"][b] == pick % V).all()
        assert np.abs(outs[1]["score"][b] - s2[pick]).max() < 2e-6
        pairs = np.stack([t1[pick // V], pick % V], axis=1)
        # level 3
        cands = []
        for r, (a1, a2) in enumerate(pairs.tolist()):
            lp3 = grid[a1, a2] - s2[pick[r]]
            top = np.argsort(-lp3, kind="stable")[:K]
            cands += [(-grid[a1, a2, v], r, int(v)) for v in top if bitmap[a1, a2, v]]
        cands.sort()
        n = int(outs[2]["count"][b])
        assert n == min(K, len(cands)) and n > 128
        assert [(c[1], c[2]) for c in cands[:n]] == list(zip(outs[2]["parent"][b, :n].tolist(),
                                                             outs[2]["code"][b, :n].tolist()))
        assert np.abs(outs[2]["score"][b, :n] + np.array([c[0] for c in cands[:n]])).max() < 3e-6
