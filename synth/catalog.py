"""Synthetic item catalogs (sets of distinct semantic-ID tuples) and verifier
queries.  Tuples are int32 arrays [n, L], level 1 in column 0.

The tuple space [0,V)^L is enumerated here in numpy's row-major order (level 1
most significant).  That is only this generator's way of walking the space;
it is unrelated to, and deliberately not, the method's key packing."""
import numpy as np
from .rng import Bijection, uniform01, mix64, raw64

_U64 = np.uint64


def _salt(seed, c):
    return _U64((int(seed) * c) & 0xFFFFFFFFFFFFFFFF)


def digits_of(flat, radices):
    """Row-major position in the grid prod(radices) -> int32 [n, L] tuples."""
    cols = np.unravel_index(np.asarray(flat, dtype=np.int64), tuple(int(r) for r in radices))
    return np.stack(cols, axis=1).astype(np.int32)


def _flat_of(tuples, radices):
    return np.ravel_multi_index(tuple(tuples[:, i].astype(np.int64) for i in range(tuples.shape[1])),
                                tuple(int(r) for r in radices))


def uniform_catalog(radices, N, seed):
    """N distinct tuples spread uniformly: images of 0..N-1 under a keyed
    permutation pi of the tuple space.  Returns (tuples, pi); pi(j) for j >= N
    is guaranteed absent."""
    size = int(np.prod([int(r) for r in radices], dtype=object))
    assert N <= size
    pi = Bijection(size, seed, key=1)
    return digits_of(pi(np.arange(N, dtype=_U64)), radices), pi


def absent_tuples(radices, N, pi, seed, n, stream=70):
    """n tuples that are not in uniform_catalog(radices, N, .) built with pi."""
    size = pi.size
    assert size > N
    u = uniform01(seed, stream, n)
    j = (N + np.floor(u * (size - N))).astype(np.int64).clip(N, size - 1)
    return digits_of(pi(j.astype(_U64)), radices)


def zipf_weights(n, s):
    w = np.arange(1, n + 1, dtype=np.float64) ** (-float(s))
    return w / w.sum()


def _allocate(N, probs, cap):
    """Integer counts proportional to probs, each <= cap, summing to N
    (water-filling: cells that would exceed cap are fixed at cap and the
    excess is shared out among the rest in proportion)."""
    n = probs.size
    assert N <= cap * n
    fixed = np.zeros(n, dtype=bool)
    target = np.zeros(n, dtype=np.float64)
    while True:
        free_mass = probs[~fixed].sum()
        rest = N - cap * fixed.sum()
        target[fixed] = cap
        target[~fixed] = rest * probs[~fixed] / free_mass if free_mass > 0 else 0.0
        over = (~fixed) & (target > cap)
        if not over.any():
            break
        fixed |= over
    counts = np.floor(target).astype(np.int64)
    short = int(N - counts.sum())
    if short > 0:
        frac = target - counts
        frac[counts >= cap] = -1.0
        order = np.argsort(-frac, kind="stable")[:short]
        counts[order] += 1
    assert counts.sum() == N and counts.max() <= cap
    return counts


def zipf_catalog(radices, N, seed, s, depth=1, cap_frac=0.5):
    """N distinct tuples whose first `depth` levels follow Zipf(s) popularity
    (rank -> code by a seeded permutation; at depth 2 the second level is Zipf
    given the first, with its own rank permutation per first-level code) and
    whose remaining levels are uniform without replacement.  The number of
    items under a prefix is capped at cap_frac of the tuples that exist there."""
    radices = [int(r) for r in radices]
    L = len(radices)
    assert 1 <= depth < L
    V1 = radices[0]
    p1 = zipf_weights(V1, s)
    code1 = Bijection(V1, seed, key=2)(np.arange(V1, dtype=_U64)).astype(np.int64)
    if depth == 1:
        probs = p1
        prefix_cols = [code1]
    else:
        V2 = radices[1]
        p2 = zipf_weights(V2, s)
        probs = (p1[:, None] * p2[None, :]).ravel()
        r1 = np.repeat(np.arange(V1), V2)
        r2 = np.tile(np.arange(V2), V1)
        # per-first-code rotation of one shared rank permutation
        perm2 = Bijection(V2, seed, key=3)(np.arange(V2, dtype=_U64)).astype(np.int64)
        rot = (mix64(code1[r1].astype(_U64) + _U64(0xC0DE)) % _U64(V2)).astype(np.int64)
        prefix_cols = [code1[r1], perm2[(r2 + rot) % V2]]
    sub = radices[depth:]
    sub_size = int(np.prod(sub, dtype=object))
    counts = _allocate(N, probs, int(cap_frac * sub_size))
    pid = np.repeat(np.arange(probs.size, dtype=np.int64), counts)
    starts = np.cumsum(counts) - counts
    local = np.arange(N, dtype=np.int64) - np.repeat(starts, counts)
    off = (mix64(pid.astype(_U64) * _U64(0x9E3779B97F4A7C15) + _U64(seed)) % _U64(sub_size)).astype(np.int64)
    pos = ((local + off) % sub_size).astype(_U64)
    lower = digits_of(Bijection(sub_size, seed, key=4)(pos), sub)
    upper = np.stack([c[pid] for c in prefix_cols], axis=1).astype(np.int32)
    return np.concatenate([upper, lower], axis=1)


def planted_catalog(radices, background, plant, ban, seed):
    """Catalog of len(background) items: the tuples in `plant`, plus background
    tuples that are in neither `plant` nor `ban`, in a seeded shuffled order."""
    N = background.shape[0]
    fb = _flat_of(background, radices)
    fp = np.unique(_flat_of(plant, radices)) if len(plant) else np.zeros(0, np.int64)
    fx = np.unique(_flat_of(ban, radices)) if len(ban) else np.zeros(0, np.int64)
    fp = fp[~np.isin(fp, fx)]
    keep = fb[~np.isin(fb, np.concatenate([fp, fx]))]
    keep = keep[: max(0, N - fp.size)]
    allf = np.concatenate([fp, keep])
    order = np.argsort(mix64(allf.astype(_U64) + _salt(seed, 0x2545F4914F6CDD1D)), kind="stable")
    return digits_of(allf[order], radices)


def plant_mask(tuples, radices, seed, percent=70):
    """Seeded per-tuple coin: True for about `percent` % of distinct tuples."""
    f = _flat_of(tuples, radices).astype(_U64)
    return (mix64(f ^ (_salt(seed, 0xD6E8FEB86659FD93))) % _U64(100)) < _U64(percent)


def stress_queries(radices, N, pi, seed, n, absent_frac=0.3, zipf=True):
    """Queries for the stand-alone verifier against uniform_catalog(radices, N):
    a fraction absent (uniform over the absent part of the tuple space), the
    rest present with popularity rank r = floor((N+1)^u) - 1 (log-uniform, the
    continuous form of Zipf(1)) or uniform rank; ranks are scattered over the
    catalog by a second permutation.  Returns (tuples [n,L], present bool[n])."""
    u_kind = uniform01(seed, 80, n)
    u_val = uniform01(seed, 81, n)
    present = u_kind >= absent_frac
    size = pi.size
    if zipf:
        rank = np.floor(np.exp(u_val * np.log(N + 1.0))).astype(np.int64) - 1
    else:
        rank = np.floor(u_val * N).astype(np.int64)
    rank = rank.clip(0, N - 1)
    item = Bijection(N, seed, key=5)(rank.astype(_U64)).astype(np.int64)
    j_abs = (N + np.floor(u_val * (size - N))).astype(np.int64).clip(N, size - 1)
    src = np.where(present, item, j_abs)
    return digits_of(pi(src.astype(_U64)), radices), present
