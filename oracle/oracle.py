"""ctypes binding of the CPU oracle.  TEST INFRASTRUCTURE ONLY: imported by the
tests, the smoke check and the CPU-baseline leg of the benchmark, never by the
GPU library or its Python binding."""
import ctypes as C
import os
import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_set_new.restype = C.c_void_p
        L.orc_set_size.restype = C.c_int64
        L.orc_set_size.argtypes = [C.c_void_p]
        L.orc_set_free.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def _p(a, ctype=C.c_void_p):
    if a is None:
        return None
    return a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def pack(codes, radices):
    """Eq. 4.  Returns (keys uint64 [n], ok bool [n])."""
    codes = _i32(codes)
    n, L = codes.shape
    rad = _i32(radices)
    keys = np.empty(n, dtype=np.uint64)
    ok = np.empty(n, dtype=np.uint8)
    rc = lib().orc_pack(_p(codes), C.c_int64(n), C.c_int32(L), _p(rad), _p(keys), _p(ok))
    if rc != 0:
        raise OverflowError("product of radices does not fit in 64 bits")
    return keys, ok.astype(bool)


def unpack(keys, radices):
    keys = np.ascontiguousarray(keys, dtype=np.uint64)
    rad = _i32(radices)
    out = np.empty((keys.size, rad.size), dtype=np.int32)
    lib().orc_unpack(_p(keys), C.c_int64(keys.size), C.c_int32(rad.size), _p(rad), _p(out))
    return out


class ItemSet:
    """The set of valid item indices of Eq. 5 (std::unordered_set)."""

    def __init__(self, codes, radices):
        codes = _i32(codes)
        self.radices = _i32(radices)
        self.L = int(self.radices.size)
        assert codes.ndim == 2 and codes.shape[1] == self.L
        err = C.c_int(0)
        self._h = lib().orc_set_new(_p(codes), C.c_int64(codes.shape[0]), C.c_int32(self.L),
                                    _p(self.radices), C.byref(err))
        if err.value != 0:
            self._h = None
            raise ValueError("code out of range or radices overflow (%d)" % err.value)

    def __len__(self):
        return int(lib().orc_set_size(C.c_void_p(self._h)))

    def contains_keys(self, keys):
        keys = np.ascontiguousarray(keys, dtype=np.uint64)
        mask = np.empty(keys.size, dtype=np.uint8)
        lib().orc_set_contains_keys(C.c_void_p(self._h), _p(keys), C.c_int64(keys.size), _p(mask))
        return mask.astype(bool).reshape(keys.shape)

    def verify_tuples(self, codes):
        """Returns (mask uint8 [n], accepted indices int64 [count])."""
        codes = _i32(codes)
        n = codes.shape[0]
        mask = np.empty(n, dtype=np.uint8)
        index = np.empty(n, dtype=np.int64)
        count = C.c_int64(0)
        lib().orc_verify_tuples(C.c_void_p(self._h), _p(codes), C.c_int64(n), _p(mask),
                                _p(index), C.byref(count))
        return mask, index[: count.value].copy()

    def close(self):
        if getattr(self, "_h", None):
            lib().orc_set_free(C.c_void_p(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def draft_level(level, L, radices, K, H_l, W_l, E_l=None, state_in=None, key_in=None,
                score_in=None, itemset=None, round_state_bf16=False, want_logp=False,
                want_state=True, threads=None, U_l=None):
    """One level (1-based) of the inference part of Alg. 3 for a batch.

    H_l [B,d] float32; W_l [(d+e),V]; E_l [V,e]; state_in [B,K_in,e] or None.
    itemset: full tuples (used at level L) or prefixes of length `level` (used at this level).
    U_l [e,e]: the recurrent Transition c' = tanh(U_l c + e_l) instead of c' = c + e_l.
    Returns dict(key, score, parent, code, count[, state][, logp])."""
    H_l = np.ascontiguousarray(H_l, dtype=np.float32)
    W_l = np.ascontiguousarray(W_l, dtype=np.float32)
    B, d = H_l.shape
    rad = _i32(radices)
    V = int(rad[level - 1])
    e = W_l.shape[0] - d
    assert W_l.shape[1] == V and e >= 0
    if state_in is not None:
        state_in = np.ascontiguousarray(state_in, dtype=np.float32)
        K_in = state_in.shape[1]
        assert state_in.shape == (B, K_in, e)
    elif key_in is not None:
        K_in = np.asarray(key_in).shape[1]
    else:
        K_in = 1
    if key_in is not None:
        key_in = np.ascontiguousarray(key_in, dtype=np.uint64)
        assert key_in.shape == (B, K_in)
    if score_in is not None:
        score_in = np.ascontiguousarray(score_in, dtype=np.float32)
        assert score_in.shape == (B, K_in)
    want_state = want_state and level < L and E_l is not None
    if E_l is not None:
        E_l = np.ascontiguousarray(E_l, dtype=np.float32)
        assert E_l.shape == (V, e)
    out = {
        "key": np.empty((B, K), dtype=np.uint64),
        "score": np.empty((B, K), dtype=np.float32),
        "parent": np.empty((B, K), dtype=np.int32),
        "code": np.empty((B, K), dtype=np.int32),
        "count": np.empty(B, dtype=np.int32),
    }
    state_out = np.empty((B, K, e), dtype=np.float32) if want_state else None
    logp = np.empty((B, K_in, V), dtype=np.float64) if want_logp else None
    if threads is None:
        threads = os.cpu_count() or 1
    if U_l is not None:
        U_l = np.ascontiguousarray(U_l, dtype=np.float32)
        assert U_l.shape == (e, e)
    rc = lib().orc_draft_level(
        C.c_int32(B), C.c_int32(L), C.c_int32(level), C.c_int32(K), C.c_int32(K_in),
        C.c_int32(d), C.c_int32(e), _p(rad), _p(H_l), C.c_int64(d), _p(W_l), _p(E_l),
        _p(state_in), _p(key_in), _p(score_in),
        C.c_void_p(itemset._h) if itemset is not None else None,
        _p(U_l), C.c_int(0 if U_l is None else 1),
        C.c_int(1 if round_state_bf16 else 0), _p(out["key"]), _p(out["score"]),
        _p(out["parent"]), _p(out["code"]), _p(state_out), _p(out["count"]), _p(logp),
        C.c_int(int(threads)))
    if rc != 0:
        raise ValueError("orc_draft_level failed (%d)" % rc)
    if want_state:
        out["state"] = state_out
    if want_logp:
        out["logp"] = logp
    return out


def decode(H, W, E, radices, K, itemset=None, round_state_bf16=False, threads=None, U=None,
           prefix_sets=None, use_state=True):
    """All L levels of Alg. 3 (inference) chained.  H [B,L,d]; W, E lists per
    level; U (optional) list of [e,e] per level below L: recurrent Transition;
    prefix_sets (optional) list of L-1 sets (or None) of valid prefixes of length 1..L-1.
    Returns the list of per-level outputs; the last one is the answer."""
    L = len(W)
    B_ = H.shape[0]
    outs = []
    state = key = score = None
    for l in range(1, L + 1):
        s = itemset if l == L else (prefix_sets[l - 1] if prefix_sets else None)
        o = draft_level(l, L, radices, K, H[:, l - 1, :], W[l - 1],
                        E[l - 1] if l < L else None, state if use_state else None, key, score,
                        s, round_state_bf16, threads=threads,
                        U_l=U[l - 1] if (U is not None and l < L) else None)
        outs.append(o)
        state, key, score = o.get("state"), o["key"], o["score"]
        if l < L and B_:
            # drop the slots that are empty in every request (without verification below the
            # last level all requests keep the same number: min(K, live beams * codes))
            cnt = int(o["count"].max())
            if not prefix_sets:
                assert (o["count"] == cnt).all()
            cnt = max(cnt, 1)
            state, key, score = state[:, :cnt], key[:, :cnt], score[:, :cnt]
    return outs
