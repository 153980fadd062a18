"""ctypes binding of libnezha.so (see include/nezha.h for the contract of each call).
Argument marshalling only."""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

NEZHA_F32, NEZHA_BF16 = 0, 1
NEZHA_TRANSITION_ADD, NEZHA_TRANSITION_RNN = 0, 1
MAX_LEVELS = 8

EXPORTS = ["nezha_last_error", "nezha_build_itemset", "nezha_itemset_info", "nezha_free_itemset",
           "nezha_verify_tuples", "nezha_verify_workspace", "nezha_draft_step",
           "nezha_draft_step_workspace", "nezha_unpack_keys", "nezha_profile_enable",
           "nezha_profile_reset", "nezha_profile_kinds", "nezha_profile_read",
           "nezha_bench_random_gather", "nezha_user_projection", "nezha_pack_weights",
           "nezha_packed_weights_bytes", "nezha_user_projection_levels", "nezha_draft_levels", "nezha_decode",
           "nezha_profile_event_overhead",
           "nezha_draft_levels_workspace", "nezha_check_itemset", "nezha_verify_tuples_static",
           "nezha_bench_mfma_rate", "nezha_bench_random_gather_depth", "nezha_bench_tile_step"]


class NezhaError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("nezha error %d: %s" % (code, text))
        self.code = code


class _StepDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("L", C.c_int32), ("level", C.c_int32), ("K", C.c_int32),
                ("K_in", C.c_int32), ("d", C.c_int32), ("e", C.c_int32),
                ("radices", C.POINTER(C.c_int32)), ("dtype", C.c_int),
                ("h_row_stride", C.c_int64), ("w_packed", C.c_int32),
                ("user_part", C.c_void_p), ("transition", C.c_int32), ("U_l", C.c_void_p),
                ("state_init", C.c_void_p)]


class _LevelIO(C.Structure):
    _fields_ = [("H_l", C.c_void_p), ("W_l", C.c_void_p), ("E_l", C.c_void_p), ("set", C.c_void_p),
                ("user_part", C.c_void_p), ("U_l", C.c_void_p), ("key_out", C.c_void_p),
                ("score_out", C.c_void_p), ("parent_out", C.c_void_p), ("code_out", C.c_void_p),
                ("state_out", C.c_void_p), ("count_out", C.c_void_p)]


def library_path():
    return os.path.join(_HERE, "libnezha.so")


def load_library():
    """Loads the built library; builds it first only if no built library exists."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    lib = C.CDLL(path)
    lib.nezha_last_error.restype = C.c_char_p
    lib.nezha_verify_workspace.restype = C.c_size_t
    lib.nezha_verify_workspace.argtypes = [C.c_int64]
    lib.nezha_draft_step_workspace.restype = C.c_size_t
    lib.nezha_draft_step_workspace.argtypes = [C.POINTER(_StepDesc)]
    lib.nezha_build_itemset.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int,
                                        C.c_double, C.c_void_p, C.POINTER(C.c_void_p)]
    lib.nezha_itemset_info.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                       C.POINTER(C.c_int32), C.c_void_p]
    lib.nezha_free_itemset.argtypes = [C.c_void_p]
    lib.nezha_verify_tuples.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.nezha_draft_step.argtypes = [C.POINTER(_StepDesc)] + [C.c_void_p] * 14 + [C.c_size_t,
                                                                                  C.c_void_p]
    lib.nezha_unpack_keys.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    lib.nezha_verify_tuples_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                               C.c_void_p, C.c_void_p, C.c_void_p]
    lib.nezha_check_itemset.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p,
                                        C.POINTER(C.c_int64)]
    _LIB = lib
    return lib


def _check(rc):
    if rc != 0:
        raise NezhaError(rc, load_library().nezha_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _radices(radices):
    arr = (C.c_int32 * len(radices))(*[int(r) for r in radices])
    return arr


class ItemSet:
    """Owner of a device-resident nezha_itemset."""

    def __init__(self, handle, L, radices):
        self._h = handle
        self.L = L
        self.radices = list(radices)

    def info(self):
        n, slots, L = C.c_int64(), C.c_int64(), C.c_int32()
        rad = (C.c_int32 * MAX_LEVELS)()
        _check(load_library().nezha_itemset_info(self._h, C.byref(n), C.byref(slots), C.byref(L), rad))
        return {"n_distinct": n.value, "n_slots": slots.value, "L": L.value,
                "radices": list(rad[:L.value])}

    def check(self, codes, stream=None):
        """nezha_check_itemset: how many of the tuples `codes` (int32 [n, L], numpy / CPU tensor or
        CUDA tensor) the set does not find; 0 for the catalog it was built from."""
        if isinstance(codes, np.ndarray):
            codes = torch.from_numpy(np.ascontiguousarray(codes, dtype=np.int32))
        codes = codes.contiguous()
        missing = C.c_int64(-1)
        _check(load_library().nezha_check_itemset(self._h, _ptr(codes) if codes.numel() else None,
                                                  codes.shape[0], 1 if codes.is_cuda else 0,
                                                  _stream(stream), C.byref(missing)))
        return missing.value

    def close(self):
        if self._h is not None:
            h, self._h = self._h, None
            _check(load_library().nezha_free_itemset(h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def build_itemset(codes, radices, load_factor=0.5, stream=None):
    """nezha_build_itemset.  codes: int32 [n, L], a CPU tensor / numpy array (host
    pointer) or a CUDA tensor (device pointer)."""
    lib = load_library()
    if isinstance(codes, np.ndarray):
        codes = torch.from_numpy(np.ascontiguousarray(codes, dtype=np.int32))
    codes = codes.contiguous()
    if codes.dtype != torch.int32 or codes.dim() != 2 or codes.shape[1] != len(radices):
        raise ValueError("codes must be int32 [n, L]")
    out = C.c_void_p()
    rad = _radices(radices)
    on_dev = 1 if codes.is_cuda else 0
    s = _stream(stream) if torch.cuda.is_available() else None
    _check(lib.nezha_build_itemset(_ptr(codes) if codes.numel() else None, codes.shape[0],
                                   len(radices), rad, on_dev, float(load_factor), s,
                                   C.byref(out)))
    return ItemSet(out, len(radices), radices)


def verify_workspace(n):
    return int(load_library().nezha_verify_workspace(int(n)))


def verify_tuples(itemset, codes, out_mask=None, out_index=None, out_count=None, workspace=None,
                  want_index=True, stream=None):
    """nezha_verify_tuples on a CUDA int32 [n, L] tensor.  Returns (mask uint8 [n],
    index int64 [n] (first count entries valid), count int64 [1]); tensors are
    allocated here unless given."""
    n = codes.shape[0]
    dev = codes.device
    if out_mask is None:
        out_mask = torch.empty(n, dtype=torch.uint8, device=dev)
    if want_index and out_index is None:
        out_index = torch.empty(n, dtype=torch.int64, device=dev)
    if want_index and out_count is None:
        out_count = torch.empty(1, dtype=torch.int64, device=dev)
    if workspace is None:
        workspace = torch.empty(max(16, verify_workspace(n)), dtype=torch.uint8, device=dev)
    _check(load_library().nezha_verify_tuples(itemset._h, _ptr(codes), n, _ptr(out_mask),
                                              _ptr(out_index), _ptr(out_count), _ptr(workspace),
                                              workspace.numel(), _stream(stream)))
    return out_mask, out_index, out_count


VERIFY_STATIC_MAX = 32 * 1024 * 1024


def verify_tuples_static(itemset, codes, out_mask, out_index=None, out_count=None, stream=None):
    """nezha_verify_tuples_static: the verifier with its scratch in a fixed device array of the
    library; the caller passes every output (nothing is allocated here or in the library)."""
    _check(load_library().nezha_verify_tuples_static(itemset._h, _ptr(codes), codes.shape[0],
                                                     _ptr(out_mask), _ptr(out_index),
                                                     _ptr(out_count), _stream(stream)))
    return out_mask, out_index, out_count


def _desc(B, L, level, K, K_in, d, e, radices, dtype, h_row_stride, w_packed=False,
          user_part=None, U_l=None, state_init=None):
    rad = _radices(radices)
    dsc = _StepDesc(B, L, level, K, K_in, d, e, C.cast(rad, C.POINTER(C.c_int32)),
                    NEZHA_BF16 if dtype == torch.bfloat16 else NEZHA_F32, h_row_stride,
                    1 if w_packed else 0, None if user_part is None else user_part.data_ptr(),
                    NEZHA_TRANSITION_ADD if U_l is None else NEZHA_TRANSITION_RNN,
                    None if U_l is None else U_l.data_ptr(),
                    None if state_init is None else state_init.data_ptr())
    dsc._keep = rad
    return dsc


class PackedWeights:
    """W_l in the kernels' operand order (nezha_pack_weights); pass it where W_l is expected."""

    def __init__(self, data, d, e, V):
        self.data, self.d, self.e, self.V = data, d, e, V

    @property
    def shape(self):
        return (self.d + self.e, self.V)

    def data_ptr(self):
        return self.data.data_ptr()


def pack_weights(level, L, radices, W_l, d, stream=None):
    """nezha_pack_weights for a bf16 W_l [(d+e), T_level]; returns a PackedWeights."""
    lib = load_library()
    V = int(radices[level - 1])
    e = W_l.shape[0] - d
    dsc = _desc(1, L, level, 1, 1, d, e, radices, W_l.dtype, d)
    lib.nezha_packed_weights_bytes.restype = C.c_size_t
    lib.nezha_packed_weights_bytes.argtypes = [C.POINTER(_StepDesc)]
    n = int(lib.nezha_packed_weights_bytes(C.byref(dsc)))
    if n == 0:
        raise NezhaError(-1, "these weights cannot be packed (bf16 only; check the shapes)")
    out = torch.empty(n, dtype=torch.uint8, device=W_l.device)
    lib.nezha_pack_weights.argtypes = [C.POINTER(_StepDesc), C.c_void_p, C.c_void_p, C.c_void_p]
    _check(lib.nezha_pack_weights(C.byref(dsc), _ptr(W_l), _ptr(out), _stream(stream)))
    return PackedWeights(out, d, e, V)


def draft_step_workspace(B, L, level, K, K_in, d, e, radices, dtype, w_packed=False):
    dsc = _desc(B, L, level, K, K_in, d, e, radices, dtype, d, w_packed)
    return int(load_library().nezha_draft_step_workspace(C.byref(dsc)))


def draft_step(level, L, radices, K, H_l, W_l, E_l=None, state_in=None, key_in=None,
               score_in=None, itemset=None, out=None, workspace=None, stream=None,
               h_row_stride=None, user_part=None, U_l=None):
    """nezha_draft_step for one level.  H_l [B, d] (a view with a row stride is
    fine), W_l [(d+e), V], E_l [V, e]; state_in [B, K_in, e], key_in int64-as-uint64
    [B, K_in], score_in float32 [B, K_in].  itemset: the items (used at level L) or the
    valid prefixes of length `level`.  U_l [e, e]: recurrent Transition (NEZHA_TRANSITION_RNN).
    `out` may hold preallocated tensors key, score, parent, code, state, count.  Returns that
    dict."""
    B, d = H_l.shape
    V = int(radices[level - 1])
    e = W_l.shape[0] - d
    dev, dt = H_l.device, H_l.dtype
    if h_row_stride is None:
        h_row_stride = H_l.stride(0) if B > 1 else d
    K_in = 1 if key_in is None and state_in is None else (
        state_in.shape[1] if state_in is not None else key_in.shape[1])
    if out is None:
        out = {}
    out.setdefault("key", torch.empty((B, K), dtype=torch.int64, device=dev))
    out.setdefault("score", torch.empty((B, K), dtype=torch.float32, device=dev))
    out.setdefault("parent", torch.empty((B, K), dtype=torch.int32, device=dev))
    out.setdefault("code", torch.empty((B, K), dtype=torch.int32, device=dev))
    out.setdefault("count", torch.empty((B,), dtype=torch.int32, device=dev))
    if level < L and "state" not in out:
        out["state"] = torch.empty((B, K, e), dtype=dt, device=dev)
    dsc = _desc(B, L, level, K, K_in, d, e, radices, dt, h_row_stride,
                isinstance(W_l, PackedWeights), user_part, U_l if level < L else None)
    if workspace is None:
        need = int(load_library().nezha_draft_step_workspace(C.byref(dsc)))
        workspace = torch.empty(max(256, need), dtype=torch.uint8, device=dev)
    _check(load_library().nezha_draft_step(
        C.byref(dsc), _ptr(H_l), _ptr(W_l), _ptr(E_l), _ptr(state_in), _ptr(key_in),
        _ptr(score_in), itemset._h if itemset is not None else None, _ptr(out["key"]),
        _ptr(out["score"]), _ptr(out["parent"]), _ptr(out["code"]), _ptr(out.get("state")),
        _ptr(out["count"]), _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def user_projection(level, L, radices, H_l, W_l, out=None, workspace=None, stream=None,
                    h_row_stride=None):
    """nezha_user_projection: float32 [B, T_level] = H_l @ W_l[:d]."""
    B, d = H_l.shape
    V = int(radices[level - 1])
    e = W_l.shape[0] - d
    if h_row_stride is None:
        h_row_stride = H_l.stride(0) if B > 1 else d
    if out is None:
        out = torch.empty((B, V), dtype=torch.float32, device=H_l.device)
    dsc = _desc(B, L, level, 1, 1, d, e, radices, H_l.dtype, h_row_stride,
                isinstance(W_l, PackedWeights))
    lib = load_library()
    if workspace is None:
        need = int(lib.nezha_draft_step_workspace(C.byref(dsc)))
        workspace = torch.empty(max(256, need), dtype=torch.uint8, device=H_l.device)
    lib.nezha_user_projection.argtypes = [C.POINTER(_StepDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_size_t, C.c_void_p]
    _check(lib.nezha_user_projection(C.byref(dsc), _ptr(H_l), _ptr(W_l), _ptr(out),
                                     _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def user_projection_levels(H, Wp, radices, out, stream=None):
    """nezha_user_projection_levels: H [B, L, d] (bf16), Wp list of PackedWeights, out list of
    float32 [B, T_l] tensors; one launch for all levels."""
    L = len(Wp)
    B, _, d = H.shape
    dsc = _desc(B, L, 1, 1, 1, d, Wp[0].e, radices, H.dtype, H.stride(0), True)
    esz = H.element_size()
    hp = (C.c_void_p * L)(*[H.data_ptr() + l * H.stride(1) * esz for l in range(L)])
    wp = (C.c_void_p * L)(*[w.data_ptr() for w in Wp])
    ap = (C.c_void_p * L)(*[o.data_ptr() for o in out])
    lib = load_library()
    lib.nezha_user_projection_levels.argtypes = [C.POINTER(_StepDesc), C.c_int32, C.c_void_p,
                                                 C.c_void_p, C.c_void_p, C.c_void_p]
    _check(lib.nezha_user_projection_levels(C.byref(dsc), L, hp, wp, ap, _stream(stream)))
    return out


class DraftBuffers:
    """Preallocated outputs and workspace for a full L-level decode, so that the
    timed loop allocates nothing."""

    def __init__(self, B, L, K, d, e, radices, dtype, device):
        self.outs = []
        need = 256
        for level in range(1, L + 1):
            K_in = 1 if level == 1 else K
            need = max(need, draft_step_workspace(B, L, level, K, K_in, d, e, radices, dtype))
            o = {"key": torch.empty((B, K), dtype=torch.int64, device=device),
                 "score": torch.empty((B, K), dtype=torch.float32, device=device),
                 "parent": torch.empty((B, K), dtype=torch.int32, device=device),
                 "code": torch.empty((B, K), dtype=torch.int32, device=device),
                 "count": torch.empty((B,), dtype=torch.int32, device=device)}
            if level < L:
                o["state"] = torch.empty((B, K, e), dtype=dtype, device=device)
            self.outs.append(o)
        self.workspace = torch.empty(need, dtype=torch.uint8, device=device)
        self.user_parts = [torch.empty((B, int(radices[l])), dtype=torch.float32, device=device)
                           for l in range(L)]


def _dp(t):
    return None if t is None else t.data_ptr()


def draft_levels(H, W, E, radices, K, itemset=None, buffers=None, stream=None, U=None,
                 prefix_sets=None, user_parts=None, state_init=None):
    """nezha_draft_levels: all L levels in one C call (one kernel launch when every level is
    small and `user_parts` are given).  Arguments as for decode(); state_init [B, 1, e]: the state
    level 1 starts from (None = zeros)."""
    L = len(W)
    B, _, d = H.shape
    e = W[0].shape[0] - d
    if buffers is None:
        buffers = DraftBuffers(B, L, K, d, e, radices, H.dtype, H.device)
    packed = all(isinstance(w, PackedWeights) for w in W)
    if not packed and any(isinstance(w, PackedWeights) for w in W):
        raise ValueError("either all or none of the W_l may be packed")
    dsc = _desc(B, L, 1, K, 1, d, e, radices, H.dtype, H.stride(0), packed, None,
                U[0] if U is not None else None, state_init)
    esz = H.element_size()
    io = (_LevelIO * L)()
    for l in range(L):
        o = buffers.outs[l]
        s = itemset if l == L - 1 else (prefix_sets[l] if prefix_sets else None)
        io[l] = _LevelIO(H.data_ptr() + l * H.stride(1) * esz, W[l].data_ptr(),
                         _dp(E[l]) if l < L - 1 else None, s._h if s is not None else None,
                         _dp(user_parts[l]) if user_parts is not None else None,
                         _dp(U[l]) if (U is not None and l < L - 1) else None,
                         o["key"].data_ptr(), o["score"].data_ptr(), o["parent"].data_ptr(),
                         o["code"].data_ptr(), _dp(o.get("state")), o["count"].data_ptr())
    lib = load_library()
    lib.nezha_draft_levels.argtypes = [C.POINTER(_StepDesc), C.POINTER(_LevelIO), C.c_void_p,
                                       C.c_size_t, C.c_void_p]
    _check(lib.nezha_draft_levels(C.byref(dsc), io, _ptr(buffers.workspace),
                                  buffers.workspace.numel(), _stream(stream)))
    return buffers.outs


class DecodePlan:
    """Everything nezha_decode needs for one fixed set of buffers, marshalled once: run() is a
    single foreign call (what a serving loop would do per batch).  bf16 with packed weights."""

    def __init__(self, H, W, E, radices, K, itemset=None, buffers=None, stream=None, U=None,
                 prefix_sets=None, state_init=None):
        L = len(W)
        B, _, d = H.shape
        if not all(isinstance(w, PackedWeights) for w in W):
            raise ValueError("DecodePlan needs weights from pack_weights")
        e = W[0].shape[0] - d
        self.buffers = buffers if buffers is not None else DraftBuffers(B, L, K, d, e, radices,
                                                                        H.dtype, H.device)
        self._keep = (H, W, E, U, itemset, prefix_sets, state_init)   # the memory the pointers refer to
        self._dsc = _desc(B, L, 1, K, 1, d, e, radices, H.dtype, H.stride(0), True, None,
                          U[0] if U is not None else None, state_init)
        esz = H.element_size()
        self._io = (_LevelIO * L)()
        for l in range(L):
            o = self.buffers.outs[l]
            s = itemset if l == L - 1 else (prefix_sets[l] if prefix_sets else None)
            self._io[l] = _LevelIO(H.data_ptr() + l * H.stride(1) * esz, W[l].data_ptr(),
                                   _dp(E[l]) if l < L - 1 else None, s._h if s is not None else None,
                                   self.buffers.user_parts[l].data_ptr(),
                                   _dp(U[l]) if (U is not None and l < L - 1) else None,
                                   o["key"].data_ptr(), o["score"].data_ptr(),
                                   o["parent"].data_ptr(), o["code"].data_ptr(),
                                   _dp(o.get("state")), o["count"].data_ptr())
        lib = load_library()
        lib.nezha_decode.argtypes = [C.POINTER(_StepDesc), C.POINTER(_LevelIO), C.c_void_p,
                                     C.c_size_t, C.c_void_p]
        self._fn = lib.nezha_decode
        self._dref = C.byref(self._dsc)
        self._ws = _ptr(self.buffers.workspace)
        self._ws_bytes = self.buffers.workspace.numel()
        self._stream = stream

    def run(self):
        rc = self._fn(self._dref, self._io, self._ws, self._ws_bytes, _stream(self._stream))
        if rc != 0:
            _check(rc)
        return self.buffers.outs


def decode(H, W, E, radices, K, itemset=None, buffers=None, stream=None, U=None,
           prefix_sets=None, use_state=True, level_events=None, state_init=None):
    """All L levels of the inference loop of Alg. 3: L calls of nezha_draft_step on one
    stream, each level's outputs feeding the next.  H [B, L, d]; W, E lists per level; U
    (optional) list of [e, e] per level below L: recurrent Transition; prefix_sets (optional)
    list of L-1 item sets (or None) of the valid prefixes of length 1..L-1; use_state=False
    never hands a state to the next level (the head then sees h_l only: the paper's ablation
    without the autoregressive state, and parallel multi-token heads when all h_l are equal).
    state_init [B, 1, e]: the state the single beam of level 1 starts from (None = zeros).
    level_events (measurement aid): L+1 pairs of torch.cuda.Event recorded on the current
    stream around the projections made ahead of the loop (pair 0) and around each level's call
    (pairs 1..L)."""
    L = len(W)
    B, _, d = H.shape
    e = W[0].shape[0] - d
    if buffers is None:
        buffers = DraftBuffers(B, L, K, d, e, radices, H.dtype, H.device)
    state, key, score = state_init, None, None
    parts = None
    if level_events is not None:
        level_events[0][0].record()
    if all(isinstance(w, PackedWeights) for w in W):
        # the projections of h_1..h_L do not depend on the beams: one launch before the loop
        parts = user_projection_levels(H, W, radices, buffers.user_parts, stream=stream)
    if level_events is not None:
        level_events[0][1].record()
    if parts is not None and use_state and level_events is None:
        # the level loop itself in one call (one launch when every level is small)
        return draft_levels(H, W, E, radices, K, itemset, buffers, stream, U, prefix_sets, parts,
                            state_init)
    for level in range(1, L + 1):
        if level_events is not None:
            level_events[level][0].record()
        o = draft_step(level, L, radices, K, H[:, level - 1, :], W[level - 1],
                       E[level - 1] if level < L else None, state if use_state else None, key,
                       score,
                       itemset if level == L else (prefix_sets[level - 1] if prefix_sets else None),
                       out=buffers.outs[level - 1],
                       workspace=buffers.workspace, stream=stream, h_row_stride=H.stride(0),
                       user_part=None if parts is None else parts[level - 1],
                       U_l=U[level - 1] if (U is not None and level < L) else None)
        if level_events is not None:
            level_events[level][1].record()
        state, key, score = o.get("state"), o["key"], o["score"]
    return buffers.outs


def bench_random_gather(buf, n, line_bytes=64, seed=1, stream=None, depth=4, lanes_per_line=1,
                        sink=None):
    """nezha_bench_random_gather_depth over the CUDA tensor `buf` (any dtype, 128-byte aligned)."""
    if sink is None:
        sink = torch.zeros(1, dtype=torch.int64, device=buf.device)
    lib = load_library()
    lib.nezha_bench_random_gather_depth.argtypes = [C.c_void_p, C.c_size_t, C.c_int64, C.c_int,
                                                    C.c_int, C.c_int, C.c_uint64, C.c_void_p,
                                                    C.c_void_p]
    _check(lib.nezha_bench_random_gather_depth(_ptr(buf), buf.numel() * buf.element_size(), int(n),
                                               int(line_bytes), int(depth), int(lanes_per_line),
                                               int(seed), _ptr(sink), _stream(stream)))
    return sink


def bench_mfma_rate(operands, iters=2000, workgroups=256, stream=None):
    """nezha_bench_mfma_rate on the values of the CUDA tensor `operands`.  Returns (TFLOP/s summed
    over the workgroups' own loop times, core clock in MHz during the loop)."""
    dev = operands.device
    ticks = torch.zeros(2 * workgroups, dtype=torch.int64, device=dev)
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    lib = load_library()
    lib.nezha_bench_mfma_rate.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
    _check(lib.nezha_bench_mfma_rate(_ptr(operands), operands.numel() * operands.element_size(),
                                     int(iters), int(workgroups), _ptr(ticks), _ptr(sink),
                                     _stream(stream)))
    torch.cuda.synchronize()
    t = ticks.cpu().numpy().reshape(workgroups, 2).astype(np.float64)
    seconds = t[:, 1] / 100e6
    flops_per_wg = 4.0 * iters * 32 * 32768
    return float((flops_per_wg / seconds).sum() / 1e12), float((t[:, 0] / t[:, 1]).mean() * 100.0)


def bench_tile_step(mode, waves_per_simd=4, iters=20000, stream=None):
    """nezha_bench_tile_step with `waves_per_simd` waves on every SIMD of the device.  Returns
    (tile steps per second and SIMD, core clock in MHz during the loop)."""
    dev = torch.device("cuda", torch.cuda.current_device())
    n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
    workgroups = n_cu * int(waves_per_simd)
    g = torch.Generator().manual_seed(1)
    values = (torch.rand(256, generator=g) - 0.5).to(dev)
    ticks = torch.zeros(2 * workgroups, dtype=torch.int64, device=dev)
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    lib = load_library()
    lib.nezha_bench_tile_step.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s = stream if stream is not None else torch.cuda.current_stream()
    for timed in (False, True):
        if timed:
            start.record(s)
        _check(lib.nezha_bench_tile_step(int(mode), int(iters), workgroups, _ptr(values),
                                         _ptr(ticks), _ptr(sink), _stream(stream)))
    stop.record(s)
    torch.cuda.synchronize()
    seconds = start.elapsed_time(stop) * 1e-3
    t = ticks.cpu().numpy().reshape(workgroups, 2).astype(np.float64)
    steps_per_simd = float(waves_per_simd) * iters      # a SIMD holds that many waves, each does iters
    return steps_per_simd / seconds, float((t[:, 0] / t[:, 1]).mean() * 100.0)


def profile_enable(on):
    _check(load_library().nezha_profile_enable(1 if on else 0))


def profile_reset():
    _check(load_library().nezha_profile_reset())


def profile_read():
    """{kernel name: (launches, total milliseconds)} for every kernel kind that ran."""
    lib = load_library()
    out = {}
    for kind in range(lib.nezha_profile_kinds()):
        name, n, ms = C.c_char_p(), C.c_int64(), C.c_double()
        _check(lib.nezha_profile_read(kind, C.byref(name), C.byref(n), C.byref(ms)))
        if n.value:
            out[name.value.decode()] = (n.value, ms.value)
    return out


def profile_event_overhead(launches=200, stream=None):
    """Microseconds the library's event bracket reports for an empty kernel."""
    lib = load_library()
    lib.nezha_profile_event_overhead.argtypes = [C.c_int, C.c_void_p, C.POINTER(C.c_double)]
    us = C.c_double()
    _check(lib.nezha_profile_event_overhead(int(launches), _stream(stream), C.byref(us)))
    return us.value


def unpack_keys(keys, radices):
    """Inverse of Eq. 4 on the host (nezha_unpack_keys): uint64/int64 [n] -> int32 [n, L]."""
    k = np.ascontiguousarray(np.asarray(keys).astype(np.uint64, copy=False).ravel())
    out = np.empty((k.size, len(radices)), dtype=np.int32)
    rad = _radices(radices)
    _check(load_library().nezha_unpack_keys(k.ctypes.data_as(C.c_void_p), k.size, len(radices),
                                            rad, out.ctypes.data_as(C.c_void_p)))
    return out
