"""Float64 CPU oracle of the DynTS decode hot path.  TEST INFRASTRUCTURE ONLY.

Thin ctypes binding of oracle/dynts_oracle.c plus `OracleLayer`, a plain driver
that takes the steps of one decode iteration in the paper's order (Sec. 4.2):
append -> attend (Eq. attn-score, Eq. attn-o) -> score accumulation
(Eq. importance-score, running form) -> on trigger: select, evict.

Nothing here is used by the product path; the HIP library never imports it and
shares no code with it.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = None

_f64 = np.float64
_i32 = np.int32
_u8 = np.uint8


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        L.dynts_oracle_break_even_volume.restype = C.c_double
        L.dynts_oracle_break_even_volume.argtypes = [C.c_double] * 3
        L.dynts_oracle_mlp_flops.restype = C.c_double
        L.dynts_oracle_mlp_flops.argtypes = [C.c_double] * 4
        L.dynts_oracle_attn_flops.restype = C.c_double
        L.dynts_oracle_attn_flops.argtypes = [C.c_double] * 3
        _lib = L
    return _lib


def _p(a, dtype):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (
        "oracle arrays must be C-contiguous %s" % dtype)
    return a.ctypes.data_as(C.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError("oracle %s failed with code %d" % (what, rc))


def max_threads():
    return int(lib().dynts_oracle_max_threads())


def set_threads(n):
    lib().dynts_oracle_set_threads(C.c_int(int(n)))


def append(K, V, S, pos, seq_len, next_pos, k_new, v_new, s_new=None, active=None):
    Nb, Hkv, cap, d = K.shape
    _check(lib().dynts_oracle_append(Nb, Hkv, d, cap, _p(k_new, _f64), _p(v_new, _f64),
                                     _p(s_new, _f64), _p(active, _u8), _p(K, _f64), _p(V, _f64),
                                     _p(S, _f64), _p(pos, _i32), _p(seq_len, _i32),
                                     _p(next_pos, _i32)), "append")


def attend(q, K, V, seq_len, scale, active=None, out=None, want_alpha=True):
    """Returns (out [Nb][Hq][d], alpha [Nb][Hq][cap] or None, lse [Nb][Hq])."""
    Nb, Hkv, cap, d = K.shape
    Hq = q.shape[1]
    if out is None:
        out = np.zeros((Nb, Hq, d), _f64)
    alpha = np.zeros((Nb, Hq, cap), _f64) if want_alpha else None
    lse = np.zeros((Nb, Hq), _f64)
    _check(lib().dynts_oracle_attend(Nb, Hq, Hkv, d, cap, _p(q, _f64), _p(K, _f64), _p(V, _f64),
                                     _p(seq_len, _i32), _p(active, _u8), C.c_double(scale),
                                     _p(out, _f64), _p(alpha, _f64), _p(lse, _f64)), "attend")
    return out, alpha, lse


def update_scores(S, alpha, seq_len, n_prompt, active=None):
    Nb, Hkv, cap = S.shape
    Hq = alpha.shape[1]
    _check(lib().dynts_oracle_update_scores(Nb, Hq, Hkv, cap, _p(alpha, _f64), _p(seq_len, _i32),
                                            _p(n_prompt, _i32), _p(active, _u8), _p(S, _f64)),
           "update_scores")


def score_block(q_blk, k_blk, K, seq_len, scale, active=None, I=None):
    """Eq. importance-score for a block of queries: q_blk [Nb][T][Hq][d], k_blk [Nb][T][Hkv][d] or None
    (the block's own keys, seen causally).  Returns I [Nb][Hkv][cap] (added to the I passed in, if any)."""
    Nb, T, Hq, d = q_blk.shape
    _, Hkv, cap, _ = K.shape
    if I is None:
        I = np.zeros((Nb, Hkv, cap), _f64)
    _check(lib().dynts_oracle_score_block(Nb, T, Hq, Hkv, d, cap, _p(q_blk, _f64), _p(k_blk, _f64), _p(K, _f64),
                                          _p(seq_len, _i32), _p(active, _u8), C.c_double(scale), _p(I, _f64)),
           "score_block")
    return I


ACT_NONE, ACT_RELU, ACT_SILU = 0, 1, 2


def predictor(h, W1, b1, W2, b2, w3, b3, act=ACT_RELU):
    """Importance Predictor MLP d -> m1 -> m2 -> 1 (Sec. 4.1, App. A): h [Nb][d] -> s [Nb]."""
    Nb, d = h.shape
    m1, m2 = W1.shape[0], W2.shape[0]
    assert W1.shape == (m1, d) and W2.shape == (m2, m1) and w3.shape == (m2,)
    s = np.zeros((Nb,), _f64)
    _check(lib().dynts_oracle_predictor(Nb, d, m1, m2, _p(h, _f64), _p(W1, _f64), _p(b1, _f64), _p(W2, _f64),
                                        _p(b2, _f64), _p(w3, _f64), _p(b3, _f64), int(act), _p(s, _f64)),
           "predictor")
    return s


def select(S, pos, seq_len, n_prompt, window, k_keep, trigger=None, keep_stride=None):
    """Returns (keep_idx [Nb][Hkv][keep_stride] (-1 padded), new_len [Nb])."""
    Nb, Hkv, cap = S.shape
    if keep_stride is None:
        keep_stride = cap
    keep_idx = np.full((Nb, Hkv, keep_stride), -1, _i32)
    new_len = np.zeros((Nb,), _i32)
    _check(lib().dynts_oracle_select(Nb, Hkv, cap, _p(S, _f64), _p(pos, _i32), _p(seq_len, _i32),
                                     _p(n_prompt, _i32), _p(trigger, _u8), int(window),
                                     int(k_keep), int(keep_stride), _p(keep_idx, _i32),
                                     _p(new_len, _i32)), "select")
    return keep_idx, new_len


def compact(K, V, S, pos, seq_len, keep_idx, new_len, trigger=None):
    Nb, Hkv, cap, d = K.shape
    _check(lib().dynts_oracle_compact(Nb, Hkv, d, cap, _p(trigger, _u8), _p(keep_idx, _i32),
                                      int(keep_idx.shape[2]), _p(new_len, _i32), _p(K, _f64),
                                      _p(V, _f64), _p(S, _f64), _p(pos, _i32), _p(seq_len, _i32)),
           "compact")


def eviction_events(M, i, B, K):
    return int(lib().dynts_oracle_eviction_events(int(M), int(i), int(B), int(K)))


def effective_length(M, i, B, K):
    return int(lib().dynts_oracle_effective_length(int(M), int(i), int(B), int(K)))


def mlp_flops(d, m1, m2, m3):
    return float(lib().dynts_oracle_mlp_flops(d, m1, m2, m3))


def attn_flops(L, d, S):
    return float(lib().dynts_oracle_attn_flops(L, d, S))


def break_even_volume(d, L, n_events):
    return float(lib().dynts_oracle_break_even_volume(d, L, n_events))


class OracleLayer:
    """One attention layer's compressed KV cache and its decode step, in float64.

    budget/window/evict_every follow the benchmark's reading of Sec. 4.2: after a
    trigger the selection window holds `budget` slots and the local window
    `window` slots; a trigger falls on the step at which a sequence's thinking
    tokens reach budget+window+evict_every, i.e. every `evict_every`-th step from
    then on.  In the paper's notation the
    total budget is B = M + budget + window + evict_every and the eviction volume
    is K = evict_every.
    """

    def __init__(self, batch, n_q_heads, n_kv_heads, head_dim, capacity, budget, window,
                 evict_every, softmax_scale=None, external_scores=False):
        self.Nb, self.Hq, self.Hkv, self.d, self.cap = batch, n_q_heads, n_kv_heads, head_dim, capacity
        self.budget, self.window, self.evict_every = budget, window, evict_every
        self.scale = float(softmax_scale) if softmax_scale else 1.0 / np.sqrt(head_dim)
        self.external = bool(external_scores)
        self.K = np.zeros((batch, n_kv_heads, capacity, head_dim), _f64)
        self.V = np.zeros_like(self.K)
        self.S = np.zeros((batch, n_kv_heads, capacity), _f64)
        self.pos = np.zeros((batch, n_kv_heads, capacity), _i32)
        self.seq_len = np.zeros((batch,), _i32)
        self.n_prompt = np.zeros((batch,), _i32)
        self.next_pos = np.zeros((batch,), _i32)
        self.steps_done = np.zeros((batch,), np.int64)

    def prefill(self, K0, V0, m):
        """Question window (Sec. 4.2): K0,V0 [Nb][Hkv][Mmax][d]; m [Nb] prompt lengths; score +inf."""
        for b in range(self.Nb):
            M = int(m[b])
            self.K[b, :, :M] = K0[b, :, :M]
            self.V[b, :, :M] = V0[b, :, :M]
            self.S[b, :, :M] = np.inf
            self.pos[b, :, :M] = np.arange(M, dtype=_i32)[None, :]
            self.seq_len[b] = M
            self.n_prompt[b] = M
            self.next_pos[b] = M

    def append(self, k_new, v_new, s_new=None, active=None):
        append(self.K, self.V, self.S, self.pos, self.seq_len, self.next_pos, k_new, v_new,
               s_new if self.external else None, active)

    def attend(self, q, active=None, out=None):
        return attend(q, self.K, self.V, self.seq_len, self.scale, active, out)

    def update_scores(self, alpha, active=None):
        if not self.external:
            update_scores(self.S, alpha, self.seq_len, self.n_prompt, active)

    def score_block(self, q_blk, k_blk=None, active=None):
        """Add the block's attention (Eq. importance-score) to the scores of the thinking slots."""
        I = score_block(q_blk, k_blk, self.K, self.seq_len, self.scale, active)
        for b in range(self.Nb):
            if active is not None and not active[b]:
                continue
            self.S[b, :, self.n_prompt[b]:self.seq_len[b]] += I[b, :, self.n_prompt[b]:self.seq_len[b]]
        return I

    def due(self, active=None):
        """Trigger mask after a step: the cache has reached its total budget (Sec. 4.2).  Sec. 5 counts
        the same events: the first when M + i reaches B, then one every K steps."""
        n_think = self.seq_len - self.n_prompt
        trig = n_think >= self.budget + self.window + self.evict_every
        if active is not None:
            trig &= active.astype(bool)
        return trig.astype(_u8)

    def select(self, trigger=None, k_keep=None):
        return select(self.S, self.pos, self.seq_len, self.n_prompt, self.window,
                      self.budget if k_keep is None else k_keep, trigger)

    def compact(self, keep_idx, new_len, trigger=None):
        compact(self.K, self.V, self.S, self.pos, self.seq_len, keep_idx, new_len, trigger)

    def step(self, q, k_new, v_new, s_new=None, active=None, out=None):
        """One decode step of every active sequence.  Returns (out, alpha, lse, trigger, keep_idx)."""
        self.append(k_new, v_new, s_new, active)
        if active is None:
            self.steps_done += 1
        else:
            self.steps_done += active.astype(np.int64)
        o, alpha, lse = self.attend(q, active, out)
        self.update_scores(alpha, active)
        trig = self.due(active)
        keep_idx = None
        if trig.any():
            keep_idx, new_len = self.select(trig)
            self.compact(keep_idx, new_len, trig)
        return o, alpha, lse, trig, keep_idx
