"""Pins of the oracle's attention and score functions against what the paper and the
mathematics fix (CPU only).  Each test is written differently from the oracle so that a
dropped term, a wrong index or a transposed operand in the oracle fails one of them."""
import numpy as np
import pytest
import torch

from oracle import dynts_oracle as orc


def _rand_case(rng, Nb=2, Hq=8, Hkv=2, d=16, cap=24, lens=(24, 17)):
    q = rng.standard_normal((Nb, Hq, d))
    K = rng.standard_normal((Nb, Hkv, cap, d))
    V = rng.standard_normal((Nb, Hkv, cap, d))
    seq_len = np.array(lens, np.int32)
    return q, K, V, seq_len


def test_attention_equals_unshifted_longdouble_definition():
    """Eq. attn-score / attn-o written literally (no max subtraction) in extended precision."""
    rng = np.random.default_rng(1)
    q, K, V, seq_len = _rand_case(rng)
    scale = 0.37
    out, alpha, lse = orc.attend(q, K, V, seq_len, scale)
    Nb, Hq, d = q.shape
    G = Hq // K.shape[1]
    for b in range(Nb):
        n = seq_len[b]
        for hq in range(Hq):
            h = hq // G
            w = np.zeros(n, np.longdouble)
            for j in range(n):
                w[j] = np.exp(np.longdouble(scale) * np.dot(q[b, hq].astype(np.longdouble),
                                                            K[b, h, j].astype(np.longdouble)))
            a = w / w.sum()
            o = (a[:, None] * V[b, h, :n].astype(np.longdouble)).sum(0)
            np.testing.assert_allclose(alpha[b, hq, :n], a.astype(np.float64), rtol=1e-12, atol=1e-15)
            assert np.all(alpha[b, hq, n:] == 0.0)
            np.testing.assert_allclose(out[b, hq], o.astype(np.float64), rtol=1e-12, atol=1e-14)
            np.testing.assert_allclose(lse[b, hq], float(np.log(w.sum())), rtol=1e-12)


def test_attention_equals_library_sdpa_with_repeated_kv_heads():
    """Library special case: float64 scaled_dot_product_attention with KV heads repeated per group."""
    rng = np.random.default_rng(2)
    q, K, V, _ = _rand_case(rng, Nb=3, Hq=12, Hkv=4, d=32, cap=40, lens=(40, 40, 40))
    seq_len = np.full(3, 40, np.int32)
    out, _, _ = orc.attend(q, K, V, seq_len, 1.0 / np.sqrt(32))
    G = 3
    tq = torch.from_numpy(q).unsqueeze(2)  # [Nb][Hq][1][d]
    tk = torch.from_numpy(K).repeat_interleave(G, dim=1)
    tv = torch.from_numpy(V).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0]
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-11, atol=1e-13)


def test_softmax_rows_sum_to_one_and_gqa_mapping():
    rng = np.random.default_rng(3)
    q, K, V, seq_len = _rand_case(rng)
    _, alpha, _ = orc.attend(q, K, V, seq_len, 0.25)
    np.testing.assert_allclose(alpha.sum(-1), 1.0, atol=1e-12)
    # heads of one group given the same query produce the same output; a different KV head does not
    q2 = q.copy()
    q2[:, 1] = q2[:, 0]
    q2[:, 4] = q2[:, 0]
    out2, _, _ = orc.attend(q2, K, V, seq_len, 0.25)
    assert np.array_equal(out2[:, 0], out2[:, 1])
    assert not np.allclose(out2[:, 0], out2[:, 4])


def test_closed_forms():
    rng = np.random.default_rng(4)
    q, K, V, _ = _rand_case(rng)
    # n = 1: output is the single value row exactly
    out, alpha, _ = orc.attend(q, K, V, np.array([1, 1], np.int32), 0.5)
    assert np.array_equal(out[:, :4], np.broadcast_to(V[:, 0:1, 0], out[:, :4].shape))
    assert np.all(alpha[:, :, 0] == 1.0)
    # q = 0: uniform weights, output = mean of the value rows
    seq_len = np.array([24, 17], np.int32)
    out, alpha, lse = orc.attend(np.zeros_like(q), K, V, seq_len, 0.5)
    for b in range(2):
        n = seq_len[b]
        np.testing.assert_allclose(alpha[b, :, :n], 1.0 / n, rtol=1e-14)
        np.testing.assert_allclose(out[b, 0], V[b, 0, :n].mean(0), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(out[b, 7], V[b, 1, :n].mean(0), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[b], np.log(n), rtol=1e-14)
    # one key far ahead of the rest: output tends to its value row
    K2 = K.copy()
    K2[0, 0, 5] = 100.0 * q[0, 0] / np.dot(q[0, 0], q[0, 0])
    K2[0, 0, :5] *= 0.01
    K2[0, 0, 6:] *= 0.01
    out, alpha, _ = orc.attend(q, K2, V, seq_len, 1.0)
    assert alpha[0, 0, 5] >= 1 - 1e-15
    np.testing.assert_allclose(out[0, 0], V[0, 0, 5], rtol=1e-12, atol=1e-14)


def test_invariances():
    rng = np.random.default_rng(5)
    q, K, V, seq_len = _rand_case(rng, lens=(24, 24))
    out, alpha, _ = orc.attend(q, K, V, seq_len, 0.3)
    # same shift of every logit (add c*q/|q|^2 to every key of a head with G=1 mapping) leaves alpha
    Nb, Hq, d = q.shape
    q1 = np.ascontiguousarray(q[:, ::4])  # one query head per KV head
    K1 = K.copy()
    for b in range(Nb):
        for h in range(2):
            K1[b, h] += 3.0 * q1[b, h] / np.dot(q1[b, h], q1[b, h])
    o0, a0, l0 = orc.attend(q1, K, V, seq_len, 0.3)
    o1, a1, l1 = orc.attend(q1, K1, V, seq_len, 0.3)
    np.testing.assert_allclose(a1, a0, rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(o1, o0, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(l1 - l0, 0.9, rtol=1e-10)
    # permuting the slots permutes alpha and leaves the output unchanged
    perm = rng.permutation(24)
    out_p, alpha_p, _ = orc.attend(q, np.ascontiguousarray(K[:, :, perm]),
                                   np.ascontiguousarray(V[:, :, perm]), seq_len, 0.3)
    np.testing.assert_allclose(alpha_p, alpha[:, :, perm], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(out_p, out, rtol=1e-11, atol=1e-13)


def test_inactive_rows_untouched():
    rng = np.random.default_rng(6)
    q, K, V, seq_len = _rand_case(rng)
    out = np.full((2, 8, 16), 7.0)
    active = np.array([0, 1], np.uint8)
    o, alpha, _ = orc.attend(q, K, V, seq_len, 0.3, active=active, out=out)
    assert np.all(o[0] == 7.0) and not np.any(o[1] == 7.0)
    assert np.all(alpha[0] == 0.0)


# ---- importance score (Eq. importance-score, running form) ----------------------------------

def _dense_no_eviction_run(rng, T=9, M=3, Hq=4, Hkv=2, d=8):
    """Decode T steps without eviction; also build the dense [T x n] attention matrix by hand."""
    cap = M + T
    lay = orc.OracleLayer(1, Hq, Hkv, d, cap, budget=10 ** 6, window=0, evict_every=1, softmax_scale=0.4)
    K0 = rng.standard_normal((1, Hkv, M, d))
    V0 = rng.standard_normal((1, Hkv, M, d))
    lay.prefill(K0, V0, [M])
    qs = rng.standard_normal((T, 1, Hq, d))
    ks = rng.standard_normal((T, 1, Hkv, d))
    vs = rng.standard_normal((T, 1, Hkv, d))
    for t in range(T):
        lay.step(qs[t], ks[t], vs[t])
    G = Hq // Hkv
    Kall = np.concatenate([K0[0], ks[:, 0].transpose(1, 0, 2)], axis=1)  # [Hkv][M+T][d]
    A = np.zeros((Hq, T, M + T))
    for hq in range(Hq):
        for t in range(T):
            n = M + t + 1
            e = 0.4 * Kall[hq // G, :n] @ qs[t, 0, hq]
            w = np.exp(e - e.max())
            A[hq, t, :n] = w / w.sum()
    return lay, A, M, T, G


def test_scores_equal_column_sums_of_dense_attention_matrix():
    """App. B.1: aggregate over heads, sum along the query dimension -> one value per token."""
    lay, A, M, T, G = _dense_no_eviction_run(np.random.default_rng(7))
    for h in range(lay.Hkv):
        col = A[h * G:(h + 1) * G].sum(axis=(0, 1))  # sum over group heads and over queries
        np.testing.assert_allclose(lay.S[0, h, M:M + T], col[M:], rtol=1e-12, atol=1e-15)
        assert np.all(np.isinf(lay.S[0, h, :M]))
    assert np.array_equal(lay.pos[0, 0, :M + T], np.arange(M + T))


def test_score_increment_mass_balance_and_uniform_case():
    rng = np.random.default_rng(8)
    Nb, Hq, Hkv, d, cap = 2, 6, 2, 8, 20
    G = Hq // Hkv
    q = rng.standard_normal((Nb, Hq, d))
    K = rng.standard_normal((Nb, Hkv, cap, d))
    V = rng.standard_normal((Nb, Hkv, cap, d))
    seq_len = np.array([20, 11], np.int32)
    n_prompt = np.array([4, 2], np.int32)
    S = np.zeros((Nb, Hkv, cap))
    for b in range(Nb):
        S[b, :, :n_prompt[b]] = np.inf
    S0 = S.copy()
    _, alpha, _ = orc.attend(q, K, V, seq_len, 0.5)
    orc.update_scores(S, alpha, seq_len, n_prompt)
    for b in range(Nb):
        M, n = n_prompt[b], seq_len[b]
        for h in range(Hkv):
            prompt_mass = alpha[b, h * G:(h + 1) * G, :M].sum()
            inc = (S[b, h, M:n] - S0[b, h, M:n]).sum()
            np.testing.assert_allclose(inc, G - prompt_mass, rtol=1e-12)
            assert np.all(np.isinf(S[b, h, :M])) and np.all(S[b, h, n:] == 0.0)
    # uniform attention: every thinking slot gains G/n
    S = S0.copy()
    _, alpha, _ = orc.attend(np.zeros_like(q), K, V, seq_len, 0.5)
    orc.update_scores(S, alpha, seq_len, n_prompt)
    for b in range(Nb):
        np.testing.assert_allclose(S[b, :, n_prompt[b]:seq_len[b]], G / seq_len[b], rtol=1e-13)


def test_new_token_receives_its_own_attention():
    """The sum of Eq. attn-score runs up to t itself: a lone thinking token gets alpha = its share."""
    lay = orc.OracleLayer(1, 2, 1, 4, 8, budget=100, window=0, evict_every=1, softmax_scale=1.0)
    lay.prefill(np.zeros((1, 1, 1, 4)), np.zeros((1, 1, 1, 4)), [1])
    o, alpha, _, _, _ = lay.step(np.zeros((1, 2, 4)), np.ones((1, 1, 4)), np.ones((1, 1, 4)))
    assert lay.seq_len[0] == 2
    np.testing.assert_allclose(lay.S[0, 0, 1], 2 * 0.5)  # two heads, uniform over two slots
    np.testing.assert_allclose(o, 0.5)
