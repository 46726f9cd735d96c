"""Pins of the oracle's block scoring (Eq. importance-score, sum over the K answer tokens; App. B.1)
against things other than itself: a library softmax on the dense causal matrix, the single-query oracle
run token by token, closed forms, mass balance and symmetries."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import dynts_oracle as orc


def _case(rng, Nb=2, T=5, Hq=6, Hkv=2, d=8, cap=40, lens=(17, 40)):
    q = rng.standard_normal((Nb, T, Hq, d))
    kb = rng.standard_normal((Nb, T, Hkv, d))
    K = rng.standard_normal((Nb, Hkv, cap, d))
    return q, kb, K, np.array(lens, np.int32)


def test_equals_library_softmax_on_the_dense_causal_matrix():
    rng = np.random.default_rng(51)
    q, kb, K, n = _case(rng)
    Nb, T, Hq, d = q.shape
    Hkv, G, scale = K.shape[1], Hq // K.shape[1], 0.37
    for use_block_keys in (True, False):
        I = orc.score_block(q, kb if use_block_keys else None, K, n, scale)
        for b in range(Nb):
            for h in range(Hkv):
                keys = K[b, h, :n[b]]
                if use_block_keys:
                    keys = np.concatenate([keys, kb[b, :, h]], 0)
                want = np.zeros(n[b])
                for g in range(G):
                    logits = q[b, :, h * G + g] @ keys.T * scale            # [T][n (+T)]
                    if use_block_keys:
                        future = np.triu(np.ones((T, T), bool), 1)         # block key i' > i is not visible
                        logits[:, n[b]:][future] = -np.inf
                    want += softmax(logits, axis=1)[:, :n[b]].sum(0)
                np.testing.assert_allclose(I[b, h, :n[b]], want, rtol=1e-12, atol=1e-15)
                assert np.all(I[b, h, n[b]:] == 0.0)


def test_equals_the_single_query_oracle_run_token_by_token():
    """Appending block token i and attending with its query is the forward pass the block form describes."""
    rng = np.random.default_rng(52)
    Nb, T, Hq, Hkv, d, M = 2, 6, 8, 2, 16, 3
    lay = orc.OracleLayer(Nb, Hq, Hkv, d, 64, 40, 8, 8)
    lay.prefill(rng.standard_normal((Nb, Hkv, M, d)), rng.standard_normal((Nb, Hkv, M, d)), [M, 2])
    for _ in range(20):
        lay.step(rng.standard_normal((Nb, Hq, d)), rng.standard_normal((Nb, Hkv, d)), rng.standard_normal((Nb, Hkv, d)))
    n0 = lay.seq_len.copy()
    q = rng.standard_normal((Nb, T, Hq, d))
    kb = rng.standard_normal((Nb, T, Hkv, d))
    I = orc.score_block(q, kb, lay.K, n0, lay.scale)
    S0 = lay.S.copy()
    for i in range(T):
        lay.append(np.ascontiguousarray(kb[:, i]), rng.standard_normal((Nb, Hkv, d)))
        _, alpha, _ = lay.attend(np.ascontiguousarray(q[:, i]))
        lay.update_scores(alpha)
    for b in range(Nb):
        m, n = int(lay.n_prompt[b]), int(n0[b])
        np.testing.assert_allclose(I[b, :, m:n], lay.S[b, :, m:n] - S0[b, :, m:n], rtol=1e-12, atol=1e-15)


def test_one_query_without_block_keys_is_the_decode_score_update():
    rng = np.random.default_rng(53)
    q, _, K, n = _case(rng, T=1)
    V = rng.standard_normal(K.shape)
    _, alpha, _ = orc.attend(np.ascontiguousarray(q[:, 0]), K, V, n, 0.5)
    S = np.zeros(K.shape[:3])
    orc.update_scores(S, alpha, n, np.zeros(2, np.int32))
    np.testing.assert_allclose(orc.score_block(q, None, K, n, 0.5), S, rtol=1e-13, atol=0)


def test_closed_forms_and_mass_balance():
    rng = np.random.default_rng(54)
    q, kb, K, n = _case(rng)
    Nb, T, Hq, d = q.shape
    Hkv, G = K.shape[1], Hq // K.shape[1]
    # zero queries: uniform attention, query i sees n + i + 1 keys
    I = orc.score_block(np.zeros_like(q), kb, K, n, 1.0)
    for b in range(Nb):
        want = G * sum(1.0 / (n[b] + i + 1) for i in range(T))
        np.testing.assert_allclose(I[b, :, :n[b]], want, rtol=1e-13)
    # no block keys: every query's weights sum to one over the cache
    I = orc.score_block(q, None, K, n, 0.8)
    np.testing.assert_allclose(I.sum(-1), T * G, rtol=1e-12)
    # with block keys the cache gets less than everything, and more than nothing
    I2 = orc.score_block(q, kb, K, n, 0.8)
    assert np.all(I2.sum(-1) < T * G) and np.all(I2 > -1e-300) and np.all(I2[:, :, 0] > 0)
    assert np.all(I2 <= I + 1e-15)   # extra keys in the denominator can only lower a cached slot's share
    # one key aligned with every query takes (almost) all of it
    K2 = K.copy()
    qq = np.abs(q) + 1.0
    K2[:, :, 5] = 50.0
    I3 = orc.score_block(qq, None, K2, n, 1.0)
    np.testing.assert_allclose(I3[:, :, 5], T * G, rtol=1e-9)


def test_symmetries():
    rng = np.random.default_rng(55)
    q, kb, K, n = _case(rng, lens=(40, 40))
    Hkv, G = K.shape[1], q.shape[2] // K.shape[1]
    I = orc.score_block(q, kb, K, n, 0.6)
    perm = rng.permutation(40)
    np.testing.assert_allclose(orc.score_block(q, kb, np.ascontiguousarray(K[:, :, perm]), n, 0.6), I[:, :, perm], rtol=1e-12)
    # heads of one group may be swapped, groups may not
    hp = np.arange(q.shape[2]); hp[[0, 1]] = hp[[1, 0]]
    np.testing.assert_allclose(orc.score_block(np.ascontiguousarray(q[:, :, hp]), kb, K, n, 0.6), I, rtol=1e-12)
    hp = np.arange(q.shape[2]); hp[[0, G]] = hp[[G, 0]]
    assert not np.allclose(orc.score_block(np.ascontiguousarray(q[:, :, hp]), kb, K, n, 0.6), I)
    # the order of the block matters only through causality: reversing queries and keys together changes I ...
    Ir = orc.score_block(np.ascontiguousarray(q[:, ::-1]), np.ascontiguousarray(kb[:, ::-1]), K, n, 0.6)
    assert not np.allclose(Ir, I)
    # ... but without block keys the queries are independent
    np.testing.assert_allclose(orc.score_block(np.ascontiguousarray(q[:, ::-1]), None, K, n, 0.6),
                               orc.score_block(q, None, K, n, 0.6), rtol=1e-12)
    # inactive sequences are skipped, bad shapes refused
    Ia = orc.score_block(q, kb, K, n, 0.6, active=np.array([1, 0], np.uint8))
    assert np.all(Ia[1] == 0) and np.allclose(Ia[0], I[0])
    with pytest.raises(Exception):
        orc.score_block(q, kb, K, np.array([41, 3], np.int32), 0.6)


def test_layer_method_adds_to_thinking_slots_only():
    rng = np.random.default_rng(56)
    lay = orc.OracleLayer(1, 4, 2, 8, 32, 16, 4, 4)
    lay.prefill(rng.standard_normal((1, 2, 5, 8)), rng.standard_normal((1, 2, 5, 8)), [5])
    for _ in range(9):
        lay.step(rng.standard_normal((1, 4, 8)), rng.standard_normal((1, 2, 8)), rng.standard_normal((1, 2, 8)))
    S0 = lay.S.copy()
    I = lay.score_block(rng.standard_normal((1, 3, 4, 8)), rng.standard_normal((1, 3, 2, 8)))
    assert np.all(np.isinf(lay.S[0, :, :5]))
    np.testing.assert_allclose(lay.S[0, :, 5:14] - S0[0, :, 5:14], I[0, :, 5:14], rtol=1e-12)
    assert np.all(lay.S[0, :, 14:] == S0[0, :, 14:])
