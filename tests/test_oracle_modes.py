"""Pins of the oracle's external-score mode and of its `active` masks (CPU only).

External mode is the paper's own inference mode (Sec. 4.1, Sec. 4.2 second paragraph): the
predictor gives ONE score per token, it is appended with the token's KV entry and never changes
afterwards; selection then ranks those scores.  The `active` mask is the reading taken for ragged
batches: a finished sequence is neither appended to, attended, scored nor triggered.

Expected values are built here from the supplied arrays with plain numpy indexing, never by
calling the function under test a second time.
"""
import numpy as np

from oracle import dynts_oracle as orc


def _layer(rng, Nb, Hq, Hkv, d, M, budget, window, E, external, lens=None):
    lay = orc.OracleLayer(Nb, Hq, Hkv, d, max(M) + budget + window + E, budget, window, E,
                          external_scores=external)
    Mmax = max(M)
    lay.prefill(rng.standard_normal((Nb, Hkv, Mmax, d)), rng.standard_normal((Nb, Hkv, Mmax, d)), M)
    return lay


def test_external_append_stores_the_score_of_its_own_sequence_and_head():
    """Catches: s_new indexed by sequence only (s_new[b]) or by head only, a score written to the
    wrong slot, a score written for a masked sequence, and external scores ignored (left at 0)."""
    rng = np.random.default_rng(41)
    Nb, Hq, Hkv, d = 3, 6, 3, 4
    M = [2, 4, 3]
    lay = _layer(rng, Nb, Hq, Hkv, d, M, 6, 2, 2, external=True)
    # distinct value per (sequence, head): 100 b + 10 h + step / 16
    want = [[[] for _ in range(Hkv)] for _ in range(Nb)]
    for t in range(1, 6):
        s_new = np.array([[100.0 * b + 10.0 * h + t / 16.0 for h in range(Hkv)] for b in range(Nb)])
        active = np.array([1, t % 2, 1], np.uint8)  # sequence 1 sits out the even steps
        lay.append(rng.standard_normal((Nb, Hkv, d)), rng.standard_normal((Nb, Hkv, d)), s_new, active)
        for b in range(Nb):
            if active[b]:
                for h in range(Hkv):
                    want[b][h].append(s_new[b, h])
    for b in range(Nb):
        n = int(lay.seq_len[b])
        assert n == M[b] + len(want[b][0])
        for h in range(Hkv):
            assert np.all(np.isposinf(lay.S[b, h, :M[b]]))               # question slots keep +inf
            assert lay.S[b, h, M[b]:n].tolist() == want[b][h]              # exact: nothing is computed
            assert np.all(lay.S[b, h, n:] == 0.0)                          # nothing written past the end


def test_external_scores_are_never_updated_by_attention():
    """Catches: an oracle that still accumulates attention in external mode (the predictor's score
    is fixed once appended)."""
    rng = np.random.default_rng(42)
    Nb, Hq, Hkv, d = 2, 4, 2, 8
    lay = _layer(rng, Nb, Hq, Hkv, d, [3, 3], 8, 2, 4, external=True)
    for t in range(1, 7):
        s_new = rng.integers(0, 50, (Nb, Hkv)).astype(np.float64)
        lay.append(rng.standard_normal((Nb, Hkv, d)), rng.standard_normal((Nb, Hkv, d)), s_new)
        before = lay.S.copy()
        _, alpha, _ = lay.attend(rng.standard_normal((Nb, Hq, d)))
        assert alpha[:, :, :lay.seq_len[0]].min() > 0.0                    # there WAS attention to add
        lay.update_scores(alpha)
        assert np.array_equal(lay.S, before)
    # the accumulate-mode layer under the same calls does change (the test would otherwise be vacuous)
    acc = _layer(rng, Nb, Hq, Hkv, d, [3, 3], 8, 2, 4, external=False)
    acc.append(rng.standard_normal((Nb, Hkv, d)), rng.standard_normal((Nb, Hkv, d)), np.ones((Nb, Hkv)))
    assert np.all(acc.S[:, :, 3] == 0.0)                                    # accumulate mode ignores s_new
    _, alpha, _ = acc.attend(rng.standard_normal((Nb, Hq, d)))
    acc.update_scores(alpha)
    assert np.all(acc.S[:, :, 3] > 0.0)


def test_selection_in_external_mode_follows_the_supplied_scores():
    """End to end through OracleLayer.step in external mode: the retained thinking tokens are exactly
    the budget-many tokens with the highest supplied score (lower position on ties), per head --
    computed here by sorting the supplied (score, position) pairs, not by the oracle's select."""
    rng = np.random.default_rng(43)
    Nb, Hq, Hkv, d = 2, 4, 2, 4
    M, budget, window, E = [2, 2], 5, 2, 3
    lay = _layer(rng, Nb, Hq, Hkv, d, M, budget, window, E, external=True)
    given = {}   # (b, h, position) -> score
    alive = [[[] for _ in range(Hkv)] for _ in range(Nb)]  # thinking positions still cached
    n_trig = 0
    for t in range(1, 32):
        s_new = rng.integers(0, 4, (Nb, Hkv)).astype(np.float64)         # few levels: ties at every cut
        pos_t = 2 + t - 1
        for b in range(Nb):
            for h in range(Hkv):
                given[(b, h, pos_t)] = s_new[b, h]
                alive[b][h].append(pos_t)
        _, _, _, trig, _ = lay.step(rng.standard_normal((Nb, Hq, d)), rng.standard_normal((Nb, Hkv, d)),
                                    rng.standard_normal((Nb, Hkv, d)), s_new)
        for b in range(Nb):
            if trig[b]:
                n_trig += 1
                for h in range(Hkv):
                    cand, recent = alive[b][h][:-window], alive[b][h][-window:]
                    ranked = sorted(cand, key=lambda p: (-given[(b, h, p)], p))
                    alive[b][h] = sorted(ranked[:budget]) + recent
            n = int(lay.seq_len[b])
            for h in range(Hkv):
                assert lay.pos[b, h, 2:n].tolist() == alive[b][h]
                assert lay.S[b, h, 2:n].tolist() == [given[(b, h, p)] for p in alive[b][h]]
    assert n_trig >= 2 * Nb and len(alive[0][0]) <= budget + window + E


def _snapshot(lay):
    return [a.copy() for a in (lay.K, lay.V, lay.S, lay.pos, lay.seq_len, lay.next_pos)]


def test_inactive_sequence_is_left_byte_identical_and_never_triggers():
    """Catches: a mask applied to the wrong sequence, a mask ignored by append / update_scores / due,
    lengths or positions advanced for a finished sequence."""
    rng = np.random.default_rng(44)
    Nb, Hq, Hkv, d = 3, 4, 2, 4
    M, budget, window, E = [2, 3, 2], 4, 2, 2
    for external in (False, True):
        lay = _layer(rng, Nb, Hq, Hkv, d, M, budget, window, E, external=external)
        frozen_at, frozen = None, None
        for t in range(1, 25):
            active = np.array([1, 1 if t <= 5 else 0, 1], np.uint8)       # sequence 1 finishes after 5 steps
            if t == 6:
                frozen_at, frozen = t, [a[1].copy() for a in _snapshot(lay)]
            out0 = np.full((Nb, Hq, d), 7.0)
            o, alpha, lse, trig, _ = lay.step(rng.standard_normal((Nb, Hq, d)), rng.standard_normal((Nb, Hkv, d)),
                                              rng.standard_normal((Nb, Hkv, d)),
                                              rng.standard_normal((Nb, Hkv)), active, out0)
            if t > 5:
                assert trig[1] == 0
                assert np.all(o[1] == 7.0)                                 # its output row is not written
                now = [a[1] for a in _snapshot(lay)]
                for a, b in zip(now, frozen):
                    assert np.array_equal(a, b)
        assert frozen_at == 6
        # the active ones kept going and did trigger
        assert lay.steps_done.tolist() == [24, 5, 24]
        assert int(lay.seq_len[1]) == M[1] + 5                              # 5 < budget+window+E: never full
        assert int(lay.next_pos[0]) == M[0] + 24 and int(lay.next_pos[1]) == M[1] + 5


def test_due_masks_a_full_but_finished_sequence():
    """`due` alone: a sequence whose cache is at the trigger level but which is masked does not
    trigger; without the mask it does.  Catches a mask that `due` ignores."""
    rng = np.random.default_rng(45)
    Nb, Hq, Hkv, d = 2, 2, 1, 4
    M, budget, window, E = [1, 1], 3, 1, 2
    lay = _layer(rng, Nb, Hq, Hkv, d, M, budget, window, E, external=False)
    for t in range(budget + window + E):
        lay.append(rng.standard_normal((Nb, Hkv, d)), rng.standard_normal((Nb, Hkv, d)))
    assert lay.due().tolist() == [1, 1]
    assert lay.due(np.array([1, 0], np.uint8)).tolist() == [1, 0]
    assert lay.due(np.array([0, 1], np.uint8)).tolist() == [0, 1]
    # update_scores with a mask: only the active sequence's thinking slots move, by the group's column sums
    _, alpha, _ = lay.attend(rng.standard_normal((Nb, Hq, d)))
    before = lay.S.copy()
    lay.update_scores(alpha, np.array([0, 1], np.uint8))
    assert np.array_equal(lay.S[0], before[0])
    n = int(lay.seq_len[1])
    want = before[1, 0, 1:n] + alpha[1, :, 1:n].sum(axis=0)
    np.testing.assert_allclose(lay.S[1, 0, 1:n], want, rtol=0, atol=1e-15)
    assert np.isposinf(lay.S[1, 0, 0])
