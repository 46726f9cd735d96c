"""Pins of the oracle's selection, eviction and schedule (CPU only)."""
import itertools
import os

import numpy as np
import pytest

from oracle import dynts_oracle as orc


def _unit(S, pos, M, W, k_keep):
    """Run the oracle's select on one unit; returns the retained slot list."""
    n = len(S)
    S3 = np.ascontiguousarray(np.asarray(S, np.float64).reshape(1, 1, n))
    p3 = np.ascontiguousarray(np.asarray(pos, np.int32).reshape(1, 1, n))
    keep, new_len = orc.select(S3, p3, np.array([n], np.int32), np.array([M], np.int32), W, k_keep)
    return keep[0, 0, :new_len[0]].tolist()


def test_select_equals_lexsort_on_random_and_tied_scores():
    rng = np.random.default_rng(11)
    for trial in range(200):
        M, W = int(rng.integers(0, 5)), int(rng.integers(0, 6))
        nc = int(rng.integers(0, 40))
        n = M + nc + W
        k = int(rng.integers(0, nc + 3))
        levels = rng.choice([2, 4, 1000])
        S = np.concatenate([np.full(M, np.inf), rng.integers(0, levels, nc + W) / 4.0])
        if trial % 3 == 0:
            S[M:] -= 1.0  # negative scores and signed zeros
            S[S == 0.0] = rng.choice([0.0, -0.0], size=(S == 0.0).sum())
        pos = np.arange(n) * 2 + 1
        got = _unit(S, pos, M, W, k)
        lo, hi = M, n - W
        order = np.lexsort((pos[lo:hi], -S[lo:hi]))  # primary: score descending, then position ascending
        chosen = sorted((lo + order[:min(k, nc)]).tolist())
        assert got == list(range(M)) + chosen + list(range(hi, n))


def test_select_is_the_best_subset_exhaustively():
    """For small windows: the kept set maximises the score sum; among maximisers it is the
    lexicographically smallest set of positions (lower position wins a tie)."""
    rng = np.random.default_rng(12)
    for trial in range(60):
        nc = int(rng.integers(1, 11))
        k = int(rng.integers(0, nc + 1))
        S = rng.integers(0, 4, nc).astype(np.float64)
        pos = np.arange(nc) + 5
        got = _unit(S, pos, 0, 0, k)
        best = None
        for sub in itertools.combinations(range(nc), k):
            key = (-sum(S[list(sub)]), sub)
            if best is None or key < best:
                best = key
        assert tuple(got) == best[1]


def test_select_special_cases():
    M, W = 3, 2
    S = np.concatenate([np.full(M, np.inf), np.full(12, 0.5)])
    pos = np.arange(15)
    # all ties: oldest k candidates survive
    assert _unit(S, pos, M, W, 4) == [0, 1, 2, 3, 4, 5, 6, 13, 14]
    # strictly increasing scores: newest k candidates survive
    S2 = np.concatenate([np.full(M, np.inf), np.arange(12.0)])
    assert _unit(S2, pos, M, W, 4) == [0, 1, 2, 9, 10, 11, 12, 13, 14]
    # k_keep = 0: question + local window only (the "Window" baseline of Table 1)
    assert _unit(S2, pos, M, W, 0) == [0, 1, 2, 13, 14]
    # fewer candidates than k_keep: nothing is evicted
    assert _unit(S2, pos, M, W, 50) == list(range(15))
    # window slots are kept even with the lowest scores; prompt kept without looking at scores
    S3 = S2.copy()
    S3[-2:] = -100.0
    assert _unit(S3, pos, M, W, 1)[-2:] == [13, 14]
    # -0.0 and +0.0 tie, the lower position wins
    assert _unit([0.0, -0.0, 0.0, -0.0], [0, 1, 2, 3], 0, 0, 2) == [0, 1]
    assert _unit([-0.0, 0.0, -0.0, 0.0], [0, 1, 2, 3], 0, 0, 2) == [0, 1]


def test_select_rejects_nan():
    with pytest.raises(RuntimeError):
        _unit([1.0, np.nan, 2.0], [0, 1, 2], 0, 0, 1)


def test_trigger_mask_and_new_len():
    rng = np.random.default_rng(13)
    S = rng.random((3, 2, 16))
    pos = np.broadcast_to(np.arange(16, dtype=np.int32), (3, 2, 16)).copy()
    seq_len = np.array([16, 12, 16], np.int32)
    n_prompt = np.array([2, 2, 4], np.int32)
    keep, new_len = orc.select(S, pos, seq_len, n_prompt, 3, 5, trigger=np.array([1, 0, 1], np.uint8))
    assert new_len.tolist() == [10, 12, 12]
    assert np.all(keep[1] == -1)
    for b in (0, 2):
        for h in range(2):
            row = keep[b, h, :new_len[b]]
            assert np.all(np.diff(row) > 0)
            assert row[:n_prompt[b]].tolist() == list(range(n_prompt[b]))
            assert row[-3:].tolist() == [13, 14, 15]


def test_compact_equals_boolean_mask_indexing():
    rng = np.random.default_rng(14)
    Nb, Hkv, cap, d = 3, 2, 20, 4
    K = rng.standard_normal((Nb, Hkv, cap, d))
    V = rng.standard_normal((Nb, Hkv, cap, d))
    S = rng.random((Nb, Hkv, cap))
    pos = np.cumsum(rng.integers(1, 4, (Nb, Hkv, cap)), axis=-1).astype(np.int32)
    seq_len = np.array([20, 15, 18], np.int32)
    n_prompt = np.array([2, 3, 0], np.int32)
    trig = np.array([1, 0, 1], np.uint8)
    keep, new_len = orc.select(S, pos, seq_len, n_prompt, 4, 6, trigger=trig)
    K0, V0, S0, p0 = K.copy(), V.copy(), S.copy(), pos.copy()
    orc.compact(K, V, S, pos, seq_len, keep, new_len, trigger=trig)
    assert seq_len.tolist() == [12, 15, 10]
    for b in range(Nb):
        for h in range(Hkv):
            if not trig[b]:
                assert np.array_equal(K[b, h], K0[b, h]) and np.array_equal(S[b, h], S0[b, h])
                continue
            m = np.zeros(cap, bool)
            m[keep[b, h, :new_len[b]]] = True
            nl = new_len[b]
            assert np.array_equal(K[b, h, :nl], K0[b, h][m])
            assert np.array_equal(V[b, h, :nl], V0[b, h][m])
            assert np.array_equal(S[b, h, :nl], S0[b, h][m])
            assert np.array_equal(pos[b, h, :nl], p0[b, h][m])
            assert np.all(np.diff(pos[b, h, :nl]) > 0)
            first_evicted = int(np.argmin(m))
            assert np.array_equal(K[b, h, :first_evicted], K0[b, h, :first_evicted])


def test_compact_rejects_bad_indices():
    K = np.zeros((1, 1, 8, 2)); V = K.copy(); S = np.zeros((1, 1, 8)); pos = np.zeros((1, 1, 8), np.int32)
    seq_len = np.array([8], np.int32)
    bad = np.array([[[0, 2, 2, 5]]], np.int32)
    with pytest.raises(RuntimeError):
        orc.compact(K, V, S, pos, seq_len, bad, np.array([4], np.int32))
    with pytest.raises(RuntimeError):
        orc.compact(K, V, S, pos, seq_len, np.array([[[0, 1, 9]]], np.int32), np.array([3], np.int32))


# ---- schedule: the paper's closed form for the effective cache length ---------------------------

def _run_schedule(M, budget, window, E, T, rng):
    Hq, Hkv, d = 2, 1, 4
    cap = M + budget + window + E
    lay = orc.OracleLayer(1, Hq, Hkv, d, cap, budget, window, E)
    lay.prefill(rng.standard_normal((1, Hkv, M, d)), rng.standard_normal((1, Hkv, M, d)), [M])
    lens, events = [], 0
    for t in range(1, T + 1):
        _, _, _, trig, _ = lay.step(rng.standard_normal((1, Hq, d)), rng.standard_normal((1, Hkv, d)),
                                    rng.standard_normal((1, Hkv, d)))
        events += int(trig[0])
        lens.append(int(lay.seq_len[0]))
    return lay, lens, events


def test_cache_length_follows_effective_length_formula():
    """Sec. 5 "Notions": S_i = M + i - n_i K, n_i = max(0, floor(((M+i)-B)/K)+1), with the total
    budget B = M + budget + window + evict_every and eviction volume K = evict_every."""
    rng = np.random.default_rng(15)
    # (the last three have budget + window not a multiple of the period, as the paper's own settings do:
    # total 5000, window 2000, retention 0.4 of the 3000 others => keep 1200, evict 1800 per trigger)
    for (M, budget, window, E, T) in [(5, 8, 4, 2, 60), (3, 6, 3, 3, 50), (0, 4, 0, 4, 40), (7, 16, 8, 8, 100),
                                      (5, 7, 4, 3, 60), (10, 12, 20, 18, 150), (4, 6, 10, 14, 120)]:
        lay, lens, events = _run_schedule(M, budget, window, E, T, rng)
        Bp = M + budget + window + E
        for i, got in enumerate(lens, start=1):
            n_i = max(0, ((M + i) - Bp) // E + 1)
            assert got == M + i - n_i * E
            assert orc.eviction_events(M, i, Bp, E) == n_i
            assert orc.effective_length(M, i, Bp, E) == got
            assert got - M <= budget + window + E - 1 or got - M == budget + window
        assert events == max(0, (T - (budget + window + E)) // E + 1)
        assert max(lens) < Bp
        # prompt never evicted, positions strictly increasing, local window = most recent tokens
        n = lens[-1]
        assert np.all(np.isinf(lay.S[0, 0, :M]))
        assert lay.pos[0, 0, :M].tolist() == list(range(M))
        assert np.all(np.diff(lay.pos[0, 0, :n]) > 0)
        assert lay.pos[0, 0, n - window:n].tolist() == list(range(M + T - window, M + T))


def test_cfg1_schedule_has_22_evictions():
    rng = np.random.default_rng(16)
    _, lens, events = _run_schedule(64, 128, 32, 16, 512, rng)
    assert events == 22 and max(lens) == 64 + 128 + 32 + 16 - 1
    assert lens[-1] == 64 + 128 + 32


def test_planted_heavy_hitters_survive_eviction():
    """Meaning check: tokens that keep receiving attention stay; the rest of the window churns."""
    rng = np.random.default_rng(17)
    M, budget, window, E, d = 2, 6, 2, 2, 8
    lay = orc.OracleLayer(1, 1, 1, d, M + budget + window + E, budget, window, E, softmax_scale=1.0)
    lay.prefill(np.zeros((1, 1, M, d)), np.zeros((1, 1, M, d)), [M])
    u = np.zeros(d); u[0] = 1.0
    hot = {3, 7, 12}
    for t in range(1, 41):
        pos = M + t - 1
        k = (6.0 * u if pos in hot else 0.1 * rng.standard_normal(d)).reshape(1, 1, d)
        lay.step((u + 0.01 * rng.standard_normal(d)).reshape(1, 1, d), k, rng.standard_normal((1, 1, d)))
    kept = set(lay.pos[0, 0, :lay.seq_len[0]].tolist())
    assert hot <= kept


# ---- cost model helpers against the values the paper prints --------------------------------------

def _golden():
    vals = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")
    for line in open(path):
        line = line.split("--")[0].strip()
        if line and not line.startswith("#"):
            k, v = line.split()
            vals[k] = float(v)
    return vals


def test_break_even_values_printed_in_the_paper():
    g = _golden()
    for hid, lay in ((g["llama_hidden"], g["llama_layers"]), (g["qwen_hidden"], g["qwen_layers"])):
        # the paper rounds (6d^2+d)/(4Ld) to 1.5d/L
        assert abs(orc.break_even_volume(hid, lay, 1.0) - g["break_even_rhs"]) < 0.01
        assert 1.5 * hid / lay == g["break_even_rhs"]
        assert orc.mlp_flops(hid, 2 * hid, hid / 2, 1) == g["mlp_flops_coeff_d2"] * hid ** 2 + g["mlp_flops_coeff_d"] * hid
        assert orc.attn_flops(lay, hid, 1000) == g["attn_flops_coeff"] * lay * hid * 1000
    assert g["eviction_volume_example"] >= g["break_even_rhs"]
