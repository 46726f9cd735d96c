"""GPU parity of the Importance Predictor head (Sec. 4.1, App. A) against the float64 oracle, synthetic weights."""
import numpy as np
import pytest
import torch

from oracle import dynts_oracle as orc
from tests.helpers import assert_close, f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2601_18383_amd import binding
    return binding


def _make(rng, d, m1, m2, bias=True):
    bf = lambda a: torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)
    W1 = bf(rng.standard_normal((m1, d)) / np.sqrt(d))
    W2 = bf(rng.standard_normal((m2, m1)) / np.sqrt(m1))
    w3 = bf(rng.standard_normal(m2) / np.sqrt(m2))
    b1 = torch.from_numpy(rng.standard_normal(m1).astype(np.float32) * 0.1) if bias else None
    b2 = torch.from_numpy(rng.standard_normal(m2).astype(np.float32) * 0.1) if bias else None
    b3 = torch.from_numpy(rng.standard_normal(1).astype(np.float32)) if bias else None
    return W1, b1, W2, b2, w3, b3


def _run(B, rng, d, m1, m2, batch, act, bias=True, n_rep=1, pack=True):
    dev = torch.device("cuda:0")
    ws = _make(rng, d, m1, m2, bias)
    h = torch.from_numpy(rng.standard_normal((batch, d)).astype(np.float32)).to(torch.bfloat16)
    pred = B.Predictor(*[w.to(dev) if w is not None else None for w in ws], activation=act, pack=pack)
    s = torch.full((batch, n_rep), 7.0, dtype=torch.float32, device=dev)
    B.dynts_predict_scores(pred, h.to(dev), s)
    ref = orc.predictor(f64(h), *[f64(w) if w is not None else None for w in ws], act)
    got = f64(s)
    for r in range(n_rep):
        worst = assert_close(got[:, r], ref, "predictor d=%d batch=%d act=%d" % (d, batch, act), tight=1e-4)
    assert np.all(got == got[:, :1])
    return worst


@pytest.mark.parametrize("act", [0, 1, 2])
@pytest.mark.parametrize("d,m1,m2,batch", [(64, 128, 32, 3), (96, 160, 48, 17), (256, 512, 128, 40),
                                            (512, 1024, 256, 128), (64, 128, 32, 1), (992, 2016, 496, 33)])
def test_small_shapes(B, d, m1, m2, batch, act):
    """Ragged feature groups (m not a multiple of 128), K slices with a partial last chunk, every batch-tile
    variant of the kernel, with and without biases."""
    rng = np.random.default_rng(d + batch + act)
    _run(B, rng, d, m1, m2, batch, act, bias=(batch % 2 == 1), n_rep=1 + batch % 4, pack=(act != 1))


@pytest.mark.parametrize("d,batch,hkv", [(3584, 32, 4), (4096, 64, 8), (4096, 128, 8)])
def test_paper_sizes(B, d, batch, hkv):
    """App. C: 3584 -> 7168 -> 1792 -> 1 (R1-Qwen) and 4096 -> 8192 -> 2048 -> 1 (R1-Llama), decode batches of the
    benchmark configs, the score written once per KV head."""
    rng = np.random.default_rng(d + batch)
    _run(B, rng, d, 2 * d, d // 2, batch, orc.ACT_RELU, n_rep=hkv)


def test_pack_is_the_documented_permutation(B):
    """[m][K] -> [m/16][K/32][16][32], bit for bit."""
    dev = torch.device("cuda:0")
    m, K = 48, 96
    W = torch.arange(m * K, dtype=torch.int32).reshape(m, K).to(torch.int16).view(torch.bfloat16).to(dev)
    got = B.dynts_predictor_pack(W).view(torch.int16).cpu().numpy().reshape(m // 16, K // 32, 16, 32)
    want = W.view(torch.int16).cpu().numpy().reshape(m // 16, 16, K // 32, 32).transpose(0, 2, 1, 3)
    assert np.array_equal(got, want)


def test_row_major_weights_at_paper_size(B):
    rng = np.random.default_rng(5)
    _run(B, rng, 3584, 7168, 1792, 32, orc.ACT_SILU, n_rep=4, pack=False)


def test_argument_errors(B):
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(0)
    ws = [w.to(dev) for w in _make(rng, 64, 128, 32)]
    pred = B.Predictor(*ws)
    h = torch.zeros((4, 64), dtype=torch.bfloat16, device=dev)
    s = torch.zeros((4, 300), dtype=torch.float32, device=dev)
    with pytest.raises(B.DyntsError):
        B.dynts_predict_scores(pred, h, s)                       # n_rep too large
    bad = B.dynts_predictor(60, 128, 32, 1, 0, 0, 0, 0, 0, 0, 0)  # d not a multiple of 32
    assert B.dynts_predict_scratch_bytes(bad, 4) == 0
    assert B.dynts_predict_scratch_bytes(pred.w, 129) == 0
    assert B.dynts_predict_scratch_bytes(pred.w, 128) > 0


def test_paper_inference_mode_end_to_end(B):
    """The paper's own inference loop (Sec. 4.1-4.2) in small: every step the predictor head turns the current
    token's hidden state into one score, the token is appended with that score (the same for every KV head),
    attention runs over the retained cache, and when the budget is reached the top-k by predicted score stay.
    HIP path (predictor + fused decode step + selection + compaction) against the oracle chain."""
    from tests.helpers import SideBySide
    rng = np.random.default_rng(77)
    dev = torch.device("cuda:0")
    Nb, Hq, Hkv, d_head, M, budget, window, E = 3, 8, 2, 64, 11, 24, 16, 20
    d_model, m1, m2 = 64, 128, 32
    ws = _make(rng, d_model, m1, m2)
    pred = B.Predictor(*[w.to(dev) for w in ws], activation=B.DYNTS_ACT_SILU)
    cap = M + budget + window + E
    cache = B.Cache(1, Nb, Hq, Hkv, d_head, cap, budget, window, E, external_scores=True)
    o = orc.OracleLayer(Nb, Hq, Hkv, d_head, cap, budget, window, E, external_scores=True)
    sbs = SideBySide(B, cache, 0, o, "step")
    bf = lambda *shape: torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).to(torch.bfloat16)
    sbs.prefill(bf(Nb, Hkv, M, d_head), bf(Nb, Hkv, M, d_head), [M, 5, 8])
    s_dev = torch.zeros((Nb, Hkv), dtype=torch.float32, device=dev)
    T = budget + window + 3 * E + 7
    for t in range(1, T + 1):
        h = bf(Nb, d_model)
        B.dynts_predict_scores(pred, h.to(dev), s_dev)
        s_ref = orc.predictor(f64(h), *[f64(w) for w in ws], orc.ACT_SILU)
        assert_close(f64(s_dev)[:, 0], s_ref, "predicted score, step %d" % t, tight=1e-4)
        # both sides append the HIP path's fp32 score, so that the selection below is decided on identical
        # numbers (the predictor's own parity is asserted just above)
        sbs.step(bf(Nb, Hq, d_head), bf(Nb, Hkv, d_head), bf(Nb, Hkv, d_head), s=s_dev.cpu(), check_scores=(t % 9 == 0))
    assert sbs.evictions == 3
    sbs.check_state()
    # external scores are never changed by attention: every retained thinking slot still holds its predicted score
    S = f64(cache.S[0])
    assert np.all(S[:, 0, :] == S[:, 1, :])
    assert int(cache.status.item()) == 0
