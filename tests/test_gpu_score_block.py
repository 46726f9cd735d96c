"""GPU parity of the block scoring (Eq. importance-score over a block of queries) against the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import dynts_oracle as orc
from paper_2601_18383_amd import configs, synth
from tests.helpers import assert_close, f64, i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2601_18383_amd import binding
    return binding


def _bf16(rng, *shape, scale=1.0):
    return torch.from_numpy(rng.standard_normal(shape).astype(np.float32) * scale).to(torch.bfloat16)


@pytest.mark.parametrize("with_block_keys", [True, False])
@pytest.mark.parametrize("d,Hq,Hkv,T", [(64, 8, 2, 5), (128, 28, 4, 37), (128, 6, 6, 16), (128, 16, 1, 70),
                                         (128, 28, 4, 1), (64, 4, 2, 300)])
def test_small_shapes_ragged(B, d, Hq, Hkv, T, with_block_keys):
    """Several row and key tiles, ragged tails in both, a cache shorter than one tile, an empty selection
    window, an inactive sequence; into the score array (question slots untouched) and into a plain buffer."""
    rng = np.random.default_rng(1000 + d + Hq + T)
    Nb, cap = 5, 333
    lens = np.array([333, 9, 200, 47, 16], np.int32)
    M = np.array([20, 9, 0, 30, 3], np.int32)
    active = np.array([1, 1, 1, 0, 1], np.uint8)
    dev = torch.device("cuda:0")
    cache = B.Cache(1, Nb, Hq, Hkv, d, cap, 100, 10, 10)
    K = _bf16(rng, Nb, Hkv, cap, d)
    S0 = torch.from_numpy(rng.random((Nb, Hkv, cap)).astype(np.float32))
    for b in range(Nb):
        S0[b, :, :M[b]] = float("inf")
    cache.K[0].copy_(K)
    cache.S[0].copy_(S0)
    cache.seq_len[0].copy_(torch.from_numpy(lens))
    cache.n_prompt.copy_(torch.from_numpy(M))
    q = _bf16(rng, Nb, T, Hq, d, scale=1.5)
    kb = _bf16(rng, Nb, T, Hkv, d) if with_block_keys else None
    scratch = torch.empty(B.dynts_score_block_scratch_bytes(cache.cfg, T), dtype=torch.uint8, device=dev)
    act = torch.from_numpy(active).to(dev)
    I_ref = orc.score_block(f64(q), f64(kb) if kb is not None else None, f64(K), lens, 1.0 / np.sqrt(d), active)

    # (1) into a plain buffer, overwriting: every slot below seq_len, question slots included
    dst = torch.full((Nb, Hkv, cap), 7.0, dtype=torch.float32, device=dev)
    B.dynts_score_block(cache.ctx, 0, q.to(dev), kb.to(dev) if kb is not None else None, scratch, dst=dst,
                        accumulate=False, active=act)
    got = f64(dst)
    for b in range(Nb):
        n = lens[b]
        if active[b]:
            assert_close(got[b, :, :n], I_ref[b, :, :n], "I[%d]" % b)
            assert np.all(got[b, :, n:] == 7.0)
        else:
            assert np.all(got[b] == 7.0)
    # (2) the same again, accumulating: exactly twice the first result plus nothing else
    B.dynts_score_block(cache.ctx, 0, q.to(dev), kb.to(dev) if kb is not None else None, scratch, dst=dst,
                        accumulate=True, active=act)
    got2 = f64(dst)
    for b in range(Nb):
        if active[b]:
            assert np.array_equal(got2[b, :, :lens[b]], 2.0 * got[b, :, :lens[b]])
    # (3) into the layer's score array: thinking slots gain I, question slots keep +inf, the rest is untouched
    B.dynts_score_block(cache.ctx, 0, q.to(dev), kb.to(dev) if kb is not None else None, scratch, active=act)
    S1 = f64(cache.S[0])
    for b in range(Nb):
        n, m = lens[b], M[b]
        if active[b]:
            assert np.all(np.isinf(S1[b, :, :m]))
            assert_close(S1[b, :, m:n], f64(S0)[b, :, m:n] + I_ref[b, :, m:n], "S[%d]" % b)
            assert np.array_equal(S1[b, :, n:], f64(S0)[b, :, n:])
        else:
            assert np.array_equal(S1[b], f64(S0)[b])
    assert int(cache.status.item()) == 0


def test_argument_errors(B):
    cache = B.Cache(1, 2, 8, 2, 64, 64, 20, 4, 4)
    dev = cache.K.device
    q = torch.zeros((2, 4, 8, 64), dtype=torch.bfloat16, device=dev)
    small = torch.empty(16, dtype=torch.uint8, device=dev)
    with pytest.raises(B.DyntsError) as e:
        B.dynts_score_block(cache.ctx, 0, q, None, small)
    assert e.value.code == B.DYNTS_EWORKSPACE
    with pytest.raises(B.DyntsError):
        B.dynts_score_block(cache.ctx, 3, q, None, small)
    assert B.dynts_score_block_scratch_bytes(cache.cfg, 0) == 0
    assert B.dynts_score_block_scratch_bytes(cache.cfg, 4) >= 2 * 2 * 16 * 4


@pytest.mark.parametrize("name,T,sample", [("cfg3", 256, [0, 31]), ("paper_llama_3000", 128, [5])])
def test_full_shape(B, name, T, sample):
    """Benchmark shapes: a generator-made steady-state cache, a block of T answer queries with their keys."""
    wl = configs.get(name)
    dev = torch.device("cuda:0")
    gen = synth.Synth(wl, dev)
    cache = B.Cache.for_workload(wl, device=dev)
    n0 = wl.steady_len + 23
    st = gen.steady_state(0, n0)
    cache.K[0, :, :, :n0] = st["K"]
    cache.S[0, :, :, :n0] = st["S"]
    cache.seq_len[0].fill_(n0)
    cache.n_prompt.fill_(wl.prompt)
    steps = torch.arange(70000, 70000 + T)
    q = gen.q(0, steps).permute(1, 0, 2, 3).contiguous()          # [Nb][T][Hq][d]
    kb = gen.kv(0, steps)[0].permute(1, 0, 2, 3).contiguous()     # [Nb][T][Hkv][d]
    scratch = torch.empty(B.dynts_score_block_scratch_bytes(cache.cfg, T), dtype=torch.uint8, device=dev)
    dst = torch.zeros((wl.batch, wl.n_kv_heads, wl.capacity), dtype=torch.float32, device=dev)
    B.dynts_score_block(cache.ctx, 0, q, kb, scratch, dst=dst, accumulate=False)
    lens = np.full(len(sample), n0, np.int32)
    Ks = np.zeros((len(sample), wl.n_kv_heads, wl.capacity, wl.head_dim))
    Ks[:, :, :n0] = f64(st["K"][sample])
    I_ref = orc.score_block(f64(q[sample]), f64(kb[sample]), Ks, lens, 1.0 / np.sqrt(wl.head_dim))
    got = f64(dst[sample])
    worst = assert_close(got[:, :, :n0], I_ref[:, :, :n0], "I full shape")
    # whole batch: every query row spends at most its whole weight on the cache
    tot = f64(dst.sum(-1))
    assert np.all(tot > 0) and np.all(tot <= T * wl.group * (1 + 1e-4))
    # planted critical keys collect far more than the median slot
    assert got[:, :, :n0].max() > 20 * np.median(got[:, :, wl.prompt:n0])
    cache.close()
