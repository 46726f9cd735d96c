"""GPU parity of the paged (block-table) cache layout: the same decode path, K/V rows found through a page
table, pages popped on append and pushed back after compaction.  Compared with the float64 oracle through a
dense view gathered from the pools."""
import numpy as np
import pytest
import torch

from oracle import dynts_oracle as orc
from paper_2601_18383_amd import configs, synth
from tests.helpers import SideBySide, assert_close, f64, i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2601_18383_amd import binding
    return binding


def _bf16(rng, *shape, scale=1.0):
    return torch.from_numpy(rng.standard_normal(shape).astype(np.float32) * scale).to(torch.bfloat16)


def _check_pages(cache):
    """Every page is either free or held by exactly one unit; the units hold what their lengths need."""
    need, missing = cache.pages_in_use()
    assert need == missing, (need, missing)
    top = int(cache.free_top.item())
    free = i32(cache.free_stack)[:top].tolist()
    L, Nb = cache.seq_len.shape
    held = []
    bt, sl = i32(cache.block_table), i32(cache.seq_len)
    for l in range(L):
        for b in range(Nb):
            for h in range(cache.cfg.n_kv_heads):
                held += bt[l, b, h, :(sl[l, b] + 63) // 64].tolist()
    assert len(set(held)) == len(held) and not (set(held) & set(free)) and len(set(free)) == len(free)
    assert sorted(held + free) == list(range(cache.n_pages))


@pytest.mark.parametrize("one_workgroup", [False, True])
@pytest.mark.parametrize("mode", ["unfused", "fused", "step", "step+hint"])
@pytest.mark.parametrize("d,Hq,Hkv", [(64, 8, 2), (128, 28, 4)])
def test_trajectory_paged(B, mode, d, Hq, Hkv, one_workgroup):
    """Several pages per unit, ragged prompts, evictions that free pages, a sequence that finishes early.
    one_workgroup: a single workgroup per unit, so that every wave walks a range of tiles behind its first one
    (the launch shape of the large workloads) instead of one tile each."""
    rng = np.random.default_rng(300 + d + Hq)
    Nb, M_max, budget, window, E, T = 3, 37, 150, 19, 91, 420
    cap = M_max + budget + window + E
    # (both initial page orders are exercised: ids in order with the single-workgroup shape, shuffled otherwise)
    cache = B.PagedCache(1, Nb, Hq, Hkv, d, cap, budget, window, E, launch_shape=(1, 8) if one_workgroup else None,
                         page_order="sequential" if one_workgroup else "shuffled")
    assert sorted(cache.free_stack.tolist()) == list(range(cache.n_pages))
    o = orc.OracleLayer(Nb, Hq, Hkv, d, cap, budget, window, E)
    sbs = SideBySide(B, cache, 0, o, mode)
    sbs.prefill(_bf16(rng, Nb, Hkv, M_max, d), _bf16(rng, Nb, Hkv, M_max, d), [37, 5, 20])
    _check_pages(cache)
    last = [T, 130, T]
    for t in range(1, T + 1):
        active = np.array([t <= last[b] for b in range(Nb)], np.uint8)
        trig = sbs.step(_bf16(rng, Nb, Hq, d, scale=1.5), _bf16(rng, Nb, Hkv, d), _bf16(rng, Nb, Hkv, d), active=active,
                        check_scores=(t % 7 == 0 or mode == "unfused"))
        if trig.any() or t % 50 == 0:
            _check_pages(cache)
    sbs.check_scores()
    sbs.check_state()
    assert sbs.evictions >= 2 and int(cache.status.item()) == 0
    assert int(cache.seq_len[0, 1].item()) == sbs.o.seq_len[1]


def test_pool_shared_between_sequences_and_exhaustion(B):
    """A pool smaller than batch x capacity: eviction returns pages that other sequences then take; when the pool
    runs dry the status word says so."""
    rng = np.random.default_rng(41)
    dev = torch.device("cuda:0")
    Nb, Hq, Hkv, d = 4, 8, 2, 64
    M, budget, window, E = 10, 64, 20, 108          # capacity 202 slots = 4 pages per unit
    cap = M + budget + window + E
    n_pages = Nb * Hkv * 3 + 2                      # not enough for everyone at full length (would be 32)
    cache = B.PagedCache(1, Nb, Hq, Hkv, d, cap, budget, window, E, n_pages=n_pages)
    o = orc.OracleLayer(Nb, Hq, Hkv, d, cap, budget, window, E)
    sbs = SideBySide(B, cache, 0, o, "step")
    sbs.prefill(_bf16(rng, Nb, Hkv, M, d), _bf16(rng, Nb, Hkv, M, d), [M] * Nb)
    # 180 steps: every unit needs 3 pages (190 slots), the pool has 26
    for t in range(1, 181):
        sbs.step(_bf16(rng, Nb, Hq, d), _bf16(rng, Nb, Hkv, d), _bf16(rng, Nb, Hkv, d), check_scores=False)
    assert int(cache.status.item()) == 0
    _check_pages(cache)
    assert int(cache.free_top.item()) == 2
    # step 182 fills the cache (10 + 192 = 202) only after a 4th page: 8 units want one, 2 are left -> exhaustion
    q, k, v = _bf16(rng, Nb, Hq, d), _bf16(rng, Nb, Hkv, d), _bf16(rng, Nb, Hkv, d)
    for t in range(181, 184):
        B.dynts_decode_step(cache.ctx, 0, q.to(dev), k.to(dev), v.to(dev), sbs.out)
    assert int(cache.status.item()) & 4
    assert int(cache.free_top.item()) == 0


def test_cfg3_full_shape_paged(B):
    """cfg3 at full shape through the paged layout: steady state reached by the path itself, sampled sequences
    against the oracle replaying the same steps from a snapshot."""
    wl = configs.get("cfg3")
    dev = torch.device("cuda:0")
    gen = synth.Synth(wl, dev)
    cache = B.PagedCache.for_workload(wl, device=dev)
    K0, V0 = gen.prompt_kv(0)
    B.dynts_prefill(cache.ctx, 0, K0, V0, torch.full((wl.batch,), wl.prompt, dtype=torch.int32, device=dev))
    out = torch.zeros((1, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    T0 = wl.budget + wl.window + wl.evict_every + 5       # just past the first eviction
    steps = torch.arange(1, T0 + 1)
    q = gen.q(0, steps).unsqueeze(1).contiguous()
    k, v = gen.kv(0, steps)
    k, v = k.unsqueeze(1).contiguous(), v.unsqueeze(1).contiguous()
    flags = torch.zeros(T0, dtype=torch.uint8)
    flags[wl.budget + wl.window + wl.evict_every - 1] = 1
    B.dynts_decode_loop(cache.ctx, T0, q, k, v, out, cache.keep_idx, cache.new_len, evict_steps=flags)
    B.dynts_update_scores(cache.ctx, 0)
    assert int(cache.status.item()) == 0
    n0 = wl.steady_len + 5
    assert np.all(i32(cache.seq_len[0]) == n0)
    _check_pages(cache)
    # snapshot -> oracle, then three more fused steps on both
    sample = [0, 17]
    o = orc.OracleLayer(len(sample), wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, wl.budget, wl.window,
                        wl.evict_every)
    Kd, Vd = cache.K[0][sample], cache.V[0][sample]
    o.K[:, :, :n0] = f64(Kd[:, :, :n0]); o.V[:, :, :n0] = f64(Vd[:, :, :n0])
    o.S[:, :, :n0] = f64(cache.S[0][sample][:, :, :n0]); o.pos[:, :, :n0] = i32(cache.pos[0][sample][:, :, :n0])
    o.seq_len[:] = n0; o.n_prompt[:] = wl.prompt; o.next_pos[:] = i32(cache.next_pos[0][sample])
    steps2 = torch.arange(T0 + 1, T0 + 4)
    q2 = gen.q(0, steps2); k2, v2 = gen.kv(0, steps2)
    o1 = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    for i in range(3):
        B.dynts_decode_step(cache.ctx, 0, q2[i], k2[i], v2[i], o1)
        o.append(f64(k2[i][sample]), f64(v2[i][sample]))
        ref, alpha, _ = o.attend(f64(q2[i][sample]))
        o.update_scores(alpha)
        assert_close(f64(o1[sample]), ref, "paged cfg3 out, step %d" % i)
    B.dynts_update_scores(cache.ctx, 0)
    n1 = n0 + 3
    assert_close(f64(cache.S[0][sample][:, :, :n1]), o.S[:, :, :n1], "paged cfg3 S")
    assert np.array_equal(f64(cache.K[0][sample][:, :, :n1]), o.K[:, :, :n1])
    cache.close()


def test_two_layers_share_one_pool(B):
    """Two layers with different inputs draw from and return to the same pool."""
    rng = np.random.default_rng(43)
    Nb, Hq, Hkv, d = 2, 8, 2, 64
    M, budget, window, E = 9, 70, 11, 75
    cap = M + budget + window + E
    cache = B.PagedCache(2, Nb, Hq, Hkv, d, cap, budget, window, E, n_pages=2 * Nb * Hkv * 3)
    layers = []
    for l in range(2):
        o = orc.OracleLayer(Nb, Hq, Hkv, d, cap, budget, window, E)
        sbs = SideBySide(B, cache, l, o, "step")
        sbs.prefill(_bf16(rng, Nb, Hkv, M, d), _bf16(rng, Nb, Hkv, M, d), [M, 4])
        layers.append(sbs)
    for t in range(1, 2 * E + budget + window + 3):
        for sbs in layers:
            sbs.step(_bf16(rng, Nb, Hq, d), _bf16(rng, Nb, Hkv, d), _bf16(rng, Nb, Hkv, d), check_scores=(t % 13 == 0))
        if t % 40 == 0:
            _check_pages(cache)
    for sbs in layers:
        sbs.check_scores()
        sbs.check_state()
        assert sbs.evictions == 2
    _check_pages(cache)
    assert int(cache.status.item()) == 0


def test_block_scoring_reads_the_paged_layout(B):
    """dynts_score_block on a paged cache equals the oracle on the dense view (keys found through the block table)."""
    rng = np.random.default_rng(44)
    dev = torch.device("cuda:0")
    Nb, Hq, Hkv, d, T = 3, 28, 4, 128, 40
    M, budget, window, E = 13, 200, 17, 90
    cap = M + budget + window + E
    cache = B.PagedCache(1, Nb, Hq, Hkv, d, cap, budget, window, E)
    o = orc.OracleLayer(Nb, Hq, Hkv, d, cap, budget, window, E)
    sbs = SideBySide(B, cache, 0, o, "step")
    sbs.prefill(_bf16(rng, Nb, Hkv, M, d), _bf16(rng, Nb, Hkv, M, d), [13, 4, 9])
    # the first trigger falls on step budget + window + E = 307 (90 slots = more than a page leave every unit);
    # 33 steps later the units have grown back over a page boundary, into pages that were returned
    for t in range(1, 341):
        sbs.step(_bf16(rng, Nb, Hq, d), _bf16(rng, Nb, Hkv, d), _bf16(rng, Nb, Hkv, d), check_scores=False)
    assert sbs.evictions == 1
    _check_pages(cache)
    sbs.check_scores()
    q = _bf16(rng, Nb, T, Hq, d, scale=1.5)
    kb = _bf16(rng, Nb, T, Hkv, d)
    scratch = torch.empty(B.dynts_score_block_scratch_bytes(cache.cfg, T), dtype=torch.uint8, device=dev)
    dst = torch.zeros((Nb, Hkv, cap), dtype=torch.float32, device=dev)
    B.dynts_score_block(cache.ctx, 0, q.to(dev), kb.to(dev), scratch, dst=dst, accumulate=False)
    I_ref = orc.score_block(f64(q), f64(kb), o.K, o.seq_len, o.scale)
    for b in range(Nb):
        n = int(o.seq_len[b])
        assert_close(f64(dst)[b, :, :n], I_ref[b, :, :n], "paged block scoring, sequence %d" % b)
