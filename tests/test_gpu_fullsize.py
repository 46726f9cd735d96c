"""GPU parity at the benchmark's full shapes, in the launch configuration bench.py times.

The cache state is made by the input generator (never by the HIP path), the HIP path then
runs whole fused steps (append + attend + deferred score update), a score flush, a selection
and a compaction on the full batch, and the float64 oracle replays the same steps for a sample
of sequences, all KV heads, from the same state."""
import numpy as np
import pytest
import torch

from oracle import dynts_oracle as orc
from paper_2601_18383_amd import configs, synth
from tests.helpers import assert_close, f64, i32, near_tie_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2601_18383_amd import binding
    return binding


def _oracle_from_state(wl, st, sample, n0, external):
    o = orc.OracleLayer(len(sample), wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, wl.budget, wl.window,
                        wl.evict_every, external_scores=external)
    o.K[:, :, :n0] = f64(st["K"][sample])
    o.V[:, :, :n0] = f64(st["V"][sample])
    o.S[:, :, :n0] = f64(st["S"][sample])
    o.pos[:, :, :n0] = i32(st["pos"][sample])
    o.seq_len[:] = n0
    o.n_prompt[:] = wl.prompt
    o.next_pos[:] = 10 ** 6
    o.steps_done[:] = 0
    return o


def _run(B, name, layers, sample, n_steps=3, n0_delta=0):
    wl = configs.get(name)
    dev = torch.device("cuda:0")
    gen = synth.Synth(wl, dev)
    cache = B.Cache.for_workload(wl, device=dev)
    n0 = wl.steady_len + n0_delta
    assert n0 + n_steps <= wl.capacity
    worst = dict(out=0.0, S=0.0)
    out = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    lse = torch.zeros((wl.batch, wl.n_q_heads), dtype=torch.float32, device=dev)
    for layer in layers:
        st = gen.steady_state(layer, n0)
        if wl.external_scores:  # scores on the 64-level grid, as the external source would have supplied them
            ext = gen.external_scores(torch.arange(1, n0 - wl.prompt + 1))            # [n_think][Nb]
            st["S"][:, :, wl.prompt:] = ext.t().unsqueeze(1).expand(wl.batch, wl.n_kv_heads, n0 - wl.prompt)
        cache.K[layer, :, :, :n0] = st["K"]
        cache.V[layer, :, :, :n0] = st["V"]
        cache.S[layer, :, :, :n0] = st["S"]
        cache.pos[layer, :, :, :n0] = st["pos"]
        cache.seq_len[layer].fill_(n0)
        cache.next_pos[layer].fill_(10 ** 6)
        cache.n_prompt.fill_(wl.prompt)
        o = _oracle_from_state(wl, st, sample, n0, wl.external_scores)
        steps = torch.arange(50000, 50000 + n_steps)
        q = gen.q(layer, steps)
        k, v = gen.kv(layer, steps)
        s = None
        if wl.external_scores:
            s = gen.external_scores(steps).unsqueeze(-1).expand(n_steps, wl.batch, wl.n_kv_heads).contiguous()
        for i in range(n_steps):
            out.fill_(7.0)
            B.dynts_decode_step(cache.ctx, layer, q[i], k[i], v[i], out, s_new=s[i] if s is not None else None,
                                lse=lse)
            o.append(f64(k[i][sample]), f64(v[i][sample]), f64(s[i][sample]) if s is not None else None)
            o_out, alpha, o_lse = o.attend(f64(q[i][sample]))
            o.update_scores(alpha)
            worst["out"] = max(worst["out"], assert_close(f64(out[sample]), o_out, "%s layer %d step %d out" % (name, layer, i)))
            assert_close(f64(lse[sample]), o_lse, "lse")
        B.dynts_update_scores(cache.ctx, layer)
        n1 = n0 + n_steps
        assert np.all(i32(cache.seq_len[layer]) == n1)
        S_gpu = f64(cache.S[layer][sample])
        worst["S"] = max(worst["S"], assert_close(S_gpu[:, :, :n1], o.S[:, :, :n1], "S after flush"))
        assert np.array_equal(f64(cache.K[layer][sample][:, :, :n1]), o.K[:, :, :n1])  # appended rows landed
        assert np.array_equal(i32(cache.pos[layer][sample][:, :, :n1]), o.pos[:, :, :n1])
        # selection on the full batch; oracle on the sampled sequences with the SAME score arrays
        cache.keep_idx.fill_(-1)
        B.dynts_select_evict(cache.ctx, layer, cache.keep_idx, cache.new_len)
        keep_gpu, len_gpu = i32(cache.keep_idx[sample]), i32(cache.new_len[sample])
        pos_gpu = i32(cache.pos[layer][sample])
        keep_same, len_same = orc.select(S_gpu, pos_gpu, o.seq_len, o.n_prompt, wl.window, wl.budget)
        assert np.array_equal(len_gpu, len_same) and np.all(len_gpu == wl.steady_len)
        assert np.array_equal(keep_gpu, keep_same), "selection differs from the oracle on identical scores"
        keep_ref, len_ref = o.select()
        for bi in range(len(sample)):
            for h in range(wl.n_kv_heads):
                assert near_tie_ok(o.S[bi, h], wl.prompt, n1 - wl.window, keep_gpu[bi, h, :len_gpu[bi]].tolist(),
                                   keep_ref[bi, h, :len_ref[bi]].tolist())
        # the retained set is the best one by the GPU's own scores: properties that hold at any size
        if wl.budget > 0:
            kk = keep_gpu[0, 0, wl.prompt:wl.prompt + wl.budget]
            cand = S_gpu[0, 0, wl.prompt:n1 - wl.window]
            cut = np.sort(cand)[::-1][wl.budget - 1]
            assert np.all(S_gpu[0, 0, kk] >= cut) and np.all(np.diff(kk) > 0)
        B.dynts_compact(cache.ctx, layer, cache.keep_idx, cache.new_len)
        o.compact(keep_same, len_same)
        n2 = wl.steady_len
        assert np.all(i32(cache.seq_len[layer]) == n2)
        assert np.array_equal(f64(cache.K[layer][sample][:, :, :n2]), o.K[:, :, :n2])
        assert np.array_equal(f64(cache.V[layer][sample][:, :, :n2]), o.V[:, :, :n2])
        assert np.array_equal(i32(cache.pos[layer][sample][:, :, :n2]), o.pos[:, :, :n2])
        assert_close(f64(cache.S[layer][sample][:, :, :n2]), o.S[:, :, :n2], "S after compaction")
        # whole-batch invariants: prompt kept, positions strictly increasing, window = newest tokens
        pos_all = i32(cache.pos[layer][:, :, :n2])
        assert np.all(pos_all[:, :, :wl.prompt] == np.arange(wl.prompt))
        assert np.all(np.diff(pos_all, axis=-1) > 0)
        assert np.all(pos_all[:, :, -1] == 10 ** 6 + n_steps - 1)
        assert np.all(np.isinf(f64(cache.S[layer][:, :, :wl.prompt])))
    assert int(cache.status.item()) == 0
    cache.close()
    del cache
    torch.cuda.empty_cache()
    return worst


def test_cfg2_full_shape(B):
    _run(B, "cfg2", [0], [0], n_steps=4, n0_delta=31)


def test_cfg3_full_shape(B):
    _run(B, "cfg3", [0], [0, 13, 31], n_steps=3, n0_delta=30)


def test_cfg4_full_shape_first_and_last_layer(B):
    _run(B, "cfg4", [0, 31], [5, 63], n_steps=2, n0_delta=17)


def test_cfg5_full_shape_heavy_tails(B):
    _run(B, "cfg5", [0, 27], [0, 77, 127], n_steps=3, n0_delta=9)


def test_cfg5b_external_scores_with_ties(B):
    _run(B, "cfg5b", [3], [1, 126], n_steps=2, n0_delta=14)


def test_paper_budget_settings_full_shape(B):
    """The paper's budget settings (Sec. 6.1): a full cache of 5000 (3000) thinking tokens, one trigger that
    keeps 0.4 (0.3) of the selection window and moves every row behind the first evicted one."""
    wl = configs.get("paper_qwen_5000")
    _run(B, "paper_qwen_5000", [0], [0, 31], n_steps=2, n0_delta=wl.evict_every - 2)
    wl = configs.get("paper_llama_3000")
    _run(B, "paper_llama_3000", [0], [7], n_steps=2, n0_delta=wl.evict_every - 2)


def test_other_policies_full_shape(B):
    """The same kernels under two other cache policies: sliding window with sinks (nothing kept by score) and
    heavy-hitter eviction of one token per step."""
    _run(B, "policy_window", [0], [3], n_steps=2, n0_delta=62)
    _run(B, "policy_h2o", [0], [9, 30], n_steps=1, n0_delta=0)


def test_ragged_batch_full_shape(B):
    """cfg3 shape with per-sequence lengths and a mask of finished sequences, through the native loop."""
    wl = configs.get("cfg3")
    dev = torch.device("cuda:0")
    gen = synth.Synth(wl, dev)
    cache = B.Cache.for_workload(wl, device=dev)
    rng = np.random.default_rng(3)
    lens = rng.integers(wl.prompt + 1, wl.capacity - 8, wl.batch).astype(np.int32)
    lens[0], lens[1] = wl.prompt + 1, wl.capacity - 8
    nmax = int(lens.max())
    st = gen.steady_state(0, nmax)
    cache.K[0, :, :, :nmax] = st["K"]; cache.V[0, :, :, :nmax] = st["V"]
    cache.S[0, :, :, :nmax] = st["S"]; cache.pos[0, :, :, :nmax] = st["pos"]
    cache.seq_len[0].copy_(torch.from_numpy(lens)); cache.next_pos[0].fill_(10 ** 6); cache.n_prompt.fill_(wl.prompt)
    T = 6
    active = (rng.random((T, wl.batch)) < 0.7).astype(np.uint8)
    active[:, 0] = 1
    active[2:, 5] = 0
    steps = torch.arange(777, 777 + T)
    q = gen.q(0, steps).unsqueeze(1).contiguous()
    k, v = gen.kv(0, steps)
    k, v = k.unsqueeze(1).contiguous(), v.unsqueeze(1).contiguous()
    outs = torch.full((T, 1, wl.batch, wl.n_q_heads, wl.head_dim), 7.0, dtype=torch.float32, device=dev)
    B.dynts_decode_loop(cache.ctx, T, q, k, v, outs, active=torch.from_numpy(active).to(dev),
                        out_step_stride=outs[0].numel())
    B.dynts_update_scores(cache.ctx, 0)
    sample = [0, 1, 5, 17]
    o = orc.OracleLayer(len(sample), wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, wl.budget, wl.window,
                        wl.evict_every)
    o.K[:, :, :nmax] = f64(st["K"][sample]); o.V[:, :, :nmax] = f64(st["V"][sample])
    o.S[:, :, :nmax] = f64(st["S"][sample]); o.pos[:, :, :nmax] = i32(st["pos"][sample])
    o.seq_len[:] = lens[sample]; o.n_prompt[:] = wl.prompt; o.next_pos[:] = 10 ** 6
    for i in range(T):
        act = np.ascontiguousarray(active[i, sample])
        o.append(f64(k[i, 0][sample]), f64(v[i, 0][sample]), None, act)
        ref = np.full((len(sample), wl.n_q_heads, wl.head_dim), 7.0)
        o_out, alpha, _ = o.attend(f64(q[i, 0][sample]), act, ref)
        o.update_scores(alpha, act)
        assert_close(f64(outs[i, 0][sample]), o_out, "ragged out step %d" % i)
    assert np.array_equal(i32(cache.seq_len[0][sample]), o.seq_len)
    assert np.array_equal(i32(cache.seq_len[0]), lens + active.sum(0))
    S_gpu = f64(cache.S[0][sample])
    for bi in range(len(sample)):
        n = int(o.seq_len[bi])
        assert_close(S_gpu[bi, :, :n], o.S[bi, :, :n], "ragged S")
        assert np.array_equal(i32(cache.pos[0][sample][bi, :, :n]), o.pos[bi, :, :n])
    assert int(cache.status.item()) == 0


def test_results_are_reproducible_bit_for_bit_and_stream_independent(B):
    """The same steps from the same state give the same bits (partials are merged in index order, every score has
    one owner), on the null stream and on a stream of the caller's own."""
    wl = configs.get("cfg3")
    dev = torch.device("cuda:0")
    gen = synth.Synth(wl, dev)
    n0 = wl.steady_len + 40
    st = gen.steady_state(0, n0)
    T = wl.evict_every - 40 + 3           # runs through one trigger
    steps = torch.arange(9000, 9000 + T)
    q = gen.q(0, steps).unsqueeze(1).contiguous()
    k, v = gen.kv(0, steps)
    k, v = k.unsqueeze(1).contiguous(), v.unsqueeze(1).contiguous()
    flags = torch.zeros(T, dtype=torch.uint8)
    flags[wl.evict_every - 40 - 1] = 1
    results = []
    for use_stream in (None, None, torch.cuda.Stream()):
        cache = B.Cache.for_workload(wl, device=dev)
        cache.K[0, :, :, :n0] = st["K"]; cache.V[0, :, :, :n0] = st["V"]
        cache.S[0, :, :, :n0] = st["S"]; cache.pos[0, :, :, :n0] = st["pos"]
        cache.seq_len[0].fill_(n0); cache.next_pos[0].fill_(10 ** 6); cache.n_prompt.fill_(wl.prompt)
        outs = torch.zeros((T, 1, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        if use_stream is None:
            B.dynts_decode_loop(cache.ctx, T, q, k, v, outs, cache.keep_idx, cache.new_len, evict_steps=flags,
                                out_step_stride=outs[0].numel())
            B.dynts_update_scores(cache.ctx, 0)
        else:
            with torch.cuda.stream(use_stream):
                B.dynts_decode_loop(cache.ctx, T, q, k, v, outs, cache.keep_idx, cache.new_len, evict_steps=flags,
                                    out_step_stride=outs[0].numel())
                B.dynts_update_scores(cache.ctx, 0)
        torch.cuda.synchronize()
        assert int(cache.status.item()) == 0 and int(cache.seq_len[0, 0].item()) == wl.steady_len + 3
        n = wl.steady_len + 3
        results.append((outs.clone(), cache.S[0, :, :, :n].clone(), cache.K[0, :, :, :n].clone(),
                        cache.pos[0, :, :, :n].clone()))
        cache.close()
    for other in results[1:]:
        for a, b in zip(results[0], other):
            assert torch.equal(a, b)
