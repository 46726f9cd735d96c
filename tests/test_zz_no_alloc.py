"""The allocation-free entry point (dynts_decode_step_static: the launch's scratch in a static device array)
against dynts_decode_step on identical inputs, called through the C ABI: two calls in a row on two contexts of
different size, the second one smaller, so that the second call finds the array as the first one left it."""
import numpy as np
import pytest
import torch

from oracle import dynts_oracle as orc
from tests.helpers import assert_close, f64, i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2601_18383_amd import binding
    return binding


def _bf16(rng, *shape, scale=1.0):
    return torch.from_numpy(rng.standard_normal(shape).astype(np.float32) * scale).to(torch.bfloat16)


def _twin(B, Nb, Hq, Hkv, d, M, budget, window, E, launch_shape):
    cap = M + budget + window + E
    a = B.Cache(1, Nb, Hq, Hkv, d, cap, budget, window, E, launch_shape=launch_shape)
    b = B.Cache(1, Nb, Hq, Hkv, d, cap, budget, window, E, launch_shape=launch_shape)
    o = orc.OracleLayer(Nb, Hq, Hkv, d, cap, budget, window, E)
    return a, b, o, cap


def _state(c):
    torch.cuda.synchronize()
    return [t.clone() for t in (c.K, c.V, c.S, c.pos, c.seq_len, c.next_pos)]


def test_static_scratch_matches_workspace_entry_point(B):
    rng = np.random.default_rng(77)
    dev = torch.device("cuda:0")
    # first a larger context whose units are split over several workgroups (partials and tickets in use),
    # then a smaller one: fewer sequences, shorter cache, other head counts
    shapes = [dict(Nb=3, Hq=28, Hkv=4, d=128, M=40, budget=300, window=30, E=50, launch_shape=(64, 8)),
              dict(Nb=1, Hq=8, Hkv=2, d=64, M=9, budget=300, window=11, E=20, launch_shape=(16, 4))]
    pairs = []
    for sh in shapes:
        a, b, o, cap = _twin(B, **sh)
        Nb, Hq, Hkv, d, M = sh["Nb"], sh["Hq"], sh["Hkv"], sh["d"], sh["M"]
        K0, V0 = _bf16(rng, Nb, Hkv, M, d), _bf16(rng, Nb, Hkv, M, d)
        m = torch.full((Nb,), M, dtype=torch.int32, device=dev)
        for c in (a, b):
            B.dynts_prefill(c.ctx, 0, K0.to(dev), V0.to(dev), m)
        o.prefill(f64(K0), f64(V0), [M] * Nb)
        pairs.append((sh, a, b, o))
    # alternate between the two contexts step by step, so every call of the small one follows one of the large one
    n_steps = 420
    outs = {}
    for i, (sh, a, b, o) in enumerate(pairs):
        Nb, Hq, d = sh["Nb"], sh["Hq"], sh["d"]
        outs[i] = [torch.zeros((Nb, Hq, d), dtype=torch.float32, device=dev) for _ in range(2)] + \
                  [torch.zeros((Nb, Hq), dtype=torch.float32, device=dev) for _ in range(2)]
    for t in range(1, n_steps + 1):
        for i, (sh, a, b, o) in enumerate(pairs):
            Nb, Hq, Hkv, d = sh["Nb"], sh["Hq"], sh["Hkv"], sh["d"]
            q, k, v = _bf16(rng, Nb, Hq, d, scale=1.5), _bf16(rng, Nb, Hkv, d), _bf16(rng, Nb, Hkv, d)
            qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
            oa, ob, la, lb = outs[i]
            B.dynts_decode_step(a.ctx, 0, qd, kd, vd, oa, lse=la)
            B.dynts_decode_step_static(b.ctx, 0, qd, kd, vd, ob, lse=lb)
            torch.cuda.synchronize()
            assert torch.equal(oa, ob), "out differs at step %d, context %d" % (t, i)
            assert torch.equal(la, lb), "lse differs at step %d, context %d" % (t, i)
            # and both against the oracle, to the tolerance of the contract
            o.append(f64(k), f64(v))
            ref, alpha, lse_ref = o.attend(f64(q))
            o.update_scores(alpha)
            assert_close(f64(ob), ref, "static entry point out, step %d" % t)
            assert_close(f64(lb), lse_ref, "static entry point lse, step %d" % t)
            trig = o.due()
            if trig.any():
                keep, new_len = o.select(trig)
                for c in (a, b):
                    B.dynts_select_evict(c.ctx, 0, c.keep_idx, c.new_len, -1)
                torch.cuda.synchronize()
                assert torch.equal(a.keep_idx, b.keep_idx) and torch.equal(a.new_len, b.new_len)
                for c in (a, b):
                    B.dynts_compact(c.ctx, 0, c.keep_idx, c.new_len)
                # the oracle follows the GPU's list (near-ties may differ in float64)
                o.compact(i32(a.keep_idx), i32(a.new_len), trig)
    for i, (sh, a, b, o) in enumerate(pairs):
        for c in (a, b):
            B.dynts_update_scores(c.ctx, 0)
        for x, y in zip(_state(a), _state(b)):
            assert torch.equal(x, y)
        n = int(o.seq_len[0])
        assert_close(f64(b.S[0])[:, :, :n], o.S[:, :, :n], "S, context %d" % i)
        assert int(a.status.item()) == 0 and int(b.status.item()) == 0
        assert int(a.seq_len[0, 0].item()) < sh["M"] + n_steps  # evictions happened


def test_static_scratch_rejects_what_does_not_fit(B):
    # 512 sequences x 8 KV heads split 2-way: partials of 8192 rows x (128 + 2) x 8 bytes > 8 MiB
    cap = 64 + 1024 + 32 + 16
    cfg = B.make_config(1, 512, 32, 8, 128, cap, 1024, 32, 16)
    ctx = B.dynts_create(cfg)
    B.dynts_set_launch_shape(ctx, 8192, 8)
    need = B.dynts_ctx_workspace_bytes(ctx)
    assert need > B.DYNTS_STATIC_SCRATCH_BYTES
    dev = torch.device("cuda:0")
    t = lambda *s, dt=torch.bfloat16: torch.zeros(s, dtype=dt, device=dev)
    K, V = t(1, 512, 8, cap, 128), t(1, 512, 8, cap, 128)
    S, pos = t(1, 512, 8, cap, dt=torch.float32), t(1, 512, 8, cap, dt=torch.int32)
    sl, npos, npr = t(1, 512, dt=torch.int32), t(1, 512, dt=torch.int32), t(512, dt=torch.int32)
    ws, st = torch.zeros(need, dtype=torch.uint8, device=dev), t(1, dt=torch.int32)
    B.dynts_bind(ctx, K, V, S, pos, sl, npos, npr, ws, st)
    q, k, v = t(512, 32, 128), t(512, 8, 128), t(512, 8, 128)
    out = t(512, 32, 128, dt=torch.float32)
    with pytest.raises(B.DyntsError) as e:
        B.dynts_decode_step_static(ctx, 0, q, k, v, out)
    assert e.value.code == B.DYNTS_EWORKSPACE
    B.dynts_destroy(ctx)
