"""Host side of the C ABI, no GPU needed: the built library loads, exports every symbol the header
declares, and turns bad arguments into error codes before anything could be launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2601_18383_amd import binding, build
    if build.is_stale():
        build.build()
    return binding


def test_library_exports_every_declared_symbol(B):
    header = open(os.path.join(ROOT, "include", "dynts.h")).read()
    declared = set(re.findall(r"\b(dynts_[a-z_]+)\s*\(", header))
    declared -= {"dynts_config", "dynts_ctx"}
    assert len(declared) >= 15
    raw = C.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(raw, name), "libdynts.so does not export %s" % name
    assert declared == set(B.EXPORTS), "binding and header disagree: %s" % (declared ^ set(B.EXPORTS))
    for name in B.EXPORTS:  # the Python binding carries the same names
        assert callable(getattr(B, name))


def test_version_and_error_strings(B):
    assert B.dynts_version() >= 100
    seen = set()
    for code in range(0, -9, -1):
        text = B.dynts_strerror(code)
        assert text and text != "unknown error"
        seen.add(text)
    assert len(seen) == 9
    assert B.dynts_strerror(-99) == "unknown error"


def _cfg(B, **kw):
    base = dict(n_layers=2, batch=3, n_q_heads=8, n_kv_heads=2, head_dim=128, capacity=400, budget=256, window=64,
                evict_every=16, softmax_scale=0.0, score_mode=0)
    base.update(kw)
    return B.make_config(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(n_layers=0), -1), (dict(batch=-1), -1), (dict(evict_every=0), -1), (dict(budget=-1), -1),
    (dict(score_mode=2), -1), (dict(softmax_scale=-1.0), -1), (dict(softmax_scale=float("nan")), -1),
    (dict(head_dim=96), -3), (dict(n_q_heads=7), -3), (dict(n_q_heads=34, n_kv_heads=2), -3),
    (dict(capacity=335), -4), (dict(n_kv_heads=128, n_q_heads=128, head_dim=128), -3),
    (dict(capacity=(1 << 22) + 1), -3),
])
def test_create_rejects_bad_config(B, kw, code):
    cfg = _cfg(B, **kw)
    ctx = C.c_void_p()
    assert B.lib.dynts_create(C.byref(cfg), C.byref(ctx)) == code
    assert not ctx.value
    assert B.dynts_workspace_bytes(cfg) == 0


def test_create_and_calls_before_bind(B):
    cfg = _cfg(B)
    assert B.dynts_workspace_bytes(cfg) > 0
    assert B.lib.dynts_create(None, C.byref(C.c_void_p())) == B.DYNTS_ENULL
    assert B.lib.dynts_create(C.byref(cfg), None) == B.DYNTS_ENULL
    ctx = B.dynts_create(cfg)
    one = C.c_void_p(16)  # a non-null, 16-byte aligned dummy address: never dereferenced before the checks fail
    assert B.lib.dynts_update_scores(ctx, 0, None) == B.DYNTS_ENOTBOUND
    assert B.lib.dynts_decode_attend(ctx, 0, one, None, one, None, None) == B.DYNTS_ENOTBOUND
    assert B.lib.dynts_compact(ctx, 0, None, one, 400, one, None) == B.DYNTS_ENOTBOUND
    assert B.lib.dynts_update_scores(None, 0, None) == B.DYNTS_ENULL
    # bind: null pointers, short or misaligned workspace
    need = B.dynts_workspace_bytes(cfg)
    args = [one] * 8
    assert B.lib.dynts_bind(ctx, *args[:7], None, need, one) == B.DYNTS_ENULL
    assert B.lib.dynts_bind(ctx, *args[:7], C.c_void_p(256), need - 1, one) == B.DYNTS_EWORKSPACE
    assert B.lib.dynts_bind(ctx, *args[:7], C.c_void_p(264), need, one) == B.DYNTS_EWORKSPACE
    assert B.lib.dynts_bind(ctx, C.c_void_p(8), *args[1:7], C.c_void_p(256), need, one) == B.DYNTS_EINVAL
    assert B.lib.dynts_bind(ctx, *args[:7], C.c_void_p(256), need, one) == B.DYNTS_OK
    # bound now: argument checks come before any launch
    assert B.lib.dynts_update_scores(ctx, 2, None) == B.DYNTS_EINVAL       # layer out of range
    assert B.lib.dynts_update_scores(ctx, 0, None) == B.DYNTS_OK           # nothing outstanding: no launch
    assert B.lib.dynts_decode_attend(ctx, 0, None, None, one, None, None) == B.DYNTS_ENULL
    assert B.lib.dynts_decode_attend(ctx, 0, C.c_void_p(8), None, one, None, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_decode_step(ctx, 0, one, None, one, None, None, one, None, None) == B.DYNTS_ENULL
    assert B.lib.dynts_prefill(ctx, 0, one, one, 0, one, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_prefill(ctx, 0, one, one, 401, one, None) == B.DYNTS_ECAPACITY
    assert B.lib.dynts_select_evict(ctx, 0, None, -1, None, 400, one, None) == B.DYNTS_ENULL
    assert B.lib.dynts_select_evict(ctx, 0, None, -1, one, 0, one, None) == B.DYNTS_ECAPACITY
    assert B.lib.dynts_compact(ctx, 0, None, one, 0, one, None) == B.DYNTS_ECAPACITY
    assert B.lib.dynts_decode_loop(ctx, -1, one, one, one, None, None, None, None, one, 0, None, None, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_decode_loop(ctx, 0, one, one, one, None, None, None, None, one, 0, None, None, None) == B.DYNTS_OK
    assert B.lib.dynts_set_kernel_events(ctx, one, None) == B.DYNTS_EINVAL
    B.dynts_destroy(ctx)
    # external-score mode requires the scores at append
    ctx = B.dynts_create(_cfg(B, score_mode=1))
    assert B.lib.dynts_bind(ctx, *args[:7], C.c_void_p(256), B.dynts_workspace_bytes(_cfg(B, score_mode=1)), one) == 0
    assert B.lib.dynts_append(ctx, 0, one, one, None, None, None) == B.DYNTS_ENULL
    assert B.lib.dynts_decode_step(ctx, 0, one, one, one, None, None, one, None, None) == B.DYNTS_ENULL
    B.dynts_destroy(ctx)


def test_argument_checks_of_the_wider_entry_points(B):
    """Block scoring, predictor, paged binding, read-stream probe: every refusal comes before any launch."""
    cfg = _cfg(B)
    one = C.c_void_p(256)
    need = B.dynts_workspace_bytes(cfg)
    ctx = B.dynts_create(cfg)
    assert B.lib.dynts_bind(ctx, *([one] * 7), one, need, one) == B.DYNTS_OK
    # block scoring
    assert B.dynts_score_block_scratch_bytes(cfg, 0) == 0 and B.dynts_score_block_scratch_bytes(cfg, 16) > 0
    sb = B.dynts_score_block_scratch_bytes(cfg, 16)
    assert B.lib.dynts_score_block(ctx, 0, None, None, 16, None, None, 1, one, sb, None) == B.DYNTS_ENULL
    assert B.lib.dynts_score_block(ctx, 0, one, None, 0, None, None, 1, one, sb, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_score_block(ctx, 0, one, None, 16, None, None, 1, one, sb - 1, None) == B.DYNTS_EWORKSPACE
    assert B.lib.dynts_score_block(ctx, 0, C.c_void_p(8), None, 16, None, None, 1, one, sb, None) == B.DYNTS_EINVAL
    # paged binding: table too short for the capacity, missing stack
    args = [one, one, 64, one, 1, one, one, one, one, one, one, one, one, need, one]
    assert B.lib.dynts_bind_paged(ctx, *args) == B.DYNTS_ECAPACITY            # 1 page of 64 slots < capacity
    args[4] = (cfg.capacity + 63) // 64
    assert B.lib.dynts_bind_paged(ctx, *(args[:5] + [None] + args[6:])) == B.DYNTS_ENULL
    assert B.lib.dynts_bind_paged(ctx, *(args[:2] + [0] + args[3:])) == B.DYNTS_EINVAL
    assert B.lib.dynts_bind_paged(ctx, *args) == B.DYNTS_OK
    B.dynts_destroy(ctx)
    # predictor
    w = B.dynts_predictor(64, 128, 32, 1, 0, 256, 0, 256, 0, 256, 0)
    assert B.dynts_predict_scratch_bytes(w, 8) > 0 and B.dynts_predict_scratch_bytes(w, 0) == 0
    nb = B.dynts_predict_scratch_bytes(w, 8)
    assert B.lib.dynts_predict_scores(C.byref(w), None, 8, one, 1, one, nb, None, None, None) == B.DYNTS_ENULL
    assert B.lib.dynts_predict_scores(C.byref(w), one, 8, one, 0, one, nb, None, None, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_predict_scores(C.byref(w), one, 8, one, 1, one, nb - 1, None, None, None) == B.DYNTS_EWORKSPACE
    assert B.lib.dynts_predict_scores(C.byref(w), one, 8, one, 1, one, nb, one, None, None) == B.DYNTS_EINVAL
    bad = B.dynts_predictor(64, 128, 40, 1, 0, 256, 0, 256, 0, 256, 0)        # m2 not a multiple of 16
    assert B.lib.dynts_predict_scores(C.byref(bad), one, 8, one, 1, one, nb, None, None, None) == B.DYNTS_ESHAPE
    assert B.lib.dynts_predictor_pack(None, 16, 32, one, None) == B.DYNTS_ENULL
    assert B.lib.dynts_predictor_pack(one, 10, 32, C.c_void_p(512), None) == B.DYNTS_ESHAPE
    assert B.lib.dynts_predictor_pack(one, 16, 32, one, None) == B.DYNTS_EINVAL   # in place is refused
    # read-stream probe
    assert B.lib.dynts_probe_read_stream(None, 1024, 4, 0, one, None, None, None) == B.DYNTS_ENULL
    assert B.lib.dynts_probe_read_stream(one, 1000, 4, 0, one, None, None, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_probe_read_stream(one, 1024, 0, 0, one, None, None, None) == B.DYNTS_EINVAL
    # the other two measurement aids
    assert B.lib.dynts_probe_exp_rate(4, 10, None, None, None, None) == B.DYNTS_ENULL
    assert B.lib.dynts_probe_exp_rate(0, 10, one, None, None, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_probe_issue_mix(4, 10, 3, None, None, None, None) == B.DYNTS_ENULL
    for what in (0, 4, -1):
        assert B.lib.dynts_probe_issue_mix(4, 10, what, one, None, None, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_probe_issue_mix(0, 10, 3, one, None, None, None) == B.DYNTS_EINVAL
    assert B.lib.dynts_probe_issue_mix(4, 0, 3, one, None, None, None) == B.DYNTS_EINVAL


def test_missing_library_is_an_import_error(monkeypatch, tmp_path):
    import importlib
    import paper_2601_18383_amd.binding as binding
    monkeypatch.setenv("DYNTS_LIBRARY", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        importlib.reload(binding)
    monkeypatch.delenv("DYNTS_LIBRARY")
    importlib.reload(binding)


def test_bench_result_line_has_the_contract_fields():
    """bench.py's output object, formatted from stand-in numbers (no GPU): every field of the contract."""
    import argparse
    import json
    import bench
    from paper_2601_18383_amd import configs
    wl = configs.get("cfg3")
    r = dict(value=1.0, ms_per_step=1.0, roofline={"bound": "hbm", "achieved": 1.0, "peak": 8000.0, "unit": "GB/s",
                                                    "frac": 0.1, "traffic": None},
             whole_step_gbs=1.0, seq_steps_per_s=1.0, evictions_timed=1, first_timed_step=1, active_min=1,
             active_max=2)
    for traj in (False, True):
        args = argparse.Namespace(steps=4, warmup=1, trajectory=traj)
        line = json.loads(json.dumps(bench.result_line(args, wl, r, None)))
        for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                    "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
            assert key in line
        assert "workload" in line["config"] and "model" not in line["config"]


def test_bench_trigger_schedule_matches_the_oracle_layer():
    """bench.py's host-side schedule (trigger steps, cache length per step) against the oracle's own run."""
    import bench
    import numpy as np
    from oracle import dynts_oracle as orc
    from paper_2601_18383_amd import configs
    import dataclasses
    rng = np.random.default_rng(0)
    for (M, budget, window, E) in [(3, 8, 4, 4), (5, 6, 10, 9), (2, 4, 12, 7)]:
        wl = dataclasses.replace(configs.get("cfg1"), prompt=M, budget=budget, window=window, evict_every=E)
        lay = orc.OracleLayer(1, 2, 1, 4, wl.capacity, budget, window, E)
        lay.prefill(rng.standard_normal((1, 1, M, 4)), rng.standard_normal((1, 1, M, 4)), [M])
        T = 90
        flags = bench.evict_flags(wl, 0, T)
        for t in range(1, T + 1):
            lay.append(rng.standard_normal((1, 1, 4)), rng.standard_normal((1, 1, 4)))
            assert int(lay.seq_len[0]) == bench.cache_len_before_step(wl, t)
            trig = lay.due()
            assert int(trig[0]) == int(flags[t - 1])
            if trig[0]:
                keep, new_len = lay.select(trig)
                lay.compact(keep, new_len, trig)
