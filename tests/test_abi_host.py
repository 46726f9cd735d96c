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


def test_missing_library_is_an_import_error(monkeypatch, tmp_path):
    import importlib
    import paper_2601_18383_amd.binding as binding
    monkeypatch.setenv("DYNTS_LIBRARY", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        importlib.reload(binding)
    monkeypatch.delenv("DYNTS_LIBRARY")
    importlib.reload(binding)
