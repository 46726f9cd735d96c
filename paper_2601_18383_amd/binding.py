"""ctypes binding of libdynts.so: the same names as include/dynts.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the decode path runs in the
library's kernels.  There is no fallback: if the library is missing, import of this module
raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DYNTS_LIBRARY") or os.path.join(_HERE, "libdynts.so")  # override: development builds

DYNTS_OK = 0
DYNTS_EINVAL, DYNTS_ENULL, DYNTS_ESHAPE, DYNTS_ECAPACITY = -1, -2, -3, -4
DYNTS_ENOTBOUND, DYNTS_EWORKSPACE, DYNTS_EHIP, DYNTS_EPENDING = -5, -6, -7, -8
DYNTS_SCORE_ACCUMULATE, DYNTS_SCORE_EXTERNAL = 0, 1

EXPORTS = [
    "dynts_version", "dynts_strerror", "dynts_create", "dynts_destroy", "dynts_workspace_bytes",
    "dynts_bind", "dynts_prefill", "dynts_append", "dynts_decode_attend", "dynts_update_scores",
    "dynts_decode_attend_update", "dynts_decode_step", "dynts_select_evict", "dynts_compact",
    "dynts_decode_loop", "dynts_set_kernel_events", "dynts_set_kernel_event_list", "dynts_probe_read_stream",
    "dynts_score_block_scratch_bytes", "dynts_score_block",
    "dynts_predict_scratch_bytes", "dynts_predict_scores", "dynts_predictor_pack", "dynts_bind_paged",
    "dynts_set_launch_shape", "dynts_ctx_workspace_bytes",
    "dynts_decode_step_static", "dynts_probe_exp_rate", "dynts_probe_issue_mix", "dynts_hint_trigger",
]


class dynts_predictor(C.Structure):
    _fields_ = [("d", C.c_int32), ("m1", C.c_int32), ("m2", C.c_int32), ("activation", C.c_int32),
                ("packed", C.c_int32), ("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
                ("w3", C.c_void_p), ("b3", C.c_void_p)]


DYNTS_ACT_NONE, DYNTS_ACT_RELU, DYNTS_ACT_SILU = 0, 1, 2


class dynts_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("capacity", C.c_int32),
                ("budget", C.c_int32), ("window", C.c_int32), ("evict_every", C.c_int32),
                ("softmax_scale", C.c_float), ("score_mode", C.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python -m paper_2601_18383_amd.build` "
            "(there is no CPU fallback for the decode path)" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.dynts_version.restype = C.c_int
    lib.dynts_strerror.restype = C.c_char_p
    lib.dynts_strerror.argtypes = [C.c_int]
    lib.dynts_create.argtypes = [C.POINTER(dynts_config), C.POINTER(vp)]
    lib.dynts_destroy.argtypes = [vp]
    lib.dynts_workspace_bytes.restype = sz
    lib.dynts_workspace_bytes.argtypes = [C.POINTER(dynts_config)]
    lib.dynts_set_launch_shape.argtypes = [vp, i32, i32]
    lib.dynts_ctx_workspace_bytes.restype = sz
    lib.dynts_ctx_workspace_bytes.argtypes = [vp]
    lib.dynts_bind.argtypes = [vp] * 9 + [sz, vp]
    lib.dynts_bind_paged.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dynts_prefill.argtypes = [vp, i32, vp, vp, i32, vp, vp]
    lib.dynts_append.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.dynts_decode_attend.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.dynts_update_scores.argtypes = [vp, i32, vp]
    lib.dynts_decode_attend_update.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.dynts_decode_step.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.dynts_decode_step_static.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.dynts_hint_trigger.argtypes = [vp, i32]
    lib.dynts_select_evict.argtypes = [vp, i32, vp, i32, vp, i32, vp, vp]
    lib.dynts_compact.argtypes = [vp, i32, vp, vp, i32, vp, vp]
    lib.dynts_decode_loop.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp]
    lib.dynts_set_kernel_events.argtypes = [vp, vp, vp]
    lib.dynts_set_kernel_event_list.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), i32]
    lib.dynts_score_block_scratch_bytes.restype = sz
    lib.dynts_score_block_scratch_bytes.argtypes = [C.POINTER(dynts_config), i32]
    lib.dynts_score_block.argtypes = [vp, i32, vp, vp, i32, vp, vp, i32, vp, sz, vp]
    lib.dynts_predict_scratch_bytes.restype = sz
    lib.dynts_predict_scratch_bytes.argtypes = [C.POINTER(dynts_predictor), i32]
    lib.dynts_predictor_pack.argtypes = [vp, i32, i32, vp, vp]
    lib.dynts_predict_scores.argtypes = [C.POINTER(dynts_predictor), vp, i32, vp, i32, vp, sz, vp, vp, vp]
    lib.dynts_probe_read_stream.argtypes = [vp, sz, i32, C.c_uint32, vp, vp, vp, vp]
    lib.dynts_probe_exp_rate.argtypes = [i32, i32, vp, vp, vp, vp]
    lib.dynts_probe_issue_mix.argtypes = [i32, i32, i32, vp, vp, vp, vp]
    for name in EXPORTS:
        getattr(lib, name)
    return lib


lib = _load()


class DyntsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, lib.dynts_strerror(code).decode(), code))


def _ptr(t, dtype=None):
    """Device (or host) address of a tensor, None -> NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors crossing the C ABI must be contiguous"
    if dtype is not None:
        assert t.dtype == dtype, "expected %s, got %s" % (dtype, t.dtype)
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc, where):
    if rc != DYNTS_OK:
        raise DyntsError(rc, where)


def dynts_version():
    return int(lib.dynts_version())


def dynts_strerror(code):
    return lib.dynts_strerror(int(code)).decode()


def make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, capacity, budget, window, evict_every,
                softmax_scale=0.0, score_mode=DYNTS_SCORE_ACCUMULATE):
    return dynts_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, capacity, budget, window,
                        evict_every, softmax_scale, score_mode)


def dynts_create(cfg):
    ctx = C.c_void_p()
    _check(lib.dynts_create(C.byref(cfg), C.byref(ctx)), "dynts_create")
    return ctx


def dynts_destroy(ctx):
    _check(lib.dynts_destroy(ctx), "dynts_destroy")


def dynts_workspace_bytes(cfg):
    return int(lib.dynts_workspace_bytes(C.byref(cfg)))


def dynts_set_launch_shape(ctx, target_workgroups=0, waves_per_workgroup=0):
    _check(lib.dynts_set_launch_shape(ctx, target_workgroups, waves_per_workgroup), "dynts_set_launch_shape")


def dynts_ctx_workspace_bytes(ctx):
    return int(lib.dynts_ctx_workspace_bytes(ctx))


def dynts_bind(ctx, K, V, S, pos, seq_len, next_pos, n_prompt, workspace, status):
    _check(lib.dynts_bind(ctx, _ptr(K, torch.bfloat16), _ptr(V, torch.bfloat16), _ptr(S, torch.float32),
                          _ptr(pos, torch.int32), _ptr(seq_len, torch.int32), _ptr(next_pos, torch.int32),
                          _ptr(n_prompt, torch.int32), _ptr(workspace), workspace.numel() * workspace.element_size(),
                          _ptr(status, torch.int32)), "dynts_bind")


def dynts_bind_paged(ctx, K_pool, V_pool, block_table, free_stack, free_top, S, pos, seq_len, next_pos, n_prompt,
                     workspace, status):
    _check(lib.dynts_bind_paged(ctx, _ptr(K_pool, torch.bfloat16), _ptr(V_pool, torch.bfloat16), K_pool.shape[0],
                                _ptr(block_table, torch.int32), block_table.shape[-1], _ptr(free_stack, torch.int32),
                                _ptr(free_top, torch.int32), _ptr(S, torch.float32), _ptr(pos, torch.int32),
                                _ptr(seq_len, torch.int32), _ptr(next_pos, torch.int32), _ptr(n_prompt, torch.int32),
                                _ptr(workspace), workspace.numel() * workspace.element_size(),
                                _ptr(status, torch.int32)), "dynts_bind_paged")


def dynts_prefill(ctx, layer, K0, V0, m, stream=None):
    _check(lib.dynts_prefill(ctx, layer, _ptr(K0, torch.bfloat16), _ptr(V0, torch.bfloat16), K0.shape[2],
                             _ptr(m, torch.int32), _stream(stream)), "dynts_prefill")


def dynts_append(ctx, layer, k_new, v_new, s_new=None, active=None, stream=None):
    _check(lib.dynts_append(ctx, layer, _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
                            _ptr(s_new, torch.float32), _ptr(active, torch.uint8), _stream(stream)), "dynts_append")


def dynts_decode_attend(ctx, layer, q, out, lse=None, active=None, stream=None):
    _check(lib.dynts_decode_attend(ctx, layer, _ptr(q, torch.bfloat16), _ptr(active, torch.uint8),
                                   _ptr(out, torch.float32), _ptr(lse, torch.float32), _stream(stream)),
           "dynts_decode_attend")


def dynts_update_scores(ctx, layer, stream=None):
    _check(lib.dynts_update_scores(ctx, layer, _stream(stream)), "dynts_update_scores")


def dynts_decode_attend_update(ctx, layer, q, out, lse=None, active=None, stream=None):
    _check(lib.dynts_decode_attend_update(ctx, layer, _ptr(q, torch.bfloat16), _ptr(active, torch.uint8),
                                          _ptr(out, torch.float32), _ptr(lse, torch.float32), _stream(stream)),
           "dynts_decode_attend_update")


def dynts_decode_step(ctx, layer, q, k_new, v_new, out, s_new=None, active=None, lse=None, stream=None):
    _check(lib.dynts_decode_step(ctx, layer, _ptr(q, torch.bfloat16), _ptr(k_new, torch.bfloat16),
                                 _ptr(v_new, torch.bfloat16), _ptr(s_new, torch.float32),
                                 _ptr(active, torch.uint8), _ptr(out, torch.float32), _ptr(lse, torch.float32),
                                 _stream(stream)), "dynts_decode_step")


def dynts_decode_step_static(ctx, layer, q, k_new, v_new, out, s_new=None, active=None, lse=None, stream=None):
    _check(lib.dynts_decode_step_static(ctx, layer, _ptr(q, torch.bfloat16), _ptr(k_new, torch.bfloat16),
                                        _ptr(v_new, torch.bfloat16), _ptr(s_new, torch.float32),
                                        _ptr(active, torch.uint8), _ptr(out, torch.float32), _ptr(lse, torch.float32),
                                        _stream(stream)), "dynts_decode_step_static")


DYNTS_STATIC_SCRATCH_BYTES = 8 << 20


def dynts_hint_trigger(ctx, layer):
    _check(lib.dynts_hint_trigger(ctx, layer), "dynts_hint_trigger")


def dynts_select_evict(ctx, layer, keep_idx, new_len, k_keep=-1, trigger=None, stream=None):
    _check(lib.dynts_select_evict(ctx, layer, _ptr(trigger, torch.uint8), k_keep, _ptr(keep_idx, torch.int32),
                                  keep_idx.shape[-1], _ptr(new_len, torch.int32), _stream(stream)),
           "dynts_select_evict")


def dynts_compact(ctx, layer, keep_idx, new_len, trigger=None, stream=None):
    _check(lib.dynts_compact(ctx, layer, _ptr(trigger, torch.uint8), _ptr(keep_idx, torch.int32),
                             keep_idx.shape[-1], _ptr(new_len, torch.int32), _stream(stream)), "dynts_compact")


def dynts_decode_loop(ctx, n_steps, q, k_new, v_new, out, keep_idx=None, new_len=None, s_new=None, active=None,
                      evict_steps=None, trigger=None, out_step_stride=0, stream=None):
    """evict_steps: host uint8 tensor [n_steps] (CPU) or None."""
    if evict_steps is not None:
        assert evict_steps.device.type == "cpu" and evict_steps.dtype == torch.uint8
    _check(lib.dynts_decode_loop(ctx, n_steps, _ptr(q, torch.bfloat16), _ptr(k_new, torch.bfloat16),
                                 _ptr(v_new, torch.bfloat16), _ptr(s_new, torch.float32),
                                 _ptr(active, torch.uint8), _ptr(evict_steps), _ptr(trigger, torch.uint8),
                                 _ptr(out, torch.float32), out_step_stride, _ptr(keep_idx, torch.int32),
                                 _ptr(new_len, torch.int32), _stream(stream)), "dynts_decode_loop")


def dynts_set_kernel_events(ctx, start, stop):
    """start, stop: raw hipEvent_t handles (ints) or None."""
    _check(lib.dynts_set_kernel_events(ctx, start, stop), "dynts_set_kernel_events")


def dynts_set_kernel_event_list(ctx, starts, stops):
    """starts, stops: equally long lists of raw hipEvent_t handles (ctypes.c_void_p or ints)."""
    n = len(starts)
    assert len(stops) == n
    arr = C.c_void_p * max(n, 1)
    a = arr(*[s.value if isinstance(s, C.c_void_p) else s for s in starts]) if n else None
    b = arr(*[s.value if isinstance(s, C.c_void_p) else s for s in stops]) if n else None
    _check(lib.dynts_set_kernel_event_list(ctx, a, b, n), "dynts_set_kernel_event_list")


def dynts_score_block_scratch_bytes(cfg, n_queries):
    return int(lib.dynts_score_block_scratch_bytes(C.byref(cfg), n_queries))


def dynts_score_block(ctx, layer, q_blk, k_blk, scratch, dst=None, accumulate=True, active=None, stream=None):
    """q_blk bf16 [Nb][T][Hq][d], k_blk bf16 [Nb][T][Hkv][d] or None, scratch: device uint8/any tensor of
    at least dynts_score_block_scratch_bytes bytes; dst fp32 [Nb][Hkv][cap] or None (= the layer's S)."""
    T = q_blk.shape[1]
    _check(lib.dynts_score_block(ctx, layer, _ptr(q_blk, torch.bfloat16), _ptr(k_blk, torch.bfloat16), T,
                                 _ptr(active, torch.uint8), _ptr(dst, torch.float32), 1 if accumulate else 0,
                                 scratch.data_ptr(), scratch.numel() * scratch.element_size(), _stream(stream)),
           "dynts_score_block")


class Predictor:
    """The Importance Predictor's weights (device tensors, kept alive here) and its scratch; marshalling only."""

    def __init__(self, W1, b1, W2, b2, w3, b3, activation=DYNTS_ACT_RELU, max_batch=128, pack=True):
        """W1 [m1][d], W2 [m2][m1] row-major bf16 device tensors; pack=True repacks them once (library kernel)."""
        m1, d = W1.shape
        m2 = W2.shape[0]
        assert W2.shape == (m2, m1) and w3.shape == (m2,)
        if pack:
            W1, W2 = dynts_predictor_pack(W1), dynts_predictor_pack(W2)
        self.t = (W1, b1, W2, b2, w3, b3)
        self.w = dynts_predictor(d, m1, m2, activation, 1 if pack else 0, _ptr(W1, torch.bfloat16),
                                 _ptr(b1, torch.float32), _ptr(W2, torch.bfloat16), _ptr(b2, torch.float32),
                                 _ptr(w3, torch.bfloat16), _ptr(b3, torch.float32))
        need = max(dynts_predict_scratch_bytes(self.w, nb) for nb in (16, 32, 64, max_batch) if nb <= max_batch)
        self.scratch = torch.zeros(max(need, 256), dtype=torch.uint8, device=W1.device)


def dynts_predictor_pack(W, stream=None):
    """Row-major bf16 device matrix -> the tiled layout (a new tensor of the same shape and size)."""
    out = torch.empty_like(W)
    _check(lib.dynts_predictor_pack(_ptr(W, torch.bfloat16), W.shape[0], W.shape[1], out.data_ptr(), _stream(stream)),
           "dynts_predictor_pack")
    return out


PAGE_SLOTS = 64


PAGED_SHUFFLE_BELOW_BYTES = 200 << 20


class PagedCache:
    """The paged layout's buffers (page pools, block table, free stack) allocated with torch and bound.
    `K` and `V` give a dense [L][Nb][Hkv][cap][d] copy gathered through the block table (for inspection)."""

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, capacity, budget, window, evict_every,
                 n_pages=None, softmax_scale=0.0, external_scores=False, device="cuda:0", launch_shape=None,
                 page_order="auto"):
        self.cfg = make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, capacity, budget, window,
                               evict_every, softmax_scale,
                               DYNTS_SCORE_EXTERNAL if external_scores else DYNTS_SCORE_ACCUMULATE)
        self.ctx = dynts_create(self.cfg)
        if launch_shape is not None:
            dynts_set_launch_shape(self.ctx, *launch_shape)
        dev = torch.device(device)
        L, Nb, Hkv, cap, d = n_layers, batch, n_kv_heads, capacity, head_dim
        self.max_pages = (cap + PAGE_SLOTS - 1) // PAGE_SLOTS
        self.n_pages = L * Nb * Hkv * self.max_pages if n_pages is None else n_pages
        self.K_pool = torch.zeros((self.n_pages, PAGE_SLOTS, d), dtype=torch.bfloat16, device=dev)
        self.V_pool = torch.zeros((self.n_pages, PAGE_SLOTS, d), dtype=torch.bfloat16, device=dev)
        self.block_table = torch.full((L, Nb, Hkv, self.max_pages), -1, dtype=torch.int32, device=dev)
        # The order of the ids in the initial free stack decides where a unit's pages lie (see dynts_bind_paged in
        # dynts.h): "sequential" (ids in order: units that append in step get neighbouring pages), "shuffled" (a
        # fixed pseudo-random permutation), "auto" = shuffled when one layer's K/V fits the 256 MB memory-side cache.
        if page_order == "auto":
            kv_layer_bytes = 2 * Nb * Hkv * cap * d * 2
            page_order = "shuffled" if kv_layer_bytes <= PAGED_SHUFFLE_BELOW_BYTES else "sequential"
        if page_order == "shuffled":
            gen = torch.Generator().manual_seed(0x5EED)
            self.free_stack = torch.randperm(self.n_pages, generator=gen).to(torch.int32).to(dev)
        elif page_order == "sequential":
            self.free_stack = torch.arange(self.n_pages, dtype=torch.int32, device=dev)
        else:
            raise ValueError("page_order must be 'auto', 'sequential' or 'shuffled'")
        self.page_order = page_order
        self.free_top = torch.full((1,), self.n_pages, dtype=torch.int32, device=dev)
        self.S = torch.zeros((L, Nb, Hkv, cap), dtype=torch.float32, device=dev)
        self.pos = torch.zeros((L, Nb, Hkv, cap), dtype=torch.int32, device=dev)
        self.seq_len = torch.zeros((L, Nb), dtype=torch.int32, device=dev)
        self.next_pos = torch.zeros((L, Nb), dtype=torch.int32, device=dev)
        self.n_prompt = torch.zeros((Nb,), dtype=torch.int32, device=dev)
        self.status = torch.zeros((1,), dtype=torch.int32, device=dev)
        self.workspace = torch.zeros((dynts_ctx_workspace_bytes(self.ctx),), dtype=torch.uint8, device=dev)
        self.keep_idx = torch.zeros((Nb, Hkv, cap), dtype=torch.int32, device=dev)
        self.new_len = torch.zeros((Nb,), dtype=torch.int32, device=dev)
        dynts_bind_paged(self.ctx, self.K_pool, self.V_pool, self.block_table, self.free_stack, self.free_top, self.S,
                         self.pos, self.seq_len, self.next_pos, self.n_prompt, self.workspace, self.status)

    @classmethod
    def for_workload(cls, wl, device="cuda:0", n_layers=None, n_pages=None, launch_shape=None, page_order="auto"):
        return cls(wl.n_layers if n_layers is None else n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads,
                   wl.head_dim, wl.capacity, wl.budget, wl.window, wl.evict_every, n_pages=n_pages,
                   external_scores=wl.external_scores, device=device, launch_shape=launch_shape,
                   page_order=page_order)

    def _dense(self, pool):
        idx = self.block_table.clamp(min=0).long()                      # [L][Nb][Hkv][max_pages]
        rows = pool[idx]                                                # [...][max_pages][64][d]
        L, Nb, Hkv, mp = idx.shape
        return rows.reshape(L, Nb, Hkv, mp * PAGE_SLOTS, pool.shape[-1])[:, :, :, :self.cfg.capacity]

    @property
    def K(self):
        return self._dense(self.K_pool)

    @property
    def V(self):
        return self._dense(self.V_pool)

    def pages_in_use(self):
        """Pages the block table should hold for the current lengths, and pages missing from the free stack."""
        per_unit = (self.seq_len + PAGE_SLOTS - 1) // PAGE_SLOTS        # [L][Nb]
        return int(per_unit.sum().item()) * self.cfg.n_kv_heads, self.n_pages - int(self.free_top.item())

    def close(self):
        if self.ctx is not None:
            dynts_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def dynts_predict_scratch_bytes(w, batch):
    return int(lib.dynts_predict_scratch_bytes(C.byref(w), batch))


def dynts_predict_scores(pred, h, s_out, start=None, stop=None, stream=None):
    """pred: Predictor; h bf16 [Nb][d]; s_out fp32 [Nb][n_rep] (or [Nb])."""
    n_rep = s_out.shape[1] if s_out.dim() == 2 else 1
    _check(lib.dynts_predict_scores(C.byref(pred.w), _ptr(h, torch.bfloat16), h.shape[0], _ptr(s_out, torch.float32),
                                    n_rep, pred.scratch.data_ptr(), pred.scratch.numel(), start, stop,
                                    _stream(stream)), "dynts_predict_scores")


def dynts_probe_read_stream(buf, n_workgroups, sink, start=None, stop=None, magic=0x9E3779B9, stream=None):
    """buf: contiguous device tensor (its byte size a multiple of 16); sink: device tensor of >= 4 bytes."""
    nbytes = buf.numel() * buf.element_size()
    _check(lib.dynts_probe_read_stream(buf.data_ptr(), nbytes, n_workgroups, magic, sink.data_ptr(), start, stop,
                                       _stream(stream)), "dynts_probe_read_stream")


def dynts_probe_exp_rate(n_workgroups, iters, sink, start=None, stop=None, stream=None):
    """sink: device float tensor of >= 1 element."""
    _check(lib.dynts_probe_exp_rate(n_workgroups, iters, sink.data_ptr(), start, stop, _stream(stream)),
           "dynts_probe_exp_rate")


def dynts_probe_issue_mix(n_workgroups, iters, what, sink, start=None, stop=None, stream=None):
    """what: 1 = the MFMAs of a block-scoring tile, 2 = its vector instructions, 3 = both; sink: device float tensor."""
    _check(lib.dynts_probe_issue_mix(n_workgroups, iters, what, sink.data_ptr(), start, stop, _stream(stream)),
           "dynts_probe_issue_mix")


class Cache:
    """Device buffers of one context, allocated with torch and bound; marshalling only."""

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, capacity, budget, window,
                 evict_every, softmax_scale=0.0, external_scores=False, device="cuda:0", launch_shape=None):
        """launch_shape: None or (target_workgroups, waves_per_workgroup) for dynts_set_launch_shape."""
        self.cfg = make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, capacity, budget, window,
                               evict_every, softmax_scale,
                               DYNTS_SCORE_EXTERNAL if external_scores else DYNTS_SCORE_ACCUMULATE)
        self.ctx = dynts_create(self.cfg)
        if launch_shape is not None:
            dynts_set_launch_shape(self.ctx, *launch_shape)
        dev = torch.device(device)
        L, Nb, Hkv, cap, d = n_layers, batch, n_kv_heads, capacity, head_dim
        self.K = torch.zeros((L, Nb, Hkv, cap, d), dtype=torch.bfloat16, device=dev)
        self.V = torch.zeros((L, Nb, Hkv, cap, d), dtype=torch.bfloat16, device=dev)
        self.S = torch.zeros((L, Nb, Hkv, cap), dtype=torch.float32, device=dev)
        self.pos = torch.zeros((L, Nb, Hkv, cap), dtype=torch.int32, device=dev)
        self.seq_len = torch.zeros((L, Nb), dtype=torch.int32, device=dev)
        self.next_pos = torch.zeros((L, Nb), dtype=torch.int32, device=dev)
        self.n_prompt = torch.zeros((Nb,), dtype=torch.int32, device=dev)
        self.status = torch.zeros((1,), dtype=torch.int32, device=dev)
        self.workspace = torch.zeros((dynts_ctx_workspace_bytes(self.ctx),), dtype=torch.uint8, device=dev)
        self.keep_idx = torch.zeros((Nb, Hkv, cap), dtype=torch.int32, device=dev)
        self.new_len = torch.zeros((Nb,), dtype=torch.int32, device=dev)
        dynts_bind(self.ctx, self.K, self.V, self.S, self.pos, self.seq_len, self.next_pos, self.n_prompt,
                   self.workspace, self.status)

    @classmethod
    def for_workload(cls, wl, device="cuda:0", n_layers=None, launch_shape=None):
        return cls(wl.n_layers if n_layers is None else n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads,
                   wl.head_dim, wl.capacity, wl.budget, wl.window, wl.evict_every,
                   external_scores=wl.external_scores, device=device, launch_shape=launch_shape)

    def close(self):
        if self.ctx is not None:
            dynts_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
