#!/usr/bin/env python3
"""Decode-step benchmark of the DynTS hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: for every layer the
fused append + decode attention + deferred score update, and on trigger steps the score
flush, top-k selection and in-place compaction -- all inside the timed region, inputs
resident in HBM.  Prints ONE JSON line (see the README for the fields).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(wl, n_list, n_active):
    """Bytes one layer-step must move (K+V rows read, scores read+written unless they come from
    outside, q in, out written, the appended K/V row written), for cache lengths n_list of the
    active sequences."""
    d, Hkv, Hq, M = wl.head_dim, wl.n_kv_heads, wl.n_q_heads, wl.prompt
    s_bytes = 0 if wl.external_scores else 8
    kv = sum(Hkv * (n * d * 2 * 2 + (n - M) * s_bytes) for n in n_list)
    return kv + n_active * Hq * d * (2 + 4) + 2 * n_active * Hkv * d * 2


class HipEvents:
    """Raw hipEvent pairs, so the library can record them around its streaming kernel."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0
            assert self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.pairs[i][0], self.pairs[i][1])
        assert rc == 0, rc
        return ms.value

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def make_pools(gen, wl, t0, n, device):
    """q [n][L][Nb][Hq][d], k/v [n][L][Nb][Hkv][d] for decode steps t0+1 .. t0+n."""
    import torch
    steps = torch.arange(t0 + 1, t0 + n + 1)
    qs, ks, vs = [], [], []
    for l in range(wl.n_layers):
        qs.append(gen.q(l, steps))
        k, v = gen.kv(l, steps)
        ks.append(k)
        vs.append(v)
    q = torch.stack(qs, 1).contiguous()
    k = torch.stack(ks, 1).contiguous()
    v = torch.stack(vs, 1).contiguous()
    s = None
    if wl.external_scores:
        s = gen.external_scores(steps).unsqueeze(-1).expand(n, wl.batch, wl.n_kv_heads).contiguous()
    return q, k, v, s


def active_pool(lengths, t0, n, device):
    """uint8 [n][Nb] on the device: is sequence b still decoding at steps t0+1 .. t0+n; None if all are."""
    import torch
    steps = torch.arange(t0 + 1, t0 + n + 1).view(-1, 1)
    act = (steps <= lengths.view(1, -1))
    if bool(act.all()):
        return None, act
    return act.to(torch.uint8).to(device).contiguous(), act


def n_triggers_through(wl, t):
    """Triggers among decode steps 1..t: the first when the thinking tokens fill budget + window +
    evict_every slots, then one every evict_every steps (Sec. 5, the count of eviction events)."""
    full = wl.budget + wl.window + wl.evict_every
    return 0 if t < full else (t - full) // wl.evict_every + 1


def evict_flags(wl, t0, n):
    """Host flags of the trigger steps among t0+1 .. t0+n."""
    import torch
    f = torch.zeros(n, dtype=torch.uint8)
    for i in range(n):
        t = t0 + 1 + i
        f[i] = n_triggers_through(wl, t) - n_triggers_through(wl, t - 1)
    return f


def cache_len_before_step(wl, t):
    """Slots attended at decode step t (after the append, before any eviction of that step)."""
    return wl.prompt + t - n_triggers_through(wl, t - 1) * wl.evict_every


def read_stream_rates(B, nbytes, dev):
    """GB/s of the library's plain read-stream probe on buffers of nbytes: the same buffer again and again
    (what a cache re-read every step can get from the memory-side cache) and a rotation of buffers that
    together exceed it (what HBM alone delivers).  Median of 20 launches each, best of three grid sizes."""
    import torch
    nbytes = max(nbytes, 1 << 20)
    n_rot = max(2, (2 << 30) // nbytes)
    bufs = [torch.ones(nbytes // 4, dtype=torch.int32, device=dev) for _ in range(n_rot)]
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    ev = HipEvents(1)
    a, b = ev.pairs[0]
    best = {"same_buffer": 0.0, "rotating_buffers": 0.0}
    for grid in (512, 1024, 2048):
        for mode in best:
            ts = []
            for it in range(24):
                buf = bufs[0] if mode == "same_buffer" else bufs[it % n_rot]
                B.dynts_probe_read_stream(buf, grid, sink, a, b)
                torch.cuda.synchronize()
                if it >= 4:
                    ts.append(ev.elapsed_ms(0))
            ts.sort()
            best[mode] = max(best[mode], nbytes / (ts[len(ts) // 2] * 1e-3) / 1e9)
    ev.close()
    return {k: round(v, 1) for k, v in best.items()}


def time_periods(B, cache, gen, wl, lengths, out, t0, dev, n_periods=5, kernel_events=0, period=None):
    """n_periods windows of evict_every whole steps each, starting at decode step t0 + 1 (t0 a step right after a
    trigger, so each window ends on its one trigger), timed with events on the launch stream and no host
    synchronisation in between.  Returns the full_period block; with kernel_events > 0 also the average
    duration of that many attend launches (dispatch-attached events) and their algorithmic bytes."""
    import torch
    E, L = period or wl.evict_every, wl.n_layers
    n = E * n_periods
    q, k, v, s = make_pools(gen, wl, t0, n, dev)
    flags = evict_flags(wl, t0, n)
    act, act_host = active_pool(lengths, t0, n, dev)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_periods + 1)]
    ev = None
    if kernel_events:
        kernel_events = min(kernel_events, n * L)
        ev = HipEvents(kernel_events)
        B.dynts_set_kernel_event_list(cache.ctx, [a for a, _ in ev.pairs], [b for _, b in ev.pairs])
    torch.cuda.synchronize()
    marks[0].record()
    for i in range(n_periods):
        a, b = i * E, (i + 1) * E
        B.dynts_decode_loop(cache.ctx, E, q[a:b], k[a:b], v[a:b], out, cache.keep_idx, cache.new_len,
                            s_new=s[a:b] if s is not None else None, active=act[a:b] if act is not None else None,
                            evict_steps=flags[a:b], trigger=act[a:b] if act is not None else None)
        marks[i + 1].record()
    torch.cuda.synchronize()
    if ev:
        B.dynts_set_kernel_event_list(cache.ctx, [], [])
    ms = sorted(marks[i].elapsed_time(marks[i + 1]) / E for i in range(n_periods))
    med = ms[len(ms) // 2]
    act_counts = [int(act_host[i].sum()) for i in range(n)]
    step_bytes = sum(algorithmic_bytes(wl, [cache_len_before_step(wl, t0 + 1 + i)] * act_counts[i], act_counts[i])
                     for i in range(n)) * L / n
    r = {"windows": n_periods, "steps_each": E, "evictions": int(flags.sum()), "first_step": t0 + 1,
         "ms_per_step_median": round(med, 5), "ms_per_step_min": round(ms[0], 5), "ms_per_step_max": round(ms[-1], 5),
         "steps_per_s": round(1e3 / med, 2), "algorithmic_GBps": round(step_bytes / (med * 1e-3) / 1e9, 1)}
    if ev:
        k_ms = [ev.elapsed_ms(i) for i in range(kernel_events)]
        ev.close()
        # launches are step-major, layer-minor: launch j belongs to step j // L
        kb = [algorithmic_bytes(wl, [cache_len_before_step(wl, t0 + 1 + j // L)] * act_counts[j // L], act_counts[j // L])
              for j in range(kernel_events)]
        k_avg = sum(k_ms) / len(k_ms)
        r["attend_kernel_us"] = round(k_avg * 1e3, 2)
        r["attend_kernel_GBps"] = round(sum(kb) / len(kb) / (k_avg * 1e-3) / 1e9, 1)
        r["attend_kernel_frac_of_peak"] = round(r["attend_kernel_GBps"] / HBM_PEAK_GBS, 4)
    return r


def steady_cache(B, gen, wl, dev, n_layers=None, n0=None):
    """A cache at steady state made by the input generator (not through the path): every layer holds
    wl.steady_len slots, as right after a trigger (or n0 slots of a cache that has not triggered yet).
    Returns (cache, t0) with t0 the decode step it stands for."""
    import torch
    L = wl.n_layers if n_layers is None else n_layers
    cache = B.Cache.for_workload(wl, device=dev, n_layers=L)
    t0 = wl.budget + wl.window + wl.evict_every   # the step of the first trigger: budget + window thinking tokens after it
    if n0 is None:
        n0 = wl.steady_len
    else:
        t0 = n0 - wl.prompt
    for l in range(L):
        st = gen.steady_state(l, n0)
        if wl.external_scores:
            ext = gen.external_scores(torch.arange(1, n0 - wl.prompt + 1))
            st["S"][:, :, wl.prompt:] = ext.t().unsqueeze(1).expand(wl.batch, wl.n_kv_heads, n0 - wl.prompt)
        cache.K[l, :, :, :n0] = st["K"]
        cache.V[l, :, :, :n0] = st["V"]
        cache.S[l, :, :, :n0] = st["S"]
        cache.pos[l, :, :, :n0] = st["pos"]
        del st
    cache.seq_len.fill_(n0)
    cache.next_pos.fill_(10 ** 6)
    cache.n_prompt.fill_(wl.prompt)
    return cache, t0


def run_other_workloads(args, main_name):
    """The other configurations of the benchmark, each at steady state for a few whole eviction periods: a bounded
    companion to the main line (cache brought to its third trigger through the path, one more period of warm-up,
    three timed; all sequences are still decoding at that point)."""
    import dataclasses
    import torch
    from paper_2601_18383_amd import binding as B, configs, synth

    dev = torch.device("cuda:0")
    res = {}
    for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg5b", "cfg4_full_kv"):
        if name == main_name:
            continue
        t_w = time.perf_counter()
        note = None
        n0 = None
        if name == "cfg4_full_kv":
            # the comparison without eviction at the END of cfg4's decode (steps 8129 .. 8192: every token still
            # cached, 8640 -> 8704 slots), attention + append only, no scores; 4 of the 32 layers (9 GB of K/V)
            base = configs.get("cfg4")
            wl = dataclasses.replace(base, name=name, n_layers=4, budget=base.steps[1], window=0, evict_every=64,
                                     external_scores=True)
            n0 = base.prompt + base.steps[1] - 64
            note = "cfg4 without eviction over decode steps 8145..8192 (8656..8704 cached slots), 4 of 32 layers, no trigger"
        else:
            wl = configs.get(name)
        gen = synth.Synth(wl, dev)
        if name == "cfg4_full_kv":   # 8640 slots through the path would take minutes: the generator makes the state
            cache, t0 = steady_cache(B, gen, wl, dev, n0=n0)
            lengths = torch.full((wl.batch,), 10 ** 6, dtype=torch.int64)
            out = torch.zeros((wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
        else:                        # through the path itself, so that the eviction pattern is the path's own
            cache, out, lengths, t0 = run_up(B, gen, wl, dev)
        period = 16 if name == "cfg4_full_kv" else wl.evict_every
        time_periods(B, cache, gen, wl, lengths, out, t0, dev, n_periods=1, period=period)                  # warm-up
        r = time_periods(B, cache, gen, wl, lengths, out, t0 + period, dev, n_periods=3, kernel_events=256, period=period)
        assert int(cache.status[0]) == 0, "device status word set in %s: %d" % (name, int(cache.status[0]))
        r["layers"] = wl.n_layers
        if note:
            r["note"] = note
        res[name] = r
        cache.close()
        del cache, out, gen
        torch.cuda.empty_cache()
        log("other workload %s: %s (%.1f s)" % (name, r, time.perf_counter() - t_w))
    return res


def run_up(B, gen, wl, dev, paged=False, launch_shape=None, t_stop=None):
    """A cache brought to steady state through the path itself (untimed): prompt rows, then decode steps up to
    the third trigger (or t_stop).  Returns (cache, out, lengths, t) with t the last step taken."""
    import torch
    cache = (B.PagedCache if paged else B.Cache).for_workload(wl, device=dev, launch_shape=launch_shape)
    L = wl.n_layers
    for l in range(L):
        K0, V0 = gen.prompt_kv(l)
        m = torch.full((wl.batch,), wl.prompt, dtype=torch.int32, device=dev)
        B.dynts_prefill(cache.ctx, l, K0, V0, m)
    out = torch.zeros((L, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    E = wl.evict_every
    t_steady = (wl.budget + wl.window + E) + 2 * E if t_stop is None else t_stop   # the step of the third trigger
    lengths = gen.decode_lengths()  # per-sequence decode lengths (ragged workloads); finished ones are masked
    per_step = L * wl.batch * (wl.n_q_heads + 2 * wl.n_kv_heads) * wl.head_dim * 2
    block = max(1, min(256, (1 << 30) // per_step))   # input pool of at most 1 GiB
    t = 0
    t_pre = time.perf_counter()
    while t < t_steady:
        n = min(block, t_steady - t)
        q, k, v, s = make_pools(gen, wl, t, n, dev)
        act, _ = active_pool(lengths, t, n, dev)
        B.dynts_decode_loop(cache.ctx, n, q, k, v, out, cache.keep_idx, cache.new_len, s_new=s, active=act,
                            evict_steps=evict_flags(wl, t, n), trigger=act)
        t += n
    torch.cuda.synchronize()
    log("%s: steady state reached at step %d in %.1f s; seq_len[0,0]=%d status=%d" %
        (wl.name, t, time.perf_counter() - t_pre, int(cache.seq_len[0, 0]), int(cache.status[0])))
    return cache, out, lengths, t


def run_gpu(args, wl):
    import torch
    from paper_2601_18383_amd import binding as B, synth

    dev = torch.device("cuda:0")
    props = torch.cuda.get_device_properties(0)
    log("device: %s, %d CUs, %.0f GiB" % (props.name, props.multi_processor_count, props.total_memory / 2 ** 30))
    gen = synth.Synth(wl, dev)
    cache, out, lengths, t = run_up(B, gen, wl, dev, paged=args.paged, launch_shape=args.launch_shape)
    L, E = wl.n_layers, wl.evict_every

    # ---- warmup + timed window, inputs resident ---------------------------------------------
    qw, kw, vw, sw = make_pools(gen, wl, t, args.warmup, dev) if args.warmup else (None,) * 4
    fw = evict_flags(wl, t, args.warmup)
    qt, kt, vt, stt = make_pools(gen, wl, t + args.warmup, args.steps, dev)
    ft = evict_flags(wl, t + args.warmup, args.steps)
    aw, _ = active_pool(lengths, t, args.warmup, dev) if args.warmup else (None, None)
    at, at_host = active_pool(lengths, t + args.warmup, args.steps, dev)
    torch.cuda.synchronize()
    if args.warmup:
        B.dynts_decode_loop(cache.ctx, args.warmup, qw, kw, vw, out, cache.keep_idx, cache.new_len, s_new=sw,
                            active=aw, evict_steps=fw, trigger=aw)
    # the K timed steps go out as up to 8 windows of whole eviction periods, with an event between them on
    # the launch stream (no host synchronisation inside the timed region)
    n_win = max(1, min(8, args.steps // E))
    win = args.steps // n_win // E * E if args.steps >= E else args.steps
    bounds = [i * win for i in range(n_win)] + [args.steps]
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_win + 1)]
    # (a single window needs no marks: the two synchronisations bracket it; an event record costs the launch
    # stream about 10 us, which a 20-step window would feel)
    use_marks = n_win > 1
    calls = []   # (the views of the resident inputs are made before the clock starts)
    for i in range(n_win):
        a, b = bounds[i], bounds[i + 1]
        calls.append((b - a, qt[a:b], kt[a:b], vt[a:b], stt[a:b] if stt is not None else None,
                      at[a:b] if at is not None else None, ft[a:b]))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if use_marks:
        marks[0].record()
    for i, (n_i, q_i, k_i, v_i, s_i, a_i, f_i) in enumerate(calls):
        B.dynts_decode_loop(cache.ctx, n_i, q_i, k_i, v_i, out, cache.keep_idx, cache.new_len,
                            s_new=s_i, active=a_i, evict_steps=f_i, trigger=a_i)
        if use_marks:
            marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    win_ms = (sorted(marks[i].elapsed_time(marks[i + 1]) / (bounds[i + 1] - bounds[i]) for i in range(n_win))
              if use_marks else [dt * 1e3 / args.steps])
    t_end = t + args.warmup + args.steps
    assert int(cache.status[0]) == 0, "device status word set: %d" % int(cache.status[0])
    longest = int(lengths.argmax())
    assert int(cache.seq_len[0, longest]) == cache_len_before_step(wl, t_end + 1) - 1

    # ---- the streaming kernel alone, timed with HIP events recorded by the library ------------
    n_prof = 64 // E * E or 64   # a pass of its own, whatever --steps says: whole periods, 64 steps
    qp, kp, vp, sp = make_pools(gen, wl, t_end, n_prof, dev)
    fp = evict_flags(wl, t_end, n_prof)
    # (the same native loop as the timed window, so the launches are back to back; every attend launch
    # of the loop takes one event pair, in call order: step-major, layer-minor)
    ap_dev, ap_host = active_pool(lengths, t_end, n_prof, dev)
    ev = HipEvents(n_prof * L)
    B.dynts_set_kernel_event_list(cache.ctx, [a for a, _ in ev.pairs], [b for _, b in ev.pairs])
    B.dynts_decode_loop(cache.ctx, n_prof, qp, kp, vp, out, cache.keep_idx, cache.new_len, s_new=sp,
                        active=ap_dev, evict_steps=fp, trigger=ap_dev)
    B.dynts_set_kernel_event_list(cache.ctx, [], [])
    launch_bytes = []
    for i in range(n_prof):
        n_act = int(ap_host[i].sum())
        launch_bytes.append(algorithmic_bytes(wl, [cache_len_before_step(wl, t_end + 1 + i)] * n_act, n_act))
    torch.cuda.synchronize()
    k_ms = [ev.elapsed_ms(i) for i in range(n_prof * L)]
    ev.close()
    k_avg_ms = sum(k_ms) / len(k_ms)
    bytes_launch = sum(launch_bytes) / len(launch_bytes)
    achieved = bytes_launch / (k_avg_ms * 1e-3) / 1e9
    traffic = None  # HBM bytes per launch from the committed rocprofv3 counter summary, if there is one
    tf = os.path.join(ROOT, "profiles", "attend_kernel_%s_hbm_counters.txt" % args.workload)
    if os.path.exists(tf):
        for ln in open(tf):
            if ln.startswith("hbm_bytes_per_launch:"):
                traffic = int(ln.split(":")[1])
    # ---- whole eviction periods (the "+evict" leg of the metric), when the requested window is too short to
    # hold several: 5 in-stream windows of one period each, every one with exactly one trigger in it
    full_period = None
    if args.steps < 5 * E:
        # (as many windows, up to 5, as end before the shortest sequence does: the batch stays full)
        n_per = min(5, (int(lengths.min()) - (t_end + n_prof)) // E)
        if n_per >= 1:
            full_period = time_periods(B, cache, gen, wl, lengths, out, t_end + n_prof, dev, n_periods=n_per)
    stream = read_stream_rates(B, int(bytes_launch) // 16 * 16, dev)
    roofline = {"bound": "hbm", "kernel": "attend_kernel<%d,attend,pending,append>" % wl.head_dim,
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": ("profiles/attend_kernel_%s_hbm_counters.txt: rocprofv3 --pmc FETCH_SIZE and "
                                   "WRITE_SIZE of this workload's steady state, scaled by a 1 GiB copy; a committed "
                                   "summary, not measured in this run" % args.workload) if traffic else None,
                "kernel_avg_us": round(k_avg_ms * 1e3, 2), "algorithmic_bytes_per_launch": int(bytes_launch),
                "launches_timed": len(k_ms), "plain_read_stream_GBps": stream,
                "frac_of_plain_read_stream": round(achieved / max(stream.values()), 4)}
    act_counts = [int(at_host[i].sum()) for i in range(args.steps)]
    step_bytes = sum(algorithmic_bytes(wl, [cache_len_before_step(wl, t + args.warmup + 1 + i)] * act_counts[i],
                                       act_counts[i]) for i in range(args.steps)) * L
    return dict(value=args.steps / dt, ms_per_step=dt / args.steps * 1e3, roofline=roofline,
                whole_step_gbs=step_bytes / dt / 1e9, seq_steps_per_s=sum(act_counts) / dt,
                evictions_timed=int(ft.sum()), first_timed_step=t + args.warmup + 1,
                active_min=min(act_counts), active_max=max(act_counts), full_period=full_period,
                page_order=getattr(cache, "page_order", None),
                windows={"n": n_win, "steps_each": win, "ms_per_step_median": round(win_ms[len(win_ms) // 2], 5),
                         "ms_per_step_min": round(win_ms[0], 5), "ms_per_step_max": round(win_ms[-1], 5)})


def run_trajectory(args, wl):
    """The whole decode of the workload, from the prompt to the end of the longest sequence, through
    the native loop; finished sequences of a ragged batch are masked out.  Inputs are generated block
    by block (untimed); only the loops are timed, one host synchronisation per block."""
    import torch
    from paper_2601_18383_amd import binding as B, synth

    dev = torch.device("cuda:0")
    gen = synth.Synth(wl, dev)
    cache = (B.PagedCache if args.paged else B.Cache).for_workload(wl, device=dev)
    L = wl.n_layers
    for l in range(L):
        K0, V0 = gen.prompt_kv(l)
        m = torch.full((wl.batch,), wl.prompt, dtype=torch.int32, device=dev)
        B.dynts_prefill(cache.ctx, l, K0, V0, m)
    out = torch.zeros((L, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    lengths = gen.decode_lengths()
    t_max = int(lengths.max()) if not args.max_steps else min(int(lengths.max()), args.max_steps)
    per_step = L * wl.batch * (wl.n_q_heads + 2 * wl.n_kv_heads) * wl.head_dim * 2
    block = max(1, min(256, (1 << 30) // per_step))
    t, busy, seq_steps, alg_bytes, n_evict, t_log = 0, 0.0, 0, 0, 0, time.perf_counter()
    while t < t_max:
        n = min(block, t_max - t)
        q, k, v, s = make_pools(gen, wl, t, n, dev)
        act, act_host = active_pool(lengths, t, n, dev)
        flags = evict_flags(wl, t, n)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.dynts_decode_loop(cache.ctx, n, q, k, v, out, cache.keep_idx, cache.new_len, s_new=s, active=act,
                            evict_steps=flags, trigger=act)
        torch.cuda.synchronize()
        busy += time.perf_counter() - t0
        for i in range(n):
            na = int(act_host[i].sum())
            seq_steps += na
            alg_bytes += L * algorithmic_bytes(wl, [cache_len_before_step(wl, t + 1 + i)] * na, na)
        n_evict += int(flags.sum())
        t += n
        if time.perf_counter() - t_log > 20:
            t_log = time.perf_counter()
            log("  step %d of %d, %.1f s in the loops so far" % (t, t_max, busy))
    assert int(cache.status[0]) == 0, "device status word set: %d" % int(cache.status[0])
    longest = int(lengths.argmax())
    if t_max == int(lengths.max()):
        assert int(cache.seq_len[0, longest]) == cache_len_before_step(wl, t_max + 1) - 1
    roofline = {"bound": "hbm", "kernel": "whole run, all kernels", "achieved": round(alg_bytes / busy / 1e9, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(alg_bytes / busy / 1e9 / HBM_PEAK_GBS, 4),
                "traffic": None}
    return dict(value=t_max / busy, ms_per_step=busy / t_max * 1e3, roofline=roofline,
                whole_step_gbs=alg_bytes / busy / 1e9, seq_steps_per_s=seq_steps / busy, evictions_timed=n_evict,
                first_timed_step=1, active_min=int(act_host[-1].sum()), active_max=wl.batch, steps=t_max)


def run_score_block(args, wl):
    """Block scoring (Eq. importance-score over a block of T answer queries with their own keys) on a
    generator-made steady-state cache of layer 0: both kernels of one call, timed with events on the
    launch stream.  A step is one call on the full batch."""
    import torch
    from paper_2601_18383_amd import binding as B, synth

    dev = torch.device("cuda:0")
    gen = synth.Synth(wl, dev)
    cache = B.Cache.for_workload(wl, device=dev)
    T, n0 = args.score_block, wl.steady_len + wl.evict_every // 2
    st = gen.steady_state(0, n0)
    cache.K[0, :, :, :n0] = st["K"]
    cache.S[0, :, :, :n0] = st["S"]
    cache.seq_len[0].fill_(n0)
    cache.n_prompt.fill_(wl.prompt)
    steps = torch.arange(70000, 70000 + T)
    q = gen.q(0, steps).permute(1, 0, 2, 3).contiguous()
    kb = gen.kv(0, steps)[0].permute(1, 0, 2, 3).contiguous()
    scratch = torch.empty(B.dynts_score_block_scratch_bytes(cache.cfg, T), dtype=torch.uint8, device=dev)
    dst = torch.zeros((wl.batch, wl.n_kv_heads, wl.capacity), dtype=torch.float32, device=dev)
    for _ in range(args.warmup):
        B.dynts_score_block(cache.ctx, 0, q, kb, scratch, dst=dst, accumulate=False)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        B.dynts_score_block(cache.ctx, 0, q, kb, scratch, dst=dst, accumulate=False)
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1) / args.steps
    # the second roofline: exponentials.  Rate of the vector ALUs measured by the library's probe (2048 workgroups
    # of 256 lanes, 4000 x 8 exponentials + subtractions per lane), in the same process
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    hev = HipEvents(1)
    rates = []
    for _ in range(4):
        B.dynts_probe_exp_rate(2048, 4000, sink, hev.pairs[0][0], hev.pairs[0][1])
        torch.cuda.synchronize()
        rates.append(2048 * 256 * 4000 * 8 / (hev.elapsed_ms(0) * 1e-3))
    hev.close()
    exp_rate = max(rates[1:])
    # the third: the kernels' own instruction mix without memory (16 MFMA + 16 x (fma, exp2, add) per wave and
    # streamed 16-row tile), three waves per SIMD as the kernels run; time per tile and SIMD
    hev = HipEvents(1)
    mix_ns = {}
    for what, name in ((1, "mfma_only"), (2, "vector_only"), (3, "both")):
        best = None
        for _ in range(3):
            B.dynts_probe_issue_mix(768, 20000, what, sink, hev.pairs[0][0], hev.pairs[0][1])
            torch.cuda.synchronize()
            t = hev.elapsed_ms(0) * 1e6 / 20000 / 3
            best = t if best is None or t < best else best
        mix_ns[name] = round(best, 1)
    hev.close()
    units, R, d = wl.batch * wl.n_kv_heads, T * wl.group, wl.head_dim
    # the contraction the method defines: every query row against the cached slots and its visible block keys
    flops = units * 2.0 * d * (R * n0 + wl.group * T * (T + 1) / 2)
    executed = units * 2.0 * d * (2 * R * n0 + wl.group * T * (T + 1) / 2)   # the logits are formed twice
    peak = 2500.0
    roofline = {"bound": "mfma", "kernel": "score_block_stats_kernel + score_block_colsum_kernel",
                "achieved": round(flops / (ev_ms * 1e-3) / 1e12, 1), "peak": peak, "unit": "TFLOP/s",
                "frac": round(flops / (ev_ms * 1e-3) / 1e12 / peak, 4), "traffic": None,
                "call_avg_us": round(ev_ms * 1e3, 1), "algorithmic_flops_per_call": flops,
                "executed_mfma_flops_per_call": executed, "exp2_per_call": units * (2.0 * R * n0),
                "second_bound": {"kind": "v_exp_f32 issue (one exponential and one subtraction per (query row, slot) "
                                         "and pass, two passes)",
                                 "peak_exp2_per_s": round(exp_rate / 1e12, 2), "unit": "T/s, measured by "
                                 "dynts_probe_exp_rate in this run",
                                 "achieved_exp2_per_s": round(units * (2.0 * R * n0) / (ev_ms * 1e-3) / 1e12, 2),
                                 "frac": round(units * (2.0 * R * n0) / (ev_ms * 1e-3) / exp_rate, 4)},
                "issue_bound": {"kind": "the kernels' instruction mix with no memory access: 16 MFMA + 16 x (fma, exp2, "
                                        "add) per wave and streamed 16-row tile, 3 waves per SIMD (dynts_probe_issue_mix "
                                        "in this run)",
                                "ns_per_tile_and_simd": mix_ns,
                                "wave_tiles_per_call": executed / (16 * 16384.0),
                                "floor_ms_per_call": round(executed / (16 * 16384.0) / 1024 * mix_ns["both"] * 1e-6, 4),
                                "frac": round(executed / (16 * 16384.0) / 1024 * mix_ns["both"] * 1e-6 / ev_ms, 4)}}
    return dict(value=args.steps / dt, ms_per_step=dt / args.steps * 1e3, roofline=roofline,
                whole_step_gbs=0.0, seq_steps_per_s=args.steps * wl.batch / dt, evictions_timed=0,
                first_timed_step=0, active_min=wl.batch, active_max=wl.batch)


def run_predictor(args, wl):
    """The Importance Predictor head with synthetic weights at the size of the workload's model shape
    (28 query heads: 3584 -> 7168 -> 1792 -> 1, else 4096 -> 8192 -> 2048 -> 1), one score per sequence
    written once per KV head (the layout dynts_decode_step takes as s_new).  A step is one call."""
    import torch
    from paper_2601_18383_amd import binding as B

    dev = torch.device("cuda:0")
    d = 3584 if wl.n_q_heads == 28 else 4096
    m1, m2, nb = 2 * d, d // 2, min(wl.batch, 128)
    g = torch.Generator(device="cpu").manual_seed(wl.seed)
    rnd = lambda *shape: torch.randn(*shape, generator=g)
    W1 = (rnd(m1, d) / d ** 0.5).to(torch.bfloat16).to(dev)
    W2 = (rnd(m2, m1) / m1 ** 0.5).to(torch.bfloat16).to(dev)
    w3 = (rnd(m2) / m2 ** 0.5).to(torch.bfloat16).to(dev)
    b1, b2, b3 = (rnd(m1) * 0.1).to(dev), (rnd(m2) * 0.1).to(dev), rnd(1).to(dev)
    pred = B.Predictor(W1, b1, W2, b2, w3, b3, activation=B.DYNTS_ACT_RELU, max_batch=nb)
    n_pool = 8  # rotate hidden states; the weights are the traffic
    hs = [rnd(nb, d).to(torch.bfloat16).to(dev) for _ in range(n_pool)]
    s = torch.zeros((nb, wl.n_kv_heads), dtype=torch.float32, device=dev)
    for i in range(args.warmup):
        B.dynts_predict_scores(pred, hs[i % n_pool], s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        B.dynts_predict_scores(pred, hs[i % n_pool], s)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n_ev = min(args.steps, 64)
    ev = HipEvents(n_ev)
    for i in range(n_ev):
        B.dynts_predict_scores(pred, hs[i % n_pool], s, ev.pairs[i][0], ev.pairs[i][1])
    torch.cuda.synchronize()
    call_ms = sum(ev.elapsed_ms(i) for i in range(n_ev)) / n_ev
    ev.close()
    alg = 2 * (m1 * d + m2 * m1 + m2) + 4 * (m1 + m2 + 1) + nb * d * 2 + nb * wl.n_kv_heads * 4
    achieved = alg / (call_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "mlp_gemm x2 + reductions (one dynts_predict_scores call)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None, "call_avg_us": round(call_ms * 1e3, 2),
                "algorithmic_bytes_per_call": alg, "flops_per_call": 2.0 * nb * (m1 * d + m2 * m1 + m2)}
    return dict(value=args.steps / dt, ms_per_step=dt / args.steps * 1e3, roofline=roofline, whole_step_gbs=alg / dt *
                args.steps / 1e9, seq_steps_per_s=args.steps * nb / dt, evictions_timed=0, first_timed_step=0,
                active_min=nb, active_max=nb, mode="Importance Predictor %d -> %d -> %d -> 1, batch %d" % (d, m1, m2, nb))


def run_cpu_baseline(wl, budget_s=15.0):
    """The float64 oracle, as it stands, on the host cores: whole decode steps of the same
    workload from a generator-made steady state (one layer's worth scaled to all layers)."""
    import numpy as np
    import torch
    from oracle import dynts_oracle as orc
    from paper_2601_18383_amd import synth

    gen = synth.Synth(wl, "cpu")
    E = wl.evict_every
    n0 = wl.steady_len
    st = gen.steady_state(0, n0)
    o = orc.OracleLayer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.capacity, wl.budget, wl.window,
                        E, external_scores=wl.external_scores)
    o.K[:, :, :n0] = st["K"].to(torch.float64).numpy()
    o.V[:, :, :n0] = st["V"].to(torch.float64).numpy()
    o.S[:, :, :n0] = st["S"].to(torch.float64).numpy()
    o.pos[:, :, :n0] = st["pos"].numpy()
    o.seq_len[:] = n0
    o.n_prompt[:] = wl.prompt
    o.next_pos[:] = o.pos[:, :, n0 - 1].max(axis=1) + 1
    o.steps_done[:] = wl.budget + wl.window + E  # a multiple of E: the next trigger is E steps away
    threads = orc.max_threads()
    n_multi = max(4 * E, 1024)                      # at most this many steps on all threads ...
    steps = torch.arange(10 ** 5, 10 ** 5 + n_multi + 32)   # ... and up to 32 more on one thread
    q = gen.q(0, steps).to(torch.float64).numpy()
    k, v = gen.kv(0, steps)
    k, v = k.to(torch.float64).numpy(), v.to(torch.float64).numpy()
    s = None
    if wl.external_scores:
        s = gen.external_scores(steps).unsqueeze(-1).expand(len(steps), wl.batch, wl.n_kv_heads)
        s = s.to(torch.float64).contiguous().numpy()
    done, t0 = 0, time.perf_counter()
    while done < n_multi:
        o.step(q[done], k[done], v[done], s[done] if s is not None else None)
        done += 1
        if time.perf_counter() - t0 > budget_s and done >= 2:
            break
    dt = time.perf_counter() - t0
    layer_steps_per_s = done / dt
    # the same oracle on one thread, a few more steps (bounded to ~5 s)
    orc.set_threads(1)
    one, t1 = 0, time.perf_counter()
    while done + one < len(steps) and (one < 2 or time.perf_counter() - t1 < 5.0):
        i = done + one
        o.step(q[i], k[i], v[i], s[i] if s is not None else None)
        one += 1
    dt1 = time.perf_counter() - t1
    orc.set_threads(threads)
    return {"value": layer_steps_per_s / wl.n_layers, "unit": "decode steps/s", "cores": threads,
            "one_thread_value": (one / dt1 / wl.n_layers) if one else None,
            "kind": "oracle",
            "sample": "%d whole layer-steps (append+attend+score%s) of %s, full batch, from a synthetic steady "
                      "state of %d slots, %.1f s; divided by %d layers" %
                      (done, ", incl. 1 select+compact" if done >= E else "", wl.name, n0, dt, wl.n_layers)}


def result_line(args, wl, r, cpu):
    """The one JSON object bench.py prints."""
    line = {
        "metric": "predictor calls/sec, 1 MI355X" if getattr(args, "predictor", False) else
                  "block-scoring calls/sec, 1 MI355X" if getattr(args, "score_block", 0) else
                  "decode steps/sec (attn+score+evict), 1 MI355X", "value": round(r["value"], 2),
        "unit": "calls/s" if getattr(args, "score_block", 0) or getattr(args, "predictor", False) else "decode steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d layer(s), batch %d, %d q / %d kv heads, head_dim %d, prompt %d, budget %d, "
                               "window %d, evict every %d; %s, %d-%d of %d sequences active" %
                               (wl.name, wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.prompt,
                                wl.budget, wl.window, wl.evict_every,
                                r["mode"] if "mode" in r else
                                "block scoring of %d queries per sequence on a steady-state cache" % args.score_block
                                if getattr(args, "score_block", 0) else
                                "whole decode from the prompt" if args.trajectory else
                                "steady state, paged layout (initial page order: %s)" % r.get("page_order")
                                if getattr(args, "paged", False) else "steady state",
                                r["active_min"], r["active_max"], wl.batch),
                   "first_timed_step": r["first_timed_step"], "evictions_in_window": r["evictions_timed"],
                   "sequence_steps_per_s": round(r["seq_steps_per_s"], 1), "timed_windows": r.get("windows"),
                   "whole_step_algorithmic_GBps": round(r["whole_step_gbs"], 1),
                   "full_period": r.get("full_period"), "other_workloads": r.get("other_workloads"),
                   "memory_note": r.get("memory_note")},
        "roofline": r["roofline"], "cpu_baseline": cpu,
    }
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--layers", type=int, default=0, help="run only this many layers of the workload's stack "
                    "(a tuning aid; the workload line says so)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the bounded runs of the other configurations that accompany the main line")
    ap.add_argument("--trajectory", action="store_true",
                    help="time the whole decode from the prompt to the end of the longest sequence (ragged "
                         "batches decay) instead of a steady-state window; --steps/--warmup are ignored")
    ap.add_argument("--max-steps", type=int, default=0, help="with --trajectory: stop after this many steps")
    ap.add_argument("--score-block", type=int, default=0, metavar="T",
                    help="time dynts_score_block for a block of T queries (with their keys) on a steady-state "
                         "cache instead of the decode path")
    ap.add_argument("--paged", action="store_true",
                    help="steady-state run on the paged (block-table) cache layout instead of the dense one")
    ap.add_argument("--predictor", action="store_true",
                    help="time the Importance Predictor head (synthetic weights at the workload's model size)")
    ap.add_argument("--full-kv", action="store_true",
                    help="the comparison run without eviction: same inputs, a cache that holds every token, "
                         "attention only (no score is kept)")
    ap.add_argument("--launch-shape", default=None, metavar="WGS,WAVES",
                    help="tuning: dynts_set_launch_shape(target workgroups, waves per workgroup) instead of the default")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (a kernel of known traffic, for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.launch_shape:
        args.launch_shape = tuple(int(x) for x in args.launch_shape.split(","))
    if args.gpus != 1:
        sys.exit("bench.py measures one MI355X: the decode path shards over sequences and KV heads "
                 "without communication, and this build runs on a single GPU only (--gpus 1).")
    from paper_2601_18383_amd import configs
    wl = configs.get(args.workload)
    if args.layers:
        import dataclasses
        wl = dataclasses.replace(wl, name="%s[%d of %d layers]" % (wl.name, args.layers, wl.n_layers),
                                 n_layers=args.layers)
    if args.full_kv:
        import dataclasses
        hi = wl.steps[1] if not args.max_steps else min(wl.steps[1], args.max_steps)
        wl = dataclasses.replace(wl, name=wl.name + " full-KV (no eviction, no scores)", budget=hi, window=0,
                                 evict_every=1, external_scores=True)
        args.trajectory = True
    log("host cores: %d; workload %s" % (os.cpu_count(), wl))
    if args.predictor:
        r = run_predictor(args, wl)
        args.no_cpu_baseline = True
    elif args.score_block:
        r = run_score_block(args, wl)
        args.no_cpu_baseline = True
    elif args.trajectory:
        r = run_trajectory(args, wl)
        args.steps, args.warmup, args.no_cpu_baseline = r["steps"], 0, True
    else:
        r = run_gpu(args, wl)
        kv_mb = 4.0 * wl.batch * wl.n_kv_heads * wl.steady_len * wl.head_dim / 1e6
        r["memory_note"] = ("%.0f MB of K/V per layer-step, %d layer(s): %s" %
                            (kv_mb, wl.n_layers, "re-read every step and below the 256 MB memory-side cache, which "
                             "therefore serves part of it; cfg4 / cfg5 in other_workloads are the HBM-only cases"
                             if kv_mb * wl.n_layers < 256 else "beyond the 256 MB memory-side cache: HBM only"))
        if not args.no_other_workloads:
            r["other_workloads"] = run_other_workloads(args, args.workload)
    if args.copy_calibration:
        import torch
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    cpu = None if args.no_cpu_baseline else run_cpu_baseline(wl)
    line = result_line(args, wl, r, cpu)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
