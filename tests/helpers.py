"""Shared machinery of the GPU parity tests: run the HIP path and the float64 oracle side by
side on the same seeded inputs and compare them.

Tolerance (stated by the benchmark spec): |gpu - oracle| <= 2e-3 * max(1, |oracle|) for
attention outputs, log-sum-exp and scores (bf16 inputs, fp32 accumulation); selection,
positions, lengths and compacted K/V rows are compared bit for bit.

Beside that contract every comparison also holds a second, much tighter regression bound TIGHT:
the kernels keep ~16 bits of each softmax weight (bf16 high + low part) and accumulate in fp32,
which puts the scaled error near 1e-6; a path that lost one of the halves, or rounded an
intermediate to bf16 (relative 2^-9 per term), lands between 1e-4 and the contract bound and
would otherwise pass unnoticed.
"""
import numpy as np
import torch

from oracle import dynts_oracle as orc

TOL = 2e-3
TIGHT = 5e-5


def assert_close(got, ref, what, tol=TOL, tight=TIGHT):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    fin = np.isfinite(ref)
    assert np.array_equal(got[~fin], ref[~fin]), "%s: non-finite entries differ" % what
    err = np.abs(got[fin] - ref[fin]) / np.maximum(1.0, np.abs(ref[fin]))
    worst = float(err.max()) if err.size else 0.0
    assert worst <= tol, "%s: max scaled error %.3e > %.1e" % (what, worst, tol)
    if tight is not None:
        assert worst <= tight, "%s: max scaled error %.3e is inside the contract but above the regression " \
                               "bound %.1e (precision lost somewhere?)" % (what, worst, tight)
    return worst


def f64(t):
    """torch tensor (any device, bf16/fp32/int) -> numpy float64 copy."""
    return t.detach().to("cpu").to(torch.float64).numpy().copy()


def i32(t):
    return t.detach().to("cpu").to(torch.int32).numpy().copy()


def near_tie_ok(S_ref_unit, lo, hi, got_slots, ref_slots, tol=TOL):
    """Two selections from the same window may differ only by slots whose oracle score is within
    2*tol (scaled) of the cut."""
    got, ref = set(got_slots), set(ref_slots)
    if got == ref:
        return True
    cand = S_ref_unit[lo:hi]
    cut = min(S_ref_unit[j] for j in ref_slots if lo <= j < hi)
    for j in got ^ ref:
        if not (lo <= j < hi):
            return False
        if abs(S_ref_unit[j] - cut) > 2 * tol * max(1.0, abs(cut)):
            return False
    return True


class SideBySide:
    """One layer of the HIP cache and the oracle layer, stepped together."""

    def __init__(self, B, cache, layer, oracle_layer, mode="step"):
        self.B, self.c, self.layer, self.o, self.mode = B, cache, layer, oracle_layer, mode
        cfg = cache.cfg
        dev = cache.K.device
        self.out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), 7.0, dtype=torch.float32, device=dev)
        self.lse = torch.full((cfg.batch, cfg.n_q_heads), 7.0, dtype=torch.float32, device=dev)
        self.out_ref = np.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), 7.0)
        self.worst = dict(out=0.0, lse=0.0, S=0.0)
        self.evictions = 0
        self.adopted = 0

    def prefill(self, K0, V0, m):
        """K0, V0 bf16 CPU tensors [Nb][Hkv][Mmax][d]; m list of prompt lengths."""
        dev = self.c.K.device
        mt = torch.tensor(m, dtype=torch.int32, device=dev)
        self.B.dynts_prefill(self.c.ctx, self.layer, K0.to(dev).contiguous(), V0.to(dev).contiguous(), mt)
        self.o.prefill(f64(K0), f64(V0), m)

    def step(self, q, k, v, s=None, active=None, check_scores=True):
        """q,k,v bf16 CPU tensors of one step; s fp32 [Nb][Hkv] or None; active uint8 numpy or None."""
        B, c, L = self.B, self.c, self.layer
        dev = c.K.device
        qd, kd, vd = q.to(dev).contiguous(), k.to(dev).contiguous(), v.to(dev).contiguous()
        sd = s.to(dev).contiguous() if s is not None else None
        ad = torch.from_numpy(active).to(dev) if active is not None else None
        if self.mode.endswith("+hintall"):
            # a hint before every step: mostly no trigger follows, and the kept logits are applied by the next step
            B.dynts_hint_trigger(c.ctx, L)
        elif self.mode.endswith("+hint"):
            # announce the trigger that will follow this step (the oracle's rule, evaluated before the append), so that
            # the step keeps its logits and the score update owed at the trigger is applied from them
            o = self.o
            act_b = np.ones(c.cfg.batch, bool) if active is None else active.astype(bool)
            if (act_b & (o.seq_len - o.n_prompt + 1 >= o.budget + o.window + o.evict_every)).any():
                B.dynts_hint_trigger(c.ctx, L)
        if self.mode == "unfused":
            B.dynts_append(c.ctx, L, kd, vd, sd, ad)
            B.dynts_decode_attend(c.ctx, L, qd, self.out, self.lse, ad)
            B.dynts_update_scores(c.ctx, L)
        elif self.mode.startswith("fused"):
            B.dynts_append(c.ctx, L, kd, vd, sd, ad)
            B.dynts_decode_attend_update(c.ctx, L, qd, self.out, self.lse, ad)
        else:
            B.dynts_decode_step(c.ctx, L, qd, kd, vd, self.out, sd, ad, self.lse)
        # oracle, in the paper's order
        o = self.o
        o.append(f64(k), f64(v), f64(s) if s is not None else None, active)
        o.steps_done += 1 if active is None else active.astype(np.int64)
        out_ref, alpha, lse_ref = o.attend(f64(q), active, self.out_ref)
        o.update_scores(alpha, active)
        self.worst["out"] = max(self.worst["out"], assert_close(f64(self.out), out_ref, "out"))
        act = np.ones(c.cfg.batch, bool) if active is None else active.astype(bool)
        self.worst["lse"] = max(self.worst["lse"], assert_close(f64(self.lse)[act], lse_ref[act], "lse"))
        assert np.array_equal(i32(c.seq_len[L]), o.seq_len)
        if check_scores:
            self.check_scores()
        trig = o.due(active)
        if trig.any():
            self.evict(trig)
        return trig

    def check_scores(self):
        B, c, L, o = self.B, self.c, self.layer, self.o
        B.dynts_update_scores(c.ctx, L)  # apply whatever the fused path still owes
        S = f64(c.S[L])
        for b in range(c.cfg.batch):
            n = int(o.seq_len[b])
            self.worst["S"] = max(self.worst["S"], assert_close(S[b, :, :n], o.S[b, :, :n], "S[%d]" % b))

    def evict(self, trig):
        B, c, L, o = self.B, self.c, self.layer, self.o
        dev = c.K.device
        td = torch.from_numpy(trig).to(dev)
        c.keep_idx.fill_(-1)
        B.dynts_select_evict(c.ctx, L, c.keep_idx, c.new_len, -1, td)
        keep_gpu, len_gpu = i32(c.keep_idx), i32(c.new_len)
        S_gpu, pos_gpu = f64(c.S[L]), i32(c.pos[L])
        # (1) same function on the same score array: bit-exact
        keep_same, len_same = orc.select(S_gpu, pos_gpu, o.seq_len, o.n_prompt, o.window, o.budget, trig)
        assert np.array_equal(len_gpu, len_same)
        assert np.array_equal(keep_gpu, keep_same), "selection differs from the oracle on identical scores"
        # (2) against the oracle's own float64 scores: identical, or differing only by near-ties
        keep_ref, len_ref = o.select(trig)
        assert np.array_equal(len_gpu, len_ref)
        if not np.array_equal(keep_gpu, keep_ref):
            for b in np.nonzero(trig)[0]:
                n, M = int(o.seq_len[b]), int(o.n_prompt[b])
                for h in range(c.cfg.n_kv_heads):
                    assert near_tie_ok(o.S[b, h], M, n - o.window, keep_gpu[b, h, :len_gpu[b]].tolist(),
                                       keep_ref[b, h, :len_ref[b]].tolist())
            self.adopted += 1
            c.keep_idx.copy_(torch.from_numpy(keep_ref).to(dev))  # the HIP path follows the oracle
        B.dynts_compact(c.ctx, L, c.keep_idx, c.new_len, td)
        o.compact(keep_ref, len_ref, trig)
        self.evictions += 1
        self.check_state()

    def check_state(self):
        """Cache contents after compaction: K, V, pos, seq_len bit-exact; S within tolerance."""
        c, L, o = self.c, self.layer, self.o
        assert np.array_equal(i32(c.seq_len[L]), o.seq_len)
        K, V, S, pos = f64(c.K[L]), f64(c.V[L]), f64(c.S[L]), i32(c.pos[L])
        for b in range(c.cfg.batch):
            n = int(o.seq_len[b])
            assert np.array_equal(K[b, :, :n], o.K[b, :, :n]), "K rows differ after compaction"
            assert np.array_equal(V[b, :, :n], o.V[b, :, :n]), "V rows differ after compaction"
            assert np.array_equal(pos[b, :, :n], o.pos[b, :, :n]), "pos differs after compaction"
            self.worst["S"] = max(self.worst["S"], assert_close(S[b, :, :n], o.S[b, :, :n], "S after compaction"))
