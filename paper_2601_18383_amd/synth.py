"""Seeded synthetic inputs for the DynTS decode path (no method arithmetic lives here).

A counter-based generator written with integer torch ops, so the same call
gives bit-identical tensors on the CPU and on a GPU: every element is
    u64 = splitmix64_finalise(key(seed, stream, layer) + counter * GOLDEN)
    value = LUT[u64 >> 48]
where LUT is a 65,536-entry bf16 table of inverse-CDF values (standard normal
or Student-t with 3 degrees of freedom) built once on the host in float64.
Stands in for the q/k/v streams of real reasoning traces: only shapes, length
scales and the "few decision-critical tokens" structure are taken from the
paper (Sec. 3.1, Sec. 6.1).

Planted critical tokens: per (layer, KV head) a unit direction u; every query
is z + d^(1/4) u, so its mean is mu = d^(1/4) u; a token is critical with
probability p and then its key is 4*mu on every KV head, which puts its logit
near +4 while ordinary logits stay near N(0, 1.1).
"""
import numpy as np
import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_STEP_BIAS = 1 << 20  # prompt tokens sit at negative step indices

STREAM_Q, STREAM_K, STREAM_V, STREAM_PLANT, STREAM_DIR, STREAM_LEN, STREAM_SCORE = 1, 2, 3, 4, 5, 6, 7


def _s64(x: int) -> int:
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(x: int) -> int:
    x &= _M64
    x = ((x ^ (x >> 30)) * _C1) & _M64
    x = ((x ^ (x >> 27)) * _C2) & _M64
    return x ^ (x >> 31)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _s64(_C1)
    x = (x ^ _lsr(x, 27)) * _s64(_C2)
    return x ^ _lsr(x, 31)


def stream_key(seed: int, stream: int, layer: int) -> int:
    return _mix_py(seed ^ _mix_py(stream * 0x100000001B3 + layer))


def hash_u64(key: int, counter: torch.Tensor) -> torch.Tensor:
    """int64 tensor of hashed bits (two's complement view of the u64)."""
    return _mix(counter * _s64(_GOLDEN) + _s64(key))


def _top16(h: torch.Tensor) -> torch.Tensor:
    return _lsr(h, 48)


_lut_cache = {}


def lut(kind: str, device) -> torch.Tensor:
    """bf16 [65536] inverse-CDF table: 'normal' or 'student_t3'."""
    k = (kind, str(device))
    if k not in _lut_cache:
        if (kind, "cpu") not in _lut_cache:
            from scipy import special, stats
            u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
            if kind == "normal":
                x = special.ndtri(u)
            elif kind == "student_t3":
                x = stats.t.ppf(u, 3)
            else:
                raise ValueError(kind)
            _lut_cache[(kind, "cpu")] = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16)
        _lut_cache[k] = _lut_cache[(kind, "cpu")].to(device)
    return _lut_cache[k]


class Synth:
    """Input streams of one workload (see configs.Workload) on one device."""

    def __init__(self, wl, device="cpu"):
        self.wl = wl
        self.device = torch.device(device)

    # -- element counters -------------------------------------------------
    def _counter(self, steps: torch.Tensor, heads: int, comps: int) -> torch.Tensor:
        """[steps][Nb][heads][comps] int64 counter; steps may be negative (prompt)."""
        dev = self.device
        b = torch.arange(self.wl.batch, device=dev, dtype=torch.int64).view(1, -1, 1, 1)
        t = (steps.to(dev).to(torch.int64) + _STEP_BIAS).view(-1, 1, 1, 1)
        h = torch.arange(heads, device=dev, dtype=torch.int64).view(1, 1, -1, 1)
        c = torch.arange(comps, device=dev, dtype=torch.int64).view(1, 1, 1, -1)
        return ((b * (2 * _STEP_BIAS) + t) * 64 + h) * 256 + c

    def _draw(self, stream, layer, steps, heads, comps, kind="normal"):
        h = hash_u64(stream_key(self.wl.seed, stream, layer), self._counter(steps, heads, comps))
        return lut(kind, self.device)[_top16(h)]

    # -- planted structure ------------------------------------------------
    def mean_query(self, layer: int) -> torch.Tensor:
        """mu [Hkv][d] fp32 = d^(1/4) * unit direction of (layer, KV head)."""
        wl = self.wl
        z = Synth(wl, "cpu")._draw(STREAM_DIR, layer, torch.zeros(1, dtype=torch.int64),
                                   wl.n_kv_heads, wl.head_dim)[0, 0].to(torch.float64)
        u = z / z.norm(dim=-1, keepdim=True)
        return (u * wl.head_dim ** 0.25).to(torch.float32).to(self.device)

    def critical(self, layer: int, steps: torch.Tensor) -> torch.Tensor:
        """bool [steps][Nb]: is the token generated at this step a planted critical one."""
        p = self.wl.plant_fraction(layer)
        h = hash_u64(stream_key(self.wl.seed, STREAM_PLANT, layer), self._counter(steps, 1, 1))
        return (_lsr(h, 32) < int(p * (1 << 32)))[:, :, 0, 0]

    # -- per-step tensors -------------------------------------------------
    def q(self, layer: int, steps: torch.Tensor) -> torch.Tensor:
        """bf16 [steps][Nb][Hq][d]."""
        wl = self.wl
        z = self._draw(STREAM_Q, layer, steps, wl.n_q_heads, wl.head_dim).to(torch.float32)
        if wl.plant[1] > 0.0:
            mu = self.mean_query(layer).repeat_interleave(wl.group, dim=0)  # [Hq][d]
            z = z + mu.view(1, 1, wl.n_q_heads, wl.head_dim)
        return z.to(torch.bfloat16)

    def kv(self, layer: int, steps: torch.Tensor):
        """(k, v) bf16 [steps][Nb][Hkv][d]; negative steps are prompt tokens."""
        wl = self.wl
        k = self._draw(STREAM_K, layer, steps, wl.n_kv_heads, wl.head_dim, wl.k_dist)
        v = self._draw(STREAM_V, layer, steps, wl.n_kv_heads, wl.head_dim)
        if wl.plant[1] > 0.0:
            crit = self.critical(layer, steps) & (steps.to(self.device) > 0).view(-1, 1)
            kc = (4.0 * self.mean_query(layer)).to(torch.bfloat16)  # [Hkv][d]
            k = torch.where(crit.view(crit.shape[0], crit.shape[1], 1, 1), kc.view(1, 1, *kc.shape), k)
        return k, v

    def prompt_kv(self, layer: int):
        """(K0, V0) bf16 [Nb][Hkv][M][d]: prompt rows, steps -M..-1."""
        steps = torch.arange(-self.wl.prompt, 0, dtype=torch.int64)
        k, v = self.kv(layer, steps)
        return k.permute(1, 2, 0, 3).contiguous(), v.permute(1, 2, 0, 3).contiguous()

    def decode_lengths(self) -> torch.Tensor:
        """int64 [Nb] on the CPU: decode steps of each sequence, uniform in [lo, hi]."""
        lo, hi = self.wl.steps
        b = torch.arange(self.wl.batch, dtype=torch.int64)
        h = hash_u64(stream_key(self.wl.seed, STREAM_LEN, 0), b)
        return lo + _lsr(h, 33) % (hi - lo + 1)

    def external_scores(self, steps: torch.Tensor) -> torch.Tensor:
        """fp32 [steps][Nb]: one score per token on a 64-level grid, floor(8|t3|) clamped to 63."""
        h = hash_u64(stream_key(self.wl.seed, STREAM_SCORE, 0), self._counter(steps, 1, 1))
        t = lut("student_t3", self.device)[_top16(h)].to(torch.float32)[:, :, 0, 0]
        return torch.clamp(torch.floor(t.abs() * 8.0), max=63.0)

    # -- a whole cache state without running the path ------------------------
    def steady_state(self, layer: int, n: int, seq_slice=None):
        """A plausible mid-decode cache: n slots per sequence (prompt, then thinking
        tokens at ascending positions drawn with gaps), scores from a hash.

        Returns dict(K, V bf16 [Nb][Hkv][n][d], S fp32 [Nb][Hkv][n], pos int32 [Nb][Hkv][n]).
        Positions and scores differ per KV head, as after per-head selection.
        """
        wl, dev = self.wl, self.device
        M = wl.prompt
        assert n >= M
        nt = n - M
        # thinking positions: cumulative sum of hashed gaps in {1,2,3}, per (b, head)
        idx = self._counter(torch.arange(nt, dtype=torch.int64), wl.n_kv_heads, 1)[..., 0]  # [nt][Nb][Hkv]
        gap = 1 + _lsr(hash_u64(stream_key(wl.seed, STREAM_LEN, layer + 1), idx), 40) % 3
        tpos = M - 1 + torch.cumsum(gap, dim=0)  # [nt][Nb][Hkv] position of each thinking slot
        pos = torch.cat([torch.arange(M, device=dev, dtype=torch.int64).view(M, 1, 1).expand(M, wl.batch, wl.n_kv_heads),
                         tpos], dim=0)  # [n][Nb][Hkv]
        step_of = pos - M + 1  # decode step that produced the token (<=0: prompt)
        step_of = torch.where(step_of > 0, step_of, pos - M)
        # gather K/V rows for those steps: counter built per (slot, b, head, comp)
        b = torch.arange(wl.batch, device=dev, dtype=torch.int64).view(1, -1, 1, 1)
        h = torch.arange(wl.n_kv_heads, device=dev, dtype=torch.int64).view(1, 1, -1, 1)
        c = torch.arange(wl.head_dim, device=dev, dtype=torch.int64).view(1, 1, 1, -1)
        ctr = ((b * (2 * _STEP_BIAS) + (step_of.unsqueeze(-1) + _STEP_BIAS)) * 64 + h) * 256 + c
        K = lut(wl.k_dist, dev)[_top16(hash_u64(stream_key(wl.seed, STREAM_K, layer), ctr))]
        V = lut("normal", dev)[_top16(hash_u64(stream_key(wl.seed, STREAM_V, layer), ctr))]
        if wl.plant[1] > 0.0:
            p = wl.plant_fraction(layer)
            cb = ((b * (2 * _STEP_BIAS) + (step_of.unsqueeze(-1) + _STEP_BIAS)) * 64) * 256
            crit = (_lsr(hash_u64(stream_key(wl.seed, STREAM_PLANT, layer), cb), 32) < int(p * (1 << 32)))
            crit = crit & (step_of.unsqueeze(-1) > 0)
            kc = (4.0 * self.mean_query(layer)).to(torch.bfloat16).view(1, 1, wl.n_kv_heads, wl.head_dim)
            K = torch.where(crit, kc, K)
        sc = hash_u64(stream_key(wl.seed, STREAM_SCORE, layer + 1), idx)
        x = _lsr(sc, 40).to(torch.float32) * (1.0 / (1 << 24))
        x = x * x
        S = x * x * 8.0  # heavy-ish tail in [0, 8); plain multiplications only, so CPU and GPU agree bit for bit
        S = torch.cat([torch.full((M, wl.batch, wl.n_kv_heads), float("inf"), device=dev), S], dim=0)
        out = dict(K=K.permute(1, 2, 0, 3).contiguous(), V=V.permute(1, 2, 0, 3).contiguous(),
                   S=S.permute(1, 2, 0).contiguous(), pos=pos.permute(1, 2, 0).to(torch.int32).contiguous())
        if seq_slice is not None:
            out = {k: v[seq_slice] for k, v in out.items()}
        return out
