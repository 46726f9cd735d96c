"""The benchmark workloads as named presets (shapes only; all tensors are synthetic).

Shapes follow the attention geometry of the two 7-8B reasoning models the paper
evaluates (Sec. 6.1): 32 query / 8 KV heads (Llama-3-8B-shaped) and 28 query /
4 KV heads (Qwen2.5-7B-shaped), head_dim 128, decode lengths up to 16k-32k.
`budget`, `window`, `evict_every` are the selection-window size kept after a
trigger, the local-window size and the trigger period (Sec. 4.2).
"""
from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prompt: int                 # M, question-window length (same for every sequence)
    steps: Tuple[int, int]      # decode steps per sequence, uniform in [lo, hi]
    budget: int
    window: int
    evict_every: int
    plant: Tuple[float, float]  # fraction of planted critical keys, first..last layer
    k_dist: str = "normal"      # "normal" | "student_t3"
    external_scores: bool = False
    seed: int = 0xD7A50000

    @property
    def capacity(self) -> int:
        return self.prompt + self.budget + self.window + self.evict_every

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def steady_len(self) -> int:
        """Cache length right after a trigger in steady state."""
        return self.prompt + self.budget + self.window

    def plant_fraction(self, layer: int) -> float:
        lo, hi = self.plant
        if self.n_layers <= 1:
            return lo
        return lo + (hi - lo) * layer / (self.n_layers - 1)


CONFIGS = {
    "cfg1": Workload("cfg1", 1, 1, 8, 2, 64, 64, (512, 512), 128, 32, 16, (0.03, 0.03),
                     seed=0xD7A50001),
    "cfg2": Workload("cfg2", 1, 1, 32, 8, 128, 256, (16384, 16384), 4096, 128, 64, (0.02, 0.02),
                     seed=0xD7A50002),
    "cfg3": Workload("cfg3", 1, 32, 28, 4, 128, 256, (4096, 32768), 2048, 128, 64, (0.02, 0.02),
                     seed=0xD7A50003),
    "cfg4": Workload("cfg4", 32, 64, 32, 8, 128, 512, (8192, 8192), 2048, 64, 32, (0.01, 0.05),
                     seed=0xD7A50004),
    "cfg5": Workload("cfg5", 28, 128, 28, 4, 128, 128, (1024, 32768), 1024, 32, 16, (0.0, 0.0),
                     k_dist="student_t3", seed=0xD7A50005),
}
# Same streams as cfg5, scores supplied from outside on a 64-level grid so that
# every trigger has exact ties at the cut.
CONFIGS["cfg5b"] = replace(CONFIGS["cfg5"], name="cfg5b", external_scores=True)




def paper_schedule(name, n_q_heads, n_kv_heads, total, window, retention, batch=32, prompt=256,
                   steps=16384, seed=0xD7A50010) -> Workload:
    """A workload with the budget settings of the paper's own runs (Sec. 6.1, inference settings):
    `total` thinking tokens fill the cache, the newest `window` of them are the local window, and a
    trigger keeps the fraction `retention` of the others.  One trigger therefore evicts
    (1 - retention) * (total - window) tokens at once, and the next one comes that many steps later
    (e.g. 3000 / 1500 / 0.4 evicts 900, the eviction volume the paper quotes in Sec. 6.3)."""
    keep = int(round(retention * (total - window)))
    return Workload(name, 1, batch, n_q_heads, n_kv_heads, 128, prompt, (steps, steps), keep, window,
                    total - window - keep, (0.02, 0.02), seed=seed)


# The paper's budget settings on the two model shapes: hard benchmarks 5000 / 2000, simpler ones
# 3000 / 1500 (R1-Qwen-shaped, retention 0.4) and 3000 / 1000 (R1-Llama-shaped, retention 0.3).
CONFIGS["paper_qwen_5000"] = paper_schedule("paper_qwen_5000", 28, 4, 5000, 2000, 0.4, seed=0xD7A50011)
CONFIGS["paper_qwen_3000"] = paper_schedule("paper_qwen_3000", 28, 4, 3000, 1500, 0.4, seed=0xD7A50012)
CONFIGS["paper_llama_5000"] = paper_schedule("paper_llama_5000", 32, 8, 5000, 2000, 0.3, seed=0xD7A50013)
CONFIGS["paper_llama_3000"] = paper_schedule("paper_llama_3000", 32, 8, 3000, 1000, 0.3, seed=0xD7A50014)


# Other cache policies expressed through the same selection rule (Sec. 6.1 lists them as baselines; here
# they only serve like-for-like kernel measurements on the cfg3 shape and streams):
#  * sliding window with attention sinks (StreamingLLM-style): question slots + the most recent tokens,
#    nothing selected by score -> budget 0, the whole thinking budget is the local window;
#  * heavy-hitter eviction (H2O-style): accumulated attention as the score, a local window, and ONE token
#    evicted per step once the cache is full -> evict_every 1.
CONFIGS["policy_window"] = replace(CONFIGS["cfg3"], name="policy_window", budget=0, window=2176, evict_every=64)
CONFIGS["policy_h2o"] = replace(CONFIGS["cfg3"], name="policy_h2o", budget=2048, window=128, evict_every=1)


def get(name: str) -> Workload:
    return CONFIGS[name]
