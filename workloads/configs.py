"""The five synthetic workload configurations of the benchmark contract.

Notation: P prompts, G responses per prompt, T maximum response length,
R = P*G responses, N = R*T token slots, d hidden size, V vocabulary size.
Slot i = (p*G + g)*T + t; a slot is valid iff t < len[p*G + g] (right padding).
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class Workload:
    index: int            # position in the benchmark's config list (seeds depend on it)
    name: str
    P: int
    G: int
    T: int
    d: int
    V: int
    dtype: str            # "f32" or "bf16": storage type of H and W
    tok_dist: str         # "uniform" | "zipf1.1"
    len_dist: str         # "uniform" | "loguniform"
    len_lo: int
    len_hi: int
    reward_dist: str      # "bernoulli" | "uniform"
    reward_p: float       # Bernoulli probability (unused for "uniform")
    loss: str             # "grpo" | "flowrl"
    beta: float = 1.0     # FlowRL reward scale
    clip_eps: float = 0.2
    kl_coef: float = 0.04
    log_z: str = "zero"   # "zero" | "normal"
    want_entropy: bool = False
    recompute_old_ref: bool = False  # old/ref log-probs are part of the timed step

    @property
    def R(self) -> int:
        return self.P * self.G

    @property
    def N(self) -> int:
        return self.P * self.G * self.T

    def scaled(self, **kw) -> "Workload":
        """Same distributions at other sizes (used for parity cases the oracle can afford).

        Length bounds follow T with the same ratio unless given explicitly.
        """
        if "T" in kw and "len_lo" not in kw and "len_hi" not in kw:
            t_new = kw["T"]
            kw["len_lo"] = max(1, (self.len_lo * t_new) // self.T)
            kw["len_hi"] = max(1, (self.len_hi * t_new) // self.T)
        return replace(self, **kw)


CONFIGS = [
    Workload(0, "tiny-f32-grpo", P=2, G=4, T=32, d=256, V=4096, dtype="f32",
             tok_dist="uniform", len_dist="uniform", len_lo=8, len_hi=32,
             reward_dist="bernoulli", reward_p=0.5, loss="grpo", beta=1.0,
             clip_eps=0.2, kl_coef=0.04, log_z="zero"),
    Workload(1, "bf16-8x8x256-grpo", P=8, G=8, T=256, d=2048, V=151936, dtype="bf16",
             tok_dist="zipf1.1", len_dist="uniform", len_lo=64, len_hi=256,
             reward_dist="bernoulli", reward_p=0.3, loss="grpo"),
    # Lengths scale with T like the other configs: uniform in [T/4, T].
    Workload(2, "bf16-32x8x2048-grpo", P=32, G=8, T=2048, d=4096, V=151936, dtype="bf16",
             tok_dist="zipf1.1", len_dist="uniform", len_lo=512, len_hi=2048,
             reward_dist="bernoulli", reward_p=0.3, loss="grpo"),
    Workload(3, "bf16-16x16x4096-flowrl", P=16, G=16, T=4096, d=3584, V=152064, dtype="bf16",
             tok_dist="zipf1.1", len_dist="loguniform", len_lo=32, len_hi=4096,
             reward_dist="uniform", reward_p=0.0, loss="flowrl", beta=15.0, log_z="normal"),
    Workload(4, "bf16-8x16x8192-grpo-entropy", P=8, G=16, T=8192, d=5120, V=151936, dtype="bf16",
             tok_dist="zipf1.1", len_dist="uniform", len_lo=1024, len_hi=8192,
             reward_dist="bernoulli", reward_p=0.2, loss="grpo", want_entropy=True,
             recompute_old_ref=True),
]


def get_config(i: int) -> Workload:
    return CONFIGS[i]
