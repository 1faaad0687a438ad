"""The five workload shapes of the draft+verify step (Vicuna-shaped, synthetic).

Index 0 is the tiny fp32 case a CPU finishes in milliseconds; 1-3 are single
sequence 7B / 7B-long / 13B shapes; 4 is a batch of eight ragged sequences.
V is the vocabulary WITHOUT the blank; the draft head has V+1 rows and the blank
is row V.
"""
from dataclasses import dataclass
from typing import Tuple


@dataclass(frozen=True)
class StepConfig:
    name: str
    B: int            # independent sequences
    D: int            # hidden size
    V: int            # vocabulary size without blank (blank id == V)
    T: int            # draft slots
    k: int            # top-k per slot
    beam: int         # max collapsed candidates kept
    max_nodes: int    # max tree nodes, root included
    H: int            # attention heads
    dh: int           # head dim
    ctx: Tuple[int, int]  # KV context length range [lo, hi] (lo == hi: fixed)
    kv_cap: int       # KV rows allocated per head
    dtype: str        # storage dtype of hidden/W/Q/K/V: "f32" or "bf16"
    blank_bias: float  # additive logit bias of the blank row
    rms_norm: bool    # draft hidden states normalised to unit RMS per row
    n_layers: int = 0  # attention layers of the base model the shape is borrowed from (0: none stated)

    @property
    def Vp1(self) -> int:
        return self.V + 1

    @property
    def blank_id(self) -> int:
        return self.V

    @property
    def n_align(self) -> int:
        return self.k ** self.T


CONFIGS = (
    StepConfig("tiny", B=1, D=64, V=100, T=4, k=2, beam=16, max_nodes=128, H=4, dh=16,
               ctx=(32, 32), kv_cap=32, dtype="f32", blank_bias=1.5, rms_norm=False),
    StepConfig("7b_ctx512", B=1, D=4096, V=32000, T=8, k=4, beam=64, max_nodes=128, H=32, dh=128,
               ctx=(512, 512), kv_cap=512, dtype="bf16", blank_bias=1.0, rms_norm=True, n_layers=32),
    StepConfig("7b_ctx2048", B=1, D=4096, V=32000, T=8, k=4, beam=128, max_nodes=128, H=32, dh=128,
               ctx=(2048, 2048), kv_cap=2048, dtype="bf16", blank_bias=1.0, rms_norm=True, n_layers=32),
    StepConfig("13b_ctx2048", B=1, D=5120, V=32000, T=8, k=4, beam=128, max_nodes=128, H=40, dh=128,
               ctx=(2048, 2048), kv_cap=2048, dtype="bf16", blank_bias=1.0, rms_norm=True, n_layers=40),
    StepConfig("7b_batch8_ragged", B=8, D=4096, V=32000, T=8, k=4, beam=64, max_nodes=64, H=32, dh=128,
               ctx=(256, 2048), kv_cap=2048, dtype="bf16", blank_bias=1.0, rms_norm=True, n_layers=32),
)


def get_config(which) -> StepConfig:
    """Look a config up by index or by name."""
    if isinstance(which, int):
        return CONFIGS[which]
    for c in CONFIGS:
        if c.name == which:
            return c
    raise KeyError(which)
