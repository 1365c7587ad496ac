"""Synthetic workloads: GPT-shaped fp32 tensor lists and the scalar settings of
the five benchmark configurations.  No optimizer arithmetic lives here.

The tensor lists stand in for the GPT-2 small / medium / XL and 7B models the
paper pretrains (section "Experiments"); only shapes and hyper-parameters carry
over, gradients are synthetic (see generator.py).
"""
from dataclasses import dataclass, field
from typing import List, Tuple


def gpt_tensor_list(L: int, d: int, vocab: int, ctx: int = 1024) -> List[Tuple[str, int]]:
    """(name, numel) in a fixed order: embeddings, then per layer the 12 tensors
    of a GPT-2 block, then the final LayerNorm."""
    out = [("wte", vocab * d), ("wpe", ctx * d)]
    for l in range(L):
        pre = f"h{l}."
        out += [
            (pre + "ln1.g", d), (pre + "ln1.b", d),
            (pre + "attn.qkv.w", d * 3 * d), (pre + "attn.qkv.b", 3 * d),
            (pre + "attn.proj.w", d * d), (pre + "attn.proj.b", d),
            (pre + "ln2.g", d), (pre + "ln2.b", d),
            (pre + "mlp.fc.w", d * 4 * d), (pre + "mlp.fc.b", 4 * d),
            (pre + "mlp.proj.w", 4 * d * d), (pre + "mlp.proj.b", d),
        ]
    out += [("ln_f.g", d), ("ln_f.b", d)]
    return out


@dataclass
class Workload:
    name: str
    L: int
    d: int
    vocab: int
    ctx: int
    G: int                      # group replicas
    H: int                      # inner steps per outer round (the paper's r)
    rounds: int                 # outer rounds the parity case runs
    T: int                      # total iterations, places rounds in the schedule (0: fixed scalars)
    grad_bf16: bool = False
    offload: bool = False       # anchor + outer momentum in pinned host memory
    fixed_outer: Tuple[float, float] = None   # (outer lr, mu) when T == 0
    # inner AdamW scalars (config 1's; the other configs name none)
    lr: float = 3e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    param_std: float = 0.02
    grad_std: float = 1e-3
    seed: int = 0
    tensors: List[Tuple[str, int]] = field(default_factory=list)

    def __post_init__(self):
        if not self.tensors:
            self.tensors = gpt_tensor_list(self.L, self.d, self.vocab, self.ctx)

    @property
    def numels(self) -> List[int]:
        return [n for _, n in self.tensors]

    @property
    def N(self) -> int:
        return sum(self.numels)


def workloads():
    """The five configurations, by name."""
    w = [
        # 1 outer Nesterov step with DiLoCo's fixed scalars.
        Workload("tiny", L=2, d=256, vocab=8192, ctx=1024, G=2, H=4, rounds=1, T=0,
                 fixed_outer=(0.7, 0.9)),
        # T = 1100: syncs at t = 50, 100 fall in the lazy-start phase (t <= 110),
        # t = 150 in the mu = 0.99 band, t = 200 in the mu = 0.95 band.
        Workload("gpt2_small", L=12, d=768, vocab=50257, ctx=1024, G=4, H=50, rounds=4, T=1100),
        # T = 1800: t = 100 lazy start, 200 -> mu 0.99, 300 -> mu 0.95.
        Workload("gpt2_medium", L=24, d=1024, vocab=50257, ctx=1024, G=8, H=100, rounds=3, T=1800,
                 grad_bf16=True),
        # steady state: mu 0.9, outer lr 1.1.
        Workload("gpt2_xl", L=48, d=1600, vocab=50257, ctx=1024, G=8, H=100, rounds=1, T=0,
                 fixed_outer=(1.1, 0.9)),
        Workload("gpt_7b", L=32, d=4096, vocab=50257, ctx=1024, G=2, H=100, rounds=1, T=0,
                 fixed_outer=(1.1, 0.9), offload=True),
    ]
    return {x.name: x for x in w}


# Stream identifiers of the counter-based generator (generator.py): gradients of
# replica g use stream g; parameter initialisation uses a stream no replica has.
PARAM_STREAM = 0xFFFF
