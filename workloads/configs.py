"""Workload shapes.

The five workloads are synthetic stand-ins with the entity / relation / edge
counts of the knowledge graphs in the paper's KG-statistics table (FB15k-237,
NELL995, ogbl-wikikg2, a 4-5M-entity text-attributed graph) and the paper's
hyper-parameter table (d = 400, batch 512, Adam 1e-4).  The 14 query
patterns are the ones the problem formulation names (1p ... pni).
"""
from dataclasses import dataclass, field
from typing import Dict, Tuple

# Template trees over: ('e',) anchor entity, ('p', x) relational projection,
# ('i', x1, .., xk) intersection, ('n', x) negation, ('u', x1, x2) union.
_E = ("e",)


def _p(x):
    return ("p", x)


TEMPLATES: Dict[str, tuple] = {
    "1p": _p(_E),
    "2p": _p(_p(_E)),
    "3p": _p(_p(_p(_E))),
    "2i": ("i", _p(_E), _p(_E)),
    "3i": ("i", _p(_E), _p(_E), _p(_E)),
    "ip": _p(("i", _p(_E), _p(_E))),
    "pi": ("i", _p(_p(_E)), _p(_E)),
    "2u": ("u", _p(_E), _p(_E)),
    "up": _p(("u", _p(_E), _p(_E))),
    "2in": ("i", _p(_E), ("n", _p(_E))),
    "3in": ("i", _p(_E), _p(_E), ("n", _p(_E))),
    "inp": _p(("i", _p(_E), ("n", _p(_E)))),
    "pin": ("i", _p(_p(_E)), ("n", _p(_E))),
    "pni": ("i", ("n", _p(_p(_E))), _p(_E)),
}

ALL14 = ("1p", "2p", "3p", "2i", "3i", "ip", "pi", "2u", "up",
         "2in", "3in", "inp", "pin", "pni")
# the union/intersection/projection patterns (no negation): what the box family can express
EPFO9 = ("1p", "2p", "3p", "2i", "3i", "ip", "pi", "2u", "up")


def _uniform(names):
    return {n: 1.0 / len(names) for n in names}


def _weighted_mix():
    # 40 % path queries, 30 % intersection, 20 % negation, 10 % union.
    mix = {}
    for names, w in ((("1p", "2p", "3p"), 0.40),
                     (("2i", "3i", "ip", "pi"), 0.30),
                     (("2in", "3in", "inp", "pin", "pni"), 0.20),
                     (("2u", "up"), 0.10)):
        for n in names:
            mix[n] = w / len(names)
    return mix


@dataclass(frozen=True)
class Config:
    name: str
    index: int
    N: int            # entities
    R: int            # relations
    T: int            # distinct directed triples
    alpha: float      # power-law exponent of the degree weights
    d: int            # embedding width
    h: int            # MLP hidden width
    K: int            # negatives per query
    B: int            # queries per batch
    gamma: float      # margin
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    mix: Dict[str, float] = field(default_factory=dict)
    d_sem: int = 0    # width of the frozen text feature (0 = none)
    streams: int = 2  # 1 = the caller's stream only; more = a library stream takes the independent work
    score_queries: int = 0   # all-entity ranking pass: number of queries
    topk: int = 0

    @property
    def seed(self) -> int:
        return 1000 + self.index


CONFIGS: Tuple[Config, ...] = (
    Config("tiny", 0, N=1000, R=20, T=10_000, alpha=2.1, d=32, h=64, K=8, B=64,
           gamma=12.0, mix=_uniform(("1p", "2p", "2i", "2in", "2u")), streams=1),
    Config("fb15k237", 1, N=15_000, R=474, T=310_000, alpha=2.1, d=400, h=800,
           K=128, B=512, gamma=24.0, mix=_uniform(ALL14)),
    Config("nell", 2, N=63_000, R=400, T=140_000, alpha=2.1, d=400, h=800,
           K=128, B=1024, gamma=24.0, mix=_uniform(ALL14), streams=4),
    Config("wikikg2", 3, N=2_500_000, R=1070, T=17_000_000, alpha=1.8, d=400,
           h=800, K=1024, B=4096, gamma=24.0, mix=_weighted_mix()),
    Config("semantic", 4, N=5_000_000, R=2000, T=40_000_000, alpha=2.1, d=400,
           h=800, K=1024, B=4096, gamma=24.0, mix=_uniform(ALL14), d_sem=1024,
           score_queries=1024, topk=10),
)


def get_config(key) -> Config:
    """Look a workload up by position (0..4) or by name."""
    if isinstance(key, int):
        return CONFIGS[key]
    for c in CONFIGS:
        if c.name == key:
            return c
    raise KeyError(key)
