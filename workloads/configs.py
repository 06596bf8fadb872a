"""The benchmark configurations as data (schedule, stage load, graph recipe, caps, seed).

Stage indices are 0-based, like the paper's stage numbering (Section 2.2.1, Figure 1).
"""
from dataclasses import dataclass
from typing import Optional

from . import graphs


@dataclass(frozen=True)
class GptLoad:
    """GEMM burst shaped like `layers` GPT blocks: hidden h, feed-forward width ffn, tokens = seq * microbatch."""
    layers: int
    hidden: int
    ffn: int
    tokens: int


@dataclass(frozen=True)
class Config:
    name: str
    schedule: str            # "1f1b" or "gpipe"
    p: int                   # pipeline stages
    m: int                   # micro-batches per epoch
    stage: int               # emulated stage, 0-based
    graph: str               # "rmat" or "fixed_outdeg"
    scale: int               # log2(vertices)
    edges: int
    iterations: int
    seed: int
    damping: float = 0.85
    busy_fp_ns: Optional[int] = None   # timed busy-wait stage load (config 1)
    busy_bp_ns: Optional[int] = None
    load: Optional[GptLoad] = None     # GEMM burst stage load
    mem_cap_bytes: Optional[int] = None
    cu_count: int = 256

    @property
    def vertices(self) -> int:
        return 1 << self.scale

    def build_graph(self) -> graphs.Csr:
        if self.graph == "rmat":
            return graphs.rmat_csr(self.scale, self.edges, self.seed)
        if self.graph == "fixed_outdeg":
            return graphs.fixed_outdeg_csr(self.vertices, self.edges // self.vertices, self.seed)
        raise ValueError(self.graph)


_GPT4096 = GptLoad(layers=4, hidden=4096, ffn=16384, tokens=2048)
_GPT8192 = GptLoad(layers=4, hidden=8192, ffn=32768, tokens=4096)

CONFIGS = [
    Config("cfg1", "1f1b", 4, 8, 2, "rmat", 14, 1 << 18, 30, 0, busy_fp_ns=2_000_000, busy_bp_ns=4_000_000),
    Config("cfg2", "1f1b", 4, 8, 2, "rmat", 22, 1 << 26, 50, 1, load=_GPT4096),
    Config("cfg3", "1f1b", 8, 16, 7, "rmat", 24, 1 << 28, 50, 2, load=_GPT4096, mem_cap_bytes=16 << 30),
    Config("cfg4", "1f1b", 8, 32, 0, "fixed_outdeg", 23, 1 << 28, 100, 3, load=_GPT4096, cu_count=64),
    Config("cfg5", "gpipe", 16, 16, 8, "rmat", 26, 1 << 30, 100, 4, load=_GPT8192, mem_cap_bytes=40 << 30),
]


def by_name(name: str) -> Config:
    for c in CONFIGS:
        if c.name == name:
            return c
    raise KeyError(name)
