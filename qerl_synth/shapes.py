"""Layer shapes of the benchmark configurations (Qwen2.5-family decoder
blocks, the models the paper trains).  Config numbers are 1-based."""
from __future__ import annotations

from dataclasses import dataclass


@dataclass(frozen=True)
class LinearShape:
    name: str
    K: int          # input features
    N: int          # output features
    noisy_input: bool  # fed by an AQN RMSNorm (q, k, v, gate, up)

    @property
    def packed_bytes(self) -> int:
        """E2M1 codes + E4M3 scale bytes = 0.5625 B per weight."""
        return self.N * self.K // 2 + self.N * self.K // 16


def _block(hidden: int, kv: int, inter: int):
    return [
        LinearShape("q", hidden, hidden, True),
        LinearShape("k", hidden, kv, True),
        LinearShape("v", hidden, kv, True),
        LinearShape("o", hidden, hidden, False),
        LinearShape("gate", hidden, inter, True),
        LinearShape("up", hidden, inter, True),
        LinearShape("down", inter, hidden, False),
    ]


CONFIGS = {
    1: dict(model="single-2048", hidden=2048, layers=1, r=16, alpha=32.0, M=[1],
            linears=[LinearShape("lin", 2048, 2048, False)]),
    2: dict(model="qwen2.5-7b", hidden=3584, layers=28, r=32, alpha=64.0, M=[8],
            linears=_block(3584, 512, 18944)),
    3: dict(model="qwen2.5-7b", hidden=3584, layers=28, r=32, alpha=64.0, M=[32, 64, 128],
            linears=_block(3584, 512, 18944)),
    4: dict(model="qwen2.5-14b", hidden=5120, layers=48, r=64, alpha=128.0, M=[2048],
            linears=_block(5120, 1024, 13824)),
    5: dict(model="qwen2.5-32b", hidden=5120, layers=64, r=64, alpha=128.0,
            M=[1, 16, 128, 4096], linears=_block(5120, 1024, 27648)),
}


def config_linears(config: int):
    return list(CONFIGS[config]["linears"])
