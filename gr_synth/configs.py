"""The five benchmark workloads (shapes only)."""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class GRConfig:
    config_id: int        # 1..5; also the high digits of every RNG seed
    name: str
    B: int                # requests per batch
    L_min: int            # prompt length (L_min == L_max: fixed; else uniform integer in [L_min, L_max])
    L_max: int
    Hq: int               # query heads
    Hkv: int              # KV heads
    d: int                # head dimension
    W: int                # beam width (= top-K)
    ND: int               # decode phases = tokens per item
    V: int                # codebook size per level
    n_items: int          # valid items in the table
    zipf_a: float         # 0 = uniform first token, else Zipf exponent of first-token popularity
    logit_sigma: float    # logits = sigma * N(0,1)

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    def scaled(self, **kw) -> "GRConfig":
        return replace(self, **kw)


CONFIGS = {
    1: GRConfig(1, "tiny", 1, 256, 256, 8, 8, 64, 16, 3, 256, 2_000, 0.0, 2.0),
    2: GRConfig(2, "b8_l2048_w128", 8, 2048, 2048, 32, 8, 128, 128, 3, 8192, 1_000_000, 0.0, 2.0),
    3: GRConfig(3, "b32_l4096_w256", 32, 4096, 4096, 32, 8, 128, 256, 3, 8192, 10_000_000, 1.1, 3.0),
    4: GRConfig(4, "long_b4_l16384_w512", 4, 16384, 16384, 32, 8, 128, 512, 3, 8192, 10_000_000, 1.1, 3.0),
    5: GRConfig(5, "conc_b128_ragged_w256", 128, 512, 8192, 32, 8, 128, 256, 3, 8192, 10_000_000, 1.1, 3.0),
}


def get_config(config_id: int) -> GRConfig:
    return CONFIGS[int(config_id)]
