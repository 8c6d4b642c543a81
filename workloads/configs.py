"""The five synthetic workloads (shapes borrowed from BERT-base, OPT-1.3B,
Llama-2-7B and OPT-13B feed-forward layers) and scaled-down variants of each
that a CPU check finishes in seconds."""
from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class FFNConfig:
    name: str
    index: int                 # 1..5, enters the seed
    d_model: int
    d_ff: int
    act: str                   # "gelu" | "swiglu"
    dtype: str                 # "f32" | "bf16": storage type of X, Y and dense weights
    heavy_frac: float          # planted fraction p; k = round(p * d_ff)
    heavy_scale: float         # planted neurons' W1(/Wg) column and W2 row are scaled by this
    k: int
    rem_kind: str              # "lowrank" | "int4"
    rank: int = 0
    group: int = 0
    calib_T: int = 0
    prefill_T: int = 0
    decode_B: Tuple[int, ...] = ()
    n_layers: int = 1
    weight_std: float = 0.02
    exact_svd: bool = True     # False: seeded Gaussian factors of the right shape

    @property
    def m(self) -> int:
        return self.d_ff - self.k

    @property
    def n_up(self) -> int:
        return 2 if self.act == "swiglu" else 1

    def flops_per_token(self) -> float:
        """The split path's own multiply-adds x2 per token (padding excluded)."""
        n = self.n_up + 1
        if self.rem_kind == "lowrank":
            return 2.0 * n * (self.d_model * (self.k + self.rank) + self.rank * self.m)
        return 2.0 * n * self.d_model * self.d_ff

    def weight_bytes(self) -> float:
        """Bytes of packed weights one forward call must stream (padding excluded)."""
        n = self.n_up + 1
        esz = 4 if self.dtype == "f32" else 2
        heavy = n * self.d_model * self.k * esz
        if self.rem_kind == "lowrank":
            return heavy + n * self.rank * (self.d_model + self.m) * esz
        nib = n * self.m * self.d_model / 2.0
        scales = n * self.m * (self.d_model // self.group) * 2
        return heavy + nib + scales


C1 = FFNConfig("C1-bert-base-f32", 1, 768, 3072, "gelu", "f32", 0.05, 8.0, 154,
               "lowrank", rank=64, calib_T=512, prefill_T=128)
C2 = FFNConfig("C2-opt1.3b-bf16", 2, 2048, 8192, "gelu", "bf16", 0.03, 10.0, 246,
               "lowrank", rank=512, calib_T=4096, prefill_T=4096)
C3 = FFNConfig("C3-llama7b-swiglu-bf16", 3, 4096, 11008, "swiglu", "bf16", 0.05, 8.0, 550,
               "lowrank", rank=1024, calib_T=8192, prefill_T=4096, decode_B=(1, 8, 32))
C4 = FFNConfig("C4-llama7b-swiglu-int4", 4, 4096, 11008, "swiglu", "bf16", 0.05, 8.0, 550,
               "int4", group=128, calib_T=8192, prefill_T=0, decode_B=(1, 4, 16))
C5 = FFNConfig("C5-opt13b-stack-bf16", 5, 5120, 20480, "gelu", "bf16", 0.04, 8.0, 819,
               "lowrank", rank=1280, calib_T=16384, prefill_T=4096, decode_B=(16,),
               n_layers=40, exact_svd=False)

CONFIGS = {c.name.split("-")[0]: c for c in (C1, C2, C3, C4, C5)}


def get_config(name: str) -> FFNConfig:
    return CONFIGS[name]


def reduced(cfg: FFNConfig, d_model: int, d_ff: int, rank: int = 0, calib_T: int = 0,
            prefill_T: int = 0, n_layers: int = 0, group: int = 0) -> FFNConfig:
    """Same recipe at a smaller shape; k keeps the rule k = round(p * d_ff)."""
    k = int(round(cfg.heavy_frac * d_ff))
    return replace(cfg, name=cfg.name + "-reduced", d_model=d_model, d_ff=d_ff, k=k,
                   rank=rank or cfg.rank, calib_T=calib_T or cfg.calib_T,
                   prefill_T=prefill_T or cfg.prefill_T,
                   n_layers=n_layers or cfg.n_layers, group=group or cfg.group)
