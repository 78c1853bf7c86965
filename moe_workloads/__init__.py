"""Seeded synthetic inputs for the MoE-layer workloads.

This module only DRAWS numbers and describes shapes; it holds none of the
layer's arithmetic, and it is the one piece of code that both the CPU oracle's
tests and the HIP path's tests/benchmark use, so that both sides see the very
same bits.

The five workloads stand in for the models the paper evaluates (section 5.1:
Mixtral 8x7B, Mixtral 8x22B, DBRX) at micro-batch sizes from the top of its
kernel sweep (section 6.2, mu = 32..256) up to the large-batch regime it argues
for (section 1).  A layer only ever sees a [mu, h1] activation matrix and n_e
weight sets, so no dataset or trained checkpoint is needed: activations are
N(0,1), weights and router N(0, 0.02) (standard deviations), drawn in float32
and rounded once to the storage type.

Every tensor comes from its own numpy Philox stream keyed by (seed, tensor tag,
expert), so a single expert's matrix can be regenerated alone and generation
can run on several threads without changing the values.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Optional, Tuple

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    name: str
    dtype: str          # "f32" | "bf16"
    T: int              # tokens in the micro-batch (mu)
    H: int              # h1, model hidden size
    F: int              # h2, expert intermediate size
    E: int              # n_e
    k: int              # top-k
    page_bytes: int     # fixed size of one expert-weight page
    seed: int
    bias: Tuple[Tuple[int, float], ...] = ()   # (expert, router bias) pairs; empty = no bias
    streamed: bool = False                     # expert pages live in pinned host memory

    @property
    def R(self) -> int:
        return self.T * self.k

    @property
    def dtype_code(self) -> int:
        return 1 if self.dtype == "bf16" else 0

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def ffn_flops(self) -> float:
        return 6.0 * self.R * self.H * self.F

    @property
    def router_flops(self) -> float:
        return 2.0 * self.T * self.H * self.E


KiB, MiB = 1024, 1024 * 1024

CONFIGS: Dict[str, MoEConfig] = {
    "c1_tiny_f32": MoEConfig("c1_tiny_f32", "f32", 64, 256, 512, 8, 2, 64 * KiB, seed=0),
    "c2_mixtral8x7b_t256": MoEConfig("c2_mixtral8x7b_t256", "bf16", 256, 4096, 14336, 8, 2, 2 * MiB, seed=1),
    "c3_mixtral8x7b_t4096": MoEConfig("c3_mixtral8x7b_t4096", "bf16", 4096, 4096, 14336, 8, 2, 2 * MiB, seed=2),
    # expert 0 takes ~40 % of the assignments, expert 7 under 2 %
    "c4_mixtral8x22b_t8192_skew": MoEConfig("c4_mixtral8x22b_t8192_skew", "bf16", 8192, 6144, 16384, 8, 2,
                                            4 * MiB, seed=3, bias=((0, 2.5), (7, -1.9))),
    "c5_dbrx_t16384_streamed": MoEConfig("c5_dbrx_t16384_streamed", "bf16", 16384, 6144, 10752, 16, 4,
                                         4 * MiB, seed=4, streamed=True),
}
ORDER = list(CONFIGS)


def scaled(cfg: MoEConfig, **kw) -> MoEConfig:
    """A copy of ``cfg`` with some fields replaced (reduced-size test cases)."""
    return dataclasses.replace(cfg, **kw)


_TAGS = {"x": 1, "Wr": 2, "W1": 3, "W3": 4, "W2": 5}


def _normal(seed: int, tag: str, index: int, shape, std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=[(seed << 16) ^ _TAGS[tag], index]))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def _to_storage(a: np.ndarray, cfg: MoEConfig) -> torch.Tensor:
    t = torch.from_numpy(a)
    return t.to(torch.bfloat16) if cfg.dtype == "bf16" else t


def bias_vector(cfg: MoEConfig) -> Optional[torch.Tensor]:
    if not cfg.bias:
        return None
    b = torch.zeros(cfg.E, dtype=torch.float32)
    for e, v in cfg.bias:
        b[e] = v
    return b


def make_activations(cfg: MoEConfig) -> torch.Tensor:
    return _to_storage(_normal(cfg.seed, "x", 0, (cfg.T, cfg.H), 1.0), cfg)


def make_router(cfg: MoEConfig) -> torch.Tensor:
    return _to_storage(_normal(cfg.seed, "Wr", 0, (cfg.E, cfg.H), 0.02), cfg)


def make_expert_matrix(cfg: MoEConfig, which: str, e: int) -> torch.Tensor:
    """One expert's dense matrix: W1/W3 are [F,H], W2 is [H,F] (out-features major)."""
    shape = (cfg.F, cfg.H) if which in ("W1", "W3") else (cfg.H, cfg.F)
    return _to_storage(_normal(cfg.seed, which, e, shape, 0.02), cfg)


def make_inputs(cfg: MoEConfig, threads: int = 8, identical_experts: bool = False) -> Dict[str, torch.Tensor]:
    """All tensors of a workload as CPU torch tensors in the storage type.

    x[T,H], Wr[E,H], bias[E] (float32) or None, W1[E,F,H], W3[E,F,H], W2[E,H,F].
    ``identical_experts`` copies expert 0's matrices into every expert (used by
    the routing-independence invariant).
    """
    out: Dict[str, torch.Tensor] = {"x": make_activations(cfg), "Wr": make_router(cfg), "bias": bias_vector(cfg)}
    W1 = torch.empty((cfg.E, cfg.F, cfg.H), dtype=cfg.torch_dtype)
    W3 = torch.empty((cfg.E, cfg.F, cfg.H), dtype=cfg.torch_dtype)
    W2 = torch.empty((cfg.E, cfg.H, cfg.F), dtype=cfg.torch_dtype)
    dst = {"W1": W1, "W3": W3, "W2": W2}

    def job(args):
        which, e = args
        dst[which][e].copy_(make_expert_matrix(cfg, which, 0 if identical_experts else e))

    jobs = [(w, e) for e in range(cfg.E) for w in ("W1", "W3", "W2")]
    with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
        list(pool.map(job, jobs))
    out.update(dst)
    return out


def prompt_lengths(n: int, seed: int, s_avg: int = 77, s_max: int = 418, s_min: int = 4) -> np.ndarray:
    """n seeded prompt lengths standing in for a request mix of which the paper gives the average
    and the maximum (its table of workload configurations; the defaults are the MTBench row).
    Log-normal (sigma 0.7: most prompts short, a long tail), clipped to [s_min, s_max], scaled so that
    the mean comes out at s_avg; the longest request is set to s_max.  The shape of the distribution
    is this module's choice: the paper prints only the two numbers."""
    rng = np.random.Generator(np.random.Philox(key=[(seed << 16) ^ 0x4c45, 0]))
    z = np.exp(0.7 * rng.standard_normal(n))
    scale = s_avg / z.mean()
    for _ in range(20):                                   # the clipping moves the mean: a few fixed-point steps
        lens = np.clip(np.rint(z * scale), s_min, s_max)
        scale *= s_avg / lens.mean()
    lens = np.clip(np.rint(z * scale), s_min, s_max).astype(np.int64)
    lens[int(np.argmax(lens))] = s_max
    return lens


def oracle_view(t: Optional[torch.Tensor]) -> Optional[np.ndarray]:
    """The numpy array the oracle takes for a CPU tensor: float32 as is,
    bfloat16 as its uint16 bit patterns (no copy)."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
