"""Seeded synthetic inputs for the FlatParameter data path.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds shapes and random draws only: none of the method's
arithmetic (no layout computation, no cast, no reduction, no optimizer) lives
here.  Sizes that depend on the layout (the padded length P, the unpadded
length N) are passed in by the caller, who obtained them from whichever side
is under test.

The unit shapes stand in for the paper's evaluation models (Sec. 5: T5,
minGPT-175B, DHEN); the path is data-independent, so only shapes, dtypes, the
world size W and value distributions matter.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import torch

BASE_SEED = 20230411

Shape = Tuple[int, ...]


def gpt_block_shapes(d: int, ffn: int) -> List[Shape]:
    """GPT-style transformer block in flatten order: four weights, four biases,
    then two LayerNorm weight/bias pairs."""
    return [
        (3 * d, d), (d, d), (ffn, d), (d, ffn),
        (3 * d,), (d,), (ffn,), (d,),
        (d,), (d,), (d,), (d,),
    ]


def llama_block_shapes(d: int, ffn: int) -> List[Shape]:
    """Llama-style block: q, k, v, o projections, SwiGLU gate/up/down, two
    RMSNorm weights; no biases."""
    return [
        (d, d), (d, d), (d, d), (d, d),
        (ffn, d), (ffn, d), (d, ffn),
        (d,), (d,),
    ]


@dataclass(frozen=True)
class Unit:
    name: str
    shapes: Tuple[Shape, ...]


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration: a list of FSDP units processed in
    order, the simulated world size, and the gradient dtype / distribution."""
    name: str
    units: Tuple[Unit, ...]
    world_size: int
    grad_dtype: str            # "f32" or "bf16"
    outlier_frac: float = 0.0  # fraction of grad elements multiplied by outlier_scale
    outlier_scale: float = 1.0
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    notes: str = ""
    distinct_units: Tuple[int, ...] = field(default=())  # indices of units with distinct shapes


def _cfg0() -> Workload:
    u = Unit("gpt2s.block", tuple(gpt_block_shapes(768, 3072)))
    return Workload("cfg0_gpt2s_block_w8", (u,), 8, "f32", distinct_units=(0,))


def _cfg1() -> Workload:
    root = Unit("gpt2s.root", ((50257, 768), (1024, 768), (768,), (768,)))
    blocks = tuple(Unit(f"gpt2s.block{i}", tuple(gpt_block_shapes(768, 3072))) for i in range(12))
    return Workload("cfg1_gpt2s_full_w8", (root,) + blocks, 8, "f32", distinct_units=(0, 1))


def _cfg2() -> Workload:
    blocks = tuple(Unit(f"gpt1p3b.block{i}", tuple(gpt_block_shapes(2048, 8192))) for i in range(24))
    return Workload("cfg2_1p3b_w12", blocks, 12, "f32", outlier_frac=0.01, outlier_scale=1e3,
                    distinct_units=(0,))


def _cfg3() -> Workload:
    blocks = tuple(Unit(f"llama7b.block{i}", tuple(llama_block_shapes(4096, 11008))) for i in range(32))
    return Workload("cfg3_llama7b_w64", blocks, 64, "bf16", distinct_units=(0,))


def _cfg4() -> Workload:
    u = Unit("gpt3_175b.block", tuple(gpt_block_shapes(12288, 49152)))
    return Workload("cfg4_gpt3_175b_block_w16", (u,), 16, "bf16", distinct_units=(0,))


def config(i: int) -> Workload:
    return (_cfg0, _cfg1, _cfg2, _cfg3, _cfg4)[i]()


NUM_CONFIGS = 5


def ragged_unit() -> Unit:
    """A small unit whose parameter sizes are deliberately not multiples of any
    vector width, including a 0-dim scalar and an empty tensor."""
    return Unit("ragged", ((3, 5), (7,), (1,), (), (0, 4), (13, 17), (2, 3, 5), (1023,), (4097,), (31, 33)))


# ---------------------------------------------------------------------------
# random draws
# ---------------------------------------------------------------------------

def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def numel(shape: Sequence[int]) -> int:
    n = 1
    for s in shape:
        n *= int(s)
    return n


def gen_params(unit: Unit, unit_index: int, device="cpu", seed: int = BASE_SEED,
               std: float = 0.02) -> List[torch.Tensor]:
    """fp32 master parameters ~ N(0, std), one tensor per shape, in unit order."""
    g = _gen(seed + 1000 * unit_index, device)
    out = []
    for shp in unit.shapes:
        t = torch.empty(tuple(shp), dtype=torch.float32, device=device)
        if t.numel():
            t.normal_(0.0, std, generator=g)
        out.append(t)
    return out


def gen_rank_grad(P: int, N: int, rank: int, unit_index: int, grad_dtype: str, device="cpu",
                  seed: int = BASE_SEED, std: float = 1e-3, outlier_frac: float = 0.0,
                  outlier_scale: float = 1.0, out: torch.Tensor | None = None) -> torch.Tensor:
    """Rank `rank`'s unsharded flat gradient buffer: P elements, the first N
    ~ N(0, std) (a Bernoulli(outlier_frac) subset multiplied by outlier_scale),
    the trailing P-N pad positions zero.  bf16 buffers are drawn in fp32 and
    stored as bf16."""
    g = _gen(seed + 7919 * unit_index + rank + 1, device)
    x = torch.empty(P, dtype=torch.float32, device=device)
    if N:
        x[:N].normal_(0.0, std, generator=g)
    if outlier_frac > 0.0 and N:
        mask = torch.rand(N, generator=g, device=device) < outlier_frac
        x[:N] = torch.where(mask, x[:N] * outlier_scale, x[:N])
        del mask
    x[N:].zero_()
    dt = {"f32": torch.float32, "bf16": torch.bfloat16}[grad_dtype]
    if out is None:
        return x.to(dt)
    out.copy_(x)
    return out
