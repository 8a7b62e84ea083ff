"""Plumbing shared by the GPU parity tests: building the HIP library if it is
not there, moving tensors to numpy bit patterns, carving deliberately
misaligned device buffers.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2304_11277_amd import build as fbuild


def load_product():
    fbuild.build_lib(force=False)
    import paper_2304_11277_amd as f
    return f


def np_bits(t: torch.Tensor) -> np.ndarray:
    """Device or host tensor -> numpy array of raw bit patterns (uint32 for
    fp32, uint16 for bf16)."""
    t = t.detach().contiguous().cpu()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy().view(np.uint32)
    raise TypeError(t.dtype)


def np_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().cpu().numpy()


def np_grad(t: torch.Tensor) -> np.ndarray:
    """Gradient buffer -> what the oracle takes (float32 array or uint16 bf16 bits)."""
    return np_bits(t) if t.dtype in (torch.bfloat16, torch.float16) else np_f32(t)


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    ia = a.view(np.uint32) if a.dtype == np.float32 else a
    ib = b.view(np.uint32) if b.dtype == np.float32 else b
    return ia.shape == ib.shape and ia.dtype == ib.dtype and bool(np.array_equal(ia, ib))


def first_diff(a: np.ndarray, b: np.ndarray) -> str:
    ia = a.view(np.uint32) if a.dtype == np.float32 else a
    ib = b.view(np.uint32) if b.dtype == np.float32 else b
    if ia.shape != ib.shape:
        return f"shape {ia.shape} vs {ib.shape}"
    bad = np.flatnonzero(ia != ib)
    if bad.size == 0:
        return "equal"
    k = int(bad[0])
    return f"{bad.size} of {ia.size} differ; first at {k}: {hex(int(ia[k]))} vs {hex(int(ib[k]))}"


def carve(n: int, dtype, elem_offset: int, device="cuda", fill=None) -> torch.Tensor:
    """A tensor of n elements whose address is the allocator's (256-byte
    aligned) base plus elem_offset elements."""
    base = torch.empty(n + elem_offset + 64, dtype=dtype, device=device)
    if fill is not None:
        base.view(torch.int16 if dtype in (torch.bfloat16, torch.float16) else torch.int32).fill_(fill)
    return base[elem_offset:elem_offset + n]


POISON32 = 0x7FC0DEAD - (1 << 32) if 0x7FC0DEAD >= (1 << 31) else 0x7FC0DEAD   # a NaN pattern
POISON16 = 0x7FCD


from adam_parity import adam_close, assert_adam_bits, assert_adam_parity  # noqa: E402,F401  (re-exported for the GPU tests)
