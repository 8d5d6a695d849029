"""Device-memory plumbing shared by bench.py, the driver hooks and the tests: descriptor from a
synthetic configuration, host array -> device tensor in the storage type, workspace allocation.
PyTorch is used for allocations only; nothing of the method's arithmetic lives here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as bx
from . import synth

DEV = "cuda:0"


def desc_of(cfg: synth.XattnConfig, flags=0, scale=0.0, block_offsets=None, rope_base=0.0, rope_positions=None, **packed):
    """block_offsets / rope_positions / cu_seqlens_*: optional int32 device tensors (the caller keeps them alive)."""
    return bx.make_desc(block_offsets=block_offsets, rope_base=rope_base, rope_positions=rope_positions, **packed, batch=cfg.batch, seq_q=cfg.seq_q, seq_kv=cfg.seq_kv, hidden=cfg.hidden,
                        n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                        block_size=cfg.block_size, block_offset=cfg.block_offset,
                        io_dtype=bx.BEAGLE_BF16 if cfg.dtype == "bf16" else bx.BEAGLE_F32,
                        softmax_scale=scale, flags=flags)


def tdtype(cfg):
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


def to_dev(a: np.ndarray, cfg) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, np.float32))
    if cfg.dtype == "bf16":
        t = t.to(torch.bfloat16)      # exact: the values are bf16-representable
    return t.to(DEV).contiguous()


def workspace(desc, which):
    n = bx.beagle_xattn_workspace_bytes(desc, which)
    assert n > 0
    return torch.empty(n, dtype=torch.uint8, device=DEV)
