"""PyTorch custom operators over the C-ABI library (drop-in sampling calls for a
point-network stage: sample, then gather what the next layer consumes).

    import paper_2604_17720_amd.torch_ops          # registers torch.ops.flashfps.*
    idx = torch.ops.flashfps.fps_exact(xyz, 1024, 0)                       # [B, 1024] int32
    idx = torch.ops.flashfps.fps_prune(xyz, 1024, 1, 4, 3, 0, 0)           # p = 75 %, CP+IP
    all_ = torch.ops.flashfps.fps_stages(xyz, [1024, 256, 64], 0, 1, 1, 0, 0, 0)  # [B, 1344]
    pts = torch.ops.flashfps.gather_rows(xyz, idx)                         # [B, 1024, 3]

Sampling is not differentiable (indices); gather_rows is registered without an
autograd formula as well: it is an inference-path helper."""
from __future__ import annotations

from typing import List

import torch

from . import binding as fb


@torch.library.custom_op("flashfps::fps_exact", mutates_args=(), device_types="cuda")
def fps_exact(xyz: torch.Tensor, M: int, start_idx: int) -> torch.Tensor:
    return fb.ffps_exact(xyz.contiguous(), M, start_idx)


@fps_exact.register_fake
def _(xyz, M, start_idx):
    return xyz.new_empty((xyz.shape[0] if xyz.dim() == 3 else 1, M), dtype=torch.int32)


@torch.library.custom_op("flashfps::fps_prune", mutates_args=(), device_types="cuda")
def fps_prune(xyz: torch.Tensor, M: int, keep_num: int, keep_den: int, flags: int,
              start_idx: int, seed: int) -> torch.Tensor:
    return fb.ffps_prune(xyz.contiguous(), M, keep_num, keep_den, flags, start_idx, seed=seed)[0]


@fps_prune.register_fake
def _(xyz, M, keep_num, keep_den, flags, start_idx, seed):
    return xyz.new_empty((xyz.shape[0] if xyz.dim() == 3 else 1, M), dtype=torch.int32)


@torch.library.custom_op("flashfps::fps_stages", mutates_args=(), device_types="cuda")
def fps_stages(xyz: torch.Tensor, M_stages: List[int], mode: int, keep_num: int, keep_den: int,
               flags: int, start_idx: int, seed: int) -> torch.Tensor:
    x = xyz.contiguous()
    B = x.shape[0] if x.dim() == 3 else 1
    out = torch.empty((B, sum(M_stages)), dtype=torch.int32, device=x.device)
    fb.ffps_cached_stages(x, M_stages, mode, keep_num, keep_den, flags, start_idx, seed=seed, out=out)
    return out


@fps_stages.register_fake
def _(xyz, M_stages, mode, keep_num, keep_den, flags, start_idx, seed):
    return xyz.new_empty((xyz.shape[0] if xyz.dim() == 3 else 1, sum(M_stages)), dtype=torch.int32)


@torch.library.custom_op("flashfps::gather_rows", mutates_args=(), device_types="cuda")
def gather_rows(rows: torch.Tensor, idx: torch.Tensor) -> torch.Tensor:
    return fb.ffps_gather_rows(rows.contiguous(), idx)


@gather_rows.register_fake
def _(rows, idx):
    return rows.new_empty((rows.shape[0], idx.shape[1], rows.shape[2]))
