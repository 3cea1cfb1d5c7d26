"""Device-memory plumbing for one OSP job: torch allocates the arenas and the
workspace, the library does all the arithmetic.  No method logic here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B


class DeviceJob:
    """PS arenas, N worker replicas and the workspace of one job on cuda:0,
    bound to a library context."""

    def __init__(self, numel, offset, arena_elems: int, n_workers: int, lr: float,
                 momentum: float, params_host: np.ndarray,
                 worker_weight=None, element_keys: bool = False, chunk_elems: int = 0,
                 param_stride: Optional[int] = None, device: str = "cuda:0",
                 pad_fill: Optional[float] = None, declare_in_sync: bool = True):
        self.dev = torch.device(device)
        self.arena = int(arena_elems)
        self.N = int(n_workers)
        self.param_stride = int(param_stride) if param_stride else self.arena
        self.ctx = B.Context(numel, offset, arena_elems, n_workers, lr, momentum,
                             worker_weight=worker_weight, element_keys=element_keys,
                             chunk_elems=chunk_elems)
        p = torch.from_numpy(np.ascontiguousarray(params_host, np.float32))
        self.P = p.to(self.dev)
        self.V = torch.zeros(self.arena, dtype=torch.float32, device=self.dev)
        self.Pw = torch.zeros((self.N, self.param_stride), dtype=torch.float32, device=self.dev)
        if pad_fill is not None:
            self.Pw.fill_(pad_fill)
        self.Pw[:, :self.arena] = self.P[None, :]
        nbytes = self.ctx.osp_workspace_bytes()
        # torch's caching allocator hands out 512-byte aligned blocks
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.dev)
        # the replicas were just filled from P, so the job may say so
        self.ctx.osp_bind(self.P, self.V, self.Pw, self.param_stride, self.workspace, nbytes,
                          replicas_in_sync=declare_in_sync)

    def upload_grads(self, grads_host: np.ndarray) -> torch.Tensor:
        assert grads_host.dtype == np.float32 and grads_host.ndim == 2
        return torch.from_numpy(grads_host).to(self.dev)

    def upload_grads_bf16(self, grads_bf16_host: np.ndarray) -> torch.Tensor:
        """bfloat16 bit patterns (uint16, [N, stride]) as a device tensor of int16."""
        assert grads_bf16_host.dtype == np.uint16 and grads_bf16_host.ndim == 2
        return torch.from_numpy(grads_bf16_host.view(np.int16)).to(self.dev)

    def sync_step_bf16(self, grads: torch.Tensor, granularity: int, budget_elems: int) -> None:
        c, s = self.ctx, grads.shape[1]
        c.osp_ps_aggregate_update_bf16(1, grads, s)
        c.osp_apply_stage(1)
        c.osp_lgp_correct_bf16(grads, s)
        c.osp_ps_aggregate_update_bf16(2, grads, s)
        c.osp_apply_stage(2)
        c.osp_split(granularity, budget_elems)

    def sync_step_windows_bf16(self, grads: torch.Tensor, granularity: int, budget_elems: int) -> None:
        c, s = self.ctx, grads.shape[1]
        c.osp_rs_window_bf16(grads, s)
        c.osp_ics_window_bf16(grads, s, granularity, budget_elems)

    # the six calls of one synchronization step, in the paper's order
    def sync_step(self, grads: torch.Tensor, granularity: int, budget_elems: int) -> None:
        c, s = self.ctx, grads.shape[1]
        c.osp_ps_aggregate_update(1, grads, s)
        c.osp_apply_stage(1)
        c.osp_lgp_correct(grads, s)
        c.osp_ps_aggregate_update(2, grads, s)
        c.osp_apply_stage(2)
        c.osp_split(granularity, budget_elems)

    # the same step as its two windows
    def sync_step_windows(self, grads: torch.Tensor, granularity: int, budget_elems: int) -> None:
        c, s = self.ctx, grads.shape[1]
        c.osp_rs_window(grads, s)
        c.osp_ics_window(grads, s, granularity, budget_elems)

    def download(self):
        torch.cuda.synchronize(self.dev)
        return self.P.cpu().numpy(), self.V.cpu().numpy(), self.Pw.cpu().numpy()
