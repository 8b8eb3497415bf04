"""Moves a seeded workload to the GPU and calls the C ABI through the binding."""
from __future__ import annotations

import numpy as np
import torch

import paper_2511_01633_amd as glm

TOL = 4e-3   # max abs error of fp32 output vs the fp64 oracle on identical bf16 inputs


def dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def host_u16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


class DeviceWorkload:
    def __init__(self, w):
        self.w = w
        self.pool = dev(w.pool)
        self.q = dev(w.q)
        self.tables = dev(w.block_tables)
        self.seq_lens = dev(w.seq_lens)
        self.cu = dev(w.cu_q_lens) if w.cu_q_lens is not None else None
        self.out = torch.full((w.sum_q, w.geom.num_q_heads, w.geom.head_dim), float("nan"), dtype=torch.float32,
                              device="cuda")

    def decode(self, plan=None, workspace=None, tables=None, seq_lens=None):
        w = self.w
        if workspace is None:
            nbytes = plan.workspace_bytes if plan is not None else glm.glm_attn_workspace_bytes(
                w.geom, w.B, 0, w.max_blocks * w.geom.block_size)
            workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.out.fill_(float("nan"))
        glm.glm_attn_decode(w.geom, self.pool, self.q, self.out, self.tables if tables is None else tables,
                            w.max_blocks, self.seq_lens if seq_lens is None else seq_lens, w.B, w.scale, plan, workspace)
        torch.cuda.synchronize()
        return self.out.cpu().numpy().astype(np.float64)

    def prefill(self, plan=None, workspace=None):
        w = self.w
        self.out.fill_(float("nan"))
        ws = workspace
        if plan is not None and plan.workspace_bytes > 0:
            ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
        glm.glm_attn_prefill_on_prefix(w.geom, self.pool, self.q, self.out, self.tables, w.max_blocks, self.seq_lens,
                                       self.cu, w.B, w.sum_q, int(w.q_lens.max()) if w.B else 0, w.scale, plan, ws)
        torch.cuda.synchronize()
        return self.out.cpu().numpy().astype(np.float64)

    def make_plan(self):
        w = self.w
        return glm.glm_plan_create(w.geom, w.block_tables, w.max_blocks, w.seq_lens, w.q_lens, w.B)
