"""Convenience wrapper: owns the context, the state and workspace tensors (device memory
from PyTorch) and the pointer arrays.  All arithmetic happens in libadapm.so."""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import torch

from . import binding as B
from .workloads import BlockSpec, Workload

_DT = {"f32": B.ADAPM_F32, "bf16": B.ADAPM_BF16}
_MOM = {"none": B.ADAPM_MOM_NONE, "full": B.ADAPM_MOM_FULL, "lowrank": B.ADAPM_MOM_LOWRANK}
_VM = {"element": B.ADAPM_V_ELEMENT, "rowgroup": B.ADAPM_V_ROWGROUP, "whole": B.ADAPM_V_WHOLE}


def to_c_block(b: BlockSpec) -> B.adapm_block_t:
    return B.adapm_block_t(b.rows, b.cols, _DT[b.param_dtype], _DT[b.grad_dtype], _MOM[b.mom], b.rank,
                           _VM[b.v_mode], b.v_group_rows, b.lr_scale, b.weight_decay)


def make_hparams(beta1=0.9, beta2=0.95, eps=1e-8, clip=1.0, adam_debias=0, K=5, T=1, bias_correction=1,
                 contraction=B.ADAPM_CONTRACT_AUTO, seed=0x5EED, normalise=0) -> B.adapm_hparams_t:
    return B.adapm_hparams_t(beta1, beta2, eps, clip if math.isfinite(clip) else float("inf"), adam_debias, K, T,
                             bias_correction, contraction, normalise, seed)


class AdaPM:
    def __init__(self, blocks: Sequence[BlockSpec], hp: B.adapm_hparams_t, device="cuda:0", allocate=True,
                 grad_clip: float = 0.0):
        self.blocks = list(blocks)
        self.hp = hp
        self.ctx = B.adapm_init([to_c_block(b) for b in self.blocks], hp)
        if grad_clip:
            B.adapm_set_grad_clip(self.ctx, grad_clip)
        self.state_bytes = B.adapm_state_bytes(self.ctx)
        self.workspace_bytes = B.adapm_workspace_bytes(self.ctx)
        self.device = torch.device(device)
        self.state = self.workspace = None
        self._ptr_key = None
        if allocate:
            self.state = torch.empty(max(self.state_bytes, 256), dtype=torch.uint8, device=self.device)
            self.workspace = torch.empty(max(self.workspace_bytes, 256), dtype=torch.uint8, device=self.device)
            B.adapm_state_init(self.ctx, self.state.data_ptr(), torch.cuda.current_stream(self.device).cuda_stream)

    def close(self):
        if self.ctx is not None:
            B.adapm_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, params: List[torch.Tensor], grads: List[torch.Tensor], t: int, lr: float):
        key = (tuple(p.data_ptr() for p in params), tuple(g.data_ptr() for g in grads))
        if key != self._ptr_key:
            self._pp, self._gp = B.ptr_array(key[0]), B.ptr_array(key[1])
            self._ptr_key = key
        B.adapm_step(self.ctx, self._pp, self._gp, self.state.data_ptr(), self.workspace.data_ptr(), t, lr,
                     torch.cuda.current_stream(self.device).cuda_stream)

    def last_grad_norm(self):
        """(norm, factor) of the last step with global gradient clipping."""
        return B.adapm_last_grad_norm(self.ctx, self.workspace.data_ptr(), torch.cuda.current_stream(self.device).cuda_stream)

    # views into the flat state buffer (fp32), for tests and checkpoints
    def state_view(self, i: int):
        b = self.blocks[i]
        oL, oR, om, ov = B.adapm_state_offsets(self.ctx, i)
        f = self.state.view(torch.float32)
        out = {}
        if oL is not None:
            out["L"] = f[oL // 4: oL // 4 + b.rows * b.rank].view(b.rows, b.rank)
            out["R"] = f[oR // 4: oR // 4 + b.rank * b.cols].view(b.rank, b.cols)
        if om is not None:
            out["m"] = f[om // 4: om // 4 + b.rows * b.cols].view(b.rows, b.cols)
        nv = b.rows * b.cols if b.v_mode == "element" else (b.rows // b.v_group_rows if b.v_mode == "rowgroup" else 1)
        out["v"] = f[ov // 4: ov // 4 + nv]
        return out
