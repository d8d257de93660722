"""Seeded synthetic workloads: block tables of the five benchmark shapes and the
low-rank-plus-tail gradient stream that stands in for real training gradients.

This module holds NO arithmetic of the optimizer itself.  It serves the tests,
the smoke check and the benchmark, which hand the same bits to the HIP library
and (in tests) to the CPU oracle.  The gradient model imitates what the paper
reports about transformer gradients (Sec. 3.2: energy concentrated in the top
few singular values with a long tail; slowly moving dominant subspace):

    G_t = D * ( U diag(s * a_t) V^T + sigma N_t ),   s_i = i^-p,
    a_1 = 1,  a_t = rho a_{t-1} + sqrt(1-rho^2) xi_t        (AR(1) in time)

with U, V orthonormal (QR of seeded Gaussians), N_t iid N(0,1), D a row scale.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional

import torch


@dataclass(frozen=True)
class BlockSpec:
    name: str
    rows: int
    cols: int
    param_dtype: str = "f32"        # "f32" | "bf16"
    grad_dtype: str = "f32"
    mom: str = "full"               # "none" | "full" | "lowrank"
    rank: int = 0
    v_mode: str = "element"         # "element" | "rowgroup" | "whole"
    v_group_rows: int = 1
    lr_scale: float = 1.0
    weight_decay: float = 0.0
    head_rows: int = 0              # rows per attention head (0: not an attention block)
    is_norm: bool = False

    @property
    def numel(self) -> int:
        return self.rows * self.cols


@dataclass(frozen=True)
class Workload:
    name: str
    blocks: tuple
    steps: int
    seed: int = 0
    spectrum_p: float = 1.5         # s_i = i^-p
    signal_rank: int = 256          # k (capped by min(rows, cols))
    noise_std: float = 1e-4
    ar_rho: float = 0.9
    row_scale: str = "none"         # "none" | "row_loguniform" | "head_loguniform"
    lr: float = 1e-3
    # optimizer hyper-parameters used by the paper's pre-training runs
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    clip: float = 1.0
    K: int = 5

    @property
    def numel(self) -> int:
        return sum(b.numel for b in self.blocks)


def _mat(name, rows, cols, pd, gd, rank, wd=0.1, head_rows=0, v_mode="element", v_group_rows=1):
    return BlockSpec(name, rows, cols, pd, gd, "lowrank", rank, v_mode, v_group_rows, 1.0, wd, head_rows)


def _full(name, rows, cols, pd, gd, wd=0.1, v_mode="element", v_group_rows=1, is_norm=False):
    return BlockSpec(name, rows, cols, pd, gd, "full", 0, v_mode, v_group_rows, 1.0, wd, 0, is_norm)


def tiny_block() -> Workload:
    """Config 1: one transformer block, d=256, 4 heads, SwiGLU FFN 1024, fp32, r=8, 10 steps."""
    d, f, r, hd = 256, 1024, 8, 64
    b = [_mat(f"attn.{n}", d, d, "f32", "f32", r, head_rows=hd) for n in ("q", "k", "v", "o")]
    b += [_mat("ffn.up", f, d, "f32", "f32", r), _mat("ffn.gate", f, d, "f32", "f32", r),
          _mat("ffn.down", d, f, "f32", "f32", r)]
    b += [_full(f"norm{i}", d, 1, "f32", "f32", wd=0.0, is_norm=True) for i in (1, 2)]
    return Workload("tiny_block", tuple(b), steps=10, seed=0, spectrum_p=1.5, signal_rank=32)


def llama_60m() -> Workload:
    """Config 2: 8 layers, d=512, SwiGLU 1376, vocab 32000 tied; fp32 params, bf16 grads, r=32."""
    d, f, r, hd, L = 512, 1376, 32, 64, 8
    b = [_full("embed", 32000, d, "f32", "bf16")]
    for l in range(L):
        b += [_mat(f"l{l}.attn.{n}", d, d, "f32", "bf16", r, head_rows=hd) for n in ("q", "k", "v", "o")]
        b += [_mat(f"l{l}.ffn.gate", f, d, "f32", "bf16", r), _mat(f"l{l}.ffn.up", f, d, "f32", "bf16", r),
              _mat(f"l{l}.ffn.down", d, f, "f32", "bf16", r)]
        b += [_full(f"l{l}.norm{i}", d, 1, "f32", "bf16", wd=0.0, is_norm=True) for i in (1, 2)]
    b.append(_full("norm_f", d, 1, "f32", "bf16", wd=0.0, is_norm=True))
    return Workload("llama_60m", tuple(b), steps=100, seed=0, spectrum_p=1.5, row_scale="row_loguniform")


def gpt2_350m() -> Workload:
    """Config 3: 24 layers, d=1024, FFN 4096, vocab 50304, positions 1024; bf16 params, r=64."""
    d, f, r, hd, L = 1024, 4096, 64, 64, 24
    b = [_full("wte", 50304, d, "bf16", "bf16"), _full("wpe", 1024, d, "bf16", "bf16")]
    for l in range(L):
        b += [_mat(f"h{l}.attn.{n}", d, d, "bf16", "bf16", r, head_rows=hd) for n in ("q", "k", "v", "o")]
        b += [_mat(f"h{l}.mlp.fc", f, d, "bf16", "bf16", r), _mat(f"h{l}.mlp.proj", d, f, "bf16", "bf16", r)]
        b += [_full(f"h{l}.ln{i}", d, 1, "bf16", "bf16", wd=0.0, is_norm=True) for i in (1, 2)]
    b.append(_full("ln_f", d, 1, "bf16", "bf16", wd=0.0, is_norm=True))
    return Workload("gpt2_350m", tuple(b), steps=100, seed=0, spectrum_p=1.2)


def llama_1b() -> Workload:
    """Config 4: 24 layers, d=2048, SwiGLU 5461, vocab 32000 untied; bf16 params, r=128,
    full momentum on embedding and output head, per-head gradient scale spread."""
    d, f, r, hd, L = 2048, 5461, 128, 128, 24
    b = [_full("embed", 32000, d, "bf16", "bf16")]
    for l in range(L):
        b += [_mat(f"l{l}.attn.{n}", d, d, "bf16", "bf16", r, head_rows=hd) for n in ("q", "k", "v", "o")]
        b += [_mat(f"l{l}.ffn.gate", f, d, "bf16", "bf16", r), _mat(f"l{l}.ffn.up", f, d, "bf16", "bf16", r),
              _mat(f"l{l}.ffn.down", d, f, "bf16", "bf16", r)]
        b += [_full(f"l{l}.norm{i}", d, 1, "bf16", "bf16", wd=0.0, is_norm=True) for i in (1, 2)]
    b += [_full("norm_f", d, 1, "bf16", "bf16", wd=0.0, is_norm=True), _full("lm_head", 32000, d, "bf16", "bf16")]
    return Workload("llama_1b", tuple(b), steps=50, seed=0, spectrum_p=1.5, row_scale="head_loguniform")


def gpt2_1p5b() -> Workload:
    """Config 5: 48 layers, d=1600, 25 heads, FFN 6400, vocab 50257, positions 1024; bf16
    params, fp32 state, blockwise v (per head for Q,K; per output row elsewhere; one
    value per norm vector); r=128 on the layer matrices, full momentum elsewhere."""
    d, f, r, hd, L = 1600, 6400, 128, 64, 48
    b = [_full("wte", 50257, d, "bf16", "bf16", v_mode="rowgroup"),
         _full("wpe", 1024, d, "bf16", "bf16", v_mode="rowgroup")]
    for l in range(L):
        b += [_mat(f"h{l}.attn.{n}", d, d, "bf16", "bf16", r, head_rows=hd, v_mode="rowgroup", v_group_rows=hd)
              for n in ("q", "k")]
        b += [_mat(f"h{l}.attn.{n}", d, d, "bf16", "bf16", r, head_rows=hd, v_mode="rowgroup") for n in ("v", "o")]
        b += [_mat(f"h{l}.mlp.fc", f, d, "bf16", "bf16", r, v_mode="rowgroup"),
              _mat(f"h{l}.mlp.proj", d, f, "bf16", "bf16", r, v_mode="rowgroup")]
        b += [_full(f"h{l}.ln{i}", d, 1, "bf16", "bf16", wd=0.0, v_mode="whole", is_norm=True) for i in (1, 2)]
    b += [_full("ln_f", d, 1, "bf16", "bf16", wd=0.0, v_mode="whole", is_norm=True),
          _full("lm_head", 50257, d, "bf16", "bf16", v_mode="rowgroup")]
    return Workload("gpt2_1p5b", tuple(b), steps=20, seed=0, spectrum_p=1.5)


def paper_partition(shape: str = "gpt2_1p5b", mini: bool = False) -> Workload:
    """The paper's own assignment of momentum regimes (Sec. 4.1) on the two shapes of its memory table
    (Table 2): embeddings and the attention output projection carry no momentum and run at 0.75 x lr
    (Sec. 5.1, set-ups); query, key and MLP matrices carry low-rank momentum with r = 5 % of the smaller
    dimension; value matrices (and the norm vectors, which the paper does not mention) keep full momentum.
    mini = False: per-element second moment ("AdaPM"); mini = True: blockwise second moment in the
    Adam-mini partition ("AdaPM-mini": per head for Q, K, per output row elsewhere, one value per norm).
    bf16 parameters and gradients, weight decay 0.1 on matrices, tied input / output embedding."""
    if shape == "gpt2_1p5b":
        L, d, f, hd, vocab, pos, gated = 48, 1600, 6400, 64, 50257, 1024, False
    elif shape == "llama_350m":
        L, d, f, hd, vocab, pos, gated = 24, 1024, 2736, 64, 32000, 0, True
    else:
        raise ValueError(shape)
    pd = gd = "bf16"
    rg = dict(v_mode="rowgroup") if mini else {}

    def rank(rows, cols):
        return max(1, round(0.05 * min(rows, cols)))

    def none(name, rows, cols, **kw):
        return BlockSpec(name, rows, cols, pd, gd, "none", 0, kw.get("v_mode", "element"), kw.get("v_group_rows", 1),
                         0.75, 0.1, kw.get("head_rows", 0))

    b = [none("wte", vocab, d, **rg)]
    if pos:
        b.append(none("wpe", pos, d, **rg))
    for l in range(L):
        for n in ("q", "k"):
            kw = dict(v_mode="rowgroup", v_group_rows=hd) if mini else {}
            b.append(_mat(f"h{l}.attn.{n}", d, d, pd, gd, rank(d, d), head_rows=hd, **kw))
        b.append(_full(f"h{l}.attn.v", d, d, pd, gd, **rg))
        b.append(none(f"h{l}.attn.o", d, d, head_rows=hd, **rg))
        mlp = (("gate", f, d), ("up", f, d), ("down", d, f)) if gated else (("fc", f, d), ("proj", d, f))
        for n, rows, cols in mlp:
            b.append(_mat(f"h{l}.mlp.{n}", rows, cols, pd, gd, rank(rows, cols), **rg))
        for i in (1, 2):
            b.append(_full(f"h{l}.ln{i}", d, 1, pd, gd, wd=0.0, v_mode="whole" if mini else "element", is_norm=True))
    b.append(_full("ln_f", d, 1, pd, gd, wd=0.0, v_mode="whole" if mini else "element", is_norm=True))
    return Workload(f"{shape}_paper{'_mini' if mini else ''}", tuple(b), steps=20, seed=0, spectrum_p=1.5)


CONFIGS = {
    "gpt2_1p5b_paper": lambda: paper_partition("gpt2_1p5b", False),
    "gpt2_1p5b_paper_mini": lambda: paper_partition("gpt2_1p5b", True),
    "llama_350m_paper": lambda: paper_partition("llama_350m", False),
    "llama_350m_paper_mini": lambda: paper_partition("llama_350m", True),
    "tiny_block": tiny_block,
    "llama_60m": llama_60m,
    "gpt2_350m": gpt2_350m,
    "llama_1b": llama_1b,
    "gpt2_1p5b": gpt2_1p5b,
}


def subset(wl: Workload, names_or_idx) -> Workload:
    """A workload restricted to some blocks (blocks are independent in the method)."""
    pick = []
    for x in names_or_idx:
        pick.append(wl.blocks[x] if isinstance(x, int) else next(b for b in wl.blocks if b.name == x))
    return replace(wl, blocks=tuple(pick))


_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def _gen(device, *keys) -> torch.Generator:
    g = torch.Generator(device=device)
    s = 0x9E3779B97F4A7C15
    for k in keys:
        s = (s * 6364136223846793005 + (int(k) & 0xFFFFFFFFFFFF) + 1442695040888963407) % (1 << 63)
    g.manual_seed(s)
    return g


def initial_params(wl: Workload, device="cpu") -> List[torch.Tensor]:
    """W_0 ~ N(0, 0.02^2) for matrices and embeddings, ones for norm vectors."""
    out = []
    for i, b in enumerate(wl.blocks):
        if b.is_norm:
            w = torch.ones(b.rows, b.cols, device=device)
        else:
            w = torch.randn(b.rows, b.cols, device=device, generator=_gen(device, wl.seed, i, 1)) * 0.02
        out.append(w.to(_TORCH_DT[b.param_dtype]).contiguous())
    return out


class GradientStream:
    """Per-block seeded gradient generator; `next()` returns the list of G_t tensors
    (in each block's gradient dtype) and advances the AR(1) state."""

    def __init__(self, wl: Workload, device="cpu", scale: float = 1.0):
        self.wl, self.device, self.scale = wl, device, scale
        self.t = 0
        self.U, self.V, self.s, self.a, self.D, self.gens = [], [], [], [], [], []
        for i, b in enumerate(wl.blocks):
            g = _gen(device, wl.seed, i, 2)
            self.gens.append(g)
            if b.cols == 1:
                self.U.append(None); self.V.append(None); self.s.append(None); self.D.append(None)
                self.a.append(torch.randn(b.rows, 1, device=device, generator=g))
                continue
            k = min(wl.signal_rank, b.rows, b.cols)
            # orthonormal bases from a CPU-seeded QR: the same U, V whatever the device
            gc = _gen("cpu", wl.seed, i, 3)
            U, _ = torch.linalg.qr(torch.randn(b.rows, k, generator=gc))
            V, _ = torch.linalg.qr(torch.randn(b.cols, k, generator=gc))
            self.U.append(U.to(device)); self.V.append(V.t().contiguous().to(device))
            self.s.append(torch.arange(1, k + 1, device=device, dtype=torch.float32) ** (-wl.spectrum_p))
            self.a.append(torch.ones(k, device=device))
            D = None
            if wl.row_scale == "row_loguniform":
                e = torch.rand(b.rows, 1, device=device, generator=g)
                D = 10.0 ** (-4.0 + 2.0 * e)                      # log-uniform in [1e-4, 1e-2]
            elif wl.row_scale == "head_loguniform" and b.head_rows:
                e = torch.rand(b.rows // b.head_rows, 1, device=device, generator=g)
                D = (10.0 ** (-2.0 + 2.0 * e)).repeat_interleave(b.head_rows, dim=0)   # two decades
            self.D.append(D)

    def next(self) -> List[torch.Tensor]:
        wl, rho = self.wl, self.wl.ar_rho
        out = []
        for i, b in enumerate(wl.blocks):
            g = self.gens[i]
            if self.t > 0:
                xi = torch.randn(self.a[i].shape, device=self.device, generator=g)
                self.a[i] = rho * self.a[i] + math.sqrt(1.0 - rho * rho) * xi
            if b.cols == 1:
                G = 1e-2 * self.a[i]
            else:
                G = (self.U[i] * (self.s[i] * self.a[i])) @ self.V[i]
                G = G + wl.noise_std * torch.randn(b.rows, b.cols, device=self.device, generator=g)
                if self.D[i] is not None:
                    G = G * self.D[i]
            out.append((self.scale * G).to(_TORCH_DT[b.grad_dtype]).contiguous())
        self.t += 1
        return out
