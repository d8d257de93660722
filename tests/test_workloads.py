"""The synthetic workloads: block tables of the five shapes and the gradient model."""
import numpy as np
import pytest
import torch

from paper_2510_09103_amd import workloads as WL


@pytest.mark.parametrize("name,nblocks,numel,lr_numel", [
    ("tiny_block", 9, 1_049_088, 1_048_576),
    ("llama_60m", 74, 41_689_600, 25_296_896),
    ("gpt2_350m", 195, 354_599_936, 301_989_888),
    ("llama_1b", 219, 1_339_082_752, 1_207_910_400),
    ("gpt2_1p5b", 388, 1_637_176_000, 1_474_560_000),
])
def test_block_tables(name, nblocks, numel, lr_numel):
    wl = WL.CONFIGS[name]()
    assert len(wl.blocks) == nblocks and wl.numel == numel
    assert sum(b.numel for b in wl.blocks if b.mom == "lowrank") == lr_numel
    for b in wl.blocks:
        if b.mom == "lowrank":
            assert 1 <= b.rank <= min(b.rows, b.cols)
        if b.v_mode == "rowgroup":
            assert b.rows % b.v_group_rows == 0


def test_gpt2_1p5b_blockwise_v_count():
    wl = WL.gpt2_1p5b()
    nv = sum(b.rows // b.v_group_rows if b.v_mode == "rowgroup" else 1 for b in wl.blocks)
    assert nv == 641_635


def test_gradient_stream_structure_and_determinism():
    wl = WL.subset(WL.tiny_block(), ["attn.q", "ffn.up", "norm1"])
    s1, s2 = WL.GradientStream(wl), WL.GradientStream(wl)
    g1 = [s1.next() for _ in range(6)]
    g2 = [s2.next() for _ in range(6)]
    for a, b in zip(g1, g2):
        for x, y in zip(a, b):
            assert torch.equal(x, y)
    G0 = g1[0][0].double().numpy()
    s = np.linalg.svd(G0, compute_uv=False)
    assert abs(s[0] - 1.0) < 0.05                       # s_1 a_1 = 1
    assert abs(s[7] / 8 ** -1.5 - 1) < 0.1              # power-law head, s_i = i^-1.5
    assert s[40] < 5e-3 and s[40] > 1e-4                # noise tail (sigma 1e-4, sqrt(m)+sqrt(n) scaling)
    # dominant subspace moves slowly: AR(1) with rho = 0.9 keeps consecutive steps correlated
    c = np.sum(g1[0][0].numpy() * g1[1][0].numpy()) / np.linalg.norm(g1[0][0]) / np.linalg.norm(g1[1][0])
    assert c > 0.5
    assert g1[0][2].shape == (256, 1) and abs(g1[0][2].std().item() / 1e-2 - 1) < 0.3


def test_row_scales():
    wl = WL.subset(WL.llama_60m(), ["l0.attn.q"])
    G = WL.GradientStream(wl).next()[0].float()
    assert G.dtype == torch.float32 and WL.GradientStream(wl).next()[0].dtype == torch.bfloat16
    rn = G.norm(dim=1)
    assert rn.max() / rn.min() > 5                       # log-uniform row scales spread the row norms
    assert G.abs().max() < 1e-2
