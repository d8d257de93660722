"""GPU parity: the HIP library against the CPU oracle, element by element, on the same
seeded inputs.  Tolerances (relative, per element, with a block-RMS floor):
  TOL32   1e-5  fp32 parameters and their state on the exact (fp64) contraction path;
  TOLX    2e-4  fp32 parameters and any state on the split-bf16 MFMA path, runs of up to 20 steps (worst seen 1.1e-4);
  TOLX_LONG 4e-3  the same over 50 - 100 steps.  Alg. 2 is a warm-started iteration whose state is carried from step
                to step, and it amplifies perturbations: rounding the ORACLE's own state to fp32 once per step
                (6e-8) already moves its product L R by 4e-5 after 100 steps.  The MFMA path perturbs every step
                by ~1e-6 (fp32 accumulation, operands split to 2^-17), so its distance from the oracle grows with
                the step count: product L R of config 3 1e-4 after 20 steps, 2e-4 after 30, 2.2e-3 after 100
                (bound: twice that); the exact (fp64) contraction path stays at 5e-6 (config 2, and config 3's
                strata re-run on it below);
  bf16 parameters: 2e-3 or a bounded number of representable values, with asserted flip fractions
                (parity_util.compare_params)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import adapm_oracle as O
from paper_2510_09103_amd import binding as B
from paper_2510_09103_amd import workloads as WL
from paper_2510_09103_amd.workloads import BlockSpec
from parity_util import Pair, to_np

pytestmark = pytest.mark.gpu

TOL32 = 1e-5
TOLX = 2e-4
TOLX_LONG = 4e-3
TOL16 = TOLX      # state and fp32 parameters of runs on the MFMA path


def run(wl, steps, hp=None, tol_state=TOL32, tol_param=TOL32, check_every=None, **kw):
    pair = Pair(wl, hp, **kw)
    pair.flip_per_step = max(pair.flip_per_step, 10.0 * tol_state)
    rep = None
    for t in range(1, steps + 1):
        pair.step()
        if check_every and t % check_every == 0:
            rep = pair.compare(tol_state, tol_param)
    rep = pair.compare(tol_state, tol_param)
    print(f"{wl.name} hp={hp} steps={steps}: {rep}", flush=True)
    return pair, rep


def test_seeded_start_is_bit_identical():
    wl = WL.subset(WL.llama_60m(), ["l0.attn.q", "l0.ffn.down"])
    pair = Pair(wl, dict(seed=12345))
    for i in range(2):
        sv = pair.opt.state_view(i)
        assert np.array_equal(sv["R"].cpu().numpy(), pair.state_o[i]["R"])
        assert float(sv["L"].abs().max()) == 0.0 and float(sv["v"].abs().max()) == 0.0
    pair0 = Pair(wl, dict(seed=0))
    assert float(pair0.opt.state_view(0)["R"].abs().max()) == 0.0


@pytest.mark.parametrize("T", [1, 4])
def test_config1_tiny_block(T):
    run(WL.tiny_block(), 10, dict(T=T), check_every=1)


def mixed_table(pd="f32", gd="f32"):
    mk = BlockSpec
    return WL.Workload("mixed", (
        mk("none_mat", 100, 37, pd, gd, "none", 0, "element", 1, 0.75, 0.1),
        mk("full_rg3", 129, 67, "bf16", "bf16", "full", 0, "rowgroup", 3, 1.0, 0.1),
        mk("vec_whole", 1000, 1, pd, "bf16", "full", 0, "whole", 1, 1.0, 0.0),
        mk("lr_ragged", 200, 131, pd, gd, "lowrank", 5, "rowgroup", 1, 1.0, 0.1),
        mk("lr_heads", 96, 160, "bf16", "bf16", "lowrank", 16, "rowgroup", 32, 1.0, 0.1, 32),
        mk("full_whole_big", 300, 200, pd, gd, "full", 0, "whole", 1, 1.0, 0.05),
        mk("lr_fullrank_wide", 64, 1000, pd, "bf16", "lowrank", 64, "element", 1, 1.0, 0.1),
        mk("one", 1, 1, pd, gd, "full", 0, "element", 1, 1.0, 0.0),
        mk("none_vec", 77, 1, pd, gd, "none", 0, "rowgroup", 7, 0.75, 0.0),
        mk("lr_rank1", 70, 66, pd, gd, "lowrank", 1, "whole", 1, 1.0, 0.1),
    ), steps=6, seed=3, signal_rank=24)


@pytest.mark.parametrize("hp", [
    dict(T=1), dict(T=3), dict(T=1, adam_debias=1, clip=float("inf")), dict(T=2, bias_correction=0),
    dict(T=1, bias_correction=0, K=3), dict(T=1, K=1), dict(T=2, K=1), dict(T=1, beta1=0.0),
])
def test_mixed_table_all_modes(hp):
    wl = mixed_table()
    # every mode on the exact (fp64 contraction) path at the fp32 tolerance; the MFMA path has its own
    # tables below.  bf16-parameter blocks are held to the bf16 criterion inside compare_params
    hp = dict(hp, contraction=B.ADAPM_CONTRACT_F64)
    run(wl, 6, hp, tol_state=TOL32, tol_param=TOL32, check_every=2)


def ragged_bf16_table():
    """bf16 blocks on the MFMA path whose sizes are not multiples of the 64-row stripes, the
    64-column chunks, the 128 x 128 GEMM tiles or the 8-element vectors; every rank class; every kind of v."""
    mk = BlockSpec
    return WL.Workload("ragged_bf16", (
        mk("r32_cols1000", 200, 1000, "bf16", "bf16", "lowrank", 32, "rowgroup", 1, 1.0, 0.1),
        mk("r64_small", 96, 136, "bf16", "bf16", "lowrank", 64, "element", 1, 1.0, 0.1),
        mk("r128_rows130", 130, 264, "bf16", "bf16", "lowrank", 128, "rowgroup", 65, 1.0, 0.1),
        mk("r32_f32params", 70, 72, "f32", "bf16", "lowrank", 32, "whole", 1, 1.0, 0.0),
        mk("r64_heads16", 192, 320, "bf16", "bf16", "lowrank", 64, "rowgroup", 16, 1.0, 0.1, 16),
        # columns that are not a multiple of 8: rows of G, W and v start at any 2-byte (4-byte) alignment and the
        # last cols mod 8 columns of every row are done element by element
        mk("r32_cols1001", 200, 1001, "bf16", "bf16", "lowrank", 32, "rowgroup", 1, 1.0, 0.1),
        mk("r64_cols77_elem", 96, 77, "bf16", "bf16", "lowrank", 64, "element", 1, 1.0, 0.1),
        mk("r128_cols333_f32params", 136, 333, "f32", "bf16", "lowrank", 128, "element", 1, 1.0, 0.0),
        mk("r32_cols70_whole", 130, 70, "bf16", "bf16", "lowrank", 20, "whole", 1, 1.0, 0.1),
    ), steps=6, seed=5, signal_rank=40)


@pytest.mark.parametrize("hp", [
    dict(T=1), dict(T=3), dict(T=2, bias_correction=0), dict(T=1, adam_debias=1, clip=float("inf")),
    dict(T=2, K=1), dict(T=1, beta1=0.0),
])
def test_ragged_shapes_on_the_mfma_path(hp):
    hp = dict(hp, contraction=B.ADAPM_CONTRACT_BF16X2)
    run(ragged_bf16_table(), 6, hp, tol_state=TOL16, tol_param=TOL16, check_every=2)


@pytest.mark.parametrize("hp", [dict(T=1), dict(T=3)])
def test_both_contraction_paths_in_one_table(hp):
    """Automatic choice of the contraction: the fp32-parameter blocks of the table take the exact path, the bf16 ones
    the MFMA path.  With T > 1 the exact path's step with R held needs scratch in every step while the MFMA path's
    bf16 copies of R have to survive beside it (the layout that may not put the one over the other)."""
    run(ragged_bf16_table(), 6, dict(hp), tol_state=TOL16, tol_param=TOL16, check_every=2)


def odd_rank_table():
    """bf16 blocks whose rank is not 32, 64 or 128 (the paper takes r = 5 % of the smaller dimension): the
    MFMA kernels run them in the next rank class with zero-padded images of the factors.  Ranks that are
    and are not multiples of 4 (vector / scalar access to the rows of L), rows that are and are not
    multiples of 8 (stripe products / batched GEMM in Alg. 2)."""
    mk = BlockSpec
    return WL.Workload("odd_ranks", (
        mk("r8", 136, 200, "bf16", "bf16", "lowrank", 8, "rowgroup", 1, 1.0, 0.1),
        mk("r20_rows130", 130, 264, "bf16", "bf16", "lowrank", 20, "element", 1, 1.0, 0.1),
        mk("r51", 264, 1024, "bf16", "bf16", "lowrank", 51, "rowgroup", 1, 1.0, 0.1),
        mk("r80_f32params", 160, 320, "f32", "bf16", "lowrank", 80, "whole", 1, 1.0, 0.0),
        mk("r100", 256, 136, "bf16", "bf16", "lowrank", 100, "rowgroup", 64, 1.0, 0.1),
    ), steps=6, seed=9, signal_rank=40)


@pytest.mark.parametrize("hp", [dict(T=1), dict(T=3)])
def test_ranks_between_the_classes_on_the_mfma_path(hp):
    hp = dict(hp, contraction=B.ADAPM_CONTRACT_BF16X2)
    run(odd_rank_table(), 6, hp, tol_state=TOL16, tol_param=TOL16, check_every=2)


def random_table(rng, case):
    """A few low-rank bf16-gradient blocks with random sizes (mostly multiples of 8, which Alg. 2 takes as stripe
    products with the GD step riding on them; otherwise any size), ranks on and between the class and vector
    boundaries, every kind of second moment."""
    blocks = []
    for b in range(rng.randint(2, 4)):
        if rng.random() < 0.7:
            m, n = 8 * rng.randint(2, 90), 8 * rng.randint(2, 90)
        else:
            m, n = rng.randint(9, 500), rng.randint(9, 500)
        r = min(rng.choice([1, 3, 4, 7, 8, 16, 20, 31, 32, 33, 48, 51, 64, 65, 80, 100, 127, 128]), m, n)
        vm = rng.choice(["element", "rowgroup", "rowgroup", "whole"])
        g = rng.choice([d for d in (1, 2, 3, 4, 5, 8, 16, 32, 64, 128) if m % d == 0]) if vm == "rowgroup" else 1
        pd = rng.choice(["bf16", "bf16", "f32"])
        blocks.append(BlockSpec(f"c{case}b{b}_{m}x{n}_r{r}_{vm}{g}_{pd}", m, n, pd, "bf16", "lowrank", r, vm, g, 1.0,
                                rng.choice([0.0, 0.1])))
    return WL.Workload(f"random{case}", tuple(blocks), steps=5, seed=100 + case, signal_rank=24)


@pytest.mark.parametrize("seed", [2, 3])
def test_random_tables_on_the_mfma_path(seed):
    import random
    rng = random.Random(seed)
    for case in range(10):
        wl = random_table(rng, case)
        hp = dict(T=rng.choice([1, 1, 2, 3]), K=rng.choice([2, 3, 5, 5]), contraction=B.ADAPM_CONTRACT_BF16X2)
        if rng.random() < 0.25:
            hp["normalise"] = 1
        if rng.random() < 0.2:
            hp["bias_correction"] = 0
        clip = rng.choice([None, None, 0.5])
        print([b.name for b in wl.blocks], hp, clip, flush=True)
        run(wl, 5, hp, tol_state=TOL16, tol_param=TOL16, grad_clip=clip)


def test_random_tables_of_every_regime_on_the_exact_path():
    """Random sizes (vectors included), regimes, dtypes, second-moment kinds and flags at the fp32 tolerance."""
    import random
    rng = random.Random(1)
    for case in range(12):
        blocks = []
        for b in range(rng.randint(2, 5)):
            mom = rng.choice(["none", "full", "full", "lowrank", "lowrank"])
            m, n = (rng.randint(1, 3000), 1) if rng.random() < 0.2 else (rng.randint(1, 400), rng.randint(1, 400))
            if mom == "lowrank" and (m < 2 or n < 2):
                mom = "full"
            r = max(1, min(rng.choice([1, 2, 5, 8, 16, 33, 64]), m, n)) if mom == "lowrank" else 0
            vm = rng.choice(["element", "rowgroup", "rowgroup", "whole"])
            g = rng.choice([d for d in (1, 2, 3, 4, 5, 7, 8, 16, 25, 32, 64, 100, 128) if m % d == 0]) if vm == "rowgroup" else 1
            pd, gd = rng.choice(["bf16", "f32"]), rng.choice(["bf16", "f32"])
            blocks.append(BlockSpec(f"c{case}b{b}_{mom}_{m}x{n}_r{r}_{vm}{g}_{pd}{gd}", m, n, pd, gd, mom, r, vm, g,
                                    0.75 if mom == "none" else 1.0, rng.choice([0.0, 0.1])))
        hp = dict(T=rng.choice([1, 1, 2, 3]), K=rng.choice([1, 2, 3, 5, 5]), contraction=B.ADAPM_CONTRACT_F64)
        if rng.random() < 0.25:
            hp["normalise"] = 1
        if rng.random() < 0.2:
            hp["bias_correction"] = 0
        if rng.random() < 0.2:
            hp.update(adam_debias=1, clip=float("inf"))
        clip = rng.choice([None, None, 0.5])
        wl = WL.Workload(f"random_exact{case}", tuple(blocks), steps=5, seed=200 + case, signal_rank=24)
        print([b.name for b in wl.blocks], hp, clip, flush=True)
        run(wl, 5, hp, tol_state=TOL32, tol_param=TOL32, grad_clip=clip)


@pytest.mark.parametrize("shape,mini", [("gpt2_1p5b", False), ("gpt2_1p5b", True), ("llama_350m", False), ("llama_350m", True)])
def test_paper_partition_layer(shape, mini):
    """One layer (plus an embedding-like block) of the paper's own partition (Sec. 4.1): no momentum at
    0.75 x lr, full momentum, low-rank momentum with r = 5 % (80 resp. 51: between the rank classes)."""
    full = WL.paper_partition(shape, mini)
    names = [b.name for b in full.blocks if b.name.startswith("h0.")]
    if shape == "gpt2_1p5b":
        names = ["wpe"] + names
    run(WL.subset(full, names), 5, dict(T=3), tol_state=TOL16, tol_param=TOL16, check_every=2)


@pytest.mark.parametrize("hp", [dict(T=1), dict(T=3)])
def test_global_gradient_clipping_on_the_exact_path(hp):
    """Sec. 5.1 set-ups: global gradient-norm clipping folded into the step (every regime, every kind of v)."""
    hp = dict(hp, contraction=B.ADAPM_CONTRACT_F64)
    pair, _ = run(mixed_table(), 6, hp, tol_state=TOL32, tol_param=TOL32, check_every=2, grad_clip=1.0)
    assert pair.opt.last_grad_norm()[1] < 1.0              # the clipping was active


@pytest.mark.parametrize("hp", [dict(T=1), dict(T=3), dict(T=2, bias_correction=0)])
def test_global_gradient_clipping_on_the_mfma_path(hp):
    hp = dict(hp, contraction=B.ADAPM_CONTRACT_BF16X2)
    pair, _ = run(ragged_bf16_table(), 6, hp, tol_state=TOL16, tol_param=TOL16, check_every=2, grad_clip=0.5)
    assert pair.opt.last_grad_norm()[1] < 1.0
    run(odd_rank_table(), 4, hp, tol_state=TOL16, tol_param=TOL16, check_every=2, grad_clip=0.5)


def test_global_gradient_clipping_above_the_norm_changes_nothing():
    wl = ragged_bf16_table()
    a, _ = run(wl, 3, dict(T=2, contraction=B.ADAPM_CONTRACT_BF16X2), tol_state=TOL16, tol_param=TOL16, grad_clip=1e9)
    b, _ = run(wl, 3, dict(T=2, contraction=B.ADAPM_CONTRACT_BF16X2), tol_state=TOL16, tol_param=TOL16)
    assert a.opt.last_grad_norm()[1] == 1.0
    for x, y in zip(a.params, b.params):
        assert torch.equal(x, y)


@pytest.mark.parametrize("hp", [dict(T=1), dict(T=3)])
def test_scale_normalised_alg2_on_the_exact_path(hp):
    """The optional normalised step sizes of Alg. 2 (beyond the paper), every regime, also at a gradient scale where
    the printed iteration overflows."""
    hp = dict(hp, contraction=B.ADAPM_CONTRACT_F64, normalise=1)
    run(mixed_table(), 6, hp, tol_state=TOL32, tol_param=TOL32, check_every=2)
    run(mixed_table(), 4, hp, tol_state=TOL32, tol_param=TOL32, check_every=2, grad_scale=40.0)


@pytest.mark.parametrize("hp", [dict(T=1), dict(T=3), dict(T=2, bias_correction=0)])
def test_scale_normalised_alg2_on_the_mfma_path(hp):
    hp = dict(hp, contraction=B.ADAPM_CONTRACT_BF16X2, normalise=1)
    run(ragged_bf16_table(), 6, hp, tol_state=TOL16, tol_param=TOL16, check_every=2)
    run(odd_rank_table(), 4, hp, tol_state=TOL16, tol_param=TOL16, check_every=2, grad_scale=0.01)


def test_literal_zero_start_stays_zero_on_gpu():
    wl = WL.subset(WL.tiny_block(), ["attn.q"])
    pair, _ = run(wl, 3, dict(seed=0))
    sv = pair.opt.state_view(0)
    assert float(sv["L"].abs().max()) == 0.0 and float(sv["R"].abs().max()) == 0.0


# ---------------------------------------------------------------------------------------------------------------
# The five configurations at their own step counts.  Blocks are independent in the method, so where the oracle would
# need too long for a whole table it follows a stratified subset at full size: one block of every distinct
# (shape, momentum regime, kind of second moment).  Embedding-sized full-momentum blocks (tens of millions of
# elements, seconds per oracle step) are followed for a few steps only: their update is a linear recursion per
# element with no iteration whose error could grow.
# ---------------------------------------------------------------------------------------------------------------
def f32_params(wl):
    """The same workload with fp32 parameters (bf16 gradients kept): on the MFMA path this shows the arithmetic
    itself, without the bf16 rounding of W."""
    return dataclasses.replace(wl, blocks=tuple(dataclasses.replace(b, param_dtype="f32") for b in wl.blocks))


def test_config2_llama60m_whole_table():
    """All 74 blocks (embedding with full momentum, 56 low-rank matrices at r = 32, 17 norm vectors)."""
    run(WL.llama_60m(), 10, dict(T=1), check_every=5)


def test_config2_llama60m_layer_100_steps():
    full = WL.llama_60m()
    names = [b.name for b in full.blocks if b.name.startswith("l0.")] + ["norm_f"]
    run(WL.subset(full, names), 100, dict(T=1), check_every=10)


def test_config2_llama60m_layer_100_steps_R_held():
    full = WL.llama_60m()
    run(WL.subset(full, ["l0.attn.q", "l0.ffn.gate", "l0.ffn.down", "l0.norm1"]), 100, dict(T=10), check_every=10)


C3_STRATA = ["wpe", "h3.attn.q", "h3.mlp.fc", "h3.mlp.proj", "h3.ln1"]


def test_config3_gpt2_350m_strata_100_steps():
    run(WL.subset(WL.gpt2_350m(), C3_STRATA), 100, dict(T=1), tol_state=TOLX_LONG, tol_param=TOLX_LONG, check_every=10)


def test_config3_gpt2_350m_strata_100_steps_R_held():
    run(WL.subset(WL.gpt2_350m(), ["h3.attn.q", "h3.mlp.proj", "h3.ln1"]), 100, dict(T=100), tol_state=TOLX_LONG,
        tol_param=TOLX_LONG, check_every=10)


def test_config3_strata_100_steps_on_the_exact_path():
    """The same bf16-parameter strata with the fp64 contractions: state at the fp32 tolerance after 100 steps,
    parameters by the bf16 criterion."""
    run(WL.subset(WL.gpt2_350m(), ["h3.attn.q", "h3.mlp.proj", "h3.ln1"]), 100, dict(T=1, contraction=B.ADAPM_CONTRACT_F64),
        tol_state=TOL32, tol_param=TOL32, check_every=20)


def test_config3_gpt2_350m_embedding():
    run(WL.subset(WL.gpt2_350m(), ["wte"]), 3, dict(T=1), tol_state=TOLX, tol_param=TOLX)


def test_config3_strata_with_fp32_parameters_on_the_mfma_path():
    """The arithmetic of the MFMA path without the bf16 rounding of W: parameters, state and product L R of the
    warm-started iteration against the oracle after 100 steps."""
    wl = f32_params(WL.subset(WL.gpt2_350m(), ["h3.attn.q", "h3.mlp.proj"]))
    run(wl, 100, dict(T=1, contraction=B.ADAPM_CONTRACT_BF16X2), tol_state=TOLX_LONG, tol_param=TOLX_LONG, check_every=10)


def test_config4_llama1b_strata_50_steps():
    """2048 x 2048 and 2048 x 5461 (rows of G at 2-byte alignment), per-head gradient scales over two decades."""
    run(WL.subset(WL.llama_1b(), ["l5.attn.k", "l5.ffn.down", "l5.norm1"]), 50, dict(T=1), tol_state=TOLX_LONG,
        tol_param=TOLX_LONG, check_every=10)


def test_config4_llama1b_odd_row_count():
    """5461 x 2048: the last stripes of rows and of columns of G are ragged."""
    run(WL.subset(WL.llama_1b(), ["l5.ffn.gate"]), 10, dict(T=1), tol_state=TOLX_LONG, tol_param=TOLX_LONG)


def test_config4_llama1b_strata_R_held():
    run(WL.subset(WL.llama_1b(), ["l5.attn.k"]), 50, dict(T=100), tol_state=TOLX_LONG, tol_param=TOLX_LONG, check_every=10)
    run(WL.subset(WL.llama_1b(), ["l5.ffn.down", "l5.ffn.gate"]), 6, dict(T=100), tol_state=TOLX_LONG, tol_param=TOLX_LONG)


def test_config4_llama1b_output_head():
    run(WL.subset(WL.llama_1b(), ["lm_head"]), 2, dict(T=1), tol_state=TOLX, tol_param=TOLX)      # embed: same shape and regime


def test_config4_strata_with_fp32_parameters_on_the_mfma_path():
    wl = f32_params(WL.subset(WL.llama_1b(), ["l5.attn.k", "l5.ffn.down"]))
    run(wl, 10, dict(T=1, contraction=B.ADAPM_CONTRACT_BF16X2), tol_state=TOLX_LONG, tol_param=TOLX_LONG, check_every=5)


C5_STRATA = ["h7.attn.q", "h7.attn.v", "h7.mlp.fc", "h7.mlp.proj", "h7.ln1", "wpe"]


@pytest.mark.parametrize("T", [1, 100])
def test_config5_gpt2_1p5b_strata_20_steps(T):
    """Per-head v (Q), per-row v (V, MLP), one v per norm vector, per-row v with full momentum (positions)."""
    run(WL.subset(WL.gpt2_1p5b(), C5_STRATA), 20, dict(T=T), tol_state=TOLX, tol_param=TOLX, check_every=10)


def test_config5_gpt2_1p5b_output_head():
    run(WL.subset(WL.gpt2_1p5b(), ["lm_head"]), 2, dict(T=1), tol_state=TOLX, tol_param=TOLX)


def test_config5_strata_with_fp32_parameters_on_the_mfma_path():
    wl = f32_params(WL.subset(WL.gpt2_1p5b(), ["h7.attn.q", "h7.mlp.fc", "h7.mlp.proj"]))
    run(wl, 20, dict(T=1, contraction=B.ADAPM_CONTRACT_BF16X2), tol_state=TOLX, tol_param=TOLX, check_every=10)


@pytest.mark.parametrize("T", [1, 100])
def test_config5_full_size_sampled_blocks(T):
    """All 388 blocks in the launch configurations the benchmark times (T = 100: one step that runs Alg. 2, then R
    held; T = 1: Alg. 2 every step, the whole-model work lists of its stripe, Gram and update launches); the oracle
    follows a sample of blocks (blocks are independent), the rest is checked for sanity."""
    wl = WL.gpt2_1p5b()
    names = [b.name for b in wl.blocks]
    sample = [names.index(n) for n in ("h0.attn.q", "h23.attn.o", "h47.mlp.fc", "h11.mlp.proj", "h30.ln2", "ln_f",
                                       "wpe")]
    pair = Pair(wl, dict(T=T))
    w0 = pair.params[names.index("h40.attn.k")].clone()
    for t in range(1, 4):
        pair.step(oracle_only=sample)
    rep = pair.compare(TOLX, TOLX, only=sample)
    print(f"gpt2_1p5b full size, T={T}, sampled blocks:", rep, flush=True)
    torch.cuda.synchronize()
    for i, p in enumerate(pair.params):
        assert bool(torch.isfinite(p.float()).all()), names[i]
    assert bool(torch.isfinite(pair.opt.state.view(torch.float32)).all())
    # blocks the oracle did not follow did move
    assert not torch.equal(pair.params[names.index("h40.attn.k")], w0)


def test_held_R_kernel_that_reads_G_once(monkeypatch):
    """ADAPM_PROJ_KEEP=1: blocks of rank class 128 with bf16 parameters, a blockwise v and at most 1600 columns take
    the step with R held in 64-row stripes whose gradient stays in registers between the two passes.  Same parity bar
    as the two-read kernel; ragged rows, short last chunks, a rank between the classes, v groups inside and beyond
    the stripe."""
    monkeypatch.setenv("ADAPM_PROJ_KEEP", "1")
    mk = BlockSpec
    wl = WL.Workload("keep", (
        mk("heads64", 1600, 1600, "bf16", "bf16", "lowrank", 128, "rowgroup", 64, 1.0, 0.1, 64),
        mk("rows130_cols264_g65", 130, 264, "bf16", "bf16", "lowrank", 128, "rowgroup", 65, 1.0, 0.1),
        mk("r100_g16", 208, 136, "bf16", "bf16", "lowrank", 100, "rowgroup", 16, 1.0, 0.1),
        mk("r80_whole", 96, 1600, "bf16", "bf16", "lowrank", 80, "whole", 1, 1.0, 0.0),
        mk("wide_two_read", 136, 1608, "bf16", "bf16", "lowrank", 128, "rowgroup", 1, 1.0, 0.1),
    ), steps=6, seed=21, signal_rank=40)
    pair = Pair(wl, dict(T=3, contraction=B.ADAPM_CONTRACT_BF16X2))
    for t in range(1, 7):
        if t == 3:
            B.adapm_profile_enable(pair.opt.ctx, True)
        pair.step()
        if t == 3:
            torch.cuda.synchronize()
            labels = set(B.adapm_profile_read(pair.opt.ctx))
            B.adapm_profile_enable(pair.opt.ctx, False)
            assert {"fused_project_keep_r128", "fused_project_r128"} <= labels, labels
    rep = pair.compare(TOLX, TOLX)
    print("held-R kernel that keeps G on chip:", rep, flush=True)
    run(WL.subset(WL.gpt2_1p5b(), ["h7.attn.q", "h7.mlp.fc"]), 4, dict(T=100), tol_state=TOLX, tol_param=TOLX)


def test_rank_deficient_R_passes_the_orthonormalisation_unchanged():
    """T > 1 with factors that are exactly zero (a restored state whose R = 0): R R^T has no Cholesky factor, the
    library leaves such a block's (L, R) as Alg. 2 left them instead of writing NaN, and the steps then equal the
    literal zero start of Alg. 1 (factors stay 0, m^c = G), which the oracle computes with seed = 0, T = 1."""
    for names, wl0 in ((["attn.q"], WL.tiny_block()), (["h0.attn.q"], WL.gpt2_350m())):
        wl = WL.subset(wl0, names)
        pair = Pair(wl, dict(T=2))
        pair.opt.state_view(0)["R"].zero_()
        B.adapm_state_loaded(pair.opt.ctx)
        hp_o = O.HParams(beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, clip=wl.clip, K=wl.K, T=1, seed=0)
        st_o = O.init_state(pair.blocks_o, hp_o)
        W_o = pair.W_o
        for t in range(1, 4):
            grads = pair.stream.next()
            pair.opt.step(pair.params, grads, t, wl.lr)
            W_o, st_o = O.step(pair.blocks_o, hp_o, W_o, [to_np(g) for g in grads], st_o, t, wl.lr)
        torch.cuda.synchronize()
        sv = pair.opt.state_view(0)
        assert float(sv["L"].abs().max()) == 0.0 and float(sv["R"].abs().max()) == 0.0
        assert bool(torch.isfinite(pair.params[0].float()).all())
        pair.W_o, pair.state_o, pair.t = W_o, st_o, 3
        pair.compare(TOLX, TOL32 if wl.blocks[0].param_dtype == "f32" else TOLX)


def test_two_runs_are_bit_identical_and_resume_from_a_state_copy():
    wl = mixed_table()
    hp = dict(T=2)

    def go(nsteps, resume_at=None):
        pair = Pair(wl, hp)
        saved = None
        for t in range(1, nsteps + 1):
            if resume_at is not None and t == resume_at + 1:
                # checkpoint = the flat state buffer (+ step count): restore into a fresh optimizer
                from paper_2510_09103_amd.optimizer import AdaPM
                fresh = AdaPM(wl.blocks, pair.hp_c)
                fresh.state.copy_(saved)
                B.adapm_state_loaded(fresh.ctx)
                pair.opt = fresh
            grads = pair.stream.next()
            pair.t = t
            pair.opt.step(pair.params, grads, t, wl.lr)
            if resume_at is not None and t == resume_at:
                torch.cuda.synchronize()
                saved = pair.opt.state.clone()
        torch.cuda.synchronize()
        return [p.clone() for p in pair.params], pair.opt.state.clone()

    p1, s1 = go(6)
    p2, s2 = go(6)
    p3, s3 = go(6, resume_at=3)
    for a, b, c in zip(p1, p2, p3):
        assert torch.equal(a, b) and torch.equal(a, c)
    assert torch.equal(s1, s2) and torch.equal(s1, s3)


def test_restoring_a_state_into_a_live_optimizer():
    """bf16 blocks on the MFMA path keep derived copies of R between refreshes: after the caller
    overwrites the state buffer, adapm_state_loaded() must make the next step rebuild them."""
    wl = WL.subset(WL.gpt2_350m(), ["h0.attn.q", "h0.mlp.fc"])
    hp = dict(T=4)
    a = Pair(wl, hp)
    for _ in range(6):
        a.step()                                  # t = 5 refreshed; the copies of R belong to that refresh
    torch.cuda.synchronize()
    b = Pair(wl, hp)
    for _ in range(2):
        b.step()                                  # t = 1 refreshed
    torch.cuda.synchronize()
    saved_state, saved_params = b.opt.state.clone(), [p.clone() for p in b.params]
    # continue b to t = 3 for the expected result
    g3 = b.step()
    torch.cuda.synchronize()
    want = [p.clone() for p in b.params]
    # restore b's t = 2 checkpoint into optimizer a (same workspace as its last refresh) and redo t = 3
    a.opt.state.copy_(saved_state)
    B.adapm_state_loaded(a.opt.ctx)
    a.opt.step(saved_params, g3, 3, wl.lr)
    torch.cuda.synchronize()
    for x, y in zip(saved_params, want):
        assert torch.equal(x, y)


@pytest.mark.parametrize("hp", [dict(T=1), dict(T=3)])
def test_degenerate_inputs_zero_gradients_and_zero_step_size(hp):
    """Two degenerate inputs on both contraction paths.  (i) Gradients that are exactly zero from the first step
    on: v stays 0, every momentum stays 0, only the decoupled decay moves W.  (ii) lr = 0: the state advances,
    the parameters must not change by a single bit."""
    wl = WL.Workload("degenerate", ragged_bf16_table().blocks[:3] + WL.subset(WL.tiny_block(), ["attn.q", "norm1"]).blocks,
                     steps=4, seed=3, signal_rank=16)
    pair, _ = run(wl, 4, hp, tol_state=TOL16, tol_param=TOL16, grad_scale=0.0)
    for i in range(len(wl.blocks)):
        sv = pair.opt.state_view(i)
        assert float(sv["v"].abs().max()) == 0.0
        if "L" in sv:
            assert float(sv["L"].abs().max()) == 0.0
    frozen = Pair(wl, hp)
    before = [p.clone() for p in frozen.params]
    for _ in range(3):
        frozen.step(lr=0.0)
    torch.cuda.synchronize()
    for a, b in zip(before, frozen.params):
        assert torch.equal(a, b)
    frozen.compare(TOL16, TOL16)


@pytest.mark.parametrize("rows,cols", [(136, 1 << 21), (1 << 21, 136)])
def test_largest_blocks_of_the_mfma_path_agree_with_the_exact_path(rows, cols):
    """Maximum sizes: 2^21 columns is the widest block the MFMA kernels take (32-bit offsets inside a stripe),
    2^21 rows the tallest one whose transposed copy still runs as stripe products.  The oracle needs minutes at
    these sizes, so the property checked is that the two contraction paths of the library, which share no kernel
    for low-rank blocks, agree on the same inputs."""
    from paper_2510_09103_amd.optimizer import AdaPM, make_hparams
    wl = WL.Workload("largest", (BlockSpec("big", rows, cols, "bf16", "bf16", "lowrank", 32, "rowgroup", 1, 1.0, 0.1),),
                     steps=3, seed=11, signal_rank=8)
    stream = WL.GradientStream(wl, device="cuda:0")
    grads = [[g.clone() for g in stream.next()] for _ in range(3)]
    out = []
    for mode in (B.ADAPM_CONTRACT_BF16X2, B.ADAPM_CONTRACT_F64):
        hp = make_hparams(beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, clip=wl.clip, K=wl.K, T=2, contraction=mode)
        opt = AdaPM(wl.blocks, hp)
        assert B.adapm_block_contraction(opt.ctx, 0) == mode
        params = WL.initial_params(wl, device="cuda:0")
        for t in range(1, 4):
            opt.step(params, grads[t - 1], t, wl.lr)
        torch.cuda.synchronize()
        sv = opt.state_view(0)
        out.append((params[0].float().clone(), (sv["L"].double()[:4096] @ sv["R"].double()[:, :4096]).clone(), sv["v"].clone()))
        opt.close()
        del opt
    (w_a, lr_a, v_a), (w_b, lr_b, v_b) = out
    scale = float(w_b.abs().mean())
    assert float((w_a - w_b).abs().max()) <= 2 * 2.0 ** -8 * max(float(w_b.abs().max()), scale)     # two bf16 ulps
    assert float((w_a != w_b).float().mean()) < 5e-3
    rms = float(lr_b.pow(2).mean().sqrt())
    assert float((lr_a - lr_b).abs().max()) <= TOL16 * max(float(lr_b.abs().max()), rms)
    assert torch.allclose(v_a, v_b, rtol=1e-5, atol=0.0)


def test_one_context_serving_two_state_buffers():
    """The derived copies of R in the workspace belong to one state buffer: a context that steps two replicas
    (two state buffers, one workspace) in turn must rebuild them whenever the state buffer changes."""
    from paper_2510_09103_amd.optimizer import AdaPM, make_hparams
    wl = WL.subset(WL.gpt2_350m(), ["h0.attn.q", "h0.mlp.fc"])
    hp = make_hparams(beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, clip=wl.clip, K=wl.K, T=4)
    stream = WL.GradientStream(wl, device="cuda:0")
    grads = [[g.clone() for g in stream.next()] for _ in range(6)]
    seqs = [grads, grads[::-1]]                      # the two replicas see different gradients
    want = []
    for k in (0, 1):                                 # each replica with a context of its own
        opt = AdaPM(wl.blocks, hp)
        params = WL.initial_params(wl, device="cuda:0")
        for t in range(1, 7):
            opt.step(params, seqs[k][t - 1], t, wl.lr)
        torch.cuda.synchronize()
        want.append((params, opt.state.clone()))
    shared = AdaPM(wl.blocks, hp)
    states = [shared.state, shared.state.clone()]    # the seeded start is the same for both
    params = [WL.initial_params(wl, device="cuda:0"), WL.initial_params(wl, device="cuda:0")]
    for t in range(1, 7):
        for k in (0, 1):
            shared.state = states[k]
            shared.step(params[k], seqs[k][t - 1], t, wl.lr)
    torch.cuda.synchronize()
    for k in (0, 1):
        for x, y in zip(params[k], want[k][0]):
            assert torch.equal(x, y), f"replica {k}"
        assert torch.equal(states[k], want[k][1]), f"replica {k}"


def test_step_rejects_bad_arguments_on_device():
    wl = WL.subset(WL.tiny_block(), ["norm1"])
    pair = Pair(wl)
    g = pair.stream.next()
    with pytest.raises(B.AdapmError) as e:
        pair.opt.step(pair.params, g, 0, 1e-3)
    assert e.value.status == B.ADAPM_ESTATE
    w_before = pair.params[0].clone()
    pair.opt.step(pair.params, g, 1, 1e-3)
    torch.cuda.synchronize()
    assert not torch.equal(w_before, pair.params[0])
