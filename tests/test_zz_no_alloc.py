"""adapm_step_static (the entry point that allocates nothing: the library's own scratch array in place of a
caller-allocated workspace) against adapm_step on the same seeded inputs, through the C ABI.  Both run the same
kernels in the same order, so parameters and state must agree bit for bit.  Two contexts share the array: a larger
table first, then a smaller one, then the larger one again (whose copies of R kept in scratch between steps the
smaller table's call has overwritten in the meantime)."""
import pytest
import torch

from paper_2510_09103_amd import binding as B
from paper_2510_09103_amd import workloads as WL
from paper_2510_09103_amd.optimizer import AdaPM, make_hparams

pytestmark = pytest.mark.gpu


class Run:
    """One table stepped twice on the same gradients: by adapm_step with its own workspace (reference) and by
    adapm_step_static."""

    def __init__(self, wl, T):
        self.wl = wl
        hp = make_hparams(beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, clip=wl.clip, K=wl.K, T=T)
        self.ref = AdaPM(wl.blocks, hp)
        self.sta = AdaPM(wl.blocks, hp)
        assert self.sta.workspace_bytes <= B.adapm_static_scratch_bytes()
        self.sta.workspace = None                      # the static path gets no workspace from the caller
        self.p_ref = WL.initial_params(wl, device="cuda:0")
        self.p_sta = WL.initial_params(wl, device="cuda:0")
        self.stream = WL.GradientStream(wl, device="cuda:0")
        self.t = 0

    def step(self):
        self.t += 1
        grads = self.stream.next()
        s = torch.cuda.current_stream().cuda_stream
        self.ref.step(self.p_ref, grads, self.t, self.wl.lr)
        pp = B.ptr_array([p.data_ptr() for p in self.p_sta])
        gp = B.ptr_array([g.data_ptr() for g in grads])
        B.adapm_step_static(self.sta.ctx, pp, gp, self.sta.state.data_ptr(), self.t, self.wl.lr, s)
        torch.cuda.synchronize()

    def check(self):
        for i, (a, b) in enumerate(zip(self.p_ref, self.p_sta)):
            assert torch.equal(a, b), f"{self.wl.name} step {self.t}: parameters of block {i} ({self.wl.blocks[i].name}) differ"
        assert torch.equal(self.ref.state, self.sta.state), f"{self.wl.name} step {self.t}: state differs"
        assert bool(torch.isfinite(self.sta.state.view(torch.float32)).all())


def test_static_scratch_entry_point_matches_adapm_step():
    # larger input: one full-size bf16 layer slice on the MFMA path plus full-momentum blocks, R held between refreshes
    big = Run(WL.subset(WL.gpt2_350m(), ["wpe", "h0.attn.q", "h0.mlp.fc", "h0.ln1"]), T=3)
    # smaller input: the fp32 tiny block (exact contraction path), Alg. 2 every step
    small = Run(WL.subset(WL.tiny_block(), ["attn.q", "ffn.down", "norm1"]), T=1)
    big.step(); big.check()            # first call
    small.step(); small.check()        # second call in a row, smaller input, same scratch array
    big.step(); big.check()            # holds R: its copies in scratch were overwritten by the small table's call
    small.step(); small.check()
    big.step(); big.check()
    big.step(); big.check()            # t = 4 runs Alg. 2 again


def test_static_scratch_entry_point_rejects_what_it_cannot_serve():
    wl = WL.gpt2_350m()                # the whole table needs far more scratch than the array holds
    hp = make_hparams(beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, clip=wl.clip, K=wl.K, T=1)
    ctx = B.adapm_init([__import__("paper_2510_09103_amd.optimizer", fromlist=["to_c_block"]).to_c_block(b) for b in wl.blocks], hp)
    assert B.adapm_workspace_bytes(ctx) > B.adapm_static_scratch_bytes()
    n = len(wl.blocks)
    with pytest.raises(B.AdapmError) as e:
        B.adapm_step_static(ctx, B.ptr_array([256] * n), B.ptr_array([256] * n), 4096, 1, 1e-3)
    assert e.value.status == B.ADAPM_EINVAL and "scratch" in str(e.value)
    B.adapm_destroy(ctx)
    # a context that was never set up on the device: the call would have to allocate
    wl = WL.subset(WL.tiny_block(), ["norm1"])
    opt = AdaPM(wl.blocks, make_hparams(), allocate=False)
    with pytest.raises(B.AdapmError) as e:
        B.adapm_step_static(opt.ctx, B.ptr_array([256]), B.ptr_array([512]), 4096, 1, 1e-3)
    assert e.value.status == B.ADAPM_ESTATE
    opt.close()
