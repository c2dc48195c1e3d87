"""Workload shapes: the five benchmark configurations, the capacity-table shares, scaled-down cousins.

B batch, S sequence length, D model width, H heads held locally, dh head
width, F feed-forward width held locally, L layers, V vocabulary.  H*dh may
differ from D: that is one tensor-parallel device's share of a wider block
(heads and feed-forward columns split over the model axis, Sec. 3.2).
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class BlockShape:
    B: int
    S: int
    D: int
    H: int
    dh: int
    F: int
    dtype: str = "bf16"          # "f32" or "bf16"
    gelu: str = "tanh"           # "tanh" or "erf"
    ln_eps: float = 1e-5
    sigma_w: float = 0.02
    L: int = 1

    @property
    def T(self):
        return self.B * self.S

    @property
    def Hd(self):
        return self.H * self.dh

    def scaled(self, **kw):
        return replace(self, **kw)

    def block_param_count(self):
        D, Hd, F = self.D, self.Hd, self.F
        return 2 * D + D * 3 * Hd + 3 * Hd + Hd * D + D + 2 * D + D * F + F + F * D + D

    def block_gemm_flops_fwd(self):
        return 2 * self.T * (3 * self.D * self.Hd + self.Hd * self.D + 2 * self.D * self.F)

    def block_attn_flops_fwd(self, causal_half=True):
        full = 4 * self.B * self.S * self.S * self.Hd
        return full // 2 if causal_half else full

    def block_flops_fwd_bwd(self, causal_half=True):
        return 3 * (self.block_gemm_flops_fwd() + self.block_attn_flops_fwd(causal_half))


@dataclass(frozen=True)
class ModelShape:
    blk: BlockShape
    V: int
    S_max: int

    @property
    def L(self):
        return self.blk.L

    def param_count(self):
        b = self.blk
        return self.V * b.D + self.S_max * b.D + 2 * b.D + b.L * b.block_param_count()

    def flops_fwd_bwd(self, causal_half=True):
        b = self.blk
        head = 2 * b.T * b.D * self.V
        return b.L * b.block_flops_fwd_bwd(causal_half) + 3 * head

    def scaled(self, V=None, S_max=None, **kw):
        return ModelShape(self.blk.scaled(**kw), V or self.V, S_max or self.S_max)


CONFIGS = {
    # tiny fp32 block: fwd + bwd + one AdamW step
    "cfg1": BlockShape(B=2, S=64, D=128, H=4, dh=32, F=512, dtype="f32", sigma_w=0.02, L=1),
    # 2-layer bf16 stack with fp32 master weights and AdamW state
    "cfg2": BlockShape(B=8, S=1024, D=1024, H=16, dh=64, F=4096, dtype="bf16", sigma_w=0.02, L=2),
    # one large bf16 block: the throughput target
    "cfg3": BlockShape(B=4, S=2048, D=4096, H=32, dh=128, F=16384, dtype="bf16",
                       sigma_w=0.02 / (2 * 32) ** 0.5, L=1),
    # one device's share of a D=12288, 96-head, F=49152 block split 8 ways
    "cfg4": BlockShape(B=8, S=2048, D=12288, H=12, dh=128, F=6144, dtype="bf16", sigma_w=0.006, L=1),
    # GPT-style train step with a tied vocabulary of 51200
    "cfg5": ModelShape(BlockShape(B=8, S=2048, D=2048, H=16, dh=128, F=8192, dtype="bf16",
                                  sigma_w=0.02, L=12), V=51200, S_max=2048),
    # One tensor-parallel rank's block at the operating point of the capacity table (Table 1):
    # batch 1, sequence 2048, hidden 5120 / 10240 / 16384, "maximal tensor parallelism".  The
    # paper does not say how many heads or which feed-forward width; taken here: 128-wide heads,
    # F = 4 D, split 8 ways (one 8-GPU node as the model axis), biases and weight scale as cfg4.
    "t1_5120": BlockShape(B=1, S=2048, D=5120, H=5, dh=128, F=2560, dtype="bf16", sigma_w=0.006, L=1),
    "t1_10240": BlockShape(B=1, S=2048, D=10240, H=10, dh=128, F=5120, dtype="bf16", sigma_w=0.006, L=1),
    "t1_16384": BlockShape(B=1, S=2048, D=16384, H=16, dh=128, F=8192, dtype="bf16", sigma_w=0.006, L=1),
    # The model of the per-phase timing figure (Fig. 4): "124M parameters", batch 32, sequence 2048.
    # The paper gives the size only; taken here: 12 layers, D = 768, 12 heads of 64, F = 3072 and a
    # vocabulary of 50304 (125.3M parameters, 85.1M of them in the blocks), everything else as cfg5.
    "fig4_124m": ModelShape(BlockShape(B=32, S=2048, D=768, H=12, dh=64, F=3072, dtype="bf16",
                                       sigma_w=0.02, L=12), V=50304, S_max=2048),
}

ADAMW_DEFAULT = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.01)


def get_config(name):
    return CONFIGS[name]
