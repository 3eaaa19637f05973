"""Workload shapes: the five benchmark configurations plus reduced shapes for tests.

Only shapes and scalar settings live here.  Field names follow the C header
(`include/fastardiff.h`), whose structs they fill one to one.
"""
from __future__ import annotations

import copy
from dataclasses import dataclass, field, asdict

ACT_GELU, ACT_SWIGLU = 0, 1
NORM_LAYER, NORM_RMS = 0, 1
POS_LEARNED, POS_ROPE = 0, 1
DT_F32, DT_BF16 = 0, 1
ENT_FEATURE, ENT_ATTN = 0, 1


@dataclass
class TfCfg:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_head: int
    d_ff: int
    act: int = ACT_GELU
    norm: int = NORM_LAYER
    pos: int = POS_LEARNED
    has_bias: int = 1
    norm_eps: float = 1e-5
    rope_theta: float = 1e4
    d_latent: int = 16
    n_cond_ids: int = 0
    d_out: int = 0          # feature width after the optional up-projection (0 -> d_model)
    max_pos: int = 0        # rows of the learned position table (pos == POS_LEARNED)

    def out_dim(self) -> int:
        return self.d_out if self.d_out else self.d_model


@dataclass
class HeadCfg:
    n_blocks: int
    width: int
    d_cond: int
    d_latent: int = 16
    n_steps: int = 1
    t_freq_dim: int = 256
    t_scale: float = 1000.0
    sigma_last: float = 0.25
    temperature: float = 1.0
    renoise: int = 1


@dataclass
class RoundCfg:
    target: TfCfg
    draft: TfCfg
    head: HeadCfg
    K: int
    max_batch: int
    max_ctx: int
    entropy_layer: int = 1      # 1-indexed draft layer whose output feeds the entropy
    entropy_mode: int = ENT_FEATURE
    prefix_rule: int = 1
    dtype: int = DT_BF16
    tau_ent: float = 0.0
    # workload description (not part of the C struct)
    name: str = ""
    batch: int = 1
    n_ctx: int = 64

    def to_dict(self):
        return asdict(self)


def _ln_gelu(L, d, H, F, max_pos, n_cond=0):
    return TfCfg(n_layers=L, d_model=d, n_heads=H, n_kv_heads=H, d_head=d // H, d_ff=F,
                 act=ACT_GELU, norm=NORM_LAYER, pos=POS_LEARNED, has_bias=1, norm_eps=1e-5,
                 n_cond_ids=n_cond, max_pos=max_pos)


def config(idx: int) -> RoundCfg:
    """BASELINE configurations 0..4."""
    if idx == 0:
        return RoundCfg(name="cfg0-tiny-fp32",
                        target=_ln_gelu(4, 256, 4, 1024, 128), draft=_ln_gelu(1, 256, 4, 1024, 128),
                        head=HeadCfg(3, 256, 256, n_steps=1), K=4, max_batch=1, max_ctx=128,
                        entropy_layer=1, dtype=DT_F32, batch=1, n_ctx=64)
    if idx == 1:
        return RoundCfg(name="cfg1-classcond-L24-d1024",
                        target=_ln_gelu(24, 1024, 16, 4096, 288, 1000),
                        draft=_ln_gelu(2, 1024, 16, 4096, 288, 1000),
                        head=HeadCfg(6, 1024, 1024, n_steps=2), K=8, max_batch=32, max_ctx=288,
                        entropy_layer=1, batch=32, n_ctx=129)
    if idx == 2:
        return RoundCfg(name="cfg2-classcond-L32-d1280",
                        target=_ln_gelu(32, 1280, 20, 5120, 288, 1000),
                        draft=_ln_gelu(3, 1280, 20, 5120, 288, 1000),
                        head=HeadCfg(8, 1280, 1280, n_steps=2), K=8, max_batch=64, max_ctx=288,
                        entropy_layer=2, batch=64, n_ctx=129)
    if idx == 3:
        tgt = TfCfg(n_layers=40, d_model=5120, n_heads=40, n_kv_heads=8, d_head=128, d_ff=13824,
                    act=ACT_SWIGLU, norm=NORM_RMS, pos=POS_ROPE, has_bias=0, norm_eps=1e-6)
        drf = TfCfg(n_layers=4, d_model=2048, n_heads=16, n_kv_heads=4, d_head=128, d_ff=5632,
                    act=ACT_SWIGLU, norm=NORM_RMS, pos=POS_ROPE, has_bias=0, norm_eps=1e-6, d_out=5120)
        return RoundCfg(name="cfg3-t2i-14B", target=tgt, draft=drf,
                        head=HeadCfg(12, 1536, 5120, n_steps=4), K=8, max_batch=8, max_ctx=1312,
                        entropy_layer=1, batch=8, n_ctx=768)
    if idx == 4:
        c = config(2)
        c.name = "cfg4-prefilter-stress"
        c.target.max_pos = c.draft.max_pos = 1056
        c.max_batch = c.batch = 256
        c.max_ctx = 1056
        c.n_ctx = 1024
        return c
    raise ValueError(idx)


def reduced(kind: str) -> RoundCfg:
    """Small shapes that exercise every code path in seconds on the CPU."""
    if kind == "ln-gelu-bf16":      # configs[1] family, shrunk
        return RoundCfg(name="mini-ln-gelu",
                        target=_ln_gelu(3, 128, 4, 256, 96, 10), draft=_ln_gelu(2, 128, 4, 256, 96, 10),
                        head=HeadCfg(2, 128, 128, n_steps=2), K=4, max_batch=3, max_ctx=96,
                        entropy_layer=1, batch=3, n_ctx=37)
    if kind == "gqa-rope-bf16":     # configs[3] family, shrunk (GQA 5:1, head dim 128)
        tgt = TfCfg(n_layers=2, d_model=640, n_heads=5, n_kv_heads=1, d_head=128, d_ff=384,
                    act=ACT_SWIGLU, norm=NORM_RMS, pos=POS_ROPE, has_bias=0, norm_eps=1e-6)
        drf = TfCfg(n_layers=2, d_model=256, n_heads=2, n_kv_heads=1, d_head=128, d_ff=192,
                    act=ACT_SWIGLU, norm=NORM_RMS, pos=POS_ROPE, has_bias=0, norm_eps=1e-6, d_out=640)
        return RoundCfg(name="mini-gqa-rope", target=tgt, draft=drf,
                        head=HeadCfg(2, 192, 640, n_steps=4), K=8, max_batch=2, max_ctx=160,
                        entropy_layer=1, batch=2, n_ctx=70)
    if kind == "ln-gelu-f32":
        c = reduced("ln-gelu-bf16")
        c.name = "mini-ln-gelu-f32"
        c.dtype = DT_F32
        return c
    if kind == "mid-bf16":          # several GEMM tiles per dimension, ragged tails
        return RoundCfg(name="mid-ln-gelu",
                        target=_ln_gelu(4, 512, 8, 2048, 160, 100), draft=_ln_gelu(2, 512, 8, 2048, 160, 100),
                        head=HeadCfg(3, 512, 512, n_steps=2), K=8, max_batch=13, max_ctx=160,
                        entropy_layer=1, batch=13, n_ctx=75)
    raise ValueError(kind)


def clone(c: RoundCfg) -> RoundCfg:
    return copy.deepcopy(c)
