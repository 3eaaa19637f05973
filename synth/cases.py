"""Seeded benchmark / test cases: a configuration's weights, synthetic KV caches and round inputs.

Shapes and seeded draws only (no arithmetic of the method): both the HIP library's callers and the CPU oracle's
callers build their inputs here, so the two sides see the same bits.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import gen
from .configs import RoundCfg, reduced, config, clone


@dataclass
class Case:
    rc: RoundCfg
    W: dict
    cache_t: list          # per target layer (k, v) numpy [B, Hkv, n_ctx, dh]
    cache_d: list
    inp: dict
    B: int
    n_ctx: int
    seed: int
    shared_layers: bool = True


def build_case(kind, seed=0, n_ctx=None, B=None, affine=True, w_std=None, same_draft=False, cache_layers_shared=False,
               std_overrides=None, peaky=False, deep_gain=1.0, lazy=False) -> Case:
    rc = kind if isinstance(kind, RoundCfg) else (config(kind) if isinstance(kind, int) else reduced(kind))
    rc = clone(rc)
    if same_draft:
        rc.draft = clone(rc).target
    B = rc.batch if B is None else B
    n_ctx = rc.n_ctx if n_ctx is None else n_ctx
    if peaky:
        # QKV weights scaled so that attention scores have a standard deviation near 2: the softmax
        # is far from uniform (a wrong K/Q layout shows) yet bf16 rounding of q, k stays within the bar
        std_overrides = dict(std_overrides or {})
        std_overrides["wqkv"] = 1.4 / np.sqrt(min(rc.target.d_model, rc.draft.d_model))
    # the workload recipe: N(0, 0.02) up to 2048 channels; wider models draw N(0, (0.64 / sqrt(d_model))^2), the std at
    # which a projection's gain std * sqrt(fan_in) is what 0.02 gives the 1024-wide configuration (with 0.02 itself a
    # 5120-wide pre-norm stack amplifies every rounding error: see the design notes)
    def recipe_std(cfg):
        if w_std is not None:
            return w_std
        return 0.02 if cfg.d_model <= 2048 else 0.64 / float(np.sqrt(cfg.d_model))
    std_t, std_d, std_h = recipe_std(rc.target), recipe_std(rc.draft), (0.02 if w_std is None else w_std)
    same_shape = (rc.draft.d_model, rc.draft.n_heads, rc.draft.n_kv_heads, rc.draft.d_ff) == \
                 (rc.target.d_model, rc.target.n_heads, rc.target.n_kv_heads, rc.target.d_ff)
    # lazy: the weights are drawn tensor by tensor when read (gen.LazyWeights) instead of all at once; same values
    W = gen.tf_weights(rc.target, seed, "target", rc.dtype, w_std=std_t, affine=affine, std_overrides=std_overrides,
                       deep_from=rc.draft.n_layers, deep_gain=deep_gain, recipes_only=lazy)
    aliases = {}
    if same_shape:
        if lazy:
            aliases = gen.truncated_draft(W, rc.target, rc.draft, names_only=True)
        else:
            W.update(gen.truncated_draft(W, rc.target, rc.draft))
    else:
        W.update(gen.tf_weights(rc.draft, seed, "draft", rc.dtype, w_std=std_d, affine=affine, std_overrides=std_overrides,
                                recipes_only=lazy))
    W.update(gen.head_weights(rc.head, seed, rc.dtype, w_std=std_h, affine=affine, recipes_only=lazy))
    if lazy:
        numel = {}
        for pre, shapes in (("target", gen.tf_weight_shapes(rc.target)), ("draft", gen.tf_weight_shapes(rc.draft)),
                            ("head", gen.head_weight_shapes(rc.head))):
            for name, (shape, _) in shapes.items():
                numel[f"{pre}.{name}"] = int(np.prod(shape))
        W = gen.LazyWeights(W, aliases, numel=numel)
    cache_t, cache_d = [], []
    for l in range(rc.target.n_layers):
        src = 0 if cache_layers_shared else l
        cache_t.append(gen.kv_cache(rc.target, seed, "target", src, B, n_ctx, rc.dtype) if (l == 0 or not cache_layers_shared)
                       else cache_t[0])
    for l in range(rc.draft.n_layers):
        if same_shape:
            cache_d.append(cache_t[l])
        else:
            cache_d.append(gen.kv_cache(rc.draft, seed, "draft", l, B, n_ctx, rc.dtype))
    inp = gen.round_inputs(rc, seed, B)
    return Case(rc, W, cache_t, cache_d, inp, B, n_ctx, seed, same_shape)
