"""Seeded tensor generators: weights, KV caches, latents, noise, uniforms.

Every tensor has its own sub-stream, keyed by (master seed, tensor name), so the
order in which tensors are drawn never changes their values.  Values that the
bf16 path stores in bf16 are rounded to bf16 (round-to-nearest-even) once, here,
and returned as float32 arrays holding exactly those values: the oracle widens
them to float64, the HIP path narrows them to bf16, both without further error.
"""
from __future__ import annotations

import zlib

import numpy as np

from .configs import (RoundCfg, TfCfg, HeadCfg, ACT_GELU, ACT_SWIGLU, NORM_LAYER, NORM_RMS,
                      POS_LEARNED, DT_BF16)


# --------------------------------------------------------------------------- bf16 helpers
def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bf16-exact (or get rounded here)."""
    return (bf16_round(x).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def rng_for(seed: int, name: str) -> np.random.Generator:
    key = zlib.crc32(name.encode())
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), key])))


def _store(x: np.ndarray, dtype: int) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    return bf16_round(x) if dtype == DT_BF16 else x


def normal(seed, name, shape, std, dtype, mean=0.0):
    g = rng_for(seed, name)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return _store(x, dtype)


# --------------------------------------------------------------------------- weights
def tf_weight_shapes(c: TfCfg) -> dict:
    """name -> (shape, kind); kind in {'w', 'b', 'g'} (matrix / bias / gain)."""
    d, H, Hk, dh, F, D = c.d_model, c.n_heads, c.n_kv_heads, c.d_head, c.d_ff, c.d_latent
    s = {"in.w": ((D, d), "w"), "in.b": ((d,), "b")}
    if c.pos == POS_LEARNED:
        s["pos"] = ((c.max_pos, d), "w")
    if c.n_cond_ids > 0:
        s["cond"] = ((c.n_cond_ids, d), "w")
    for i in range(c.n_layers):
        p = f"L{i}."
        s[p + "n1.g"] = ((d,), "g")
        s[p + "n2.g"] = ((d,), "g")
        if c.norm == NORM_LAYER:
            s[p + "n1.b"] = ((d,), "b")
            s[p + "n2.b"] = ((d,), "b")
        s[p + "wqkv"] = ((d, (H + 2 * Hk) * dh), "w")
        s[p + "wo"] = ((H * dh, d), "w")
        if c.has_bias:
            s[p + "bqkv"] = (((H + 2 * Hk) * dh,), "b")
            s[p + "bo"] = ((d,), "b")
        if c.act == ACT_GELU:
            s[p + "w1"] = ((d, F), "w")
            s[p + "w2"] = ((F, d), "w")
            if c.has_bias:
                s[p + "b1"] = ((F,), "b")
                s[p + "b2"] = ((d,), "b")
        else:
            s[p + "wg"] = ((d, F), "w")
            s[p + "wu"] = ((d, F), "w")
            s[p + "wd"] = ((F, d), "w")
    s["nf.g"] = ((d,), "g")
    if c.norm == NORM_LAYER:
        s["nf.b"] = ((d,), "b")
    if c.d_out and c.d_out != c.d_model:
        s["up.w"] = ((d, c.d_out), "w")
    return s


def head_weight_shapes(h: HeadCfg) -> dict:
    w, D = h.width, h.d_latent
    s = {"in.w": ((D, w), "w"), "in.b": ((w,), "b"),
         "c.w": ((h.d_cond, w), "w"), "c.b": ((w,), "b"),
         "t1.w": ((h.t_freq_dim, w), "w"), "t1.b": ((w,), "b"),
         "t2.w": ((w, w), "w"), "t2.b": ((w,), "b")}
    for j in range(h.n_blocks):
        p = f"B{j}."
        s[p + "mod.w"] = ((w, 3 * w), "w")
        s[p + "mod.b"] = ((3 * w,), "b")
        s[p + "w1"] = ((w, w), "w")
        s[p + "b1"] = ((w,), "b")
        s[p + "w2"] = ((w, w), "w")
        s[p + "b2"] = ((w,), "b")
    s["f.mod.w"] = ((w, 2 * w), "w")
    s["f.mod.b"] = ((2 * w,), "b")
    s["out.w"] = ((w, D), "w")
    s["out.b"] = ((D,), "b")
    return s


def _weight_recipes(shapes, seed, prefix, dtype, w_std, affine, std_overrides=None):
    """name -> zero-argument function that draws the tensor (its own sub-stream: the order of the calls never matters).
    affine=False: gains 1, biases 0 (the benchmark recipe).  affine=True: gains 1 + N(0, 0.1), biases N(0, 0.05) so
    that a wrong gain/bias index changes results."""
    out = {}
    for name, (shape, kind) in shapes.items():
        full = f"{prefix}.{name}"
        if kind == "w":
            std = w_std
            if std_overrides:
                for key, val in std_overrides.items():
                    if name.endswith(key):
                        std = val
            out[full] = (lambda full=full, shape=shape, std=std: normal(seed, full, shape, std, dtype))
        elif kind == "g":
            out[full] = ((lambda full=full, shape=shape: normal(seed, full, shape, 0.1, dtype, mean=1.0)) if affine
                         else (lambda shape=shape: np.ones(shape, np.float32)))
        else:
            out[full] = ((lambda full=full, shape=shape: normal(seed, full, shape, 0.05, dtype)) if affine
                         else (lambda shape=shape: np.zeros(shape, np.float32)))
    return out


def _draw_all(recipes: dict, workers: int = 8) -> dict:
    """Draws every tensor; large sets on a few threads (numpy's generators release the GIL while they fill)."""
    names = list(recipes)
    if len(names) < 8:
        return {n: recipes[n]() for n in names}
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=workers) as ex:
        vals = list(ex.map(lambda n: recipes[n](), names))
    return dict(zip(names, vals))


def _draw_weights(shapes, seed, prefix, dtype, w_std, affine, layers=None, std_overrides=None):
    return _draw_all(_weight_recipes(shapes, seed, prefix, dtype, w_std, affine, std_overrides))


class LazyWeights:
    """A weight set that is drawn tensor by tensor on demand instead of being held whole (the 11 B parameters of the
    text-to-image configuration are 44 GB as float32).  Reading `W[name]` draws the tensor from its own sub-stream
    (the same values as the eager dictionaries) and keeps it in a least-recently-used cache of `budget_bytes`;
    `as_f64=True` hands out float64 arrays (what the CPU oracle widens to anyway).  `items()` walks all tensors in
    order with `prefetch` of them being drawn ahead on threads (for uploading a whole set with bounded host memory)."""

    def __init__(self, recipes: dict, aliases: dict | None = None, budget_bytes: int = 6 << 30, as_f64: bool = False,
                 prefetch: int = 6, readahead: int = 0, numel: dict | None = None):
        self._rec = dict(recipes)
        self._alias = dict(aliases or {})
        self._budget = int(budget_bytes)
        self._f64 = as_f64
        self._prefetch = prefetch
        self._readahead = readahead                        # tensors drawn ahead of a reader that follows the listed order
        self._numel = dict(numel or {})                    # name -> element count (sizes of tensors still being drawn)
        self._names = list(self._rec)
        self._order = {n: i for i, n in enumerate(self._names)}
        self._pool = None
        from collections import OrderedDict
        self._cache = OrderedDict()
        self._sizes = {}
        self._bytes = 0

    def _draw(self, name):
        x = self._rec[self._alias.get(name, name)]()
        return x.astype(np.float64) if self._f64 else x

    def keys(self):
        return list(self._rec) + list(self._alias)

    def __iter__(self):
        return iter(self.keys())

    def __len__(self):
        return len(self._rec) + len(self._alias)

    def __contains__(self, name):
        return name in self._rec or name in self._alias

    def __getitem__(self, name):
        if name not in self:
            raise KeyError(name)
        key = self._alias.get(name, name)
        self._read_ahead(key)
        if key in self._cache:
            self._cache.move_to_end(key)
            x = self._cache[key]
            if hasattr(x, "result"):                       # still being drawn on a thread
                x = x.result()
                self._cache[key] = x
            return x
        x = self._draw(key)
        self._put(key, x, x.nbytes)
        return x

    def _put(self, key, val, nbytes):
        self._cache[key] = val
        self._sizes[key] = nbytes
        self._bytes += nbytes
        while self._bytes > self._budget and len(self._cache) > 1:
            k, _ = self._cache.popitem(last=False)
            self._bytes -= self._sizes.pop(k)

    def _read_ahead(self, key):
        """A reader that walks the tensors in their listed order (a forward pass does) finds the next few already
        being drawn on threads."""
        if self._readahead <= 0 or key not in self._order:
            return
        if self._pool is None:
            from concurrent.futures import ThreadPoolExecutor
            self._pool = ThreadPoolExecutor(max_workers=self._readahead)
        i = self._order[key]
        for nxt in self._names[i + 1:i + 1 + self._readahead]:
            if nxt not in self._cache:
                self._put(nxt, self._pool.submit(self._draw, nxt), self._nbytes(nxt))

    def _nbytes(self, key):
        return self._numel.get(key, 0) * (8 if self._f64 else 4)

    def view(self, as_f64: bool, budget_bytes: int | None = None, readahead: int = 0) -> "LazyWeights":
        """The same tensors through a cache of its own (e.g. float64 for the oracle beside float32 for the upload)."""
        return LazyWeights(self._rec, self._alias, self._budget if budget_bytes is None else budget_bytes, as_f64,
                           self._prefetch, readahead, self._numel)

    def items(self):
        from concurrent.futures import ThreadPoolExecutor
        names = self.keys()
        with ThreadPoolExecutor(max_workers=self._prefetch) as ex:
            pending = []
            it = iter(names)
            for n in it:
                pending.append((n, ex.submit(self._draw, n)))
                if len(pending) >= self._prefetch:
                    break
            while pending:
                n, fut = pending.pop(0)
                nxt = next(it, None)
                if nxt is not None:
                    pending.append((nxt, ex.submit(self._draw, nxt)))
                yield n, fut.result()


def tf_weights(c: TfCfg, seed: int, prefix: str, dtype: int, w_std=0.02, affine=False,
               std_overrides=None, deep_from=None, deep_gain=1.0, recipes_only=False) -> dict:
    """deep_from / deep_gain: the output projections (wo, w2 / wd) of layers >= deep_from are drawn
    with std w_std * deep_gain.  With deep_from = L_draft this makes the deep layers refinements of
    the shallow ones, so that a draft made of the first L_draft layers predicts the target's feature
    about as well as a trained draft would (acceptance well inside (0, 1))."""
    ov = dict(std_overrides or {})
    if deep_from is not None and deep_gain != 1.0:
        for l in range(deep_from, c.n_layers):
            for nm in ("wo", "w2", "wd"):
                ov[f"L{l}.{nm}"] = w_std * deep_gain
    rec = _weight_recipes(tf_weight_shapes(c), seed, prefix, dtype, w_std, affine, std_overrides=ov)
    return rec if recipes_only else _draw_all(rec)


def head_weights(h: HeadCfg, seed: int, dtype: int, w_std=0.02, affine=False,
                 std_overrides=None, recipes_only=False) -> dict:
    rec = _weight_recipes(head_weight_shapes(h), seed, "head", dtype, w_std, affine, std_overrides=std_overrides)
    return rec if recipes_only else _draw_all(rec)


def truncated_draft(target_w: dict, tc: TfCfg, dc: TfCfg, names_only=False) -> dict:
    """Draft = the target's embeddings, its first L_d layers and its final norm
    (a draft 'initialised with the target').  Needs equal widths.  names_only: draft name -> target name."""
    assert (tc.d_model, tc.n_heads, tc.n_kv_heads, tc.d_ff) == (dc.d_model, dc.n_heads, dc.n_kv_heads, dc.d_ff)
    out = {}
    for name in tf_weight_shapes(dc):
        out["draft." + name] = "target." + name if names_only else target_w["target." + name]
    return out


# --------------------------------------------------------------------------- caches / inputs
def kv_cache(c: TfCfg, seed: int, which: str, layer: int, B: int, n: int, dtype: int, std=0.64):
    """Synthetic cache entries K, V of shape [B, H_kv, n, d_head] for one layer."""
    shape = (B, c.n_kv_heads, n, c.d_head)
    k = normal(seed, f"cache.{which}.L{layer}.k", shape, std, dtype)
    v = normal(seed, f"cache.{which}.L{layer}.v", shape, std, dtype)
    return k, v


def latents(seed: int, name: str, shape, dtype: int):
    return normal(seed, name, shape, 1.0, dtype)


def noise(seed: int, name: str, shape):
    """fp32 Gaussian noise (never rounded to bf16: the sampler works in fp32)."""
    return rng_for(seed, name).standard_normal(size=shape, dtype=np.float32)


def uniforms(seed: int, name: str, shape):
    """fp32 U[0,1) draws for the accept test."""
    return rng_for(seed, name).random(size=shape, dtype=np.float32)


def round_inputs(rc: RoundCfg, seed: int, B: int | None = None) -> dict:
    B = rc.batch if B is None else B
    D, K, S = rc.target.d_latent, rc.K, rc.head.n_steps
    return {
        "pending": latents(seed, "pending", (B, D), rc.dtype),
        "eps_draft": noise(seed, "eps", (S + 1, B, K + 1, D)),   # shared by draft and target
        "r": uniforms(seed, "r", (B, K)),
    }


# --------------------------------------------------------------------------- entropy stress features
def stress_features(seed: int, B: int, K: int, d: int, cut: np.ndarray, dtype: int,
                    spike: float = 14.0, base_std: float = 0.25):
    """Draft shallow features whose softmax entropy is ~ln(d) for draft positions
    i < cut[b] and ~0 from cut[b] on: f = base_std*g + spike*onehot(j) on the low rows.
    `cut[b]` in [0, K] is the number of leading high-entropy rows of sample b."""
    g = rng_for(seed, "stress.g").standard_normal(size=(B, K, d), dtype=np.float32) * np.float32(base_std)
    j = rng_for(seed, "stress.j").integers(0, d, size=(B, K))
    low = np.arange(K)[None, :] >= np.asarray(cut)[:, None]
    bi, ki = np.nonzero(low)
    g[bi, ki, j[bi, ki]] += np.float32(spike)
    return _store(g, dtype)


def cuts_for_fraction(seed: int, B: int, K: int, frac_filtered: float, ragged: bool) -> np.ndarray:
    """Per-sample cut positions with mean K*(1-frac): uniform, or ragged around that mean."""
    keep = K * (1.0 - frac_filtered)
    if not ragged:
        return np.full(B, int(round(keep)), dtype=np.int64)
    g = rng_for(seed, "stress.cut")
    lo = np.floor(keep)
    c = lo + (g.random(B) < (keep - lo))
    jitter = g.integers(-2, 3, size=B)
    c = np.clip(c + jitter, 0, K)
    # re-centre so that the mean stays at `keep` (to the nearest achievable integer total)
    diff = int(round(keep * B - c.sum()))
    idx = g.permutation(B)
    for t in idx:
        if diff == 0:
            break
        step = 1 if diff > 0 else -1
        if 0 <= c[t] + step <= K:
            c[t] += step
            diff -= step
    return c.astype(np.int64)
