"""ctypes binding of libfastardiff.so: argument marshalling only.

Function names mirror include/fastardiff.h.  torch provides device memory and the stream;
every step of the path runs inside the library's kernels.  There is no CPU fallback: a missing
library raises at import of this module.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  (first: the library must bind to the HIP runtime torch has already loaded)

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libfastardiff.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2512_08537_amd.build` "
                      "(or __graft_entry__.build()).  There is no CPU fallback.")
lib = C.CDLL(LIB_PATH)

FARD_F32, FARD_BF16 = 0, 1
TARGET, DRAFT = 0, 1
STATUS = {0: "FARD_OK", -1: "FARD_EINVAL", -2: "FARD_ESHAPE", -3: "FARD_ECAPACITY", -4: "FARD_ENOMEM",
          -5: "FARD_EHIP", -6: "FARD_ESTATE"}


class TfCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "d_head", "d_ff",
                                         "act", "norm", "pos", "has_bias")] + \
               [("norm_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("d_latent", "n_cond_ids", "d_out", "max_pos")]


class HeadCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_blocks", "width", "d_cond", "d_latent", "n_steps", "t_freq_dim")] + \
               [("t_scale", C.c_float), ("sigma_last", C.c_float), ("temperature", C.c_float), ("renoise", C.c_int32)]


class RoundCfg(C.Structure):
    _fields_ = [("target", TfCfg), ("draft", TfCfg), ("head", HeadCfg)] + \
               [(n, C.c_int32) for n in ("K", "max_batch", "max_ctx", "entropy_layer", "entropy_mode",
                                         "prefix_rule", "dtype")] + [("tau_ent", C.c_float)]


class Tensor(C.Structure):
    _fields_ = [("name", C.c_char_p), ("data", C.c_void_p), ("numel", C.c_int64), ("dtype", C.c_int32),
                ("on_device", C.c_int32)]


_vp, _i32, _f32 = C.c_void_p, C.c_int32, C.c_float
_SIGS = {
    "spec_round_init": [C.POINTER(RoundCfg), C.POINTER(Tensor), _i32, _vp, C.POINTER(_vp)],
    "spec_round_destroy": [_vp],
    "spec_kv_reset": [_vp, _i32, _vp, _i32],
    "spec_kv_restore": [_vp, _i32, _vp, _i32, _i32],
    "spec_kv_load": [_vp, _i32, _i32, _vp, _vp, _i32, _i32],
    "spec_kv_lengths": [_vp, _i32, _vp, _i32],
    "spec_kv_commit": [_vp, _i32, _vp, _i32],
    "spec_forward": [_vp, _i32, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp],
    "entropy_prefilter": [_vp, _vp, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp],
    "entropy_prefilter_static": [_vp, _i32, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp, _vp],
    "diffhead_decode": [_vp, _vp, _vp, _i32, _vp, _vp, _vp],
    "spec_draft": [_vp, _vp, _vp, _vp, _f32, _i32, _vp, _vp, _vp, _vp, _vp],
    "spec_draft_step": [_vp, _i32, _vp, _vp, _vp, _f32, _i32, _vp, _vp, _vp, _vp, _vp],
    "spec_verify": [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _i32, _vp, _vp, _vp, _vp],
    "spec_accept": [_vp, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _i32, _vp, _vp, _vp],
    "spec_round": [_vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _f32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp],
    "spec_resample": [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _i32, _i32, _vp, _vp],
    "spec_generate": [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _f32, _f32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp,
                      _vp],
    "spec_gemm": [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp],
    "spec_gemm_narrow": [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp],
    "spec_gemm_norm": [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _f32, _i32, _vp],
    "spec_graph_enable": [_vp, _i32],
    "spec_entropy_loss": [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp],
    "spec_smooth_l1": [_vp, _vp, _vp, C.c_int64, _f32, _vp, _vp],
    "spec_prefill": [_vp, _i32, _vp, _vp, C.POINTER(C.c_int32), _i32, _i32, _vp],
    "spec_peak_probe": [_vp, _i32, _vp, C.c_int64, _i32, _i32, C.POINTER(C.c_float), C.POINTER(C.c_double)],
    "spec_profile_enable": [_vp, _i32],
    "spec_profile_read": [_vp, _i32, C.POINTER(C.c_float), C.POINTER(C.c_int64), C.POINTER(C.c_double),
                          C.POINTER(C.c_double)],
}
EXPORTS = list(_SIGS) + ["entropy_threshold", "spec_last_error"]
for _name, _args in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.argtypes = _args
    _fn.restype = C.c_int
lib.entropy_threshold.argtypes = [_f32, _f32]
lib.entropy_threshold.restype = _f32
lib.spec_last_error.argtypes = [_vp]
lib.spec_last_error.restype = C.c_char_p


class FardError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


def _fill(struct, obj):
    for name, _ in struct._fields_:
        v = getattr(obj, name)
        setattr(struct, name, v)
    return struct


def make_cfg(rc) -> RoundCfg:
    """rc: synth.configs.RoundCfg (or anything with the same attribute names)."""
    out = RoundCfg()
    _fill(out.target, rc.target)
    _fill(out.draft, rc.draft)
    _fill(out.head, rc.head)
    for n in ("K", "max_batch", "max_ctx", "entropy_layer", "entropy_mode", "prefix_rule", "dtype", "tau_ent"):
        setattr(out, n, getattr(rc, n))
    return out


def _ptr(t):
    if t is None:
        return None
    return C.c_void_p(t.data_ptr())


def entropy_prefilter_static(feat, tau, out, stream=None):
    """feat: device tensor [B, K, L], float32 or bfloat16; out: dict of preallocated device tensors H [B,K] f32,
    keep [B,K] u8, n_keep [B] i32, surv_idx [B*K] i32, n_surv [1] i32.  Allocates nothing."""
    import torch
    B, K, L = feat.shape
    dt = FARD_BF16 if feat.dtype == torch.bfloat16 else FARD_F32
    code = lib.entropy_prefilter_static(_ptr(feat), dt, B, K, L, float(tau), _ptr(out["H"]), _ptr(out["keep"]),
                                        _ptr(out["n_keep"]), _ptr(out["surv_idx"]), _ptr(out["n_surv"]),
                                        None if stream is None else C.c_void_p(stream.cuda_stream))
    if code != 0:
        raise FardError(code, "entropy_prefilter_static")
    return out


def entropy_threshold(mean_h: float, std_h: float) -> float:
    return float(lib.entropy_threshold(mean_h, std_h))


class Context:
    """Owns one fard_ctx.  `weights`: dict name -> numpy float32 array (values already exact in the
    storage type) or torch tensor; uploaded to the GPU in the storage type and handed to
    spec_round_init as device tensors."""

    def __init__(self, rc, weights: dict, device="cuda:0", stream=None):
        import torch
        self.torch = torch
        self.rc = rc
        self.dev = torch.device(device)
        self.bf16 = rc.dtype == FARD_BF16
        self.tdtype = torch.bfloat16 if self.bf16 else torch.float32
        self.stream_ptr = None if stream is None else C.c_void_p(stream.cuda_stream)
        cfg = make_cfg(rc)
        names, keep = [], []
        arr = (Tensor * len(weights))()
        for i, (name, w) in enumerate(weights.items()):
            t = torch.from_numpy(np.ascontiguousarray(w)) if isinstance(w, np.ndarray) else w
            small = t.dim() == 1
            t = t.to(self.dev, dtype=torch.float32 if small else self.tdtype).contiguous()
            keep.append(t)
            names.append(name.encode())
            arr[i].name = names[-1]
            arr[i].data = t.data_ptr()
            arr[i].numel = t.numel()
            arr[i].dtype = FARD_F32 if t.dtype == torch.float32 else FARD_BF16
            arr[i].on_device = 1
        torch.cuda.synchronize(self.dev)
        h = C.c_void_p()
        code = lib.spec_round_init(C.byref(cfg), arr, len(weights), self.stream_ptr, C.byref(h))
        if code != 0:
            raise FardError(code, "spec_round_init failed (message on stderr)")
        self.h = h
        del keep

    # ------------------------------------------------------------------ helpers
    def _chk(self, code):
        if code != 0:
            raise FardError(code, lib.spec_last_error(self.h).decode())

    def close(self):
        if getattr(self, "h", None):
            lib.spec_round_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def dev_f32(self, a):
        t = self.torch
        return t.as_tensor(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev) if not isinstance(a, t.Tensor) \
            else a.to(self.dev, dtype=t.float32).contiguous()

    def dev_store(self, a):
        """numpy float32 (exact in storage type) -> device tensor of the storage type."""
        t = self.torch
        x = t.as_tensor(np.ascontiguousarray(a, dtype=np.float32)) if not isinstance(a, t.Tensor) else a
        return x.to(self.dev, dtype=self.tdtype).contiguous()

    def dev_i32(self, a):
        t = self.torch
        return t.as_tensor(np.ascontiguousarray(a, dtype=np.int32)).to(self.dev) if not isinstance(a, t.Tensor) \
            else a.to(self.dev, dtype=t.int32).contiguous()

    def empty(self, shape, dtype):
        return self.torch.empty(shape, dtype=dtype, device=self.dev)

    def sync(self):
        self.torch.cuda.synchronize(self.dev)

    # ------------------------------------------------------------------ C ABI, one method per entry point
    def spec_kv_reset(self, which, cache_len=None, B=None):
        if cache_len is None:
            self._chk(lib.spec_kv_reset(self.h, which, None, self.rc.max_batch if B is None else B))
        else:
            a = np.ascontiguousarray(cache_len, dtype=np.int32)
            self._chk(lib.spec_kv_reset(self.h, which, a.ctypes.data_as(C.c_void_p), len(a)))

    def spec_kv_restore(self, which, cache_len_dev, len_hi):
        """cache_len_dev: device int32 [B]; len_hi: host upper bound of its values."""
        self._chk(lib.spec_kv_restore(self.h, which, _ptr(cache_len_dev), cache_len_dev.numel(), int(len_hi)))

    def spec_kv_load(self, which, layer, k, v):
        """k, v: device tensors [B, H_kv, n, d_head] of the storage type."""
        B, _, n, _ = k.shape
        self._chk(lib.spec_kv_load(self.h, which, layer, _ptr(k), _ptr(v), B, n))

    def spec_kv_lengths(self, which, B):
        out = np.zeros(B, dtype=np.int32)
        self._chk(lib.spec_kv_lengths(self.h, which, out.ctypes.data_as(C.c_void_p), B))
        return out

    def spec_kv_commit(self, which, n_accept):
        self._chk(lib.spec_kv_commit(self.h, which, _ptr(n_accept), n_accept.numel()))

    def spec_forward(self, which, x_in, n_q, cond_id=None, commit=True, want_shallow=False, want_h_attn=False,
                     nq_max=None):
        """n_q: host array (its maximum becomes nq_max) or a device tensor (then pass nq_max)."""
        t = self.torch
        tc = self.rc.target if which == TARGET else self.rc.draft
        if not isinstance(n_q, t.Tensor):
            n_q = np.ascontiguousarray(n_q, dtype=np.int32)
            nq_max = max(int(n_q.max()), 1) if nq_max is None else nq_max
            n_q = self.dev_i32(n_q)
        if nq_max is None:
            raise ValueError("nq_max is required when n_q lives on the device")
        M, B = x_in.shape[0], n_q.numel()
        z = self.empty((M, tc.d_out or tc.d_model), self.tdtype)
        sh = self.empty((M, tc.d_model), t.float32) if want_shallow else None
        ha = self.empty((M,), t.float32) if want_h_attn else None
        self._chk(lib.spec_forward(self.h, which, _ptr(x_in), _ptr(cond_id), _ptr(n_q), int(nq_max), B, M, int(commit),
                                   _ptr(z), _ptr(sh), _ptr(ha)))
        return z, sh, ha

    def spec_prefill(self, which, x, n, first_id=None, want_z=True):
        """x: device fp32 [B, n_max, D]; n: host int32 [B]; first_id: device int32 [B] or None."""
        B, n_max, _ = x.shape
        n = np.ascontiguousarray(n, dtype=np.int32)
        assert n.shape == (B,)
        tc = self.rc.target if which == TARGET else self.rc.draft
        z = self.empty((B, tc.d_out or tc.d_model), self.tdtype) if want_z else None
        if z is not None:
            z.zero_()
            self.torch.cuda.synchronize()
        self._chk(lib.spec_prefill(self.h, which, _ptr(x), _ptr(first_id), n.ctypes.data_as(C.POINTER(C.c_int32)), n_max, B,
                                   _ptr(z)))
        return z

    def entropy_prefilter(self, feat, tau):
        t = self.torch
        B, K, L = feat.shape
        H = self.empty((B, K), t.float32)
        keep = self.empty((B, K), t.uint8)
        n_keep = self.empty((B,), t.int32)
        surv = self.empty((max(B * K, 1),), t.int32)
        n_surv = self.empty((1,), t.int32)
        self._chk(lib.entropy_prefilter(self.h, _ptr(feat), B, K, L, float(tau), _ptr(H), _ptr(keep), _ptr(n_keep),
                                        _ptr(surv), _ptr(n_surv)))
        return H, keep, n_keep, surv, n_surv

    def diffhead_decode(self, z, eps, n_rows=None):
        t = self.torch
        n = z.shape[0]
        D = self.rc.head.d_latent
        mu = t.zeros((n, D), dtype=t.float32, device=self.dev)
        x = t.zeros((n, D), dtype=t.float32, device=self.dev)
        self._chk(lib.diffhead_decode(self.h, _ptr(z), _ptr(n_rows), n, _ptr(eps), _ptr(mu), _ptr(x)))
        return mu, x

    def _round_bufs(self, B):
        t = self.torch
        K, D = self.rc.K, self.rc.head.d_latent
        return dict(H=self.empty((B, K), t.float32), keep=self.empty((B, K), t.uint8),
                    n_keep=self.empty((B,), t.int32), x_draft=self.empty((B, K, D), t.float32),
                    mu_q=self.empty((B, K, D), t.float32), n_accept=self.empty((B,), t.int32),
                    log_ratio=self.empty((B, K), t.float32), mu_p=self.empty((B, K + 1, D), t.float32))

    def spec_draft(self, x_pending, eps, tau, pending_id=None, out=None):
        B = x_pending.shape[0]
        o = out or self._round_bufs(B)
        self._chk(lib.spec_draft(self.h, _ptr(x_pending), _ptr(pending_id), _ptr(eps), float(tau), B, _ptr(o["H"]),
                                 _ptr(o["keep"]), _ptr(o["n_keep"]), _ptr(o["x_draft"]), _ptr(o["mu_q"])))
        return o

    def spec_draft_step(self, i, x_prev, eps, tau, out, prev_id=None):
        """One draft step; out: the dict of _round_bufs that all steps of the stage share."""
        B = out["n_keep"].numel()
        self._chk(lib.spec_draft_step(self.h, int(i), _ptr(x_prev), _ptr(prev_id), _ptr(eps), float(tau), B, _ptr(out["H"]),
                                      _ptr(out["keep"]), _ptr(out["n_keep"]), _ptr(out["x_draft"]), _ptr(out["mu_q"])))
        return out

    def spec_verify(self, x_pending, x_draft, mu_q, n_keep, r, eps, log_sigma=0.0, sigma_p=None, sigma_q=None,
                    pending_id=None, want_z=False, out=None):
        B = x_pending.shape[0]
        s = self.rc.head.sigma_last * self.rc.head.temperature
        sigma_p = s if sigma_p is None else sigma_p
        sigma_q = s if sigma_q is None else sigma_q
        o = out or self._round_bufs(B)
        tc = self.rc.target
        z = self.empty((B, self.rc.K + 1, tc.d_out or tc.d_model), self.tdtype) if want_z else None
        self._chk(lib.spec_verify(self.h, _ptr(x_pending), _ptr(pending_id), _ptr(x_draft), _ptr(mu_q), _ptr(n_keep),
                                  _ptr(r), _ptr(eps), float(log_sigma), float(sigma_p), float(sigma_q), B,
                                  _ptr(o["n_accept"]), _ptr(o["log_ratio"]), _ptr(o["mu_p"]), _ptr(z)))
        o["z_p"] = z
        return o

    def spec_accept(self, x_draft, mu_p, mu_q, r, n_keep, log_sigma, sigma_p, sigma_q):
        t = self.torch
        B, K, _ = x_draft.shape
        n_acc = self.empty((B,), t.int32)
        lr = self.empty((B, K), t.float32)
        acc = self.empty((B, K), t.uint8)
        self._chk(lib.spec_accept(self.h, _ptr(x_draft), _ptr(mu_p), _ptr(mu_q), _ptr(r), _ptr(n_keep),
                                  float(log_sigma), float(sigma_p), float(sigma_q), B, _ptr(n_acc), _ptr(lr), _ptr(acc)))
        return n_acc, lr, acc

    def spec_round(self, x_pending, eps, r, tau, log_sigma=0.0, sigma_p=None, sigma_q=None, pending_id=None, out=None):
        B = x_pending.shape[0]
        s = self.rc.head.sigma_last * self.rc.head.temperature
        sigma_p = s if sigma_p is None else sigma_p
        sigma_q = s if sigma_q is None else sigma_q
        o = out or self._round_bufs(B)
        self._chk(lib.spec_round(self.h, _ptr(x_pending), _ptr(pending_id), _ptr(eps), _ptr(r), float(tau),
                                 float(log_sigma), float(sigma_p), float(sigma_q), B, _ptr(o["H"]), _ptr(o["keep"]),
                                 _ptr(o["n_keep"]), _ptr(o["x_draft"]), _ptr(o["mu_q"]), _ptr(o["n_accept"]),
                                 _ptr(o["log_ratio"]), _ptr(o["mu_p"])))
        return o

    def _sigmas(self, sigma_p, sigma_q):
        s = self.rc.head.sigma_last * self.rc.head.temperature
        return float(s if sigma_p is None else sigma_p), float(s if sigma_q is None else sigma_q)

    def spec_resample(self, mu_p, mu_q, eps, n_accept, n_keep, eps_res, u_res, log_sigma=0.0, sigma_p=None, sigma_q=None):
        B, J = u_res.shape
        D = mu_p.shape[-1]
        sp, sq = self._sigmas(sigma_p, sigma_q)
        x_next = self.empty((B, D), self.torch.float32)
        tries = self.empty((B,), self.torch.int32)
        self._chk(lib.spec_resample(self.h, _ptr(mu_p), _ptr(mu_q), _ptr(eps), _ptr(n_accept), _ptr(n_keep), _ptr(eps_res),
                                    _ptr(u_res), float(log_sigma), sp, sq, B, J, _ptr(x_next), _ptr(tries)))
        return x_next, tries

    def spec_generate(self, x_first, eps, r, eps_res, u_res, tau, first_id=None, log_sigma=0.0, sigma_p=None, sigma_q=None,
                      out=None):
        """eps [R,S+1,B,K+1,D], r [R,B,K], eps_res [R,B,J,D], u_res [R,B,J] (device fp32).  out: the dict of a
        previous call with the same shapes (its buffers are reused; with spec_graph_enable that keeps the recorded
        round valid from the first round on)."""
        t = self.torch
        R, B, K = r.shape
        J = u_res.shape[2]
        D = x_first.shape[1]
        sp, sq = self._sigmas(sigma_p, sigma_q)
        if out is not None:
            o = out
            o["tokens"].zero_()
        else:
            o = dict(tokens=t.zeros((B, R * (K + 1), D), dtype=t.float32, device=self.dev),
                     n_tokens=self.empty((B,), t.int32), H=self.empty((R, B, K), t.float32),
                     n_keep=self.empty((R, B), t.int32), n_accept=self.empty((R, B), t.int32), tries=self.empty((R, B), t.int32))
        if self.stream_ptr is not None:
            t.cuda.current_stream().synchronize()        # torch zeroed `tokens` on its own stream
        self._chk(lib.spec_generate(self.h, _ptr(x_first), _ptr(first_id), _ptr(eps), _ptr(r), _ptr(eps_res), _ptr(u_res), float(tau),
                                    float(log_sigma), sp, sq, B, R, J, _ptr(o["tokens"]), _ptr(o["n_tokens"]), _ptr(o["H"]),
                                    _ptr(o["n_keep"]), _ptr(o["n_accept"]), _ptr(o["tries"])))
        return o

    def spec_gemm(self, A, W, bias=None, act=0):
        M, K = A.shape
        N = W.shape[1]
        out = self.empty((M, N), self.tdtype)
        self._chk(lib.spec_gemm(self.h, _ptr(A), _ptr(W), _ptr(bias), M, K, N, act, _ptr(out)))
        return out

    def spec_gemm_narrow(self, A, W, out, bias=None, gate=None, epi=0, act=0, out_bf16=None):
        """`out` is written (epi 0, 1) or accumulated into (epi 2, 3) in place and returned."""
        M, K = A.shape
        N = W.shape[1]
        self._chk(lib.spec_gemm_narrow(self.h, _ptr(A), _ptr(W), _ptr(bias), _ptr(gate), M, K, N, epi, act, _ptr(out),
                                       _ptr(out_bf16)))
        return out

    def spec_gemm_norm(self, x, W, g, beta=None, bias=None, norm_type=0, eps=1e-5, act=0):
        M, K = x.shape
        N = W.shape[1]
        out = self.empty((M, N), self.torch.bfloat16)
        self._chk(lib.spec_gemm_norm(self.h, _ptr(x), _ptr(W), _ptr(g), _ptr(beta), _ptr(bias), M, K, N, norm_type, float(eps),
                                     act, _ptr(out)))
        return out

    def spec_entropy_loss(self, q, k, want_rows=True, want_dq=True, want_dk=True):
        """q: [B, H, R, dh], k: [B, Hkv, R, dh] device tensors of the storage type."""
        t = self.torch
        B, H, R, dh = q.shape
        Hkv = k.shape[1]
        loss = self.empty((1,), t.float32)
        hr = self.empty((B, H, R), t.float32) if want_rows else None
        dq = self.empty(tuple(q.shape), t.float32) if want_dq else None
        dk = self.empty(tuple(k.shape), t.float32) if want_dk else None
        self._chk(lib.spec_entropy_loss(self.h, _ptr(q), _ptr(k), B, H, Hkv, R, dh, _ptr(loss), _ptr(hr), _ptr(dq), _ptr(dk)))
        return loss, hr, dq, dk

    def spec_smooth_l1(self, pred, target, beta=1.0, want_grad=True):
        t = self.torch
        n = pred.numel()
        loss = self.empty((1,), t.float32)
        g = self.empty(tuple(pred.shape), t.float32) if want_grad else None
        self._chk(lib.spec_smooth_l1(self.h, _ptr(pred), _ptr(target), n, float(beta), _ptr(loss), _ptr(g)))
        return loss, g

    def spec_graph_enable(self, on: bool):
        self._chk(lib.spec_graph_enable(self.h, 1 if on else 0))

    def spec_peak_probe(self, kind: int, buf=None, iters: int = 0, reps: int = 10):
        """kind 0: streaming read of the device tensor buf; kind 1: MFMA loop.  Returns (ms per launch, bytes or flop per launch)."""
        ms, units = C.c_float(), C.c_double()
        nbytes = 0 if buf is None else buf.numel() * buf.element_size()
        self._chk(lib.spec_peak_probe(self.h, kind, _ptr(buf), nbytes, iters, reps, C.byref(ms), C.byref(units)))
        return ms.value, units.value

    def spec_profile_enable(self, on: bool):
        self._chk(lib.spec_profile_enable(self.h, int(on)))

    def spec_profile_read(self, cls: int):
        ms, n, fl, by = C.c_float(), C.c_int64(), C.c_double(), C.c_double()
        self._chk(lib.spec_profile_read(self.h, cls, C.byref(ms), C.byref(n), C.byref(fl), C.byref(by)))
        return dict(ms=ms.value, launches=n.value, flops=fl.value, bytes=by.value)
