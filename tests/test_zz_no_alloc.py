"""The allocation-free pre-filter entry point (entropy_prefilter_static) against entropy_prefilter: same kernels, so
every output is bit-identical; two calls in a row on one GPU, the second on a smaller input (the shared scratch array
keeps the first call's counts)."""
import numpy as np
import pytest
import torch

from synth import gen
from tests.harness import build_case, make_ctx

pytestmark = pytest.mark.gpu


def _bufs(B, K, dev):
    return dict(H=torch.full((B, K), -7.0, dtype=torch.float32, device=dev), keep=torch.full((B, K), 9, dtype=torch.uint8, device=dev),
                n_keep=torch.full((B,), -3, dtype=torch.int32, device=dev),
                surv_idx=torch.full((max(B * K, 1),), -5, dtype=torch.int32, device=dev),
                n_surv=torch.full((1,), -1, dtype=torch.int32, device=dev))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_prefilter_equals_context_prefilter_on_two_calls_in_a_row(lib, dtype):
    case = build_case("ln-gelu-bf16" if dtype == torch.bfloat16 else "ln-gelu-f32", seed=0)
    ctx = make_ctx(case)
    dev = ctx.dev
    K, L, tau = 8, 1280, 2.14
    # both above 1024 samples (the path that uses the scratch array), the second smaller and ragged; then a small one
    for B, frac, seed in ((4099, 0.5, 1), (1537, 0.25, 2), (37, 0.75, 3)):
        cut = gen.cuts_for_fraction(seed, B, K, frac, ragged=True)
        feat = ctx.dev_store(gen.stress_features(seed, B, K, L, cut, case.rc.dtype)).to(dtype)
        out = _bufs(B, K, dev)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(dev)
        lib.entropy_prefilter_static(feat, tau, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(dev) == before
        H, keep, n_keep, surv, n_surv = ctx.entropy_prefilter(feat, tau)
        ctx.sync()
        ns = int(n_surv.item())
        assert int(out["n_surv"].item()) == ns == int(cut.sum())
        assert torch.equal(out["H"], H)
        assert torch.equal(out["keep"], keep)
        assert torch.equal(out["n_keep"], n_keep)
        assert torch.equal(out["surv_idx"][:ns], surv[:ns])
        assert np.array_equal(n_keep.cpu().numpy(), cut)
    ctx.close()


def test_static_prefilter_limits_and_empty_input(lib):
    dev = torch.device("cuda:0")
    out = _bufs(4, 8, dev)
    one = torch.zeros((1, 8, 64), dtype=torch.bfloat16, device=dev)
    with pytest.raises(lib.FardError) as e:
        lib.entropy_prefilter_static(one.expand((1 << 21) + 1, 8, 64), 1.0, out)     # shape only: rejected before any launch
    assert e.value.code == -3
    empty = torch.zeros((4, 0, 64), dtype=torch.bfloat16, device=dev)
    lib.entropy_prefilter_static(empty, 1.0, out)
    torch.cuda.synchronize()
    assert int(out["n_surv"].item()) == 0 and not out["n_keep"].any()
