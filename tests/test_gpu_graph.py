"""Graph replay of spec_round (spec_graph_enable) against the kernel-by-kernel launch of the same round.

Every replay is compared bit for bit with the eager result (the kernels of this configuration use no atomics),
with eager work and synchronisations of the same context between replays, at changed cache lengths and
after a change of arguments."""
import numpy as np
import pytest

from tests.harness import build_case, load_caches, gpu_inputs, to_np

pytestmark = pytest.mark.gpu


def _ctx(case, with_stream=True):
    import torch
    from paper_2512_08537_amd import binding
    stream = torch.cuda.Stream() if with_stream else None
    ctx = binding.Context(case.rc, case.W, stream=stream)
    load_caches(ctx, case)
    return ctx


def _reset(ctx, case, n):
    from paper_2512_08537_amd import binding
    lens = np.full(case.B, n, dtype=np.int32)
    ctx.spec_kv_reset(binding.TARGET, lens)
    ctx.spec_kv_reset(binding.DRAFT, lens)


def _round(ctx, case, gi, out, tau, n):
    from paper_2512_08537_amd import binding
    load_caches(ctx, case)                               # (a round at a shorter length overwrites context rows)
    _reset(ctx, case, n)
    ctx.spec_round(gi["pending"], gi["eps"], gi["r"], tau, out=out)
    ctx.sync()
    res = to_np(out)
    res["len_t"] = ctx.spec_kv_lengths(binding.TARGET, case.B)
    res["len_d"] = ctx.spec_kv_lengths(binding.DRAFT, case.B)
    return res


def _same(a, b):
    return all(np.array_equal(a[k], b[k]) for k in a)


def test_graph_replays_equal_eager_rounds():
    import torch
    case = build_case(1, seed=3, affine=False, B=8, deep_gain=0.02)
    ctx = _ctx(case)
    gi = gpu_inputs(ctx, case)
    out = ctx._round_bufs(case.B)
    n0 = case.n_ctx
    cal = _round(ctx, case, gi, out, -1.0, n0)
    tau = float(np.median(cal["H"]))                     # some samples stop early, some do not
    ref = {n: _round(ctx, case, gi, out, tau, n) for n in (n0, n0 - 5)}
    ref_all = _round(ctx, case, gi, out, -1.0, n0)
    assert 0 < ref[n0]["n_keep"].sum() < case.B * case.rc.K
    assert not _same(ref[n0], ref[n0 - 5])

    ctx.spec_graph_enable(True)
    feat = ctx.dev_store(np.random.default_rng(0).standard_normal((4, case.rc.K, 64)).astype(np.float32))
    for i in range(5):                                   # call 0 eager, call 1 records and launches, 2.. replay
        for v in out.values():
            v.zero_()
        torch.cuda.synchronize()                         # (torch's stream is not the context's)
        got = _round(ctx, case, gi, out, tau, n0)
        assert _same(got, ref[n0]), f"call {i}"
        ctx.entropy_prefilter(feat, 0.5)                 # eager work of the same context between replays
        ctx.sync()
    # the replayed kernels read the cache lengths on the device
    for i in range(2):
        got = _round(ctx, case, gi, out, tau, n0 - 5)
        assert _same(got, ref[n0 - 5])
    # other arguments: eager again, then a new graph
    for i in range(4):
        got = _round(ctx, case, gi, out, -1.0, n0)
        assert _same(got, ref_all), f"call {i} after the change of tau"
    # switched off: kernel by kernel again
    ctx.spec_graph_enable(False)
    assert _same(_round(ctx, case, gi, out, tau, n0), ref[n0])
    ctx.close()


def test_generation_rounds_as_graph_replays_equal_eager_generation():
    """spec_generate with graph replay on: the first round of a new argument set is launched kernel by kernel, the
    second is recorded, later ones and every round of a repeated call replay; all records and tokens must equal the
    eager run bit for bit."""
    import torch
    from synth import gen
    case = build_case(1, seed=3, affine=False, B=8, deep_gain=0.02)
    rc = case.rc
    ctx = _ctx(case)
    gi = gpu_inputs(ctx, case)
    B, K, D, S, R, J = case.B, rc.K, rc.target.d_latent, rc.head.n_steps, 6, 8
    eps = ctx.dev_f32(np.stack([gen.noise(9, f"e{t}", (S + 1, B, K + 1, D)) for t in range(R)]))
    r = ctx.dev_f32(np.stack([gen.uniforms(9, f"r{t}", (B, K)) for t in range(R)]))
    er = ctx.dev_f32(np.stack([gen.noise(9, f"er{t}", (B, J, D)) for t in range(R)]))
    ur = ctx.dev_f32(np.stack([gen.uniforms(9, f"ur{t}", (B, J)) for t in range(R)]))
    ids = ctx.dev_i32(np.arange(B, dtype=np.int32) * 7 % 1000)
    cal = _round(ctx, case, gi, ctx._round_bufs(B), -1.0, case.n_ctx)
    tau = float(np.median(cal["H"]))

    def run(out=None, first_id=None):
        load_caches(ctx, case)
        _reset(ctx, case, case.n_ctx)
        o = ctx.spec_generate(gi["pending"], eps, r, er, ur, tau, first_id=first_id, out=out)
        ctx.sync()
        return o, {k: v.clone() for k, v in o.items()}

    for first_id in (None, ids):
        _, ref = run(first_id=first_id)
        assert int(ref["n_tokens"].sum()) >= R * B
        ctx.spec_graph_enable(True)
        o, got = run(first_id=first_id)                              # round 0 eager, round 1 recorded, 2.. replayed
        assert all(torch.equal(got[k], ref[k]) for k in ref), "first graph-mode call"
        for i in range(2):
            for k in ("H", "n_keep", "n_accept", "tries", "n_tokens"):
                o[k].zero_()
            torch.cuda.synchronize()
            _, got = run(out=o, first_id=first_id)                   # same buffers: every round replays
            assert all(torch.equal(got[k], ref[k]) for k in ref), f"repeated call {i}"
        ctx.spec_graph_enable(False)
    ctx.close()


def test_graph_replay_keeps_the_capacity_rules():
    from paper_2512_08537_amd import binding
    case = build_case("mid-bf16", seed=4)
    ctx = _ctx(case)
    gi = gpu_inputs(ctx, case)
    out = ctx._round_bufs(case.B)
    ctx.spec_graph_enable(True)
    for _ in range(3):
        _round(ctx, case, gi, out, -1.0, case.n_ctx)
    # a replay that could run past the cache is refused on the host, before anything is launched
    K = case.rc.K
    _reset(ctx, case, case.rc.max_ctx - K)               # room for the K draft rows but not for the K+1 target rows
    with pytest.raises(binding.FardError) as e:
        ctx.spec_round(gi["pending"], gi["eps"], gi["r"], -1.0, out=out)
    assert "FARD_ECAPACITY" in str(e.value)
    # two rounds in a row without a reset: the host bound of the lengths advances on replays too
    _reset(ctx, case, case.rc.max_ctx - 2 * (K + 1) + 1)
    ctx.spec_round(gi["pending"], gi["eps"], gi["r"], -1.0, out=out)
    with pytest.raises(binding.FardError):
        ctx.spec_round(gi["pending"], gi["eps"], gi["r"], -1.0, out=out)
    ctx.sync()
    ctx.close()


def test_graph_needs_a_stream_of_its_own():
    from paper_2512_08537_amd import binding
    case = build_case("ln-gelu-bf16", seed=2)
    ctx = _ctx(case, with_stream=False)
    with pytest.raises(binding.FardError) as e:
        ctx.spec_graph_enable(True)
    assert "FARD_ESTATE" in str(e.value)
    ctx.close()
