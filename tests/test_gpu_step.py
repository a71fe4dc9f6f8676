"""Parity of fc_denoise_step / fc_denoise_resume (through the C ABI) against the CPU
oracle on the seeded workloads, plus API error paths and the resume invariants the
paper states (a hit runs the same step function, only later: Sec. 2.2, Sec. 3.2)."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import dit, sampler
from paper_2501_04012_amd import synth
from util import cached_weights, dev, host, max_abs, record, rel_l2, run_step_gpu

pytestmark = pytest.mark.gpu

# tolerances of the parity bar: bf16 rel-L2 <= 1e-2 and max-abs <= 5e-2 per step; fp32 rel-L2 <= 1e-4
BF16_REL, BF16_ABS, F32_REL = 1e-2, 5e-2, 1e-4


def oracle_step(w, cfg, W, inputs, step, dtype=np.float64):
    lat, cond, null = inputs
    return sampler.denoise_step(cfg, W, lat, cond, null, w.schedule, step, dtype=dtype, return_eps=True)


def check(got_lat, got_eps, want_lat, want_eps, bf16):
    rl, re_ = rel_l2(got_lat, want_lat), rel_l2(got_eps, want_eps)
    ma = max_abs(got_lat, want_lat)
    record(latent_rel_l2=rl, latent_max_abs=ma, eps_rel_l2=re_)
    if bf16:
        assert rl <= BF16_REL and ma <= BF16_ABS, (rl, ma, re_)
        assert re_ <= 2e-2, re_          # the noise estimate itself, not diluted by the latent
    else:
        assert rl <= F32_REL and re_ <= F32_REL, (rl, re_)


@pytest.mark.parametrize("name", ["cfg1", "cfg3b"])
def test_tiny_fp32_configs(fc, name):
    w = synth.WORKLOADS[name]
    W = synth.make_weights(w.model, w.weight_seed)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, w.model, W, inputs, w.step)
    check(*got, *want, bf16=False)


@pytest.mark.parametrize("mode", [synth.ATTN_FACTORIZED_CROSS, synth.ATTN_FULL3D_CONCAT])
@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
def test_small_ragged_model_with_sharp_softmax(fc, mode, dtype):
    """A small model whose token counts are not multiples of any tile, weights large
    enough that softmax rows are peaked, guidance on, two requests."""
    cfg = synth.ModelConfig(frames=3, height=12, width=20, channels=4, patch=2, hidden=256, heads=4, mlp_dim=512,
                            depth=2, text_len=26, text_dim=96, attn_mode=mode, dtype=dtype)
    w = synth.Workload("small", cfg, weight_seed=7, latent_seed=8, text_seed=9, null_seed=10, requests=2)
    W = synth.make_weights(cfg, 7, std=0.08)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, cfg, W, inputs, w.step)
    check(*got, *want, bf16=dtype == synth.DT_BF16)


@pytest.mark.parametrize("frames", [16, 17, 32, 37, 64])
def test_small_factorized_model_frame_counts(fc, frames):
    """Temporal attention over up to 64 frames (one, two or four 16-token blocks per
    sequence in the matrix-core kernel, ragged last block), bf16, guidance, two requests."""
    cfg = synth.ModelConfig(frames=frames, height=8, width=12, channels=4, patch=2, hidden=256, heads=4, mlp_dim=512,
                            depth=1, text_len=26, text_dim=96, attn_mode=synth.ATTN_FACTORIZED_CROSS,
                            dtype=synth.DT_BF16)
    w = synth.Workload("frames", cfg, weight_seed=27, latent_seed=28, text_seed=29, null_seed=30, requests=2)
    W = synth.make_weights(cfg, 27, std=0.08)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, cfg, W, inputs, w.step)
    check(*got, *want, bf16=True)


@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
def test_small_model_with_16_latent_channels(fc, dtype):
    """2x2 patches of 16 channels (patch features K = 64, the shape of the full-3D
    configuration's patch embedding), ragged spatial size, guidance, two requests."""
    cfg = synth.ModelConfig(frames=3, height=12, width=20, channels=16, patch=2, hidden=256, heads=4, mlp_dim=512,
                            depth=1, text_len=26, text_dim=96, attn_mode=synth.ATTN_FULL3D_CONCAT, dtype=dtype)
    w = synth.Workload("small16", cfg, weight_seed=17, latent_seed=18, text_seed=19, null_seed=20, requests=2)
    W = synth.make_weights(cfg, 17, std=0.05)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, cfg, W, inputs, w.step)
    check(*got, *want, bf16=dtype == synth.DT_BF16)


@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
def test_small_full3d_model_with_separate_text_modulation(fc, dtype):
    """Variant: the text rows of the full-3D sequence are modulated and gated by their own
    vectors (12 chunks per block).  Two blocks so that the text rows' gated updates feed the
    video rows through the second attention; modulation weights large enough that the two
    sets differ visibly; ragged sizes, guidance, two requests."""
    cfg = synth.ModelConfig(frames=3, height=12, width=20, channels=4, patch=2, hidden=256, heads=4, mlp_dim=512,
                            depth=2, text_len=26, text_dim=96, attn_mode=synth.ATTN_FULL3D_CONCAT, dtype=dtype,
                            text_adaln=1)
    w = synth.Workload("small_text_adaln", cfg, weight_seed=37, latent_seed=38, text_seed=39, null_seed=40, requests=2)
    W = synth.make_weights(cfg, 37, std=0.08)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, cfg, W, inputs, w.step)
    check(*got, *want, bf16=dtype == synth.DT_BF16)
    # the variant is live: giving the text rows the video rows' vectors changes the result
    W_same = dict(W)
    for l in range(cfg.depth):
        for n in ("mod_w", "mod_b"):
            a = W[f"blk{l}.{n}"]
            half = a.shape[-1] // 2
            W_same[f"blk{l}.{n}"] = np.concatenate([a[..., :half], a[..., :half]], axis=-1)
    other = oracle_step(w, cfg, W_same, inputs, w.step)
    assert rel_l2(other[1], want[1]) > 10 * (2e-2 if dtype == synth.DT_BF16 else F32_REL)


@pytest.mark.parametrize("case", ["one_frame_one_text_token", "one_spatial_token", "full3d_two_tokens"])
@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
def test_degenerate_sequence_lengths(fc, case, dtype):
    """Sequences of length one: a softmax over a single key returns that key's value, so the
    temporal (one frame), spatial (one patch per frame) and cross (one text token) branches
    reduce to linear maps; the full-3D case attends over two tokens.  Guidance, three
    requests (an odd batch)."""
    shape = {"one_frame_one_text_token": dict(frames=1, height=8, width=12, text_len=1,
                                              attn_mode=synth.ATTN_FACTORIZED_CROSS),
             "one_spatial_token": dict(frames=5, height=2, width=2, text_len=3,
                                       attn_mode=synth.ATTN_FACTORIZED_CROSS),
             "full3d_two_tokens": dict(frames=1, height=2, width=2, text_len=1,
                                       attn_mode=synth.ATTN_FULL3D_CONCAT)}[case]
    cfg = synth.ModelConfig(channels=4, patch=2, hidden=256, heads=4, mlp_dim=512, depth=2, text_dim=96, dtype=dtype,
                            **shape)
    w = synth.Workload("degenerate", cfg, weight_seed=57, latent_seed=58, text_seed=59, null_seed=60, requests=3)
    W = synth.make_weights(cfg, 57, std=0.08)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, cfg, W, inputs, w.step)
    check(*got, *want, bf16=dtype == synth.DT_BF16)


def test_library_weight_counts_match_the_specification(fc):
    tiny = synth.WORKLOADS["cfg1"].model
    for cfg in (tiny, replace(tiny, attn_mode=synth.ATTN_FULL3D_CONCAT),
                replace(tiny, attn_mode=synth.ATTN_FULL3D_CONCAT, text_adaln=1)):
        m = fc.fc_model_create(cfg)
        try:
            assert fc.fc_model_weight_count(m) == synth.weight_count(cfg)
        finally:
            fc.fc_model_destroy(m)


def test_cfg2_bf16_factorized_block(fc):
    w = synth.WORKLOADS["cfg2"]
    W = synth.make_weights(w.model, w.weight_seed)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, w.model, W, inputs, w.step)
    check(*got, *want, bf16=True)


def test_cfg6_paper_shaped_latent_factorized_block(fc):
    """The latent shape the paper states for its model (64 x 40 x 64 x 4: 40 960 tokens,
    spatial sequences of 640 tokens, temporal ones of 64), one factorized bf16 block,
    against the fp32 oracle."""
    w = synth.WORKLOADS["cfg6"]
    W = synth.make_weights(w.model, w.weight_seed)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, w.model, W, inputs, w.step, dtype=np.float32)
    check(*got, *want, bf16=True)


def test_cfg4_bf16_full3d_block_every_row(fc):
    """Full-size full-3D block, the configuration the benchmark times, in the launch
    configuration it times: every one of the 17 550 output rows of the noise estimate and of
    the updated latent against the float32 oracle; then a sample of rows (random ones, the
    first and last row, the last row of the last full 512-row query tile and the first of the
    ragged one) against the oracle in float64, which separates the kernel's error from the
    float32 oracle's own."""
    w = synth.WORKLOADS["cfg4"]
    cfg = w.model
    W = synth.make_weights(cfg, w.weight_seed)
    inputs = synth.workload_inputs(w)
    lat, cond, _ = inputs
    got_lat, got_eps = run_step_gpu(fc, w, weights=W, inputs=inputs)
    assert np.isfinite(got_eps).all() and np.isfinite(got_lat).all()
    t, a_t, a_p = sampler.step_coefficients(w.schedule, w.step)

    want_eps = dit.forward(cfg, W, lat[0], cond[0], t, dtype=np.float32)
    want_lat = sampler.ddim_update(lat[0].astype(np.float64), want_eps.astype(np.float64), a_t, a_p)
    check(got_lat[0], got_eps[0], want_lat, want_eps, bf16=True)
    # per-row: no single token row is off (a mis-scattered or stale tile would be)
    ge, we = dit.patchify(got_eps[0], cfg.patch).astype(np.float64), dit.patchify(want_eps, cfg.patch).astype(np.float64)
    row_rel = np.linalg.norm(ge - we, axis=1) / np.linalg.norm(we, axis=1)
    record(worst_row_eps_rel_l2=float(row_rel.max()))
    assert row_rel.max() <= 5e-2, (int(row_rel.argmax()), float(row_rel.max()))

    rows = np.random.default_rng(0).choice(cfg.video_tokens, size=96, replace=False)
    ragged_start = (cfg.text_len + cfg.video_tokens) // 512 * 512 - cfg.text_len     # first video row of the last query tile
    rows = np.concatenate([rows, [0, cfg.video_tokens - 1, ragged_start - 1, ragged_start, 17549 - 45]])
    want = dit.forward(cfg, W, lat[0], cond[0], t, dtype=np.float64, video_rows=rows)
    got = ge[rows]
    record(sampled_eps_rel_l2=rel_l2(got, want), sampled_eps_max_abs=max_abs(got, want),
           f32_oracle_vs_f64_rel_l2=rel_l2(we[rows], want))
    assert rel_l2(got, want) <= 2e-2, rel_l2(got, want)
    assert max_abs(got, want) <= BF16_ABS
    want_l = sampler.ddim_update(dit.patchify(lat[0].astype(np.float64), cfg.patch)[rows], want, a_t, a_p)
    got_l = dit.patchify(got_lat[0], cfg.patch)[rows]
    record(sampled_latent_rel_l2=rel_l2(got_l, want_l), sampled_latent_max_abs=max_abs(got_l, want_l))
    assert rel_l2(got_l, want_l) <= BF16_REL and max_abs(got_l, want_l) <= BF16_ABS


def test_cfg3a_bf16_stack_depth4_with_guidance(fc):
    w = synth.WORKLOADS["cfg3a"]
    cfg = replace(w.model, depth=4)
    W = synth.make_weights(cfg, w.weight_seed)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, depth=4, weights=W, inputs=inputs)
    want = oracle_step(w, cfg, W, inputs, w.step, dtype=np.float32)
    check(*got, *want, bf16=True)


def test_cfg3a_bf16_full_28_block_stack_with_guidance(fc):
    """The full-size stacked configuration, one guided step, against the fp32 oracle."""
    w = synth.WORKLOADS["cfg3a"]
    W = cached_weights(w.model, w.weight_seed)
    inputs = synth.workload_inputs(w)
    got = run_step_gpu(fc, w, weights=W, inputs=inputs)
    want = oracle_step(w, w.model, W, inputs, w.step, dtype=np.float32)
    check(*got, *want, bf16=True)


def test_cfg5a_resume_steps_teacher_forced(fc):
    """Cache-hit resume at full size (4 requests x guidance pair, 28 blocks), per-step parity:
    the first remaining step after k = 10 and after k = 20, a middle one of each range and
    the last step (abar_prev = 1).  Each time all four requests run on the GPU in one batch
    and one of them (every request at least once) is checked against the fp32 oracle fed the
    same latent.  The step function does not depend on where the resume started, so the last
    step is checked once for both ranges."""
    w = synth.WORKLOADS["cfg5a"]
    W = cached_weights(w.model, w.weight_seed)
    lat, cond, null = synth.workload_inputs(w)
    for step, r in ((11, 0), (30, 1), (50, 2), (21, 3), (35, 0)):
        got_lat, got_eps = run_step_gpu(fc, w, step=step, weights=W, inputs=(lat, cond, null))
        assert np.isfinite(got_lat).all() and np.isfinite(got_eps).all()
        want_lat, want_eps = sampler.denoise_step(w.model, W, lat[r:r + 1], cond[r:r + 1], null, w.schedule, step,
                                                  dtype=np.float32, return_eps=True)
        record(step=float(step), request=float(r))
        check(got_lat[r:r + 1], got_eps[r:r + 1], want_lat, want_eps, bf16=True)


def test_cfg5a_resume_runs_the_remaining_steps(fc):
    """fc_denoise_resume at full size: k = 48 leaves two steps; it must equal two single
    steps bit for bit (same kernels, same order), and k = N must leave the latent alone."""
    import torch
    w = synth.WORKLOADS["cfg5a"]
    W = cached_weights(w.model, w.weight_seed)
    lat, cond, null = synth.workload_inputs(w)
    den = fc.Denoiser(w.model, W, w.requests, True)
    try:
        d_cond, d_null = dev(cond), dev(null)
        a, b = dev(lat), dev(lat)
        den.resume(a, d_cond, d_null, w.schedule, 48)
        den.step(b, d_cond, d_null, w.schedule, 49)
        den.step(b, d_cond, d_null, w.schedule, 50)
        torch.cuda.synchronize()
        assert torch.equal(a, b)
        assert torch.isfinite(a).all()
        c = dev(lat)
        den.resume(c, d_cond, d_null, w.schedule, 50)
        torch.cuda.synchronize()
        assert np.array_equal(host(c), lat)
    finally:
        den.close()


def test_cfg5b_resume_trajectory_and_invariants(fc):
    import torch
    w = synth.WORKLOADS["cfg5b"]
    cfg = w.model
    W = synth.make_weights(cfg, w.weight_seed)
    lat, cond, null = synth.workload_inputs(w)
    den = fc.Denoiser(cfg, W, w.requests, True)
    try:
        d_cond, d_null = dev(cond), dev(null)
        finals = {}
        for k in w.resume_k:
            d_lat = dev(lat)
            den.resume(d_lat, d_cond, d_null, w.schedule, k)
            torch.cuda.synchronize()
            finals[k] = host(d_lat)
            want = sampler.denoise_resume(cfg, W, lat, cond, null, w.schedule, k)
            record(resume_from=float(k), final_latent_rel_l2=rel_l2(finals[k], want))
            assert rel_l2(finals[k], want) <= 1e-3, (k, rel_l2(finals[k], want))
        # a hit at k followed by single steps == one resume call, bit for bit
        d_lat = dev(lat)
        for s in range(11, 21):
            den.step(d_lat, d_cond, d_null, w.schedule, s)
        den.resume(d_lat, d_cond, d_null, w.schedule, 20)
        torch.cuda.synchronize()
        d_ref = dev(lat)
        den.resume(d_ref, d_cond, d_null, w.schedule, 10)
        torch.cuda.synchronize()
        assert torch.equal(d_lat, d_ref)
        # run-to-run determinism
        assert np.array_equal(host(d_ref), finals[10])
        # k = N: untouched
        d_lat = dev(lat)
        den.resume(d_lat, d_cond, d_null, w.schedule, 50)
        torch.cuda.synchronize()
        assert np.array_equal(host(d_lat), lat)
    finally:
        den.close()


def test_flow_euler_variant_step_and_resume(fc):
    """The second step function (Euler step of a rectified-flow sampler): one step of the
    tiny fp32 configuration and of the bf16 factorized block, and a free-running tiny
    resume, against the oracle."""
    import torch
    for name, bf in (("cfg1", False), ("cfg2", True)):
        w = synth.WORKLOADS[name]
        w = replace(w, schedule=replace(w.schedule, sampler=synth.SAMPLER_FLOW_EULER))
        W = synth.make_weights(w.model, w.weight_seed)
        inputs = synth.workload_inputs(w)
        got = run_step_gpu(fc, w, weights=W, inputs=inputs)
        want = oracle_step(w, w.model, W, inputs, w.step)
        check(*got, *want, bf16=bf)
    w = synth.WORKLOADS["cfg5b"]
    sched = replace(w.schedule, sampler=synth.SAMPLER_FLOW_EULER)
    W = synth.make_weights(w.model, w.weight_seed)
    lat, cond, null = synth.workload_inputs(w)
    den = fc.Denoiser(w.model, W, w.requests, True)
    try:
        d_lat = dev(lat)
        den.resume(d_lat, dev(cond), dev(null), sched, 30)
        torch.cuda.synchronize()
        want = sampler.denoise_resume(w.model, W, lat, cond, null, sched, 30)
        record(final_latent_rel_l2=rel_l2(host(d_lat), want))
        assert rel_l2(host(d_lat), want) <= 1e-3
    finally:
        den.close()


def test_stochastic_ddim_with_counter_noise(fc):
    """eta > 0: the noise is a function of (seed, request, step, element), so the GPU step
    must reproduce the oracle's step to fp32 accuracy, per request, for the tiny
    configuration with two requests and guidance; another seed gives another latent; the
    last step draws nothing; a free-running resume stays on the oracle's trajectory."""
    import torch
    w = synth.WORKLOADS["cfg5b"]
    cfg = w.model
    W = synth.make_weights(cfg, w.weight_seed)
    lat, cond, null = synth.workload_inputs(w)
    sched = replace(w.schedule, eta=0.6, seed=(7 << 32) + 12345)
    den = fc.Denoiser(cfg, W, w.requests, True)
    try:
        d_cond, d_null = dev(cond), dev(null)
        for step in (1, 26, 49):
            d_lat = dev(lat)
            den.step(d_lat, d_cond, d_null, sched, step)
            torch.cuda.synchronize()
            want = sampler.denoise_step(cfg, W, lat, cond, null, sched, step)
            got = host(d_lat)
            record(step=float(step), latent_rel_l2=rel_l2(got, want), latent_max_abs=max_abs(got, want))
            assert rel_l2(got, want) <= F32_REL
            # the noise matters at this eta: the deterministic step is somewhere else
            assert rel_l2(sampler.denoise_step(cfg, W, lat, cond, null, replace(sched, eta=0.0), step), want) > 1e-3
        a, b = dev(lat), dev(lat)
        den.step(a, d_cond, d_null, sched, 26)
        den.step(b, d_cond, d_null, replace(sched, seed=sched.seed + 1), 26)
        c, d = dev(lat), dev(lat)
        den.step(c, d_cond, d_null, sched, 50)                     # abar_prev = 1: sigma = 0
        den.step(d, d_cond, d_null, replace(sched, eta=0.0), 50)
        torch.cuda.synchronize()
        assert not torch.equal(a, b) and torch.equal(c, d)
        x = dev(lat)
        den.resume(x, d_cond, d_null, sched, 40)
        torch.cuda.synchronize()
        want = sampler.denoise_resume(cfg, W, lat, cond, null, sched, 40)
        record(final_latent_rel_l2=rel_l2(host(x), want))
        assert rel_l2(host(x), want) <= 1e-3
    finally:
        den.close()


def test_api_errors(fc):
    import torch
    w = synth.WORKLOADS["cfg1"]
    cfg = w.model
    with pytest.raises(fc.FlexDenoiseError) as e:
        fc.fc_model_create(replace(cfg, heads=5))
    assert e.value.status == -2
    with pytest.raises(fc.FlexDenoiseError) as e:
        fc.fc_model_create(replace(cfg, height=7))
    assert e.value.status == -2
    m = fc.fc_model_create(cfg)
    try:
        lat, cond, _ = synth.workload_inputs(w)
        d_lat, d_cond = dev(lat), dev(cond)
        ws = torch.empty(fc.fc_workspace_bytes(m, 1, False), dtype=torch.uint8, device="cuda:0")
        with pytest.raises(fc.FlexDenoiseError) as e:          # weights not set
            fc.fc_denoise_step(m, d_lat, d_cond, None, w.schedule, 25, 1, None, ws)
        assert e.value.status == -7
        with pytest.raises(fc.FlexDenoiseError) as e:
            fc.fc_model_set_weights(m, np.zeros(10, dtype=np.float32))
        assert e.value.status == -2
        fc.fc_model_set_weights(m, synth.pack_weights(cfg, synth.make_weights(cfg, w.weight_seed)))
        for bad_step in (0, 51):
            with pytest.raises(fc.FlexDenoiseError) as e:
                fc.fc_denoise_step(m, d_lat, d_cond, None, w.schedule, bad_step, 1, None, ws)
            assert e.value.status == -3
        with pytest.raises(fc.FlexDenoiseError) as e:
            fc.fc_denoise_resume(m, d_lat, d_cond, None, w.schedule, 51, 1, ws)
        assert e.value.status == -3
        with pytest.raises(fc.FlexDenoiseError) as e:
            fc.fc_denoise_step(m, d_lat, d_cond, None, w.schedule, 25, 1, None, ws[:1024])
        assert e.value.status == -4
        with pytest.raises(fc.FlexDenoiseError) as e:
            fc.fc_denoise_step(m, None, d_cond, None, w.schedule, 25, 1, None, ws)
        assert e.value.status == -1
        with pytest.raises(fc.FlexDenoiseError) as e:
            fc.fc_denoise_step(m, d_lat, d_cond, None, replace(w.schedule, eta=1.5), 25, 1, None, ws)
        assert e.value.status == -3
        with pytest.raises(fc.FlexDenoiseError) as e:
            fc.fc_denoise_step(m, d_lat, d_cond, None,
                               replace(w.schedule, eta=0.5, sampler=synth.SAMPLER_FLOW_EULER), 25, 1, None, ws)
        assert e.value.status == -6
        torch.cuda.synchronize()
        assert np.array_equal(host(d_lat), lat)               # no failed call touched the latent
    finally:
        fc.fc_model_destroy(m)
    # a narrow model with very many tokens: the batch at which the row-index arithmetic of the
    # scatter epilogues would stop being exact is refused (before anything is launched)
    wide = replace(cfg, frames=64, height=40, width=64)       # 40 960 tokens of width 64
    m = fc.fc_model_create(wide)
    try:
        fc.fc_model_set_weights(m, synth.pack_weights(wide, synth.make_weights(wide, 1)))
        ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
        with pytest.raises(fc.FlexDenoiseError) as e:
            fc.fc_denoise_step(m, d_lat, d_cond, None, w.schedule, 25, 700, None, ws)
        assert e.value.status == -3
        with pytest.raises(fc.FlexDenoiseError) as e:         # a batch that is fine: only the workspace is short
            fc.fc_denoise_step(m, d_lat, d_cond, None, w.schedule, 25, 600, None, ws)
        assert e.value.status == -4
    finally:
        fc.fc_model_destroy(m)
