"""Parity of the cache-restore entry points (through the C ABI) against oracle/cache.py:
stitching is a selection (bit-exact), expansion is one fused multiply-add per element,
the reductions are compared at double-sum accuracy; plus fc_denoise_resume_ex."""
import numpy as np
import pytest

from oracle import cache as ocache
from oracle import sampler
from paper_2501_04012_amd import synth
from util import dev, host, record, rel_l2

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


# --------------------------------------------------------------------------- stitching

@pytest.mark.parametrize("shape", [(1, 1, 1, 4), (3, 5, 7, 4), (16, 32, 32, 4), (64, 40, 64, 4), (13, 60, 90, 16),
                                   (2, 9, 11, 3)])      # the last: channels not a multiple of 4 (scalar path)
@pytest.mark.parametrize("with_bg_mask", [True, False])
def test_stitch_is_bit_exact(fc, shape, with_bg_mask):
    torch = _torch()
    rng = np.random.default_rng(sum(shape))
    xo = rng.standard_normal(shape).astype(np.float32)
    xb = rng.standard_normal(shape).astype(np.float32)
    pixels = int(np.prod(shape[:-1]))
    mo = ocache.pack_mask(rng.random(pixels) < 0.4)
    mb = ocache.pack_mask(rng.random(pixels) < 0.8) if with_bg_mask else None
    want = ocache.stitch(xo, xb, mo, mb)
    out = torch.full(shape, float("nan"), device="cuda:0")
    fc.fc_cache_stitch(dev(xo), dev(xb), dev(mo), dev(mb) if with_bg_mask else None, out, pixels, shape[-1])
    torch.cuda.synchronize()
    assert np.array_equal(host(out), want)


def test_stitch_in_place_and_degenerate_masks(fc):
    torch = _torch()
    rng = np.random.default_rng(5)
    shape = (4, 8, 8, 4)
    xo, xb = rng.standard_normal(shape).astype(np.float32), rng.standard_normal(shape).astype(np.float32)
    pixels = 4 * 8 * 8
    ones, zeros = ocache.pack_mask(np.ones(pixels, bool)), ocache.pack_mask(np.zeros(pixels, bool))
    for mo, mb, want in ((ones, ones, xo), (zeros, ones, xb), (zeros, zeros, xo)):
        d_bg = dev(xb)
        fc.fc_cache_stitch(dev(xo), d_bg, dev(mo), dev(mb), d_bg, pixels, 4)      # out is x_bg itself
        torch.cuda.synchronize()
        assert np.array_equal(host(d_bg), want)
    fc.fc_cache_stitch(dev(xo), dev(xb), dev(ones), None, dev(xb), 0, 4)          # empty: nothing happens
    with pytest.raises(fc.FlexDenoiseError) as e:
        fc.fc_cache_stitch(dev(xo), dev(xb), None, None, dev(xb), pixels, 4)
    assert e.value.status == -1


# --------------------------------------------------------------------------- expanding an entry

@pytest.mark.parametrize("T,H,W,C,n_base,n_extra", [(16, 32, 32, 4, 3, 2), (64, 40, 64, 4, 5, 7), (5, 3, 3, 1, 1, 0),
                                                    (13, 60, 90, 16, 4, 1)])
def test_decompress_against_oracle(fc, T, H, W, C, n_base, n_extra):
    torch = _torch()
    rng = np.random.default_rng(T + n_base)
    F = H * W * C
    first = rng.standard_normal((H, W, C)).astype(np.float32)
    diff = rng.standard_normal((n_base, H, W, C)).astype(np.float32)
    extra = rng.standard_normal((max(n_extra, 1), H, W, C)).astype(np.float32)
    alpha = np.float32(0.8125)
    src = rng.integers(-n_extra, n_base + 1, size=T)
    src[0] = 0
    want = ocache.decompress(first.astype(np.float64), diff.astype(np.float64), float(alpha), extra.astype(np.float64), src)
    out = torch.full((T, H, W, C), float("nan"), device="cuda:0")
    fc.fc_cache_decompress(dev(first), dev(diff), n_base, float(alpha), dev(extra) if n_extra else None, n_extra, src,
                           T, F, out)
    torch.cuda.synchronize()
    got = host(out)
    # copies are exact; a restored key frame is one fp32 multiply-add (fused or not) of fp32 inputs
    copied = np.isin(src, [0]) | (src < 0)
    assert np.array_equal(got[copied], want[copied].astype(np.float32))
    np.testing.assert_allclose(got, want, rtol=0, atol=2.0 ** -22 * 8)
    record(max_abs=float(np.abs(got - want).max()))


def test_decompress_errors(fc):
    first = dev(np.zeros((2, 2, 1), np.float32))
    out = dev(np.zeros((3, 2, 2, 1), np.float32))
    with pytest.raises(fc.FlexDenoiseError) as e:
        fc.fc_cache_decompress(first, first, 1, 1.0, None, 0, [0, 2, 0], 3, 4, out)     # code 2 > n_base
    assert e.value.status == -3
    with pytest.raises(fc.FlexDenoiseError) as e:
        fc.fc_cache_decompress(first, first, 1, 1.0, None, 0, [0, -1, 0], 3, 4, out)    # no extra frames
    assert e.value.status == -3
    with pytest.raises(fc.FlexDenoiseError) as e:
        fc.fc_cache_decompress(first, first, 1, 1.0, None, 0, [0] * 300, 300, 4, out)
    assert e.value.status == -6


# --------------------------------------------------------------------------- the compressing side's reductions

@pytest.mark.parametrize("n_base,H,W,C", [(1, 3, 3, 1), (3, 32, 32, 4), (7, 40, 64, 4), (2, 60, 90, 16)])
def test_alpha_against_oracle_and_repeatable(fc, n_base, H, W, C):
    torch = _torch()
    rng = np.random.default_rng(n_base * H)
    first = rng.standard_normal((H, W, C)).astype(np.float32)
    diff = rng.standard_normal((n_base, H, W, C)).astype(np.float32)
    keys = (first[None] + 0.6 * diff + 0.2 * rng.standard_normal(diff.shape)).astype(np.float32)
    want = ocache.alpha_least_squares(first, keys, diff)
    ws = torch.empty(fc.fc_cache_workspace_bytes(0), dtype=torch.uint8, device="cuda:0")
    a1, a2 = torch.zeros(1, device="cuda:0"), torch.zeros(1, device="cuda:0")
    fc.fc_cache_alpha(dev(first), dev(keys), dev(diff), n_base, H * W * C, a1, ws)
    fc.fc_cache_alpha(dev(first), dev(keys), dev(diff), n_base, H * W * C, a2, ws)
    torch.cuda.synchronize()
    assert abs(float(a1) - want) <= 2.0 ** -23 * abs(want) * 2
    assert float(a1) == float(a2)
    record(alpha_rel_err=abs(float(a1) - want) / abs(want))


def test_alpha_of_a_motionless_base_is_zero(fc):
    """Diff_base = 0 (the common key frames repeat the first frame): Eq. 2 is 0/0; both sides
    define alpha = 0 and nothing non-finite reaches the latent."""
    torch = _torch()
    rng = np.random.default_rng(3)
    first = rng.standard_normal((8, 8, 4)).astype(np.float32)
    keys = rng.standard_normal((2, 8, 8, 4)).astype(np.float32)
    diff = np.zeros((2, 8, 8, 4), dtype=np.float32)
    ws = torch.empty(fc.fc_cache_workspace_bytes(0), dtype=torch.uint8, device="cuda:0")
    a = torch.full((1,), float("nan"), device="cuda:0")
    fc.fc_cache_alpha(dev(first), dev(keys), dev(diff), 2, 8 * 8 * 4, a, ws)
    torch.cuda.synchronize()
    assert float(a) == ocache.alpha_least_squares(first, keys, diff) == 0.0


@pytest.mark.parametrize("T,H,W,C", [(1, 4, 4, 4), (16, 32, 32, 4), (64, 40, 64, 4), (13, 60, 90, 16)])
def test_frame_similarity_and_key_frames(fc, T, H, W, C):
    torch = _torch()
    rng = np.random.default_rng(T)
    base = rng.standard_normal((4, H, W, C))
    frames = np.stack([base[rng.integers(4)] + 0.05 * rng.standard_normal((H, W, C)) for _ in range(T)]).astype(np.float32)
    want = ocache.frame_similarity(frames)
    sim = torch.full((T, T), float("nan"), device="cuda:0")
    ws = torch.empty(fc.fc_cache_workspace_bytes(T), dtype=torch.uint8, device="cuda:0")
    fc.fc_cache_frame_similarity(dev(frames), T, H * W * C, sim, ws)
    torch.cuda.synchronize()
    got = host(sim)
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-7)
    assert np.array_equal(got, got.T)
    # the decision taken from it: same key frames as the oracle (similarities of this input sit
    # near 0.9975 inside a group and near 0 across groups, far from the 0.99 threshold)
    assert np.array_equal(fc.fc_cache_select_key_frames(got, 0.99), ocache.select_key_frames(want, 0.99))


# --------------------------------------------------------------------------- compress -> restore -> stitch -> resume

def test_entry_round_trip_feeds_a_resume(fc):
    """A latent whose frames are multiples of one pattern away from its first frame is
    restored exactly (up to fp32 rounding) from first frame + alpha * base, stitched with
    a second cache, and resumed; the result equals resuming the oracle's stitched latent."""
    torch = _torch()
    w = synth.WORKLOADS["cfg5b"]
    cfg = w.model
    W = synth.make_weights(cfg, w.weight_seed)
    lat, cond, null = synth.workload_inputs(w)
    T, H, Wd, C = lat.shape[1:]
    rng = np.random.default_rng(77)
    base_step = lat[0]                                     # the "base" step of the entry
    diff_base = (base_step[1:] - base_step[0]).astype(np.float32)
    first_s = lat[1][0]
    keys_s = (first_s[None] + np.float32(0.75) * diff_base).astype(np.float32)    # step s = multiple of the base
    ws = torch.empty(fc.fc_cache_workspace_bytes(T), dtype=torch.uint8, device="cuda:0")
    a = torch.zeros(1, device="cuda:0")
    fc.fc_cache_alpha(dev(first_s), dev(keys_s), dev(diff_base), T - 1, H * Wd * C, a, ws)
    torch.cuda.synchronize()
    alpha = float(a)
    assert abs(alpha - 0.75) < 1e-6
    x_obj = torch.empty((T, H, Wd, C), device="cuda:0")
    fc.fc_cache_decompress(dev(first_s), dev(diff_base), T - 1, alpha, None, 0, list(range(T)), T, H * Wd * C, x_obj)
    x_bg = dev(lat[2])
    mo = ocache.pack_mask(rng.random(T * H * Wd) < 0.5)
    x = torch.empty((1, T, H, Wd, C), device="cuda:0")
    fc.fc_cache_stitch(x_obj, x_bg, dev(mo), None, x, T * H * Wd, C)
    torch.cuda.synchronize()
    want_alpha = ocache.alpha_least_squares(first_s, keys_s, diff_base)      # the oracle's own coefficient
    assert abs(alpha - want_alpha) <= 2.0 ** -22 * abs(want_alpha)
    want_obj = ocache.decompress(first_s.astype(np.float64), diff_base.astype(np.float64), want_alpha, None,
                                 list(range(T)))
    want_x = ocache.stitch(want_obj, lat[2].astype(np.float64), mo)[None]
    assert rel_l2(host(x), want_x) < 1e-6
    den = fc.Denoiser(cfg, W, 1, True)
    try:
        k = 45
        den.resume(x, dev(cond[:1]), dev(null), w.schedule, k)
        torch.cuda.synchronize()
        want = sampler.denoise_resume(cfg, W, want_x, cond[:1], null, w.schedule, k)
        assert rel_l2(host(x), want) < 1e-3
    finally:
        den.close()


# --------------------------------------------------------------------------- resume with key-step export

def test_resume_ex_exports_the_key_steps(fc):
    """Hit at step 10 of the tiny configuration: the latents after steps 15, 20 and 25 are
    handed out; each equals a resume that stops there (same kernels, same order: bit for
    bit) and the latent the oracle's loop holds after that step, and the final latent equals
    the plain resume."""
    torch = _torch()
    w = synth.WORKLOADS["cfg5b"]
    cfg = w.model
    W = synth.make_weights(cfg, w.weight_seed)
    lat, cond, null = synth.workload_inputs(w)
    den = fc.Denoiser(cfg, W, w.requests, True)
    try:
        d_cond, d_null = dev(cond), dev(null)
        a = dev(lat)
        exports = [torch.full_like(a, float("nan")) for _ in range(3)]
        den.resume_ex(a, d_cond, d_null, w.schedule, 10, [15, 20, 25], exports)
        b = dev(lat)
        den.resume(b, d_cond, d_null, w.schedule, 10)
        torch.cuda.synchronize()
        assert torch.equal(a, b)
        c = dev(lat)
        for s in range(11, 26):
            den.step(c, d_cond, d_null, w.schedule, s)
            if s in (15, 20, 25):
                torch.cuda.synchronize()
                assert torch.equal(exports[(s - 15) // 5], c), s
        # the exported latents are the ones the oracle's loop passes through after those steps
        # (free-running from the same stored latents; Sec. 4.2.4: these are what gets inserted)
        seen = {}
        want_final = sampler.denoise_resume(cfg, W, lat, cond, null, w.schedule, 10,
                                            on_step=lambda s, x: seen.__setitem__(s, np.array(x)))
        for e, s in enumerate((15, 20, 25)):
            err = rel_l2(host(exports[e]), seen[s])
            record(step=float(s), exported_latent_rel_l2=err)
            assert err <= 1e-3, (s, err)
        assert rel_l2(host(a), want_final) <= 1e-3
        # argument checks
        for steps in ([10], [51], [20, 15], [15, 15]):
            with pytest.raises(fc.FlexDenoiseError) as e:
                den.resume_ex(dev(lat), d_cond, d_null, w.schedule, 10, steps, exports[:len(steps)])
            assert e.value.status == -3
    finally:
        den.close()
