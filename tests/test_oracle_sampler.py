"""Pins of the sampler oracle (oracle/sampler.py): schedule closed forms, the DDIM
update for a known noise, guidance special cases and the resume semantics the
paper states (Sec. 2.2, Sec. 3.2 'Cache lookup', Sec. 4.2.2)."""
import math
from dataclasses import replace

import numpy as np
import pytest

from oracle import sampler
from paper_2501_04012_amd import synth

SCHED = synth.Schedule()


def test_alphas_cumprod_closed_form_and_shape():
    ab = sampler.alphas_cumprod(1000, 1e-4, 2e-2)
    assert ab.shape == (1000,) and ab.dtype == np.float64
    assert ab[0] == pytest.approx(1 - 1e-4, rel=1e-15)
    b1 = 1e-4 + (2e-2 - 1e-4) / 999
    assert ab[1] == pytest.approx((1 - 1e-4) * (1 - b1), rel=1e-14)
    assert np.all(np.diff(ab) < 0)
    # log-sum evaluation, a different route to the same product
    logs = sum(math.log1p(-(1e-4 + (2e-2 - 1e-4) * i / 999)) for i in range(1000))
    assert ab[-1] == pytest.approx(math.exp(logs), rel=1e-10)
    assert 3e-5 < ab[-1] < 6e-5
    # three-term schedule by hand
    np.testing.assert_allclose(sampler.alphas_cumprod(3, 0.1, 0.3), [0.9, 0.9 * 0.8, 0.9 * 0.8 * 0.7], rtol=1e-15)


def test_sampling_timesteps_and_step_coefficients():
    tau = sampler.sampling_timesteps(50, 1000)
    np.testing.assert_array_equal(tau, np.arange(50) * 20)
    ab = sampler.alphas_cumprod()
    t, a_t, a_p = sampler.step_coefficients(SCHED, 25)
    assert (t, a_t, a_p) == (500, ab[500], ab[480])          # timestep 500 -> 480
    t, a_t, a_p = sampler.step_coefficients(SCHED, 1)
    assert (t, a_t, a_p) == (980, ab[980], ab[960])
    t, a_t, a_p = sampler.step_coefficients(SCHED, 50)
    assert (t, a_t, a_p) == (0, ab[0], 1.0)                  # last step lands on the x0 estimate
    with pytest.raises(ValueError):
        sampler.step_coefficients(SCHED, 0)
    with pytest.raises(ValueError):
        sampler.step_coefficients(SCHED, 51)


def test_ddim_update_closed_form_for_known_noise():
    rng = np.random.default_rng(1)
    x0, eps = rng.standard_normal((3, 4, 5)), rng.standard_normal((3, 4, 5))
    a_t, a_p = 0.37, 0.61
    x_t = math.sqrt(a_t) * x0 + math.sqrt(1 - a_t) * eps
    got = sampler.ddim_update(x_t, eps, a_t, a_p)
    np.testing.assert_allclose(got, math.sqrt(a_p) * x0 + math.sqrt(1 - a_p) * eps, atol=1e-14)
    np.testing.assert_allclose(sampler.ddim_update(x_t, eps, a_t, 1.0), x0, atol=1e-14)
    # eps = 0: pure rescaling
    np.testing.assert_allclose(sampler.ddim_update(x_t, 0 * eps, a_t, a_p), math.sqrt(a_p / a_t) * x_t, atol=1e-14)
    # a wrong sign on the eps term would break this scalar case: x_t=1, eps=1, a_t=0.25, a_p=1 -> (1-sqrt(.75))/0.5
    assert sampler.ddim_update(np.array(1.0), np.array(1.0), 0.25, 1.0) == pytest.approx((1 - math.sqrt(0.75)) / 0.5)


def test_guidance_special_cases():
    rng = np.random.default_rng(2)
    ec, eu = rng.standard_normal(7), rng.standard_normal(7)
    np.testing.assert_allclose(sampler.guide(ec, eu, 1.0), ec, atol=1e-15)
    np.testing.assert_allclose(sampler.guide(ec, eu, 0.0), eu, atol=1e-15)
    np.testing.assert_allclose(sampler.guide(ec, ec, 7.5), ec, atol=1e-14)
    np.testing.assert_allclose(sampler.guide(ec, eu, 7.5), 7.5 * ec - 6.5 * eu, atol=1e-13)


class _Counter:
    def __init__(self, fn):
        self.fn, self.calls = fn, []

    def __call__(self, x, txt, t):
        self.calls.append(t)
        return self.fn(x, txt, t)


def test_trajectory_recovers_x0_when_network_returns_true_noise():
    """With the oracle-perfect eps* the whole N-step run lands on x0, and every
    intermediate latent is sqrt(abar) x0 + sqrt(1-abar) eps*."""
    cfg = synth.WORKLOADS["cfg1"].model
    rng = np.random.default_rng(3)
    x0 = rng.standard_normal((2, 4, 8, 8, 4)); eps = rng.standard_normal((2, 4, 8, 8, 4))
    ab = sampler.alphas_cumprod()
    x = math.sqrt(ab[980]) * x0 + math.sqrt(1 - ab[980]) * eps
    def eps_fn(xr, txt, t):
        return eps[int(txt[0, 0])]

    cond = np.zeros((2, 8, 64)); cond[1, 0, 0] = 1
    seen = {}
    out = sampler.denoise_resume(cfg, None, x, cond, None, SCHED, 0, eps_fn=eps_fn,
                                 on_step=lambda s, lat: seen.__setitem__(s, lat.copy()))
    np.testing.assert_allclose(out, x0, atol=1e-9)
    np.testing.assert_allclose(seen[25], math.sqrt(ab[480]) * x0 + math.sqrt(1 - ab[480]) * eps, atol=1e-10)
    assert sorted(seen) == list(range(1, 51))


def test_resume_semantics():
    cfg = synth.WORKLOADS["cfg1"].model
    rng = np.random.default_rng(4)
    x = rng.standard_normal((1, 4, 8, 8, 4))
    cond = rng.standard_normal((1, 8, 64)); null = rng.standard_normal((8, 64))
    fn = _Counter(lambda xr, txt, t: np.tanh(xr) * 0.5 + 0.01 * txt.sum() + 1e-3 * t)
    full = sampler.denoise_resume(cfg, None, x, cond, null, SCHED, 0, eps_fn=fn)
    assert len(fn.calls) == 100                                   # N steps x (cond, null)
    assert fn.calls[0] == fn.calls[1] == 980 and fn.calls[-1] == 0
    # run steps 1..10 one by one, then resume from the stored step-10 latent
    xk = x
    for s in range(1, 11):
        xk = sampler.denoise_step(cfg, None, xk, cond, null, SCHED, s, eps_fn=fn)
    fn2 = _Counter(fn.fn)
    resumed = sampler.denoise_resume(cfg, None, xk, cond, null, SCHED, 10, eps_fn=fn2)
    np.testing.assert_array_equal(resumed, full)                  # same function, same order: bit-exact
    assert len(fn2.calls) == 2 * 40 and fn2.calls[0] == 780       # proceeds from the 11th step
    # k = N: nothing left to do
    fn3 = _Counter(fn.fn)
    np.testing.assert_array_equal(sampler.denoise_resume(cfg, None, x, cond, null, SCHED, 50, eps_fn=fn3), x)
    assert fn3.calls == []
    # no null embedding: one evaluation per step
    fn4 = _Counter(fn.fn)
    sampler.denoise_resume(cfg, None, x, cond, None, SCHED, 20, eps_fn=fn4)
    assert len(fn4.calls) == 30
    with pytest.raises(ValueError):
        sampler.denoise_resume(cfg, None, x, cond, null, SCHED, 51, eps_fn=fn)
    with pytest.raises(ValueError):
        sampler.denoise_step(cfg, None, x, cond, null, replace(SCHED, eta=0.5), 1, eps_fn=fn)


def test_step_with_real_network_composes_forward_guidance_update():
    from oracle import dit
    w = synth.WORKLOADS["cfg3b"]
    cfg = replace(w.model, depth=2)
    W = synth.make_weights(cfg, 5)
    lat = synth.make_latent(cfg, 6, 2); cond = synth.make_text(cfg, 7, 2); null = synth.make_null_text(cfg, 8)
    out, eps = sampler.denoise_step(cfg, W, lat, cond, null, w.schedule, 25, return_eps=True)
    ab = sampler.alphas_cumprod()
    for r in range(2):
        ec = dit.forward(cfg, W, lat[r], cond[r], 500); eu = dit.forward(cfg, W, lat[r], null, 500)
        e = eu + 7.5 * (ec - eu)
        np.testing.assert_allclose(eps[r], e, atol=1e-13)
        x0 = (lat[r] - math.sqrt(1 - ab[500]) * e) / math.sqrt(ab[500])
        np.testing.assert_allclose(out[r], math.sqrt(ab[480]) * x0 + math.sqrt(1 - ab[480]) * e, atol=1e-12)


# --------------------------------------------------------------------------- Euler step of a rectified-flow sampler (variant)

def _flow_sched(n=50):
    from dataclasses import replace
    return replace(synth.Schedule(num_steps=n), sampler=synth.SAMPLER_FLOW_EULER)


def test_flow_sigmas_cover_one_to_zero():
    sched = _flow_sched(50)
    t1, s1, n1 = sampler.flow_step_sigmas(sched, 1)
    assert (t1, s1) == (1000.0, 1.0) and abs(n1 - 0.98) < 1e-15
    tN, sN, nN = sampler.flow_step_sigmas(sched, 50)
    assert abs(tN - 20.0) < 1e-12 and nN == 0.0
    prev = None
    for s in range(1, 51):
        t, a, b = sampler.flow_step_sigmas(sched, s)
        assert abs((a - b) - 1 / 50) < 1e-15 and abs(t - 1000 * a) < 1e-9
        assert prev is None or abs(prev - a) < 1e-15          # steps chain: sigma_next of one is sigma of the next
        prev = b


def test_flow_true_velocity_lands_on_the_straight_path_and_ends_at_x0():
    rng = np.random.default_rng(0)
    x0, noise = rng.standard_normal((1, 3, 4, 4, 2)), rng.standard_normal((1, 3, 4, 4, 2))
    v = noise - x0
    sched = _flow_sched(10)
    x = noise.copy()                                           # sigma = 1
    for s in range(1, 11):
        _, sig, nxt = sampler.flow_step_sigmas(sched, s)
        assert np.allclose(x, (1 - sig) * x0 + sig * noise)
        x = sampler.denoise_step(None, None, x, np.zeros((1, 1, 1)), None, sched, s, eps_fn=lambda a, b, t: v[0])
    assert np.allclose(x, x0)


def test_flow_step_dispatch_guidance_and_resume_composition():
    rng = np.random.default_rng(1)
    lat = rng.standard_normal((1, 2, 4, 4, 2))
    sched = _flow_sched(8)
    calls = []

    def net(x, txt, t):
        calls.append(t)
        return 0.3 * x + float(txt.sum()) + 0.001 * t

    cond, null = np.ones((1, 2, 3)), np.zeros((2, 3))
    got = sampler.denoise_step(None, None, lat, cond, null, sched, 3, eps_fn=net)
    t, sig, nxt = sampler.flow_step_sigmas(sched, 3)
    vc, vu = 0.3 * lat[0] + 6.0 + 0.001 * t, 0.3 * lat[0] + 0.001 * t
    want = lat[0] + (nxt - sig) * (vu + sched.guidance_scale * (vc - vu))
    assert np.allclose(got[0], want) and calls == [t, t]
    whole = sampler.denoise_resume(None, None, lat, cond, null, sched, 2, eps_fn=net)
    part = sampler.denoise_resume(None, None, lat, cond, null, sched, 2, eps_fn=net, on_step=None)
    mid = lat
    for s in range(3, 9):
        mid = sampler.denoise_step(None, None, mid, cond, null, sched, s, eps_fn=net)
    assert np.allclose(whole, mid) and np.allclose(whole, part)
