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
    with pytest.raises(ValueError):      # eta belongs to the DDIM family only
        sampler.denoise_step(cfg, None, x, cond, null,
                             replace(SCHED, eta=0.5, sampler=synth.SAMPLER_FLOW_EULER), 1, eps_fn=fn)


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


# --------------------------------------------------------------------------- eta > 0: counter-based noise

def test_philox_known_answers():
    """The known-answer vectors published with Philox4x32-10 (Random123, Salmon et al. SC'11)."""
    kat = [
        ((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
        ((0xffffffff,) * 4, (0xffffffff, 0xffffffff), (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
        ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
         (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1)),
    ]
    for ctr, key, want in kat:
        got = sampler.philox4x32_10(np.array(ctr, dtype=np.uint64), key)
        assert tuple(int(v) for v in got) == want
    # vectorised evaluation equals one block at a time
    ctrs = np.array([[1, 2, 3, 4], [5, 6, 7, 8]], dtype=np.uint64)
    both = sampler.philox4x32_10(ctrs, (9, 10))
    assert np.array_equal(both[1], sampler.philox4x32_10(ctrs[1], (9, 10)))


def test_counter_normals_are_standard_normal_and_addressable():
    z = sampler.counter_normals(1234, 0, 7, 200_003)
    assert z.shape == (200_003,) and np.all(np.isfinite(z))
    assert abs(z.mean()) < 0.01 and abs(z.var() - 1.0) < 0.01
    assert abs(np.mean(z ** 3)) < 0.03 and abs(np.mean(z ** 4) - 3.0) < 0.06
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 0.01
    # a prefix is a prefix; another step, request or seed is another stream
    assert np.array_equal(sampler.counter_normals(1234, 0, 7, 10), z[:10])
    for other in ((1234, 0, 8), (1234, 1, 7), (1235, 0, 7), (1234 + (1 << 32), 0, 7)):
        assert not np.allclose(sampler.counter_normals(*other, 10), z[:10])


def test_stochastic_ddim_special_cases():
    sched = synth.Schedule()
    rng = np.random.default_rng(0)
    x, eps, z = rng.standard_normal((3, 4)), rng.standard_normal((3, 4)), rng.standard_normal((3, 4))
    t, a_t, a_p = sampler.step_coefficients(sched, 20)
    # eta = 0 is the deterministic update
    assert np.allclose(sampler.ddim_update_stochastic(x, eps, a_t, a_p, 0.0, z), sampler.ddim_update(x, eps, a_t, a_p))
    # eta = 1: sigma^2 is the posterior variance (1-abar_prev)/(1-abar_t) * (1 - abar_t/abar_prev)
    s1 = sampler.ddim_sigma(a_t, a_p, 1.0)
    assert np.isclose(s1 ** 2, (1 - a_p) / (1 - a_t) * (1 - a_t / a_p))
    # variance bookkeeping, and the last step draws nothing (abar_prev = 1)
    for eta in (0.3, 1.0):
        s = sampler.ddim_sigma(a_t, a_p, eta)
        assert 0 < s * s < 1 - a_p
    _, a_tl, a_pl = sampler.step_coefficients(sched, sched.num_steps)
    assert a_pl == 1.0 and sampler.ddim_sigma(a_tl, a_pl, 1.0) == 0.0
    # with the true eps the step lands on the stated marginal
    x0, e_true = rng.standard_normal((3, 4)), rng.standard_normal((3, 4))
    xt = math.sqrt(a_t) * x0 + math.sqrt(1 - a_t) * e_true
    s = sampler.ddim_sigma(a_t, a_p, 0.7)
    got = sampler.ddim_update_stochastic(xt, e_true, a_t, a_p, 0.7, z)
    assert np.allclose(got, math.sqrt(a_p) * x0 + math.sqrt(1 - a_p - s * s) * e_true + s * z)


def test_eta_one_is_the_ancestral_step_in_posterior_mean_form():
    """Independent statement of the same step: at eta = 1 the DDIM family's member is the
    ancestral sampler of the discrete diffusion between the two visited timesteps,
      x_prev = (x_t - beta/sqrt(1-abar_t) eps) / sqrt(alpha) + sqrt(beta~) z,
      alpha = abar_t/abar_prev, beta = 1 - alpha, beta~ = beta (1-abar_prev)/(1-abar_t),
    written from the posterior q(x_prev | x_t, x0) and not through ddim_sigma.  A swapped
    ratio or a wrong sign in the oracle's sigma or in its eps coefficient breaks it.  For
    0 < eta < 1 the noise scale is eta times that one and the mean keeps variance
    1 - abar_prev - sigma^2 on the eps direction, checked by Monte Carlo on the marginal."""
    sched = synth.Schedule()
    rng = np.random.default_rng(3)
    x, eps, z = rng.standard_normal((5, 7)), rng.standard_normal((5, 7)), rng.standard_normal((5, 7))
    for step in (1, 20, 37, 49):
        _, a_t, a_p = sampler.step_coefficients(sched, step)
        alpha = a_t / a_p
        beta = 1.0 - alpha
        post_var = beta * (1.0 - a_p) / (1.0 - a_t)
        want = (x - beta / math.sqrt(1.0 - a_t) * eps) / math.sqrt(alpha) + math.sqrt(post_var) * z
        got = sampler.ddim_update_stochastic(x, eps, a_t, a_p, 1.0, z)
        assert np.allclose(got, want, rtol=1e-10, atol=1e-12), step
        assert math.isclose(sampler.ddim_sigma(a_t, a_p, 0.5), 0.5 * math.sqrt(post_var), rel_tol=1e-12)
    # marginal at an intermediate eta: from x_t ~ q(x_t | x0) with the true eps, x_prev ~ q(x_prev | x0),
    # i.e. (x_prev - sqrt(abar_prev) x0) has variance 1 - abar_prev whatever eta is
    _, a_t, a_p = sampler.step_coefficients(sched, 30)
    n = 400_000
    e_true, zz = rng.standard_normal(n), rng.standard_normal(n)
    x0 = 0.3
    xt = math.sqrt(a_t) * x0 + math.sqrt(1 - a_t) * e_true
    for eta in (0.4, 1.0):
        xp = sampler.ddim_update_stochastic(xt, e_true, a_t, a_p, eta, zz)
        r = xp - math.sqrt(a_p) * x0
        assert abs(r.mean()) < 4 * math.sqrt((1 - a_p) / n)
        assert abs(r.var() / (1 - a_p) - 1.0) < 0.01


def test_stochastic_step_uses_the_counter_noise_per_request():
    from dataclasses import replace
    sched = replace(synth.Schedule(num_steps=10), eta=0.5, seed=99)
    rng = np.random.default_rng(1)
    lat = rng.standard_normal((2, 2, 4, 4, 2))
    net = lambda x, txt, t: 0.1 * x
    got = sampler.denoise_step(None, None, lat, np.zeros((2, 1, 1)), None, sched, 4, eps_fn=net)
    t, a_t, a_p = sampler.step_coefficients(sched, 4)
    for r in range(2):
        z = sampler.counter_normals(99, r, 4, lat[r].size).reshape(lat[r].shape)
        assert np.allclose(got[r], sampler.ddim_update_stochastic(lat[r], 0.1 * lat[r], a_t, a_p, 0.5, z))
    again = sampler.denoise_step(None, None, lat, np.zeros((2, 1, 1)), None, sched, 4, eps_fn=net)
    assert np.array_equal(got, again)
    other = sampler.denoise_step(None, None, lat, np.zeros((2, 1, 1)), None, replace(sched, seed=100), 4, eps_fn=net)
    assert not np.allclose(got, other)
