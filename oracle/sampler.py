"""CPU oracle: noise schedule, guidance, the deterministic DDIM update, and the
cache-hit resume loop.

TEST INFRASTRUCTURE ONLY (see oracle/dit.py): never imported by the product path.

What it follows.  The paper runs a 50-step sampler of the DDIM family (Sec. 2.1;
Sec. 5 "Implementation") whose steps are strictly sequential, each step's output
being the next step's input.  On a cache hit the stored latent of step k is set
as the input and generation proceeds from the next step (Sec. 2.2; Sec. 3.2
"Cache lookup"; Sec. 4.2.2: a cache of the 10th step lets the request proceed
from the 11th).  So `denoise_resume(x_k, k)` runs steps k+1 .. N of the very same
step function a cache miss runs from k = 0.

Readings the paper leaves open, as taken here:
  * beta is linear in i between beta_start and beta_end over `train_steps`
    training timesteps; abar_t = prod_{i<=t} (1 - beta_i), evaluated in float64.
  * the N sampling timesteps are tau_j = j * (train_steps / N), j = 0..N-1, visited
    in descending order; step s (1-based) goes from t = tau_{N-s} to tau_{N-s-1},
    and the last step goes to abar_prev = 1 (it returns the x0 estimate).
  * eta = 0: no noise is drawn, the update is a deterministic function of
    (x_t, eps).  eta > 0 (the paper changes the denoising seed after a retrieval to keep
    outputs diverse, Sec. 7 "Discussions and Related Works", which needs a sampler that
    draws noise): the DDIM family's stochastic member,
      sigma = eta sqrt((1-abar_prev)/(1-abar_t)) sqrt(1 - abar_t/abar_prev),
      x_prev = sqrt(abar_prev) x0 + sqrt(1 - abar_prev - sigma^2) eps + sigma z,
    z standard normal.  z is not drawn from a stateful generator but computed from
    (seed, request, step, element) with the counter-based Philox4x32-10 of Salmon et al.
    (SC'11), so that any implementation produces the same noise: element i of request r
    at step s takes lane i % 4 of the block with counter (i // 4 low word, i // 4 high
    word, s, r) and key (seed low word, seed high word); a 32-bit output x becomes
    u = ((x >> 8) + 0.5) 2^-24 in (0, 1); lanes (0, 1) and (2, 3) are Box-Muller pairs
    (sqrt(-2 ln u_a) cos(2 pi u_b), sqrt(-2 ln u_a) sin(2 pi u_b)).
  * classifier-free guidance: eps = eps_u + s (eps_c - eps_u), eps_u from a given
    'null' text embedding.

A second step function, as a variant (sched.sampler = 1): the Euler step of a
rectified-flow sampler.  The paper fixes only that the steps are sequential and that a
hit continues with the very same step function (Sec. 2.1, Sec. 2.2), so the resume loop
is the same; what changes is the update.  The network output is read as the velocity
v = noise - x0 of the straight path x_sigma = (1 - sigma) x0 + sigma noise; sigma runs
over the uniform grid sigma_j = j / N from 1 down to 0; step s (1-based) goes from
sigma_{N-s+1} to sigma_{N-s} with x <- x + (sigma_{N-s} - sigma_{N-s+1}) v and the
network is evaluated at t = sigma_{N-s+1} * train_steps.  Guidance combines velocities
the way it combines eps.

Pins of the noise path: the three published known-answer vectors of Philox4x32-10, the
moments of the generated normals, eta = 0 equals the deterministic update, eta = 1
equals the ancestral step typed in its posterior-mean form (alpha, beta, beta~ of the
two visited timesteps; not through ddim_sigma), sigma linear in eta, and a Monte Carlo
check that the step keeps the marginal variance 1 - abar_prev for any eta.

Pins (tests/test_oracle_sampler.py): closed-form schedule values, monotonicity,
exact recovery x_prev = sqrt(abar_prev) x0 + sqrt(1-abar_prev) eps* when the
network returns the true eps*, eps = 0 scaling, guidance special cases (s = 0,
s = 1, cond == null), resume composition, resume(N) = identity, and the number
of network evaluations of resume(k).
"""
from __future__ import annotations

import math
from typing import Callable, Optional

import numpy as np

from . import dit


def alphas_cumprod(train_steps=1000, beta_start=1e-4, beta_end=2e-2):
    """abar_t for t = 0..train_steps-1, float64."""
    i = np.arange(train_steps, dtype=np.float64)
    beta = beta_start + (beta_end - beta_start) * i / (train_steps - 1)
    return np.cumprod(1.0 - beta)


def sampling_timesteps(num_steps, train_steps=1000):
    """tau_0..tau_{N-1} ascending: tau_j = j * (train_steps // N)."""
    return np.arange(num_steps, dtype=np.int64) * (train_steps // num_steps)


def step_coefficients(sched, step):
    """(t, abar_t, abar_prev) of the step-th (1-based) of sched.num_steps steps."""
    N = sched.num_steps
    if not 1 <= step <= N:
        raise ValueError("step out of range")
    tau = sampling_timesteps(N, sched.train_steps)
    abar = alphas_cumprod(sched.train_steps, sched.beta_start, sched.beta_end)
    t = int(tau[N - step])
    abar_prev = 1.0 if step == N else float(abar[tau[N - step - 1]])
    return t, float(abar[t]), abar_prev


# --------------------------------------------------------------------------- counter-based noise

_PHILOX_M0, _PHILOX_M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key):
    """counter [..., 4] and key [2] of 32-bit words -> [..., 4] uint32: ten rounds of
    (hi(M0 c0), lo(M0 c0), hi(M1 c2), lo(M1 c2)) -> (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0),
    the key bumped by the Weyl constants between rounds."""
    c = np.asarray(counter, dtype=np.uint64) & np.uint64(0xFFFFFFFF)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    mask = np.uint64(0xFFFFFFFF)
    for _ in range(10):
        p0, p1 = _PHILOX_M0 * c0, _PHILOX_M1 * c2
        hi0, lo0, hi1, lo1 = p0 >> np.uint64(32), p0 & mask, p1 >> np.uint64(32), p1 & mask
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0, k1 = (k0 + _PHILOX_W0) & 0xFFFFFFFF, (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def counter_normals(seed, request, step, n):
    """The n standard normals of (seed, request, step), float64."""
    blocks = (n + 3) // 4
    idx = np.arange(blocks, dtype=np.uint64)
    ctr = np.stack([idx & np.uint64(0xFFFFFFFF), idx >> np.uint64(32),
                    np.full(blocks, step, dtype=np.uint64), np.full(blocks, request, dtype=np.uint64)], axis=-1)
    x = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)).astype(np.float64)
    u = (np.floor(x / 256.0) + 0.5) * 2.0 ** -24
    z = np.empty((blocks, 4))
    for a, b in ((0, 1), (2, 3)):
        rad = np.sqrt(-2.0 * np.log(u[:, a]))
        z[:, a], z[:, b] = rad * np.cos(2.0 * np.pi * u[:, b]), rad * np.sin(2.0 * np.pi * u[:, b])
    return z.reshape(-1)[:n]


def ddim_sigma(abar_t, abar_prev, eta):
    return eta * math.sqrt((1.0 - abar_prev) / (1.0 - abar_t)) * math.sqrt(1.0 - abar_t / abar_prev)


def ddim_update_stochastic(x_t, eps, abar_t, abar_prev, eta, z):
    sigma = ddim_sigma(abar_t, abar_prev, eta)
    x0 = (x_t - math.sqrt(1.0 - abar_t) * eps) / math.sqrt(abar_t)
    return math.sqrt(abar_prev) * x0 + math.sqrt(max(1.0 - abar_prev - sigma * sigma, 0.0)) * eps + sigma * z


def flow_step_sigmas(sched, step):
    """(t, sigma, sigma_next) of the step-th (1-based) Euler step on the uniform sigma grid."""
    N = sched.num_steps
    if not 1 <= step <= N:
        raise ValueError("step out of range")
    sigma, sigma_next = (N - step + 1) / N, (N - step) / N
    return sigma * sched.train_steps, sigma, sigma_next


def flow_euler_update(x, v, sigma, sigma_next):
    """x_{sigma_next} = x_sigma + (sigma_next - sigma) v."""
    return x + (sigma_next - sigma) * v


def guide(eps_cond, eps_null, scale):
    """Classifier-free guidance: eps_u + s (eps_c - eps_u)."""
    return eps_null + scale * (eps_cond - eps_null)


def ddim_update(x_t, eps, abar_t, abar_prev):
    """Deterministic DDIM (eta = 0), eps-prediction:
    x0 = (x_t - sqrt(1-abar_t) eps) / sqrt(abar_t);
    x_prev = sqrt(abar_prev) x0 + sqrt(1-abar_prev) eps."""
    x0 = (x_t - math.sqrt(1.0 - abar_t) * eps) / math.sqrt(abar_t)
    return math.sqrt(abar_prev) * x0 + math.sqrt(1.0 - abar_prev) * eps


def denoise_step(cfg, weights, latent, cond, null_cond, sched, step, dtype=np.float64,
                 eps_fn: Optional[Callable] = None, return_eps=False):
    """One denoising step for R requests.

    latent [R,T,H,W,C]; cond [R,L,dt]; null_cond [L,dt] or None (no guidance).
    eps_fn(latent_r, text, t) replaces the network (used by the pins).
    Returns the latents after the step, same shape, in `dtype`."""
    flow = getattr(sched, "sampler", 0) == 1
    if sched.eta != 0.0 and flow:
        raise ValueError("eta belongs to the DDIM family; the Euler step draws no noise")
    if flow:
        t, sigma, sigma_next = flow_step_sigmas(sched, step)
    else:
        t, abar_t, abar_prev = step_coefficients(sched, step)
    if eps_fn is None:
        W = {k: np.asarray(v, dtype=dtype) for k, v in weights.items()}
        eps_fn = lambda x, txt, tt: dit.forward(cfg, W, x, txt, tt, dtype=None)
    lat = np.asarray(latent, dtype=dtype)
    out = np.empty_like(lat)
    eps_out = np.empty_like(lat)
    for r in range(lat.shape[0]):
        eps = eps_fn(lat[r], np.asarray(cond[r], dtype=dtype), t)
        if null_cond is not None:
            eps_u = eps_fn(lat[r], np.asarray(null_cond, dtype=dtype), t)
            eps = guide(eps, eps_u, sched.guidance_scale)
        eps_out[r] = eps
        if flow:
            out[r] = flow_euler_update(lat[r], eps, sigma, sigma_next)
        elif sched.eta != 0.0:
            z = counter_normals(getattr(sched, "seed", 0), r, step, lat[r].size).reshape(lat[r].shape)
            out[r] = ddim_update_stochastic(lat[r], eps, abar_t, abar_prev, sched.eta, z)
        else:
            out[r] = ddim_update(lat[r], eps, abar_t, abar_prev)
    return (out, eps_out) if return_eps else out


def denoise_resume(cfg, weights, latent, cond, null_cond, sched, k, dtype=np.float64,
                   eps_fn: Optional[Callable] = None, on_step: Optional[Callable] = None):
    """Run steps k+1 .. N from the stored step-k latent (k = 0: a full run from
    noise; k = N: nothing to do).  on_step(step, latent) is called after each step."""
    N = sched.num_steps
    if not 0 <= k <= N:
        raise ValueError("k out of range")
    x = np.asarray(latent, dtype=dtype)
    if eps_fn is None and k < N:
        W = {kk: np.asarray(v, dtype=dtype) for kk, v in weights.items()}
        eps_fn = lambda xx, txt, tt: dit.forward(cfg, W, xx, txt, tt, dtype=None)
    for s in range(k + 1, N + 1):
        x = denoise_step(cfg, None, x, cond, null_cond, sched, s, dtype=dtype, eps_fn=eps_fn)
        if on_step is not None:
            on_step(s, x)
    return x
