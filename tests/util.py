"""Helpers shared by the GPU parity tests: device staging and error measures."""
import os

import numpy as np

# measured errors of the parity tests, printed as a table at the end of the run
PARITY = []


def record(**values):
    """Notes measured errors under the running test's name."""
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split("::")[-1].split(" ")[0]
    PARITY.append((test, values))


def rel_l2(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))


def max_abs(got, want):
    return float(np.abs(np.asarray(got, dtype=np.float64) - np.asarray(want, dtype=np.float64)).max())


def dev(a, bf16=False):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


_WEIGHTS = []          # the most recent seeded weight sets: drawing a 28-block stack takes half a minute


def cached_weights(cfg, seed, std=0.02):
    """synth.make_weights, remembered for the tests that use the same model one after another."""
    from paper_2501_04012_amd import synth
    key = (cfg, seed, std)
    for k, W in _WEIGHTS:
        if k == key:
            return W
    W = synth.make_weights(cfg, seed, std=std)
    _WEIGHTS.append((key, W))
    del _WEIGHTS[:-2]
    return W


def run_step_gpu(fc, w, step=None, depth=None, weights=None, inputs=None, return_eps=True):
    """One fc_denoise_step of workload w on the GPU; returns (latent_after, eps)."""
    import torch
    from dataclasses import replace
    from paper_2501_04012_amd import synth
    cfg = w.model if depth is None else replace(w.model, depth=depth)
    W = weights if weights is not None else synth.make_weights(cfg, w.weight_seed)
    lat, cond, null = inputs if inputs is not None else synth.workload_inputs(w)
    R = lat.shape[0]
    den = fc.Denoiser(cfg, W, R, null is not None)
    try:
        d_lat, d_cond = dev(lat), dev(cond)
        d_null = dev(null) if null is not None else None
        d_eps = torch.empty_like(d_lat)
        den.step(d_lat, d_cond, d_null, w.schedule, step if step is not None else w.step, eps_out=d_eps)
        torch.cuda.synchronize()
        return host(d_lat), host(d_eps)
    finally:
        den.close()
