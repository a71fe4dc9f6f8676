"""Seeded synthetic inputs and workload descriptions for the denoising path.

This module holds no arithmetic of the method. It only
  * names the workloads (shapes of latent, text and model),
  * lists the weight tensors of a model in their fixed order (the blob format),
  * draws Gaussian latents, text embeddings and weights from seeded generators.

Both the CPU oracle's tests and the HIP path's binding are fed from here; neither
of them is imported here.

The paper (Sec. 2.1, "Diffusion Model") treats the denoiser as a given network
that maps (current latent, prompt embedding) to a noise estimate; its own model
is a trained U-Net we do not have.  The workloads below are random-init diffusion
transformers with Gaussian latents, standing in for it.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

ATTN_FACTORIZED_CROSS = 0   # spatial attn, temporal attn, text cross-attn
ATTN_FULL3D_CONCAT = 1      # one attention over [text ; video] tokens
DT_F32 = 0
DT_BF16 = 1


@dataclass(frozen=True)
class ModelConfig:
    frames: int
    height: int
    width: int
    channels: int
    patch: int
    hidden: int
    heads: int
    mlp_dim: int
    depth: int
    text_len: int
    text_dim: int
    t_embed_dim: int = 256
    attn_mode: int = ATTN_FACTORIZED_CROSS
    dtype: int = DT_F32
    ln_eps: float = 1e-6
    text_adaln: int = 0     # full-3D mode only: 1 = the text rows have modulation vectors of their own

    @property
    def spatial_tokens(self) -> int:
        return (self.height // self.patch) * (self.width // self.patch)

    @property
    def video_tokens(self) -> int:
        return self.frames * self.spatial_tokens

    @property
    def seq_tokens(self) -> int:
        """Tokens each block sees (text rows are part of the sequence in full-3D mode)."""
        extra = self.text_len if self.attn_mode == ATTN_FULL3D_CONCAT else 0
        return self.video_tokens + extra

    @property
    def patch_dim(self) -> int:
        return self.patch * self.patch * self.channels

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads


SAMPLER_DDIM = 0          # eps-prediction, deterministic DDIM update
SAMPLER_FLOW_EULER = 1    # velocity prediction, Euler step on sigma = 1 .. 0


@dataclass(frozen=True)
class Schedule:
    train_steps: int = 1000
    beta_start: float = 1e-4
    beta_end: float = 2e-2
    num_steps: int = 50
    guidance_scale: float = 7.5
    eta: float = 0.0
    sampler: int = 0          # SAMPLER_DDIM or SAMPLER_FLOW_EULER
    seed: int = 0             # key of the counter-based noise drawn when eta > 0


@dataclass(frozen=True)
class Workload:
    """One named configuration: model, seeds, batch and sampler settings."""
    name: str
    model: ModelConfig
    weight_seed: int
    latent_seed: int
    text_seed: int
    null_seed: Optional[int]      # None: no classifier-free guidance
    requests: int = 1
    step: int = 25                # 1-based step of the 50-step schedule (t=500 -> 480)
    resume_k: Tuple[int, ...] = ()
    schedule: Schedule = Schedule()


_TINY = ModelConfig(frames=4, height=8, width=8, channels=4, patch=2, hidden=64, heads=4,
                    mlp_dim=256, depth=1, text_len=8, text_dim=64,
                    attn_mode=ATTN_FACTORIZED_CROSS, dtype=DT_F32)
_FACT = ModelConfig(frames=16, height=32, width=32, channels=4, patch=2, hidden=1152, heads=16,
                    mlp_dim=4608, depth=1, text_len=120, text_dim=4096,
                    attn_mode=ATTN_FACTORIZED_CROSS, dtype=DT_BF16)
_FULL3D = ModelConfig(frames=13, height=60, width=90, channels=16, patch=2, hidden=3072, heads=48,
                      mlp_dim=12288, depth=1, text_len=226, text_dim=4096,
                      attn_mode=ATTN_FULL3D_CONCAT, dtype=DT_BF16)

WORKLOADS: Dict[str, Workload] = {
    # tiny fp32 block, one DDIM step
    "cfg1": Workload("cfg1", _TINY, weight_seed=100, latent_seed=101, text_seed=102, null_seed=None),
    # one bf16 block, factorized attention
    "cfg2": Workload("cfg2", _FACT, weight_seed=200, latent_seed=201, text_seed=202, null_seed=None),
    # 28-block stack with a classifier-free-guidance pair: wide bf16 and tiny fp32 readings
    "cfg3a": Workload("cfg3a", replace(_FACT, depth=28), weight_seed=300, latent_seed=201,
                      text_seed=202, null_seed=203),
    "cfg3b": Workload("cfg3b", replace(_TINY, depth=28), weight_seed=310, latent_seed=101,
                      text_seed=102, null_seed=103),
    # one bf16 block with full 3-D attention, text concatenated into the sequence
    "cfg4": Workload("cfg4", _FULL3D, weight_seed=400, latent_seed=401, text_seed=402, null_seed=None),
    # cache-hit resume: 4 requests, CFG pair each, restart from step k
    "cfg5a": Workload("cfg5a", replace(_FACT, depth=28), weight_seed=300, latent_seed=501,
                      text_seed=520, null_seed=503, requests=4, resume_k=(10, 20)),
    "cfg5b": Workload("cfg5b", replace(_TINY, depth=28), weight_seed=310, latent_seed=501,
                      text_seed=520, null_seed=503, requests=4, resume_k=(10, 20)),
    # a sixth, additional workload with the latent shape the paper states for its model
    # (64 frames x 40 x 64 x 4, Sec. 2.3): 40 960 tokens, spatial sequences of 640, temporal of 64
    "cfg6": Workload("cfg6", replace(_FACT, frames=64, height=40, width=64), weight_seed=600, latent_seed=601,
                     text_seed=602, null_seed=None),
}


# --------------------------------------------------------------------------- weights

def weight_spec(cfg: ModelConfig) -> List[Tuple[str, Tuple[int, ...]]]:
    """Ordered (name, shape) list of every parameter.  Linear weights are [in, out]
    row-major so that y = x @ W + b.  The flat fp32 blob handed to the library is
    the concatenation of these tensors in this order."""
    D, M, te, dt, pd = cfg.hidden, cfg.mlp_dim, cfg.t_embed_dim, cfg.text_dim, cfg.patch_dim
    nm3 = 12 if cfg.text_adaln else 6      # full-3D modulation chunks: video set (+ text set)
    spec: List[Tuple[str, Tuple[int, ...]]] = [
        ("t_w1", (te, D)), ("t_b1", (D,)), ("t_w2", (D, D)), ("t_b2", (D,)),
        ("y_w", (dt, D)), ("y_b", (D,)),
        ("p_w", (pd, D)), ("p_b", (D,)),
    ]
    for l in range(cfg.depth):
        pre = f"blk{l}."
        if cfg.attn_mode == ATTN_FACTORIZED_CROSS:
            spec += [
                (pre + "mod_w", (D, 9 * D)), (pre + "mod_b", (9 * D,)),
                (pre + "sp_qkv_w", (D, 3 * D)), (pre + "sp_qkv_b", (3 * D,)),
                (pre + "sp_proj_w", (D, D)), (pre + "sp_proj_b", (D,)),
                (pre + "tm_qkv_w", (D, 3 * D)), (pre + "tm_qkv_b", (3 * D,)),
                (pre + "tm_proj_w", (D, D)), (pre + "tm_proj_b", (D,)),
                (pre + "x_q_w", (D, D)), (pre + "x_q_b", (D,)),
                (pre + "x_kv_w", (D, 2 * D)), (pre + "x_kv_b", (2 * D,)),
                (pre + "x_proj_w", (D, D)), (pre + "x_proj_b", (D,)),
            ]
        else:
            spec += [
                (pre + "mod_w", (D, nm3 * D)), (pre + "mod_b", (nm3 * D,)),
                (pre + "qkv_w", (D, 3 * D)), (pre + "qkv_b", (3 * D,)),
                (pre + "proj_w", (D, D)), (pre + "proj_b", (D,)),
            ]
        spec += [
            (pre + "fc1_w", (D, M)), (pre + "fc1_b", (M,)),
            (pre + "fc2_w", (M, D)), (pre + "fc2_b", (D,)),
        ]
    spec += [("f_mod_w", (D, 2 * D)), ("f_mod_b", (2 * D,)), ("f_w", (D, pd)), ("f_b", (pd,))]
    return spec


def weight_count(cfg: ModelConfig) -> int:
    return int(sum(int(np.prod(s)) for _, s in weight_spec(cfg)))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array holding the nearest-even bfloat16 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _maybe_round(cfg: ModelConfig, a: np.ndarray) -> np.ndarray:
    return round_to_bf16(a) if cfg.dtype == DT_BF16 else a


def make_weights(cfg: ModelConfig, seed: int, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Every parameter (biases and modulation layers included) ~ N(0, std^2), drawn
    in spec order from one generator.  bf16 models get bf16-representable values."""
    rng = np.random.default_rng(seed)
    out: Dict[str, np.ndarray] = {}
    for name, shape in weight_spec(cfg):
        w = rng.standard_normal(shape, dtype=np.float32)
        w *= np.float32(std)
        out[name] = _maybe_round(cfg, w)
    return out


def pack_weights(cfg: ModelConfig, weights: Dict[str, np.ndarray]) -> np.ndarray:
    """Concatenate a weight dict into the flat fp32 blob, in spec order."""
    parts = []
    for name, shape in weight_spec(cfg):
        w = np.asarray(weights[name], dtype=np.float32)
        if tuple(w.shape) != tuple(shape):
            raise ValueError(f"{name}: shape {w.shape} != {shape}")
        parts.append(w.reshape(-1))
    return np.concatenate(parts)


# --------------------------------------------------------------------------- activations

def make_latent(cfg: ModelConfig, seed: int, requests: int = 1) -> np.ndarray:
    """[R, T, H, W, C] fp32 ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((requests, cfg.frames, cfg.height, cfg.width, cfg.channels),
                               dtype=np.float32)


def make_text(cfg: ModelConfig, seed: int, requests: int = 1) -> np.ndarray:
    """[R, L, dt] fp32 ~ N(0,1) (bf16-representable for bf16 models)."""
    rng = np.random.default_rng(seed)
    return _maybe_round(cfg, rng.standard_normal((requests, cfg.text_len, cfg.text_dim),
                                                 dtype=np.float32))


def make_null_text(cfg: ModelConfig, seed: int) -> np.ndarray:
    """[L, dt]: the 'empty prompt' embedding of classifier-free guidance."""
    return make_text(cfg, seed, 1)[0]


def workload_inputs(w: Workload):
    """(latent [R,...], cond [R,L,dt], null [L,dt] or None) of a named workload.

    Resume workloads: request r's stored latent is a shared seeded base plus
    0.1*N(0,1) of its own seed, and each request has its own prompt embedding."""
    cfg = w.model
    if w.resume_k:
        base = make_latent(cfg, w.latent_seed, 1)[0]
        lat = np.stack([base + np.float32(0.1) * make_latent(cfg, w.latent_seed + 9 + r, 1)[0]
                        for r in range(w.requests)]).astype(np.float32)
        cond = np.stack([make_text(cfg, w.text_seed + r, 1)[0] for r in range(w.requests)])
    else:
        lat = make_latent(cfg, w.latent_seed, w.requests)
        cond = make_text(cfg, w.text_seed, w.requests)
    null = make_null_text(cfg, w.null_seed) if w.null_seed is not None else None
    return lat, cond, null


def sharp_qkv(seed: int, n_q: int, n_k: int, d: int, gain: float = 4.0):
    """q, k, v for attention tests with peaked softmax rows (random-init models give
    near-uniform rows, which would leave max-subtraction and rescaling untested)."""
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((n_q, d), dtype=np.float32) * np.float32(gain)
    k = rng.standard_normal((n_k, d), dtype=np.float32) * np.float32(gain)
    v = rng.standard_normal((n_k, d), dtype=np.float32)
    return q, k, v


# --------------------------------------------------------------------------- FLOP accounting

def forward_flops(cfg: ModelConfig) -> Dict[str, float]:
    """Counted FLOPs of one forward pass of one sample: 2mnk per GEMM, 4*Nq*Nk*d per
    attention head; padding, softmax and elementwise work are not counted."""
    D, M, N, S, T, L = cfg.hidden, cfg.mlp_dim, cfg.video_tokens, cfg.spatial_tokens, cfg.frames, cfg.text_len
    Ns = cfg.seq_tokens
    gemm = 2.0 * L * cfg.text_dim * D + 2.0 * N * cfg.patch_dim * D * 2  # text proj, patch-embed, final
    attn = 0.0
    if cfg.attn_mode == ATTN_FACTORIZED_CROSS:
        per_gemm = 2.0 * N * D * (3 * D + D) * 2 + 2.0 * N * D * D * 2 + 2.0 * L * D * 2 * D \
            + 2.0 * N * D * M * 2
        per_attn = 4.0 * N * S * D + 4.0 * N * T * D + 4.0 * N * L * D
    else:
        per_gemm = 2.0 * Ns * D * (3 * D + D) + 2.0 * Ns * D * M * 2
        per_attn = 4.0 * Ns * Ns * D
    gemm += per_gemm * cfg.depth
    attn += per_attn * cfg.depth
    return {"gemm": gemm, "attention": attn, "total": gemm + attn,
            "block_gemm": per_gemm, "block_attention": per_attn}
