"""CPU oracle: the noise-prediction network of one denoising step.

TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition the HIP kernels are
checked against.  It shares no code with them and must never be imported by the
product path; only the tests, the smoke check and the benchmark's CPU-baseline
leg call it.

What it follows.  The paper (Sec. 2.1 "Diffusion Model") states a denoising step
as: take the current latent and the prompt embedding, predict the noise, remove
it; the denoiser is a U-Net or a diffusion transformer, and video models use
spatial-temporal transformers.  The paper gives no further detail of the network,
so the block below is the plain pre-LN adaLN diffusion transformer in its two
video forms (factorized spatial/temporal attention + text cross-attention, or one
attention over [text ; video] tokens; in the second form the text rows may carry
modulation vectors of their own, a variant in which the two modalities are normalised
and gated separately while sharing every other weight).  Every choice the paper leaves open is
written out where it is taken.

Evaluation is the textbook one: matmul for every linear layer, the full score
matrix with a max-subtracted two-pass softmax for attention, two-pass
mean/variance for LayerNorm.  `dtype` selects the arithmetic (float64 by default;
float32 is the "plain fp32" form).

Weights come as a dict of named arrays (names listed in `forward`), linear
weights stored [in, out] so that y = x @ W + b.

Pins (tests/test_oracle_*.py): brute-force attention loops, softmax row sums,
uniform-key and single-key attention, token-permutation equivariance, frame
locality of spatial / temporal attention, LayerNorm moments, GELU identities,
sinusoid norms, patchify round trip, zero-modulation identity block, and an
independently written einsum evaluation of the whole tiny network.  Separate text
modulation: equal text and video sets reproduce the shared form, zero gates of one
modality leave exactly that modality's rows unchanged, and an independently written
two-pass evaluation (text rows and video rows modulated in separate calls).
The whole network with random weights has no printed worked example in the
paper: beyond those pins its parity is unpinned by the paper.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import numpy as np

FACTORIZED_CROSS = 0
FULL3D_CONCAT = 1


# --------------------------------------------------------------------------- pointwise pieces

def silu(x):
    return x / (1.0 + np.exp(-x))


def gelu_tanh(x):
    """GELU, tanh form: 0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) ))."""
    c = math.sqrt(2.0 / math.pi)
    return 0.5 * x * (1.0 + np.tanh(c * (x + 0.044715 * x * x * x)))


def layernorm(x, eps):
    """Per-row normalisation over the last axis, biased variance, no affine."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + eps)


def modulate(u, shift, scale):
    """adaLN modulation: u * (1 + scale) + shift, vectors broadcast over tokens."""
    return u * (1.0 + scale) + shift


def softmax_rows(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v):
    """softmax(q k^T / sqrt(d)) v for [..., Nq, d], [..., Nk, d], [..., Nk, d].
    Unmasked; the whole score matrix is formed."""
    d = q.shape[-1]
    s = np.matmul(q, np.swapaxes(k, -1, -2)) / math.sqrt(d)
    return np.matmul(softmax_rows(s), v)


# --------------------------------------------------------------------------- embeddings

def timestep_embedding(t, dim=256, dtype=np.float64):
    """[cos(t f_0..f_{h-1}) | sin(t f_0..f_{h-1})], f_i = 10000^(-i/h), h = dim/2."""
    half = dim // 2
    f = np.power(10000.0, -np.arange(half, dtype=np.float64) / half)
    a = float(t) * f
    return np.concatenate([np.cos(a), np.sin(a)]).astype(dtype)


def sincos_1d(pos, dim):
    """[sin(pos w_i) | cos(pos w_i)], w_i = 10000^(-i/(dim/2)), i < dim/2; float64."""
    half = dim // 2
    w = np.power(10000.0, -np.arange(half, dtype=np.float64) / half)
    a = np.asarray(pos, dtype=np.float64)[..., None] * w
    return np.concatenate([np.sin(a), np.cos(a)], axis=-1)


def positional_embedding(frames, grid_h, grid_w, dim):
    """[T, S, D]: fixed 2-D spatial sin-cos (first D/2 dims from the patch row,
    last D/2 from the patch column) plus a 1-D temporal sin-cos on all D dims."""
    hh, ww = np.meshgrid(np.arange(grid_h), np.arange(grid_w), indexing="ij")
    spatial = np.concatenate([sincos_1d(hh.reshape(-1), dim // 2),
                              sincos_1d(ww.reshape(-1), dim // 2)], axis=-1)     # [S, D]
    temporal = sincos_1d(np.arange(frames), dim)                                 # [T, D]
    return temporal[:, None, :] + spatial[None, :, :]


def patchify(lat, p):
    """[T,H,W,C] -> [T*(H/p)*(W/p), p*p*C]; token order (t, h', w') row-major,
    feature order inside a patch (dh, dw, c)."""
    T, H, W, C = lat.shape
    x = lat.reshape(T, H // p, p, W // p, p, C).transpose(0, 1, 3, 2, 4, 5)
    return x.reshape(T * (H // p) * (W // p), p * p * C)


def unpatchify(tok, T, H, W, C, p):
    """Inverse of patchify."""
    x = tok.reshape(T, H // p, W // p, p, p, C).transpose(0, 1, 3, 2, 4, 5)
    return x.reshape(T, H, W, C)


# --------------------------------------------------------------------------- attention layers

def _split_heads(a, heads):
    """[..., n, D] -> [..., h, n, d]: heads are consecutive d-wide column groups."""
    *lead, n, D = a.shape
    return np.moveaxis(a.reshape(*lead, n, heads, D // heads), -2, -3)


def _merge_heads(a):
    """[..., h, n, d] -> [..., n, h*d]."""
    a = np.moveaxis(a, -3, -2)
    return a.reshape(*a.shape[:-2], a.shape[-2] * a.shape[-1])


def self_attention(u, w_qkv, b_qkv, w_proj, b_proj, heads, q_rows=None):
    """Multi-head self-attention.  u is [n, D] (one sequence) or [G, n, D] (G
    independent sequences); attention never crosses sequences.
    qkv = u W + b split [q | k | v].  With q_rows, only those query rows are
    evaluated (keys/values stay complete)."""
    D = u.shape[-1]
    qkv = u @ w_qkv + b_qkv
    q, k, v = qkv[..., :D], qkv[..., D:2 * D], qkv[..., 2 * D:]
    if q_rows is not None:
        q = q[..., q_rows, :]
    qh, kh, vh = _split_heads(q, heads), _split_heads(k, heads), _split_heads(v, heads)
    out = np.empty_like(qh)
    for h in range(heads):                       # one head at a time keeps the score matrix small
        out[..., h, :, :] = attention(qh[..., h, :, :], kh[..., h, :, :], vh[..., h, :, :])
    return _merge_heads(out) @ w_proj + b_proj


def cross_attention(u, y, w_q, b_q, w_kv, b_kv, w_proj, b_proj, heads):
    """Queries from u [n, D], keys/values from the projected text y [L, D]."""
    D = u.shape[1]
    q = u @ w_q + b_q
    kv = y @ w_kv + b_kv
    k, v = kv[:, :D], kv[:, D:]
    o = attention(_split_heads(q, heads), _split_heads(k, heads), _split_heads(v, heads))
    return _merge_heads(o) @ w_proj + b_proj


# --------------------------------------------------------------------------- the network

def _block_factorized(x, y, mod, W, pre, cfg):
    """x [N, D] video tokens ordered (t, s); y [L, D] projected text; mod [9D]."""
    D, T, S, h, eps = cfg.hidden, cfg.frames, cfg.spatial_tokens, cfg.heads, cfg.ln_eps
    sh_sp, sc_sp, g_sp, sh_tm, sc_tm, g_tm, sh_m, sc_m, g_m = [mod[i * D:(i + 1) * D] for i in range(9)]

    # spatial attention: each frame is its own sequence of S tokens
    u = modulate(layernorm(x, eps), sh_sp, sc_sp).reshape(T, S, D)
    a = self_attention(u, W[pre + "sp_qkv_w"], W[pre + "sp_qkv_b"],
                       W[pre + "sp_proj_w"], W[pre + "sp_proj_b"], h)            # T sequences of S
    x = x + g_sp * a.reshape(T * S, D)

    # temporal attention: each spatial position is its own sequence of T tokens
    u = modulate(layernorm(x, eps), sh_tm, sc_tm).reshape(T, S, D).transpose(1, 0, 2)
    a = self_attention(u, W[pre + "tm_qkv_w"], W[pre + "tm_qkv_b"],
                       W[pre + "tm_proj_w"], W[pre + "tm_proj_b"], h)            # S sequences of T
    x = x + g_tm * a.transpose(1, 0, 2).reshape(T * S, D)

    # text cross-attention: plain LayerNorm on the query side, no modulation, no gate
    x = x + cross_attention(layernorm(x, eps), y, W[pre + "x_q_w"], W[pre + "x_q_b"],
                            W[pre + "x_kv_w"], W[pre + "x_kv_b"],
                            W[pre + "x_proj_w"], W[pre + "x_proj_b"], h)

    # MLP
    u = modulate(layernorm(x, eps), sh_m, sc_m)
    hid = gelu_tanh(u @ W[pre + "fc1_w"] + W[pre + "fc1_b"])
    return x + g_m * (hid @ W[pre + "fc2_w"] + W[pre + "fc2_b"])


def _block_full3d(x, mod, W, pre, cfg, q_rows=None):
    """x [L+N, D] (text rows first); mod [6D], or [12D] when the text rows have their own
    modulation (cfg.text_adaln): the first 6D chunks act on the video rows, the last 6D on
    the L text rows.  With q_rows the block is evaluated for those rows only (attention
    still sees every key/value row)."""
    D, h, eps = cfg.hidden, cfg.heads, cfg.ln_eps
    sh_a, sc_a, g_a, sh_m, sc_m, g_m = [mod[i * D:(i + 1) * D] for i in range(6)]
    if getattr(cfg, "text_adaln", 0):
        # every modulation vector becomes a per-row table: text set on rows < L, video set after
        is_text = (np.arange(x.shape[0]) < cfg.text_len)[:, None]
        tsh_a, tsc_a, tg_a, tsh_m, tsc_m, tg_m = [mod[(6 + i) * D:(7 + i) * D] for i in range(6)]
        sh_a, sc_a, g_a = [np.where(is_text, tv, vv) for tv, vv in ((tsh_a, sh_a), (tsc_a, sc_a), (tg_a, g_a))]
        sh_m, sc_m, g_m = [np.where(is_text, tv, vv) for tv, vv in ((tsh_m, sh_m), (tsc_m, sc_m), (tg_m, g_m))]
    u = modulate(layernorm(x, eps), sh_a, sc_a)
    a = self_attention(u, W[pre + "qkv_w"], W[pre + "qkv_b"], W[pre + "proj_w"], W[pre + "proj_b"],
                       h, q_rows=q_rows)
    if q_rows is not None and getattr(cfg, "text_adaln", 0):
        g_a, sh_m, sc_m, g_m = g_a[q_rows], sh_m[q_rows], sc_m[q_rows], g_m[q_rows]
    xr = x if q_rows is None else x[q_rows]
    xr = xr + g_a * a
    u = modulate(layernorm(xr, eps), sh_m, sc_m)
    hid = gelu_tanh(u @ W[pre + "fc1_w"] + W[pre + "fc1_b"])
    return xr + g_m * (hid @ W[pre + "fc2_w"] + W[pre + "fc2_b"])


def forward(cfg, weights: Dict[str, np.ndarray], latent, text, t, dtype=np.float64,
            video_rows: Optional[np.ndarray] = None):
    """Predicted noise eps [T,H,W,C] for one sample.

    cfg      object with the fields of the model configuration (frames, height, width,
             channels, patch, hidden, heads, mlp_dim, depth, text_len, text_dim,
             t_embed_dim, attn_mode, ln_eps and the derived spatial_tokens).
    latent   [T,H,W,C]; text [L, text_dim]; t the integer training timestep.
    video_rows  (full-3D mode, depth 1 only) evaluate just these video-token rows and
             return their output patches [len(rows), p*p*C] instead of the latent-shaped eps.
    """
    if dtype is None:                                # weights already prepared by the caller
        W, dtype = weights, np.asarray(latent).dtype
    else:
        W = {k: np.asarray(v, dtype=dtype) for k, v in weights.items()}
    D, p = cfg.hidden, cfg.patch
    T, H, Wd, C = cfg.frames, cfg.height, cfg.width, cfg.channels
    lat = np.asarray(latent, dtype=dtype)
    txt = np.asarray(text, dtype=dtype)

    # conditioning vector from the timestep: sinusoid -> Linear -> SiLU -> Linear
    e = timestep_embedding(t, cfg.t_embed_dim, dtype)
    c = silu(e @ W["t_w1"] + W["t_b1"]) @ W["t_w2"] + W["t_b2"]
    sc = silu(c)                                    # every adaLN layer starts from SiLU(c)

    y = txt @ W["y_w"] + W["y_b"]                    # text projected to the model width
    pos = positional_embedding(T, H // p, Wd // p, D).reshape(-1, D).astype(dtype)
    x = patchify(lat, p) @ W["p_w"] + W["p_b"] + pos

    rows = None
    if cfg.attn_mode == FULL3D_CONCAT:
        x = np.concatenate([y, x], axis=0)           # text tokens first, no positions on them
        if video_rows is not None:
            if cfg.depth != 1:
                raise ValueError("row sampling is defined for a single block only")
            rows = np.asarray(video_rows) + cfg.text_len
    elif video_rows is not None:
        raise ValueError("row sampling is defined for the full-3D mode only")

    for l in range(cfg.depth):
        pre = f"blk{l}."
        mod = sc @ W[pre + "mod_w"] + W[pre + "mod_b"]
        if cfg.attn_mode == FACTORIZED_CROSS:
            x = _block_factorized(x, y, mod, W, pre, cfg)
        else:
            x = _block_full3d(x, mod, W, pre, cfg, q_rows=rows)

    if cfg.attn_mode == FULL3D_CONCAT and rows is None:
        x = x[cfg.text_len:]                         # text rows are dropped before the head
    fm = sc @ W["f_mod_w"] + W["f_mod_b"]
    out = modulate(layernorm(x, cfg.ln_eps), fm[:D], fm[D:]) @ W["f_w"] + W["f_b"]
    if rows is not None:
        return out
    return unpatchify(out, T, H, Wd, C, p)
