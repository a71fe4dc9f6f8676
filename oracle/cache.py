"""CPU oracle: restoring a cached latent (the input of the resume loop).

TEST INFRASTRUCTURE ONLY (see oracle/dit.py): never imported by the product path.

What it follows.

* Stitching (Sec. 4.2.2 "Video Latent Reconstruction").  On a decoupled hit the cache
  returns two latents of the same step, one providing the object and one the background,
  each with the 1-bit-per-pixel mask saved with it (Sec. 4.3: masks at latent
  resolution, one bit per pixel and frame).  The required part is taken from each latent;
  where the two masks do not align they are combined, and what the background video
  shows in place of its own object is replaced by the object cache's pixels at the same
  location.  Written out: with m_obj = 1 where the object video holds the object and
  m_bg = 1 where the background video holds background,
      take_obj = m_obj OR (NOT m_bg),      x = take_obj ? x_obj : x_bg,
  the same decision for every channel of a pixel.  For aligned masks (m_bg = NOT m_obj)
  this is x = m_obj * x_obj + (1 - m_obj) * x_bg.
* Intra-step compression (Sec. 4.1.1): frames are visited from the last to the first;
  the visited frame becomes a key frame and every not yet assigned frame in front of it
  whose cosine similarity with it reaches the threshold (0.99, Sec. 5 "Cache
  compressor") is mapped to it and dropped; a frame with no similar frame maps to
  itself.  Decompression repeats the key frames at the mapped positions.
* Inter-step compression (Sec. 4.1.2, Eq. 1-2): Diff_s^m = Frame_s^m - Frame_s^0; the
  differential values of another step are modelled as alpha_s * Diff_base with the single
  least-squares coefficient
      alpha_s = sum(Diff_s * Diff_base) / sum(Diff_base^2)
  summed over the pixels of all common key frames, so that a stored step is restored as
  Frame_s^m = Frame_s^0 + alpha_s * Diff_base^m; key frames a step has beyond the
  common ones are stored whole ("extra frames").

Readings the paper leaves open, as taken here: masks are packed least-significant bit
first, pixel index (t, h, w) row-major; alpha_s is one scalar per step; similarity of two
frames is the cosine of the frames flattened over (h, w, c); a restored frame is
described by a source code: 0 = the stored first frame, j in 1..n_base = first frame +
alpha * Diff_base[j-1], -(e+1) = extra frame e.

Pins (tests/test_oracle_cache.py): mask special cases (all object, all background,
invalid background), the aligned-mask blend formula, per-pixel brute force, bit order
against numpy.unpackbits; alpha against numpy.linalg.lstsq, exact recovery of a step
that is a multiple of the base, orthogonality of the residual; key-frame selection on
constructed frame sets (identical frames, orthogonal frames, a chain), and the
guarantee that every dropped frame reaches the threshold with its key frame.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- masks and stitching

def pack_mask(mask) -> np.ndarray:
    """Boolean array (any shape, pixel order row-major) -> bytes, pixel i in bit i % 8 of byte i // 8."""
    flat = np.asarray(mask, dtype=bool).reshape(-1)
    out = np.zeros((flat.size + 7) // 8, dtype=np.uint8)
    for i in np.flatnonzero(flat):
        out[i // 8] |= np.uint8(1 << (i % 8))
    return out


def unpack_mask(packed, pixels: int) -> np.ndarray:
    packed = np.asarray(packed, dtype=np.uint8)
    idx = np.arange(pixels)
    return ((packed[idx // 8] >> (idx % 8).astype(np.uint8)) & 1).astype(bool)


def stitch(x_obj, x_bg, m_obj_packed, m_bg_packed=None):
    """x_obj, x_bg: [..., C] latents of equal shape, pixels = product of the leading dims.
    m_*_packed: packed masks over the pixels; m_bg None = background valid everywhere."""
    x_obj = np.asarray(x_obj)
    x_bg = np.asarray(x_bg)
    pixels = int(np.prod(x_obj.shape[:-1]))
    take_obj = unpack_mask(m_obj_packed, pixels)
    if m_bg_packed is not None:
        take_obj = take_obj | ~unpack_mask(m_bg_packed, pixels)
    sel = take_obj.reshape(x_obj.shape[:-1] + (1,))
    return np.where(sel, x_obj, x_bg)


# --------------------------------------------------------------------------- intra-step: key frames

def frame_similarity(frames) -> np.ndarray:
    """[T, ...] -> [T, T] cosine similarities of the flattened frames (float64)."""
    f = np.asarray(frames, dtype=np.float64).reshape(len(frames), -1)
    n = np.sqrt((f * f).sum(axis=1))
    return (f @ f.T) / np.maximum(np.outer(n, n), 1e-300)


def select_key_frames(sim, threshold=0.99) -> np.ndarray:
    """sim [T, T] -> map [T]: map[f] = index of the key frame that stands for frame f
    (map[f] == f for key frames)."""
    T = sim.shape[0]
    mapping = np.full(T, -1, dtype=np.int64)
    for f in range(T - 1, -1, -1):
        if mapping[f] >= 0:
            continue                       # already stands behind a later key frame
        mapping[f] = f
        for g in range(f):
            if mapping[g] < 0 and sim[f, g] >= threshold:
                mapping[g] = f
    return mapping


def expand_key_frames(key_frames, key_index, mapping):
    """key_frames [K, ...] holding frames key_index[0..K-1]; mapping [T] -> [T, ...]."""
    where = {int(k): i for i, k in enumerate(key_index)}
    return np.stack([key_frames[where[int(m)]] for m in mapping])


# --------------------------------------------------------------------------- inter-step: alpha and restore

def alpha_least_squares(first_s, keys_s, diff_base) -> float:
    """first_s [F...], keys_s [n, F...] (the step's frames at the common key positions),
    diff_base [n, F...] -> the scalar of Eq. 2."""
    d_s = np.asarray(keys_s, dtype=np.float64) - np.asarray(first_s, dtype=np.float64)[None]
    d_b = np.asarray(diff_base, dtype=np.float64)
    den = float((d_b * d_b).sum())
    if den == 0.0:            # Diff_base == 0: Eq. 2 is indeterminate, first + alpha * 0 does not depend on alpha
        return 0.0
    return float((d_s * d_b).sum() / den)


def decompress(first, diff_base, alpha, extra, src):
    """first [F...]; diff_base [n_base, F...]; extra [n_extra, F...]; src [T] source codes
    (0: first frame; j >= 1: first + alpha * diff_base[j-1]; -(e+1): extra[e]) -> [T, F...]."""
    first = np.asarray(first)
    out = []
    for code in src:
        code = int(code)
        if code == 0:
            out.append(first.copy())
        elif code > 0:
            out.append(first + alpha * np.asarray(diff_base)[code - 1])
        else:
            out.append(np.asarray(extra)[-code - 1].copy())
    return np.stack(out)
