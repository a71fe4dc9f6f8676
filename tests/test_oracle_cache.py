"""Pins of the cache-restore oracle (stitching, key frames, inter-step coefficient)
against things other than itself: special cases the paper's description fixes,
numpy's own bit unpacking and least squares, brute force on tiny inputs."""
import numpy as np
import pytest

from oracle import cache


def _rand_mask(rng, n, p=0.5):
    return rng.random(n) < p


# --------------------------------------------------------------------------- masks

def test_pack_matches_numpy_little_endian_bits():
    rng = np.random.default_rng(0)
    for n in (1, 7, 8, 9, 64, 203):
        m = _rand_mask(rng, n)
        packed = cache.pack_mask(m)
        assert packed.size == (n + 7) // 8
        assert np.array_equal(np.unpackbits(packed, bitorder="little")[:n].astype(bool), m)
        assert np.array_equal(cache.unpack_mask(packed, n), m)


def test_mask_of_paper_sized_entry_takes_40_kilobytes():
    # Sec. 4.3: the segmentation masks of an entry take 40 KB at 1 bit per pixel: two masks
    # (object, background) over 64 frames of a 40 x 64 latent
    one = cache.pack_mask(np.zeros((64, 40, 64), dtype=bool)).nbytes
    assert 2 * one == 40 * 1024


# --------------------------------------------------------------------------- stitching (Sec. 4.2.2)

def _latents(rng, shape):
    return rng.standard_normal(shape).astype(np.float32), rng.standard_normal(shape).astype(np.float32)


def test_stitch_special_cases():
    rng = np.random.default_rng(1)
    shape = (3, 4, 5, 4)
    xo, xb = _latents(rng, shape)
    n = 3 * 4 * 5
    ones, zeros = cache.pack_mask(np.ones(n, bool)), cache.pack_mask(np.zeros(n, bool))
    assert np.array_equal(cache.stitch(xo, xb, ones, ones), xo)          # everything is object
    assert np.array_equal(cache.stitch(xo, xb, zeros, ones), xb)         # no object, clean background
    assert np.array_equal(cache.stitch(xo, xb, zeros, zeros), xo)        # background nowhere valid: object cache's pixels
    assert np.array_equal(cache.stitch(xo, xb, zeros, None), xb)


def test_stitch_aligned_masks_is_the_blend_formula():
    rng = np.random.default_rng(2)
    shape = (2, 6, 7, 3)
    xo, xb = _latents(rng, shape)
    m = _rand_mask(rng, 2 * 6 * 7)
    got = cache.stitch(xo, xb, cache.pack_mask(m), cache.pack_mask(~m))
    mm = m.reshape(2, 6, 7, 1).astype(np.float32)
    assert np.array_equal(got, mm * xo + (1 - mm) * xb)


def test_stitch_brute_force_with_misaligned_masks():
    rng = np.random.default_rng(3)
    T, H, W, C = 2, 3, 5, 2
    xo, xb = _latents(rng, (T, H, W, C))
    mo, mb = _rand_mask(rng, T * H * W, 0.4), _rand_mask(rng, T * H * W, 0.7)
    got = cache.stitch(xo, xb, cache.pack_mask(mo), cache.pack_mask(mb))
    for t in range(T):
        for h in range(H):
            for w in range(W):
                i = (t * H + h) * W + w
                # the background video's own object (mb = 0) is replaced by the object cache's pixels
                src = xo if (mo[i] or not mb[i]) else xb
                assert np.array_equal(got[t, h, w], src[t, h, w])


def test_stitch_every_output_pixel_comes_whole_from_one_source():
    rng = np.random.default_rng(4)
    xo, xb = _latents(rng, (1, 4, 4, 8))
    got = cache.stitch(xo, xb, cache.pack_mask(_rand_mask(rng, 16)), cache.pack_mask(_rand_mask(rng, 16)))
    from_o = (got == xo).all(axis=-1)
    from_b = (got == xb).all(axis=-1)
    assert (from_o | from_b).all()


# --------------------------------------------------------------------------- key frames (Sec. 4.1.1)

def test_similarity_is_cosine():
    rng = np.random.default_rng(5)
    f = rng.standard_normal((5, 3, 4, 2))
    s = cache.frame_similarity(f)
    assert np.allclose(np.diag(s), 1.0)
    a, b = f[1].ravel(), f[3].ravel()
    assert np.isclose(s[1, 3], a @ b / np.linalg.norm(a) / np.linalg.norm(b))
    assert np.allclose(s, s.T)
    assert np.isclose(cache.frame_similarity(np.stack([f[0], 3.0 * f[0], -f[0]]))[0, 1], 1.0)


def test_identical_frames_collapse_onto_the_last_one():
    f = np.tile(np.random.default_rng(6).standard_normal((1, 4, 4, 2)), (6, 1, 1, 1))
    m = cache.select_key_frames(cache.frame_similarity(f))
    assert np.array_equal(m, np.full(6, 5))          # traversal starts at the last frame: it is the key


def test_orthogonal_frames_are_all_key_frames():
    f = np.eye(5).reshape(5, 5, 1, 1)
    assert np.array_equal(cache.select_key_frames(cache.frame_similarity(f)), np.arange(5))


def test_selection_on_two_groups_and_a_loner():
    rng = np.random.default_rng(7)
    a, b, c = rng.standard_normal((3, 8, 8, 4))
    eps = 1e-3
    frames = np.stack([a, b, a + eps * rng.standard_normal(a.shape), c, b + eps * rng.standard_normal(b.shape), a])
    m = cache.select_key_frames(cache.frame_similarity(frames), 0.99)
    assert np.array_equal(m, [5, 4, 5, 3, 4, 5])
    # decompression repeats the key frames at the mapped positions
    keys = sorted(set(m.tolist()))
    rec = cache.expand_key_frames(frames[keys], keys, m)
    assert np.array_equal(rec[0], frames[5]) and np.array_equal(rec[1], frames[4]) and np.array_equal(rec[3], frames[3])


def test_every_dropped_frame_reaches_the_threshold_with_its_key_frame():
    rng = np.random.default_rng(8)
    base = rng.standard_normal((4, 6, 6, 4))
    frames = np.stack([base[rng.integers(4)] + 0.05 * rng.standard_normal((6, 6, 4)) for _ in range(24)])
    sim = cache.frame_similarity(frames)
    for thr in (0.9, 0.99):
        m = cache.select_key_frames(sim, thr)
        for f, k in enumerate(m):
            assert m[k] == k                          # maps point at key frames, never at dropped ones
            assert k >= f                             # a frame stands behind itself or a later frame
            assert f == k or sim[k, f] >= thr
        # a chain a ~ b ~ c with a !~ c must not put a behind c
    chain = np.array([[1.0, 0.995, 0.98], [0.995, 1.0, 0.995], [0.98, 0.995, 1.0]])
    assert np.array_equal(cache.select_key_frames(chain, 0.99), [0, 2, 2])


# --------------------------------------------------------------------------- inter-step coefficient (Eq. 1-2)

def test_alpha_is_the_least_squares_solution():
    rng = np.random.default_rng(9)
    first_s = rng.standard_normal((5, 6, 4))
    diff_base = rng.standard_normal((3, 5, 6, 4))
    keys_s = first_s[None] + 0.7 * diff_base + 0.1 * rng.standard_normal(diff_base.shape)
    a = cache.alpha_least_squares(first_s, keys_s, diff_base)
    A = diff_base.reshape(-1, 1)
    b = (keys_s - first_s[None]).reshape(-1)
    ref = np.linalg.lstsq(A, b, rcond=None)[0][0]
    assert np.isclose(a, ref, rtol=1e-12)
    # the residual of the restored step is orthogonal to the base (normal equation)
    res = b - a * A[:, 0]
    assert abs(res @ A[:, 0]) < 1e-9 * (A[:, 0] @ A[:, 0])
    # and no other coefficient does better
    for other in (a - 0.01, a + 0.01):
        assert np.sum((b - other * A[:, 0]) ** 2) > np.sum(res ** 2)


def test_a_step_that_is_a_multiple_of_the_base_is_restored_exactly():
    rng = np.random.default_rng(10)
    first_s = rng.standard_normal((4, 4, 2))
    diff_base = rng.standard_normal((2, 4, 4, 2))
    keys_s = first_s[None] - 1.25 * diff_base
    a = cache.alpha_least_squares(first_s, keys_s, diff_base)
    assert np.isclose(a, -1.25)
    rec = cache.decompress(first_s, diff_base, a, np.zeros((0, 4, 4, 2)), [0, 1, 2])
    assert np.allclose(rec[0], first_s) and np.allclose(rec[1:], keys_s)


def test_alpha_of_a_base_without_motion_is_zero():
    """Common key frames equal to the first frame of the base step: Diff_base = 0, Eq. 2 is 0/0.
    Every alpha then restores the same frames (first + alpha * 0), lstsq's minimum-norm answer is
    0, and the result must be finite."""
    rng = np.random.default_rng(12)
    first_s = rng.standard_normal((3, 3, 2))
    keys_s = rng.standard_normal((2, 3, 3, 2))
    diff_base = np.zeros((2, 3, 3, 2))
    a = cache.alpha_least_squares(first_s, keys_s, diff_base)
    ref = np.linalg.lstsq(diff_base.reshape(-1, 1), (keys_s - first_s[None]).reshape(-1), rcond=None)[0][0]
    assert a == 0.0 and ref == 0.0
    rec = cache.decompress(first_s, diff_base, a, None, [0, 1, 2])
    assert np.array_equal(rec, np.stack([first_s] * 3))


def test_decompress_source_codes():
    rng = np.random.default_rng(11)
    first = rng.standard_normal((3, 3, 2))
    diff = rng.standard_normal((2, 3, 3, 2))
    extra = rng.standard_normal((2, 3, 3, 2))
    out = cache.decompress(first, diff, 0.5, extra, [0, 2, -1, 1, 2, -2, 0])
    assert out.shape == (7, 3, 3, 2)
    assert np.array_equal(out[0], first) and np.array_equal(out[6], first)
    assert np.allclose(out[1], first + 0.5 * diff[1]) and np.array_equal(out[1], out[4])
    assert np.allclose(out[3], first + 0.5 * diff[0])
    assert np.array_equal(out[2], extra[0]) and np.array_equal(out[5], extra[1])
    # alpha = 0 repeats the first frame wherever a base frame is asked for
    assert np.array_equal(cache.decompress(first, diff, 0.0, extra, [1, 2])[1], first)
