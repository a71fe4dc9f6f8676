"""The entry point that allocates nothing (fc_cache_frame_similarity_noalloc: the Gram
matrix in the library's own device array) against the existing entry point with a caller
workspace, through the C ABI: same kernels, so bit for bit; two calls in a row, the
second on a smaller entry, so that what the first call left in the array is seen to be
harmless; and against the oracle."""
import numpy as np
import pytest

from oracle import cache as ocache
from util import dev, host

pytestmark = pytest.mark.gpu


def _frames(T, H, W, C, seed):
    rng = np.random.default_rng(seed)
    base = rng.standard_normal((4, H, W, C))
    return np.stack([base[rng.integers(4)] + 0.05 * rng.standard_normal((H, W, C)) for _ in range(T)]).astype(np.float32)


def test_frame_similarity_without_allocation_matches_the_workspace_form(fc):
    import torch
    for T, H, W, C in ((64, 40, 64, 4), (13, 60, 90, 16), (256, 8, 8, 4), (1, 4, 4, 4)):     # big, smaller, the maximum, one
        frames = _frames(T, H, W, C, T)
        d_frames = dev(frames)
        ws = torch.empty(fc.fc_cache_workspace_bytes(T), dtype=torch.uint8, device="cuda:0")
        want_dev = torch.full((T, T), float("nan"), device="cuda:0")
        fc.fc_cache_frame_similarity(d_frames, T, H * W * C, want_dev, ws)
        got_dev = torch.full((T, T), float("nan"), device="cuda:0")
        before = torch.cuda.memory_allocated()
        fc.fc_cache_frame_similarity_noalloc(d_frames, T, H * W * C, got_dev)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        got, want = host(got_dev), host(want_dev)
        assert np.array_equal(got, want), T
        np.testing.assert_allclose(got, ocache.frame_similarity(frames), rtol=0, atol=2e-7)
    with pytest.raises(fc.FlexDenoiseError) as e:
        fc.fc_cache_frame_similarity_noalloc(d_frames, 257, 64, got_dev)
    assert e.value.status == -6
    with pytest.raises(fc.FlexDenoiseError) as e:
        fc.fc_cache_frame_similarity_noalloc(None, 1, 64, got_dev)
    assert e.value.status == -1
