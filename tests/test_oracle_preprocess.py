"""Pins for the oracle's frame preprocessing (Sec.3: grey-scale, linear interpolation to 84x84)."""
import numpy as np
import pytest
import torch


def test_constant_and_identity(orc):
    raw = np.full((2, 210, 160), 77, np.uint8)
    out, val = orc.preprocess(raw)
    assert np.all(out == 77) and np.allclose(val, 77.0)
    rng = np.random.default_rng(0)
    same = rng.integers(0, 256, (3, 84, 84), dtype=np.uint8)      # 84x84 in: every sample point is a pixel centre
    out, _ = orc.preprocess(same)
    assert np.array_equal(out, same)


def test_linear_ramps_are_reproduced(orc):
    """Bilinear interpolation is exact on an image that is linear in x and y (away from the clamp)."""
    H, W = 210, 160
    y, x = np.mgrid[0:H, 0:W]
    lut = np.arange(256, dtype=np.float32)
    # byte = x index (0..159), table maps byte -> 1.5 * byte: a pure horizontal ramp
    raw = np.broadcast_to(x.astype(np.uint8), (1, H, W)).copy()
    out, val = orc.preprocess(raw, (1.5 * lut).astype(np.float32))
    sx = (np.arange(84) + 0.5) * W / 84 - 0.5
    assert np.allclose(val[0], np.broadcast_to(1.5 * sx, (84, 84)), atol=1e-9)
    # vertical ramp through transposition
    rawv = np.broadcast_to(y.astype(np.uint8), (1, H, W)).copy()
    out, val = orc.preprocess(rawv)
    sy = (np.arange(84) + 0.5) * H / 84 - 0.5
    assert np.allclose(val[0], np.broadcast_to(sy[:, None], (84, 84)), atol=1e-9)


@pytest.mark.parametrize("H,W", [(210, 160), (84, 84), (100, 333), (50, 40)])
def test_against_library_bilinear_resize(orc, H, W):
    """torch's bilinear interpolate with align_corners=False is the same centre-aligned rule."""
    rng = np.random.default_rng(H * W)
    raw = rng.integers(0, 256, (2, H, W), dtype=np.uint8)
    lut = (255.0 * rng.random(256)).astype(np.float32)
    out, val = orc.preprocess(raw, lut)
    grey = torch.from_numpy(lut.astype(np.float64))[torch.from_numpy(raw.astype(np.int64))]
    ref = torch.nn.functional.interpolate(grey[:, None], size=(84, 84), mode="bilinear", align_corners=False,
                                          antialias=False)[:, 0].numpy()
    assert np.allclose(val, ref, atol=1e-9)
    assert np.array_equal(out, np.clip(np.rint(val), 0, 255).astype(np.uint8))


def test_a_wrong_half_pixel_offset_would_fail(orc):
    """The corner-aligned rule (a plausible mistake) gives different values on a ramp."""
    H = W = 160
    raw = np.broadcast_to(np.arange(W, dtype=np.uint8), (1, H, W)).copy()
    _, val = orc.preprocess(raw)
    corner_aligned = np.arange(84) * (W - 1) / 83.0
    assert np.abs(val[0, 0] - corner_aligned).max() > 0.3
