"""The seeded input generators: shapes, determinism, and that they finish on every map size."""
import numpy as np
import pytest

from paper_2507_19131_amd import synth


@pytest.mark.timeout(60)
@pytest.mark.parametrize("H,W", [(5, 6), (7, 7), (8, 8), (9, 12), (14, 7)])
def test_blob_maps_finish_on_maps_of_a_few_pixels(H, W):
    """The high-magnitude regions are added until they cover about 30 % of the map without exceeding 31 %; on a map
    of a few pixels no further region may fit, and the generator has to stop instead of drawing for ever."""
    spec = synth.BlockSpec(3, H, W, 96, 3)
    x = synth.make_feature_map(spec, 220053, blobs=True)
    assert x.shape == (3, H, W, 96) and x.dtype == np.float32 and np.isfinite(x).all()
    assert np.array_equal(x, synth.make_feature_map(spec, 220053, blobs=True))


def test_feature_maps_are_seeded():
    spec = synth.BlockSpec(1, 28, 35, 96, 3)
    a = synth.make_feature_map(spec, 7, blobs=True, outlier_channels=True)
    b = synth.make_feature_map(spec, 7, blobs=True, outlier_channels=True)
    c = synth.make_feature_map(spec, 8, blobs=True, outlier_channels=True)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    plain = synth.make_feature_map(spec, 7)
    frac = float(np.mean(np.any(a != plain, axis=-1)))       # pixels touched by a region (outlier channels touch all)
    assert frac == 1.0
    blobs_only = synth.make_feature_map(spec, 7, blobs=True)
    cov = float(np.mean(np.any(blobs_only != plain, axis=-1)))
    assert 0.25 <= cov <= 0.31
