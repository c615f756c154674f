"""Host-side parts of the pipeline module (no GPU): the calibration file format."""
import numpy as np

import paper_2603_05503_amd as pkg


def test_calibration_file_round_trip(tmp_path):
    rng = np.random.default_rng(3)
    results = {
        (0, 0): pkg.CalibrationResult(mask=(rng.random((3, 5, 7)) < 0.4).astype(np.uint8), repetitive_heads=[2],
                                      scores=np.array([0.1, 0.5, 0.93]), n_prompts=64),
        (49, 39): pkg.CalibrationResult(mask=np.ones((3, 5, 7), np.uint8), repetitive_heads=[], scores=None, n_prompts=1),
        (7, 1): pkg.CalibrationResult(mask=np.zeros((3, 5, 7), np.uint8), repetitive_heads=[0, 1, 2],
                                      scores=np.array([0.9, 0.95, 0.99]), n_prompts=16),
    }
    path = str(tmp_path / "calibration.npz")
    pkg.save_calibration(path, results)
    back = pkg.load_calibration(path)
    assert set(back) == set(results)
    for key, want in results.items():
        got = back[key]
        assert got.mask.dtype == np.uint8 and np.array_equal(got.mask, want.mask)
        assert got.repetitive_heads == want.repetitive_heads and got.n_prompts == want.n_prompts
        assert (got.scores is None) == (want.scores is None)
        if want.scores is not None:
            assert np.array_equal(got.scores, want.scores)
