"""The parity figure used by the GPU tests (gpu_util.err) notices a single wrong row that the whole-tensor
relative L2 norm lets through.  CPU only."""
import numpy as np

from gpu_util import ROW_SLACK, TOL_BF16, err, rel_l2, worst_row


def test_one_wrong_row_fails_the_row_metric_but_not_the_norm():
    rng = np.random.default_rng(0)
    ref = rng.standard_normal((1, 4096, 1536))
    got = ref * (1 + 3.5e-3 * rng.standard_normal(ref.shape))        # the measured bf16 noise level
    assert err(got, ref) < TOL_BF16
    bad = got.copy()
    bad[0, 1234] = 0.3 * ref[0, 1234]                                 # one token row scaled by a wrong gate
    assert rel_l2(bad, ref) < TOL_BF16                                # the norm does not see it
    assert worst_row(bad, ref) > 0.5 and err(bad, ref) > TOL_BF16     # the row metric does
    two = np.concatenate([got, got])
    two[1, 4000] = ref[0, 4001]                                       # batch 2: a row replaced by its neighbour
    assert rel_l2(two, np.concatenate([ref, ref])) < TOL_BF16 and err(two, np.concatenate([ref, ref])) > TOL_BF16
    half = got.copy()
    half[0, 7, :768] = 0.0                                            # half of one row missing (a dropped k split)
    assert rel_l2(half, ref) < TOL_BF16 and err(half, ref) > TOL_BF16


def test_row_metric_floor_and_shapes():
    ref = np.zeros((8, 128))
    ref[:7] = 1.0
    got = ref.copy()
    got[7] += 1e-3                                                    # a zero row is measured against a typical row
    assert worst_row(got, ref) < 2e-3
    lat = np.random.default_rng(1).standard_normal((2, 16, 16, 4))    # trailing axes merged to rows of 64
    assert worst_row(lat * 1.01, lat) < 0.0101 and ROW_SLACK >= 1.0
    assert err(np.ones(5), np.ones(5)) == 0.0
