"""More than 2^19 passages on an index small enough for the inverted form: the candidate kernel for queries without a
surviving centroid then runs several workgroups per query, each on its own range of the range table, of the bitmaps of
the long lists and of the candidate words (every other test has a single such range)."""
import numpy as np
import pytest

from synth import make_workload, tiny_config

import test_gpu_parity as tp

pytestmark = pytest.mark.gpu


def test_candidates_over_two_wide_ranges(pl=None):
    import paper_2205_09707_amd as pl_
    pl_.load_library()
    w = make_workload(tiny_config(C=16, P=600_000, lo=1, hi=2, nbits=2, nq=33, seed=71), noise="calibrated")
    tp._check_workload(pl_, w, [(1, np.inf, 64, 8), (2, np.inf, 1000, 20), (2, 0.3, 64, 8)], stage2="inverted",
                       queries=[0, 1, 16, 32])
