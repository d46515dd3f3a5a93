"""CPU-only checks of the load-balancing simulation's host side: every symbol declared
in include/lbs.h is exported, and arguments outside the definition or the kernels'
limits are refused before anything is launched."""
import os
import re

import numpy as np
import pytest

import paper_2402_02447_amd as B
from paper_2402_02447_amd import lbs
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CUM = W.length_histogram_piecewise_uniform()
ENDS = W.LENGTH_STRATUM_END


def test_library_exports_every_symbol_of_lbs_h():
    L = B.load_library()
    header = open(os.path.join(ROOT, "include", "lbs.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lbs_[a-z_]+)\s*\(", header))
    assert declared == set(lbs.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_dataset_validation():
    lbs.Dataset(CUM, ENDS, device=-1).close()
    bad = CUM.copy()
    bad[100] = bad[99] - 1
    for cum, ends in [(bad, ENDS), (CUM, (128, 256, 384)), (CUM, (256, 128, 384, 512)), (np.zeros(513, np.uint32), ENDS),
                      (np.concatenate([[5], CUM[1:]]).astype(np.uint32), ENDS)]:
        with pytest.raises(lbs.LbsError) as e:
            lbs.Dataset(cum, ends, device=-1)
        assert e.value.code == -2
    with pytest.raises(lbs.LbsError) as e:
        lbs.Dataset(np.arange(2050, dtype=np.uint32), [2049], device=-1)
    assert e.value.code == -3


def test_run_validation_on_a_host_only_dataset():
    ds = lbs.Dataset(CUM, ENDS, device=-1)
    ok = dict(method=lbs.LBS_LOCAL_SNAKE, local_batch=16, gpus_per_node=8, n_gpus=1024, quota=[6, 3, 2, 5], seed=1,
              n_trials=10, sums=1 << 20)

    def code(**kw):
        with pytest.raises(lbs.LbsError) as e:
            ds.lbs_simulate(**dict(ok, **kw))
        return e.value.code
    assert code() == -5                                     # everything valid: refused only because there is no device
    assert code(method=5) == -2
    assert code(quota=[6, 3, 2, 4]) == -2                    # quotas do not add up
    assert code(quota=[6, 3, 2, 6]) == -2
    assert code(n_gpus=1020) == -2                           # not a multiple of the node size
    assert code(gpus_per_node=0) == -2
    assert code(local_batch=0) == -2
    assert code(local_batch=65, quota=[65, 0, 0, 0]) == -3
    assert code(gpus_per_node=128, n_gpus=1024) == -3        # node pool of 2048 sequences
    assert code(n_trials=1 << 31) == -3
    assert code(sums=None) == -1
    assert code(method=lbs.LBS_GLOBAL, quota=None, n_gpus=1020) == -5     # quota and node size do not matter here
    empty = CUM.copy()
    empty[129:257] = empty[128]                              # stratum 2 holds no sequences
    empty[257:] -= (CUM[256] - CUM[128])
    ds2 = lbs.Dataset(empty, ENDS, device=-1)
    with pytest.raises(lbs.LbsError) as e:
        ds2.lbs_simulate(**ok)
    assert e.value.code == -2
    with pytest.raises(lbs.LbsError) as e:
        ds2.lbs_simulate(**dict(ok, quota=[8, 0, 3, 5]))
    assert e.value.code == -5
