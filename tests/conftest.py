import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import ref
    ref.lib()
    return ref


class _LargestLayerCase:
    """Inputs of the largest benchmark layer, the declared sample of its output positions and the oracle's values
    there.  Built once per session: the inputs are 6.3 GB and take a quarter of a minute to draw."""

    def __init__(self, oracle):
        import numpy as np
        from paper_1606_05688_amd import workloads as W
        self.layer = W.CONFIGS[4]
        print(f"[largest layer] {self.layer.name}: drawing inputs", flush=True)
        self.inp, self.w, self.bias = W.make_inputs(self.layer)
        self.pts = W.sample_points(self.layer)
        print(f"[largest layer] oracle on {len(self.pts)} sampled output voxels", flush=True)
        self.exp = oracle.conv3d_points(self.inp, self.w, self.bias, self.pts, relu=self.layer.relu)
        self.tol_j = oracle.tolerance(self.inp, self.w)
        self.tol = self.tol_j[self.pts[:, 1]]
        assert np.count_nonzero(self.exp) > 0.2 * len(self.exp)      # the sample is not all rectified to zero


@pytest.fixture(scope="session")
def largest_layer_case(oracle):
    return _LargestLayerCase(oracle)
