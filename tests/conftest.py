import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def as_stored():
    """An oracle result as a tensor with the dtype and device of a GPU tensor.  The backward entry
    point takes the forward states as an input; its parity tests hand the oracle's own states, in
    the storage type, to both sides, so that nothing the oracle reads was computed on the GPU."""
    import numpy as np
    import torch

    def convert(ref, like):
        return torch.from_numpy(np.ascontiguousarray(ref)).to(like.dtype).to(like.device)
    return convert


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle.build()
    return oracle
