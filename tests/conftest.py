import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as orc

    orc.lib()
    return orc


@pytest.fixture(scope="session")
def gpu():
    """Device handle for the GPU tests: the binding, and helpers that move NumPy arrays to the MI355X and
    back.  Output tensors start as NaN so that an element a kernel fails to write is caught."""
    import numpy as np
    import torch

    from paper_2407_13726_amd import dastac

    assert torch.cuda.is_available(), "these tests need the MI355X"
    dastac.lib()

    class G:
        pass

    g = G()
    g.torch, g.d, g.dev = torch, dastac, torch.device("cuda:0")
    g.up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(g.dev)
    g.empty = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device=g.dev)
    g.down = lambda t: (torch.cuda.synchronize(), t.cpu().numpy())[1]
    return g
