import os
import shutil
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    """The CPU oracle (test infrastructure); compiled with gcc on first use."""
    from oracle import pq_oracle
    pq_oracle.build()
    return pq_oracle


@pytest.fixture(scope="session")
def pqlib_path():
    """Path of the built C-ABI library; rebuilt here only if hipcc is around and the sources are newer."""
    from paper_2408_09992_amd import build
    if build.is_stale():
        if shutil.which("hipcc") or os.path.exists("/opt/rocm/bin/hipcc"):
            build.build(force=True)
        else:
            pytest.fail("libpqtopk.so is missing or stale and hipcc is not available")
    return build.LIB


@pytest.fixture(scope="session")
def pq(pqlib_path):
    """The Python binding of the HIP library, on a machine with a GPU."""
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (select CPU tests with -m 'not gpu')")
    from paper_2408_09992_amd import binding
    binding.lib()
    return binding
