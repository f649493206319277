import os
import shutil
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _library_present():
    """Tests load the library that is built; they build it only if there is none."""
    from paper_2601_21686_amd import binding
    if not os.path.exists(binding.LIB_PATH) and (shutil.which("hipcc") or os.path.exists("/opt/rocm/bin/hipcc")):
        from paper_2601_21686_amd import build
        build.build(verbose=False)
    yield


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(params=["vector", "matrix", "vector-streamed", "matrix-streamed"])
def decode_engine(request):
    """Runs a test once per range kernel over bf16 rows (vector arithmetic, matrix cores) and per kind of
    cache load (chosen by size, which means ordinary loads at test sizes; streaming loads forced).  The
    choice travels in the flags word of every layer the test builds (the binding's default for new layers)."""
    from paper_2601_21686_amd import binding
    flags = binding.SKV_ENGINE_MATRIX if request.param.startswith("matrix") else binding.SKV_ENGINE_VECTOR
    if request.param.endswith("streamed"):
        flags |= binding.SKV_READS_STREAMING
    before = binding.DEFAULT_LAYER_FLAGS
    binding.DEFAULT_LAYER_FLAGS = flags
    yield 1 if request.param.startswith("matrix") else 0
    binding.DEFAULT_LAYER_FLAGS = before
