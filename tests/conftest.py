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


@pytest.fixture(params=[(0, 2), (1, 2), (0, 0), (1, 0)], ids=["vector", "matrix", "vector-streamed", "matrix-streamed"])
def decode_engine(request):
    """Runs a test once per range kernel over bf16 rows (vector arithmetic, matrix cores) and per kind of
    cache load (chosen by size, which means ordinary loads at test sizes; streaming loads forced)."""
    from paper_2601_21686_amd import binding
    engine, reads = request.param
    before = binding.skv_set_decode_engine(engine)
    before_reads = binding.skv_set_cache_reads(reads)
    yield engine
    binding.skv_set_decode_engine(before)
    binding.skv_set_cache_reads(before_reads)
