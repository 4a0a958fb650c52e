import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")
    # tests/test_sanitized_host_code.py re-runs the CPU tests in a child process against sanitizer builds of the
    # oracle and of the library's host side; it names those builds through these two variables.
    lib_path = os.environ.get("MOSAIC_TEST_LIBRARY")
    if lib_path:
        from paper_2601_06562_amd import binding
        binding.LIB_PATH = lib_path
    oracle_path = os.environ.get("MOSAIC_TEST_ORACLE_LIBRARY")
    if oracle_path:
        import oracle
        oracle._LIB = oracle_path


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle.build()
    return oracle
