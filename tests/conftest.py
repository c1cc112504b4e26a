import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _use_alternative_library(path):
    """Load the ctypes binding against another build of the C ABI (the host-only sanitizer build of
    tests/test_host_sanitizers.py): the binding's source with its library path replaced, registered under
    the binding's module name before anything imports it."""
    import types
    import paper_2604_06746_amd as pkg
    src_path = os.path.join(ROOT, "paper_2604_06746_amd", "binding.py")
    src = open(src_path).read()
    line = 'LIB_PATH = os.path.join(_HERE, "libstructkv.so")'
    assert line in src
    mod = types.ModuleType("paper_2604_06746_amd.binding")
    mod.__file__ = src_path
    exec(compile(src.replace(line, "LIB_PATH = %r" % path), src_path, "exec"), mod.__dict__)
    sys.modules["paper_2604_06746_amd.binding"] = mod
    pkg.binding = mod


if os.environ.get("STRUCTKV_TEST_LIB"):
    _use_alternative_library(os.environ["STRUCTKV_TEST_LIB"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle
