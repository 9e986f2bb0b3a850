import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _ensure_library():
    """Tests load the library that is built; only if none is there do they build it."""
    lib = os.path.join(ROOT, "paper_2006_05664_amd", "libopevo.so")
    if not os.path.exists(lib):
        import importlib.util as _u
        spec = _u.spec_from_file_location("_opevo_build", os.path.join(ROOT, "paper_2006_05664_amd", "build.py"))
        _b = _u.module_from_spec(spec)
        spec.loader.exec_module(_b)
        _b.build_library()


_ensure_library()
