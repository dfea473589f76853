import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

_spawner = None


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # Whatever is not built yet is built now, and the helper below is started now: both start other
    # programs, which a process must not do once it has initialised the GPU (see tests/spawner.py).
    import oracle
    oracle.build()
    from paper_2601_11743_amd import build as lib_build
    if not all(os.path.exists(p) for p in (lib_build.LIB, lib_build.SHIM, lib_build.SHIM_APP)):
        lib_build.build()
    global _spawner
    if _spawner is None:
        _spawner = subprocess.Popen([sys.executable, "-u", os.path.join(ROOT, "tests", "spawner.py")],
                                    stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True, cwd=ROOT)


def pytest_unconfigure(config):
    global _spawner
    if _spawner is not None:
        try:
            _spawner.stdin.close()
            _spawner.wait(timeout=10)
        except Exception:
            _spawner.kill()
        _spawner = None


@pytest.fixture(scope="session")
def run_program():
    """run_program(argv, env=None, timeout=60) -> {"rc", "stdout", "stderr"}: a fresh process started by
    the helper, which never touched the GPU."""
    def run(argv, env=None, timeout=60):
        assert _spawner is not None and _spawner.poll() is None, "the program-starting helper is not running"
        _spawner.stdin.write(json.dumps({"argv": list(argv), "env": env or {}, "timeout": timeout}) + "\n")
        _spawner.stdin.flush()
        return json.loads(_spawner.stdout.readline())
    return run


@pytest.fixture(scope="session")
def oracle():
    import oracle as o
    return o.Oracle()
