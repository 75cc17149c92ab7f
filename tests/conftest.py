import os
import sys
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


_capture_manager = None


def pytest_configure(config):
    global _capture_manager
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    _capture_manager = config.pluginmanager.getplugin("capturemanager")


def progress(*args):
    """A line that reaches the terminal while the test is still running, whatever pytest's capture mode: the long GPU
    tests (oracle on the host for minutes) report each step, so that a watcher can tell a slow test from a hung one."""
    line = " ".join(str(a) for a in args)
    if _capture_manager is not None:
        with _capture_manager.global_and_fixture_disabled():
            print("\n[progress] " + line, end="", file=sys.stderr, flush=True)
    else:
        print(line, file=sys.stderr, flush=True)


@pytest.fixture(scope="session")
def tiny_shape():
    import das_inputs as di
    return di.MODELS["tiny"]


@pytest.fixture(scope="session")
def tiny_oracle(tiny_shape):
    """Config-1 model: bf16-rounded N(0,0.02) weights from seed 0, widened to fp32."""
    import das_inputs as di
    import oracle
    blob = di.weights_bf16(tiny_shape, seed=0)
    return oracle.OracleModel(tiny_shape, di.bf16_to_f32(blob))
