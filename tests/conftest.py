import os
import sys
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


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
