import os
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

os.environ.setdefault("OMP_NUM_THREADS", str(min(16, os.cpu_count() or 1)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import dsa_oracle
    dsa_oracle.build()
    return dsa_oracle


_inputs_cache = {}


@pytest.fixture(scope="session")
def workload():
    """workload(name) -> DsaInputs for one of the named configs, generated once per session."""
    import dsa_inputs

    def get(name):
        key = "C4" if name in ("C4f", "C4v") else name
        cfg = dsa_inputs.CONFIGS[name]
        if key not in _inputs_cache:
            _inputs_cache[key] = dsa_inputs.make_inputs(cfg)
        x = _inputs_cache[key]
        if x.cfg is not cfg:   # C4f / C4v share tensors, differ in granularity only
            x = dsa_inputs.DsaInputs(cfg, x.Q, x.K, x.V, x.Qt, x.Kt, x.R, x.global_pos, x._bits)
        return x

    return get
