import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # load what is built; build (hipcc cross-compiles without a GPU) only if nothing is there
    import importlib.util
    spec = importlib.util.spec_from_file_location(
        "_emb_build", os.path.join(ROOT, "paper_2410_22249_amd", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.ensure_built(verbose=False)


@pytest.fixture(scope="session")
def oracle():
    from oracle import emb_bag_oracle
    emb_bag_oracle.build()
    return emb_bag_oracle
