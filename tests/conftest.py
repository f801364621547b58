import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU runner)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import salad_oracle
    salad_oracle.build()
    return salad_oracle


@pytest.fixture(scope="session", autouse=True)
def _attn_variant_from_env():
    """Development switch: SALAD_ATTN_VARIANT=n selects an attention kernel variant for the run."""
    v = os.environ.get("SALAD_ATTN_VARIANT")
    if v is not None:
        from paper_2601_16515_amd import binding as sb
        sb.salad_tune("attn_variant", int(v))
    yield
