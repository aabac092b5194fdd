import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PLAN_KNOBS = ("FLCE_WINDOWS", "FLCE_VC_TILES", "FLCE_NC_TILES", "FLCE_GENERIC", "FLCE_SPLITK_DH", "FLCE_SPLITK_DW")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def set_plan(monkeypatch, **knobs):
    """Sets launch-plan knobs (FLCE_* names) for one test and makes the library read them: it reads its tuning
    environment once per process otherwise."""
    from paper_2511_17599_amd import binding as B
    for k, v in knobs.items():
        assert k in PLAN_KNOBS, k
        monkeypatch.setenv(k, str(v))
    B.flce_tuning_reload()


@pytest.fixture(autouse=True)
def _default_plan(monkeypatch):
    """Every test starts from the default launch plan, whatever the previous test or the caller's shell set."""
    from paper_2511_17599_amd import binding as B
    for k in PLAN_KNOBS:
        monkeypatch.delenv(k, raising=False)
    if os.path.exists(B.LIB_PATH):
        B.flce_tuning_reload()
    yield
