import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# tests/test_oracle_pin_strength.py runs the pin tests against copies of the oracle with a planted mistake: the copy's
# parent directory comes first on the path, so that `import oracle` finds the copy
if os.environ.get("SPD_ORACLE_PACKAGE_ROOT"):
    sys.path.insert(0, os.environ["SPD_ORACLE_PACKAGE_ROOT"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture
def mapping_of(ctx):
    """Layout names ending in "_hpw" force the library's head-per-wave kernel mapping (it is otherwise chosen only for
    large token-major inputs) through the option SPD_OPT_HEAD_PER_WAVE of the test module's context `ctx`; returns the
    plain layout name."""
    import paper_2409_19134_amd as spd

    def apply(layout):
        if layout is not None and layout.endswith("_hpw"):
            ctx.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, 1)
            return layout[:-4]
        ctx.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, -1)
        return layout
    yield apply
    ctx.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, -1)
