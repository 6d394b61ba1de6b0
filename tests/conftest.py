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
    large token-major inputs) through the option SPD_OPT_HEAD_PER_WAVE of the test module's context `ctx`, with
    workgroups of up to eight KV heads; "_hpw4" and "_hpw2" the same with up to four and two.  Returns the plain
    layout name."""
    import re
    import paper_2409_19134_amd as spd

    def apply(layout):
        m = re.search(r"_hpw([2-8]?)$", layout or "")
        if m:
            ctx.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, int(m.group(1) or 8))
            return layout[:m.start()]
        ctx.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, -1)
        return layout
    yield apply
    ctx.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, -1)


@pytest.fixture
def in_flight(ctx):
    """The streaming kernel exists with one and with two 32-token steps in flight per wave, and the library picks by
    the size of the launch (small test inputs get the one-step form): in_flight(2) / in_flight(1) force a form through
    the option SPD_OPT_STEPS_IN_FLIGHT of the test module's context `ctx` - where the kernel has both (fp32 always
    takes one, 128-byte rows and the head-per-wave mapping always two) - and in_flight(None) leaves the choice to the
    library."""
    import paper_2409_19134_amd as spd

    def apply(steps):
        ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, -1 if steps is None else steps)
    yield apply
    ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, -1)

