"""The host-side parity tests of the kernel analyzer, the policy planner and the online monitor (C++ against
their oracles), collected a second time under the `gpu` marker so that the test run on the GPU machine records them
too.  They touch no GPU; the functions are the ones of test_planner_host.py and test_monitor_host.py."""
import pytest

from test_monitor_host import *      # noqa: F401,F403
from test_planner_host import *      # noqa: F401,F403

pytestmark = pytest.mark.gpu
