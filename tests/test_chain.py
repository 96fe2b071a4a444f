"""Profile -> planner -> stages -> schedule on a table shaped like the paper's testbed
(15 devices, Sec. 5.1; N = 34 and N = 82 layers), CPU only, from a stand-in profile.  The GPU
version of the same chain, fed by shard_profile, is in tests/test_parity_gpu.py."""
from tests import testbed


def test_chain_on_a_testbed_shaped_table(lib):
    out = testbed.check_chain(lib, testbed.STAND_IN_7B)
    assert out["t_edgeshard"] < out["t_solo"]
    print(out)
