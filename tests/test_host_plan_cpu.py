"""The library's host side without a GPU: argument checks, length and position bookkeeping and,
above all, the work partitioning of every attention call, run for real on seeded random
episodes.  The library's own evl_api.cpp is linked with launchers that check the kernel arguments
instead of launching (tests/host_probe/launch_probe.cpp, built with the undefined-behaviour
sanitizer): every work item of a grid must exist, the pieces of a key range must cover its tiles
exactly once, partial results must stay inside the workspace, apart from each other, and be
merged completely, ticket counters must not be shared.  The episodes run in a child process,
which loads the probe library only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER = os.path.join(ROOT, "tests", "host_probe", "drive.py")


@pytest.fixture(scope="module")
def probe_lib():
    from paper_2512_10310_amd import build
    if build.host_probe_is_stale():
        build.build_host_probe()
    return os.path.join(ROOT, "tests", "host_probe", "libevl_probe.so")


@pytest.mark.parametrize("first_seed", [0, 150, 300])
def test_random_episodes_give_the_kernels_what_they_assume(probe_lib, first_seed):
    r = subprocess.run([sys.executable, DRIVER, probe_lib, str(first_seed), "150"], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=300)
    tail = "\n".join(r.stdout.splitlines()[-12:])
    assert r.returncode == 0, tail
    assert "runtime error" not in r.stdout, tail          # the sanitizer's report
    assert "launches checked" in r.stdout, tail


def test_planner_choices_for_known_shapes(probe_lib):
    """What the planner does with a single sequence at the 7B-class layer shape, pinned where
    measurements fixed the right answer: the 204-token step is cut into 10 pieces of one work-group
    per CU (240) at every history length; a prefill is left unsplit (every piece would be a full
    copy of its rows); mid-size chunks get the piece count that fills whole rounds of work-groups
    on every XCD."""
    r = subprocess.run([sys.executable, DRIVER, probe_lib, "plans"], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    got = {tuple(map(int, line.split()[:2])): tuple(map(int, line.split()[2:])) for line in r.stdout.splitlines()
           if line and line[0].isdigit()}
    assert got[(6580, 204)] == got[(20452, 204)] == got[(65536, 204)] == (240, 10)
    assert got[(3316, 204)] in ((240, 10), (192, 8))     # 29.3 and 30.1 us: within 3 % of each other
    # (the first 63 tokens of a sequence see fewer than 64 keys and go to the few-keys kernel:
    # 3457 and 193 tokens are left for the matrix kernel)
    assert got[(0, 3520)] == (380, 1) and got[(0, 256)] == (24, 1) and got[(20000, 4000)] == (440, 1)
    # mid-size chunks: one round of work-groups where that is the best plan measured (224 = 28 per XCD), two
    # full rounds on every XCD where those were (9 pieces x 56 = 63 work-groups per XCD)
    assert got[(5000, 1000)] == (224, 2) and got[(60000, 500)] == (504, 9)
    assert got[(6580, 40)][0] <= 256 and got[(6580, 40)][1] > 8
    # no plan puts one work-group more than a whole number of rounds on an XCD's 32 compute units: 100 new
    # tokens are 3 row tiles x 4 KV heads, and 21 pieces would put 33 work-groups on four of the XCDs
    assert got[(60000, 100)] == (240, 20)


def test_the_probe_is_not_the_product():
    """The probe library sits with the tests and the binding never loads it by itself."""
    import paper_2512_10310_amd as evl
    assert os.path.dirname(evl.lib_path()) == os.path.join(ROOT, "paper_2512_10310_amd")
    assert "probe" not in os.path.basename(evl.lib_path())
