"""The counting logic of the in-kernel merge of the short-chunk kernel (publish the partial result,
take a ticket, the last ticket merges and resets the counter), stressed on the CPU with threads in
place of work-groups: tests/ticket_protocol/ticket_stress.cpp."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("pieces", [2, 14, 41])
def test_one_merger_per_round_and_a_clean_counter(tmp_path, pieces):
    exe = str(tmp_path / "ticket_stress")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-pthread",
                           os.path.join(ROOT, "tests", "ticket_protocol", "ticket_stress.cpp"), "-o", exe])
    r = subprocess.run([exe, str(pieces), "20000"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                       timeout=120)
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout
