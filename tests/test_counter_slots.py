"""The rule that hands sets of device counters to persistent launches, tested on the CPU: the header is
plain C++ (no HIP), the test program models which launches are still running and asserts that a slot
never serves two launches that could overlap."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_slot_table_never_shares_a_slot_between_overlapping_launches(tmp_path):
    exe = tmp_path / "counter_slots_test"
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Werror",
                    "-I", os.path.join(ROOT, "paper_2202_10217_amd", "csrc"),
                    os.path.join(ROOT, "tests", "host", "counter_slots_test.cpp"), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert "counter slots ok" in out
