"""The integer maps behind the GPU search's pruning, checked on the host.

``paper_2001_01347_amd/csrc/zl_maps.h`` holds the fine-bin grid of an instance and the value buckets of a window and
of a whole instance, with the bounds on a bucket's keys that decide which buckets are dropped unseen.  It has no
device intrinsics, so ``tests/host/check_maps.cpp`` includes it into a host program and checks every bound against
exact 128-bit arithmetic or a walk over every key: spans from 0 to 2^32 - 1, scales from 1 to 2^32 - 1, ranges up to
2^62, even, clustered and degenerate key sets; and the division by a remembered reciprocal that the predicted rows'
partition kernel uses, against the plain quotient.  A bound that is too tight would not crash anything: the search would
return a barrier that is not the best one, on the rare input that hits it.
"""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bucket_bounds_and_fine_bins_hold_for_every_key(tmp_path):
    exe = str(tmp_path / "check_maps")
    subprocess.run(["g++", "-O2", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-o", exe,
                    os.path.join(ROOT, "tests", "host", "check_maps.cpp")], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "fine-bin grid:" in r.stdout and " 0 failures" in r.stdout.splitlines()[-1]
