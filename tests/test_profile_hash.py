"""The constants bench.py takes from profiles/ belong to the kernels as they are now.

Each summary under profiles/ that bench.py reads states the hash of the kernel sources it was
measured on; bench.py drops the constants of a summary whose hash differs from the tree's.  This
test fails instead, so that a change to a kernel source is followed by new counter runs (or by a
deliberate edit of the summaries) before it is committed."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")


def _stated_hashes():
    out = {}
    for name in sorted(os.listdir(PROFILES)):
        with open(os.path.join(PROFILES, name)) as f:
            m = re.search(r"^kernel_source_sha256:\s*([0-9a-f]+)", f.read(), re.M)
        if m:
            out[name] = m.group(1)
    return out


def test_profiles_state_the_hash_of_the_kernel_sources():
    stated = _stated_hashes()
    # the files bench.py reads constants from
    for name in ("kvq_qk_kernel_c2_hbm_traffic.txt", "kvq_qk_kernel_c3_hbm_traffic.txt", "bench_c2_valu_issue.txt"):
        assert name in stated, name
    now = bench.kernel_source_hash()
    assert all(h == now for h in stated.values()), (now, stated)


def test_bench_reads_the_constants_of_matching_profiles():
    kv = bench.profile_constants("kvq_qk_kernel_c2_hbm_traffic.txt", ("dense_kernel_traffic_bytes_per_launch",))
    assert kv is not None and kv["dense_kernel_traffic_bytes_per_launch"] > 2.0e8
    kv = bench.profile_constants("bench_c2_valu_issue.txt", ("qk_valu_instructions_per_launch", "valu_issue_peak_per_s"))
    assert kv is not None and kv["qk_valu_instructions_per_launch"] > 0 and kv["valu_issue_peak_per_s"] > 0
    assert bench.profile_constants("no_such_profile.txt", ("x",)) is None
