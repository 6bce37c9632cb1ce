"""The rocprofv3 summaries under profiles/ say which build of the kernels they were taken on
(kernel_sources_digest, a hash over paper_2509_19729_amd/csrc/).  bench.py quotes a summary's
HBM traffic only when that digest matches the sources being run; this test makes a stale
summary visible as soon as a kernel source changes without the profiles being taken again."""
import glob
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_profile_summaries_were_taken_on_the_current_kernel_sources():
    import bench
    now = bench.kernel_sources_digest()
    seen = 0
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        m = re.search(r"^kernel_sources_digest (\w+)$", open(path).read(), flags=re.M)
        if m:                       # older summaries of unchanged kernels carry no digest
            seen += 1
            assert m.group(1) == now, f"{os.path.basename(path)} was taken on another build"
    assert seen >= 10


def test_reshard_summaries_carry_what_bench_quotes():
    for path in glob.glob(os.path.join(ROOT, "profiles", "reshard_*.txt")):
        text = open(path).read()
        assert re.search(r"^traffic_bytes_per_launch reshard_weights_kernel: \d+$", text, flags=re.M)
        assert re.search(r"^traffic_bytes_per_launch kv_(regroup|small)_kernel: \d+$", text, flags=re.M)
        assert "rocprofv3 --pmc FETCH_SIZE" in text and "rocprofv3 --pmc WRITE_SIZE" in text
