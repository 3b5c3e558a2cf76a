"""Host-side behaviour of bench.py that needs no GPU: more than one GPU is refused with a
message, and the names the benchmark prices kernels by exist in the library's profile table."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stderr + p.stdout) or "--gpus" in (p.stderr + p.stdout)
    assert not p.stdout.strip().startswith("{")          # no result line


def test_priced_kernel_names_exist_in_the_library():
    bench = open(os.path.join(ROOT, "bench.py")).read()
    api = open(os.path.join(ROOT, "paper_2507_17346_amd", "csrc", "ddef_api.hip")).read()
    table = re.search(r"kSlotNames\[SL_COUNT\] = \{(.*?)\};", api, re.S).group(1)
    names = set(re.findall(r'"(k_[a-z0-9_]+)"', table))
    block = re.search(r"ALGO_BYTES_PER_ELEM = \{(.*?)\n\}", bench, re.S).group(1)
    priced = set(re.findall(r'"(k_[a-z0-9_]+)"', block))
    assert priced and priced <= names, priced - names
    for name in ("k_grad", "k_ef_filter", "k_ef_filter_fused", "k_copy_f4", "k_aggregate_apply_tiles"):
        assert name in names
