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


def test_counter_figures_are_tied_to_the_sources_they_were_measured_on(monkeypatch):
    """bench.py passes on a hardware-counter figure from profiles/ only when the summary names the
    digest of the very sources of this build; otherwise traffic is null and the provenance says why."""
    sys.path.insert(0, ROOT)
    import bench
    digest = bench.source_digest()
    assert re.fullmatch(r"[0-9a-f]{16}", digest) and digest == bench.source_digest()
    fresh = {"traffic_bytes_per_launch": "12113000000", "source_digest": digest, "commit": "abc1234", "box": "mi355x"}
    monkeypatch.setattr(bench, "counter_summary", lambda kernel, workload: dict(fresh))
    value, prov = bench.measured_traffic("k_ef_filter", "C3")
    assert value == 12113000000.0 and prov["matches_this_build"] and prov["commit"] == "abc1234"
    stale = dict(fresh, source_digest="0" * 16)
    monkeypatch.setattr(bench, "counter_summary", lambda kernel, workload: dict(stale))
    value, prov = bench.measured_traffic("k_ef_filter", "C3")
    assert value is None and prov["matches_this_build"] is False and prov["source_digest"] == "0" * 16
    monkeypatch.setattr(bench, "counter_summary", lambda kernel, workload: None)
    assert bench.measured_traffic("k_ef_filter", "C3") == (None, None)


def test_the_committed_counter_summary_parses():
    sys.path.insert(0, ROOT)
    import bench
    summary = bench.counter_summary("k_ef_filter", "C3")
    assert summary is not None and float(summary["traffic_bytes_per_launch"]) > 1e10
    assert bench.VALU_PEAK_TINSTR == 157.3 / 2.0
