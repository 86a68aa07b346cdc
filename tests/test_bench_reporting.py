"""bench.py's bookkeeping that needs no GPU: the recorded HBM traffic of the dominant kernel
is reported only while it belongs to the current kernel sources, and says where it is from."""
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_recorded_traffic_is_labelled_and_goes_stale_with_the_sources(monkeypatch):
    import bench
    rec = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))["C5"]
    value, source = bench.recorded_traffic("C5")
    if rec["source_digest"] == bench.source_digest():
        assert value == rec["hbm_bytes_per_launch"] and "traffic.json" in source
        # the counters' bytes against the algorithmic ones: no wasted re-reads
        assert 1.0 <= value / rec["algorithmic_bytes"] < 1.01
    else:
        assert value is None and "older than the kernel sources" in source
    monkeypatch.setattr(bench, "source_digest", lambda: "0" * 16)
    value, source = bench.recorded_traffic("C5")
    assert value is None and "older than the kernel sources" in source
    value, source = bench.recorded_traffic("C1")
    assert value is None and "none recorded" in source


def test_algorithmic_bytes_of_a_step():
    import bench
    N, d, K_up, K_dn = 64, 110_000_000, 11_000, 11_000
    assert bench.algorithmic_bytes(N, d, K_up, K_dn) == 12 * N * d + 4 * d + 24 * N * K_up + 20 * K_dn
