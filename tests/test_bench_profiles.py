"""The committed rocprofv3 summaries cover every kernel bench.py quotes HBM traffic for: a kernel
that is renamed or re-instantiated without the summaries being regenerated fails here, on the
CPU, instead of turning into a silent null in the benchmark line."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_every_quoted_kernel_has_a_row_in_its_workload_summary():
    assert set(w for w, _ in bench.KERNEL_OF) <= set(bench.WORKLOADS)
    for (workload, leg), (prefix, _note) in bench.KERNEL_OF.items():
        full, traffic = bench.read_traffic(workload, prefix)
        assert full is not None, "profiles/%s_hbm_traffic.txt has no row for %s (leg %s)" % (workload, prefix, leg)
        assert full.startswith(prefix) and traffic is not None and traffic > 0


def test_summaries_name_their_commands_and_calibration():
    for w in bench.WORKLOADS:
        text = open(os.path.join(ROOT, "profiles", "%s_hbm_traffic.txt" % w)).read()
        assert "rocprofv3 --kernel-trace --stats" in text and "--pmc FETCH_SIZE" in text and "--pmc WRITE_SIZE" in text
        assert "bench.py --workload %s" % w in text and "cs::plain_copy_kernel" in text


def test_traffic_stays_close_to_the_algorithmic_bytes_of_the_decode_workload():
    """Counter bytes / algorithmic bytes of the decode kernel on the Llama-8B workload: wasted
    re-reads would show here first.  (Algorithmic: K/V of every key once, Q in, O out, table.)"""
    from paper_2410_01228_amd import synth
    b = synth.config_llama8b_decode()
    dec_bytes, _, _ = bench.attention_work(b)
    _, traffic = bench.read_traffic("llama8b_decode", bench.KERNEL_OF[("llama8b_decode", "paged_attention_mixed")][0])
    assert 0.98 < traffic / dec_bytes < 1.05, traffic / dec_bytes
