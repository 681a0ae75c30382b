"""Host-side checks of bench.py: the one-GPU contract of its command line and the paper's equivalent-bandwidth
model against the worked example the paper prints (tests/golden/equivalent_bandwidth_example.txt)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_equivalent_bandwidth_reproduces_the_papers_example():
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "equivalent_bandwidth_example.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 1
    C, S, K, O = (int(x) for x in rows[0][:4])
    b_pcie, b_gpu, alpha, printed, speedup = (float(x) for x in rows[0][4:])
    got = bench.equivalent_bandwidth(S, C, K, O, alpha, b_gpu, b_pcie) / 1000.0        # TB/s
    assert abs(got - printed) <= 0.05, got                                             # printed to 0.1 TB/s
    assert abs(got / (b_gpu / 1000.0) - speedup) <= 0.05
    # the other hit rates the text could suggest do not give the printed figure
    assert abs(bench.equivalent_bandwidth(S, C, K, O, 0.0, b_gpu, b_pcie) / 1000.0 - printed) > 1.0
    assert abs(bench.equivalent_bandwidth(S, C, K, O, 1.0, b_gpu, b_pcie) / 1000.0 - printed) > 1.0


def test_algorithmic_bytes_match_the_papers_traffic_terms():
    """Landmark and attended-row terms of the model, in bytes: M*S/C and 2*M*(K+O)*C with M = 2*d bytes per vector."""
    from workloads import CONFIGS
    wl = CONFIGS["c3-hbm"]
    ab = bench.algorithmic_bytes(wl)
    M, u = 2 * wl.head_dim, wl.batch * wl.n_kv_heads
    assert ab["landmarks"] == M * (wl.ctx_len // wl.chunk_size - wl.n_outlier_chunks) * u
    attended = ab["values"] + ab["resident_kv"] + ab["A_rows"] * 0            # K side of the sparse rows is rebuilt
    assert attended == (M * wl.topk_chunks * wl.chunk_size + 2 * M * (wl.n_outlier_chunks * wl.chunk_size + wl.local_len)) * u
