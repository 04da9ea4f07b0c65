"""bench.py's command line, as far as it can be checked without a GPU: more than one GPU is
refused with a message, and the CPU-oracle helpers give consistent byte counts."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one-GPU" in r.stderr and r.stdout.strip() == ""


def test_cpu_sample_counts_the_bytes_of_the_streams_it_holds():
    sys.path.insert(0, ROOT)
    import bench
    from oracle import cassandra_oracle as O
    S = bench._cpu_sample(600, 4, 2, 128)
    draft = verify = 0
    for p, X in S["mats"]:
        rows, cols = p.rows, p.cols
        bw, sw, lw, pw = O.stream_words(cols, p.K, 4)
        draft += rows * 4 * (bw + sw)
        verify += rows * 4 * (bw + sw + lw + pw)
        assert X.shape == (3, cols)
    bw, sw, lw, pw = O.stream_words(128, S["pk"].K, 4)
    draft += 2 * 128 * 4 * (bw + sw)
    verify += 2 * 128 * 4 * (bw + sw + lw + pw)
    assert (S["draft_bytes"], S["verify_bytes"]) == (draft, verify)
    assert 0.45 < draft / verify < 0.55          # 8.2 of 17 bits per value at the default format
    bench._cpu_sample_pass(S)                    # one pass of the oracle over the sample runs
