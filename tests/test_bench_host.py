"""Host-side checks of the benchmark harness that need no GPU: it refuses more than one GPU
before touching a device, its algorithmic byte counts are the formulas of the roofline table,
and the committed counter summary it reads `roofline.traffic` from parses to figures that are
consistent with those formulas."""
import os
import subprocess
import sys

import numpy as np

from paper_2509_04084_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=300)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_committed_traffic_is_close_to_the_algorithmic_bytes():
    sys.path.insert(0, ROOT)
    import bench
    traffic = bench.measured_traffic(os.path.join(ROOT, "profiles", "hbm_traffic_gpt2xl_llama7b.txt"))
    sparse, dense = synth.workload("gpt2xl"), synth.workload("llama7b")
    n, K, W = sparse.n, int(sparse.seg_k.astype(np.int64).sum()), sparse.window
    want = {
        "ld_compress_topk": 12 * n + 8 * K,                         # g and r in, r out, the records
        "ld_merge_sparse": 8 * n + 8 * K * W,                       # w in and out, every record once
        "ld_snapshot_layers": 4 * dense.n,                          # bf16 in, bf16 out
        "ld_merge_dense_adam": (24 + 2 * dense.window) * dense.n,   # w, m, v in and out, W bf16 gradients
    }
    assert set(want) <= set(traffic)
    for name, nbytes in want.items():
        ratio = traffic[name] / nbytes
        assert 0.99 <= ratio <= 1.06, (name, ratio)   # measured HBM bytes: never below, a few percent above
    assert bench.HBM_PEAK_GBS == 8000.0
    assert bench.measured_traffic(os.path.join(ROOT, "profiles", "no_such_file.txt")) == {}
