"""Host-side checks of bench.py's contract: the one-GPU rule, the byte model behind its roofline
figures, and the source stamp that gates the stored counter figure.  No GPU is needed."""
import json
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""     # no JSON line for a run that did not happen


def test_byte_model_matches_the_method_s_cost_terms():
    """Per (sequence, query head) and step: the centroid matrix shared by the G heads of a KV head, m
    rows of L entries of 8 bytes, 2 (k + t) K/V rows of 256 bytes, and q, out and the index list
    (Sec. 3.4's cost terms, in bytes)."""
    from paper_2604_08584_amd.workload import CONFIGS, algorithmic_bytes_per_head
    b = algorithmic_bytes_per_head(CONFIGS["cfg4"], 10.0)        # C = 4096, G = 8, m = 32, L = 4096, k = 6554
    assert b["centroids"] == 4096 * 128 * 2 / 8
    assert b["table_rows"] == 32 * 4096 * 8
    assert b["kv_rows"] == 2 * (6554 + 10) * 256
    assert b["io"] == 256 + 512 + 4 * 6554
    s8 = algorithmic_bytes_per_head(CONFIGS["paper_s8"], 0.0)    # 8 subspaces, one probe each, L = 6554
    assert s8["table_rows"] == 8 * 1 * 6554 * 8
    assert s8["centroids"] == 128 * 128 * 2 / 4                  # 8 x 128 centroids of 16 dimensions


def test_stored_traffic_figures_carry_a_source_stamp():
    """bench.py quotes roofline.traffic from profiles/ only while the stamp stored there equals the
    hash of the kernel sources: the files must carry a stamp of the right shape and a byte count."""
    import bench
    sha = bench.source_sha()
    assert re.fullmatch(r"[0-9a-f]{12}", sha)
    for cfg in ("cfg4", "cfg2"):
        text = open(os.path.join(ROOT, "profiles", f"attention_split_{cfg}_hbm_traffic.txt")).read()
        m = re.search(r"kernel_source_sha: ([0-9a-f]{12})", text)
        assert m, cfg
        assert re.search(r"traffic_bytes_per_launch[^\n]*: (\d+)", text), cfg
