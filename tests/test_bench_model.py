"""The byte accounting the benchmark's roofline fractions rest on, against the closed
forms of the paper's memory-traffic analysis (Sec. 4.3)."""
import subprocess
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parent.parent


def test_traffic_model_closed_forms():
    # Sec. 4.3: forward reads 5*k*nnz bytes with uint8 indices (8*k*nnz with 4-byte ones), saving
    # (4*dim - 5*k)*nnz over row-wise SpMM; backward reads 4*N*dim + 5*k*nnz and writes 4*k*nnz.
    from bench import algorithmic_bytes
    N, nnz, dim, k = 232_965, 114_848_855, 256, 32
    b = algorithmic_bytes(N, nnz, dim, k, index_bytes=1)
    assert b["fwd_cbsr_reads"] == 5 * k * nnz
    assert b["spmm_feature_reads"] - b["fwd_cbsr_reads"] == (4 * dim - 5 * k) * nnz
    assert b["bwd_paper_reads"] == 4 * N * dim + 5 * k * nnz and b["bwd_paper_writes"] == 4 * k * nnz
    assert algorithmic_bytes(N, nnz, dim, k, index_bytes=4)["fwd_cbsr_reads"] == 8 * k * nnz
    # totals used as roofline numerators add the adjacency and the compulsory output
    assert b["fwd"] == 4 * (N + 1) + 8 * nnz + 5 * k * nnz + 4 * N * dim
    assert b["bwd"] == 4 * (N + 1) + 8 * nnz + 4 * k * nnz + N * k * 5
    assert b["topk"] == 4 * N * dim + 5 * N * k
    assert b["spmm"] == 4 * (N + 1) + 8 * nnz + 4 * nnz * dim + 4 * N * dim
    # 16-bit CBSR values: 2 + ib bytes per kept position instead of 4 + ib; nothing else changes
    h = algorithmic_bytes(N, nnz, dim, k, index_bytes=1, value_bytes=2)
    assert h["fwd_cbsr_reads"] == 3 * k * nnz and b["fwd"] - h["fwd"] == 2 * k * nnz
    assert h["bwd"] == b["bwd"] and h["spmm"] == b["spmm"]


def test_headline_times_at_peak_bandwidth():
    # the per-k times a perfect 8 TB/s kernel would need on the dense workload
    from bench import algorithmic_bytes
    N, nnz, dim = 232_965, 114_848_855, 256
    want_fwd_ms = {8: 0.72, 16: 1.29, 32: 2.44, 64: 4.74, 96: 7.04, 128: 9.33}
    for k, ms in want_fwd_ms.items():
        assert abs(algorithmic_bytes(N, nnz, dim, k)["fwd"] / 8e12 * 1e3 - ms) < 0.01
    assert abs(algorithmic_bytes(N, nnz, dim, 32)["spmm"] / 8e12 * 1e3 - 14.85) < 0.01


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
