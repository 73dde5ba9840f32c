#!/usr/bin/env python3
"""Benchmark of the MaxK-GNN aggregation hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic workload, inputs already
resident in HBM:  maxk_topk_cbsr(H) -> maxk_spgemm_fwd -> maxk_sspmm_bwd(dY).
Default workload: the dense-neighbourhood graph (N=232,965, nnz=114,848,855, dim 256)
at k=32, the k the paper recommends and profiles (Tables 2-3).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dense] [--k 32]
                    [--no-sweep] [--no-cpu]

Besides the headline value the line carries: a per-k table (every k of the workload:
forward / backward ms, edges*k/s, fraction of the 8 TB/s HBM roofline by algorithmic
bytes, speedup over the same-GPU dense SpMM baseline), the roofline object for the
dominant kernel, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

L2_TO_L1_BYTES_PER_CLK_PER_CU, N_CU, CLOCK_HZ = 64.0, 256, 2.4e9  # vector L1 fill path; MI355X CUs and peak clock
INFINITY_CACHE_BYTES = 256e6


def measured_traffic(workload: str, k: int, entry: str, kernel: str):
    """L2 <-> fabric bytes per API call from the committed rocprofv3 counter summaries under profiles/ (lines of the
    form `traffic_bytes_per_call workload=... k=... entry=... kernel=... bytes=...`, written from FETCH_SIZE and
    WRITE_SIZE runs scaled by a plain copy of known size); None when no summary covers this case."""
    want = {"workload": workload, "k": str(k), "entry": entry, "kernel": kernel}
    for f in sorted((ROOT / "profiles").glob("*.txt")):
        try:
            lines = f.read_text().splitlines()
        except OSError:
            continue
        for line in lines:
            if not line.startswith("traffic_bytes_per_call"):
                continue
            kv = dict(tok.split("=", 1) for tok in line.split()[1:] if "=" in tok)
            if all(kv.get(a) == b for a, b in want.items()) and "bytes" in kv:
                return {"bytes": float(kv["bytes"]), "source": f"profiles/{f.name}"}
    return None


def lines_touched(dim: int, k: int) -> float:
    """Expected 128-byte lines of a fp32 dY row that k distinct random columns fall into."""
    per_row = dim / 32.0
    return per_row if per_row <= 1 else per_row * (1.0 - (1.0 - 1.0 / per_row) ** k)


def algorithmic_bytes(N: int, nnz: int, dim: int, k: int, index_bytes: int = 1, value_bytes: int = 4) -> dict:
    """Bytes each operator must move, from the paper's traffic model (Sec. 4.3) plus the
    adjacency and the compulsory output, which that section leaves out.

    fwd  : CSR (rowptr + col + val) + one CBSR row (k values + k indices) per stored entry + Y
           (value_bytes = 2 for the 16-bit value formats of the *_narrow entry points)
    bwd  : CSR + 4k useful sampled bytes of dY per stored entry + sp_index and dXs once
           (design-independent count; the paper's push design moves 4*N*dim + (4+ib)*k*nnz
           reads and 4*k*nnz writes, reported separately)
    topk : H once + the CBSR once
    spmm : CSR + one dense row per stored entry + Y
    """
    ib = index_bytes
    csr = 4 * (N + 1) + 8 * nnz
    return {
        "fwd_cbsr_reads": (value_bytes + ib) * k * nnz,
        "spmm_feature_reads": 4 * dim * nnz,
        "bwd_paper_reads": 4 * N * dim + (4 + ib) * k * nnz,
        "bwd_paper_writes": 4 * k * nnz,
        "fwd": csr + (value_bytes + ib) * k * nnz + 4 * N * dim,
        "bwd": csr + 4 * k * nnz + N * k * (ib + 4),
        "topk": 4 * N * dim + N * k * (4 + ib),
        "spmm": csr + 4 * nnz * dim + 4 * N * dim,
    }


def _event_ms(pairs):
    return [a.elapsed_time(b) for a, b in pairs]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="dense")
    ap.add_argument("--k", type=int, default=32)
    ap.add_argument("--no-sweep", action="store_true", help="skip the per-k table")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--sweep-reps", type=int, default=20)
    ap.add_argument("--bwd-mode", default="auto", choices=["auto", "pull", "push", "expand", "slab", "tiled"],
                    help="backward kernel used in the timed steps (default: the library's choice)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference point for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path has no collective); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2312_08656_amd as maxk
    import synth

    maxk.load_library()  # no fallback: fails here if libmaxk.so is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    k0, dim, ib = args.k, cfg.dim, cfg.index_bytes
    t_gen = time.time()
    g = synth.graph(cfg.name)
    H, dY = synth.features(cfg.name, "H"), synth.features(cfg.name, "dY")
    t_gen = time.time() - t_gen
    N, nnz = g.N, g.nnz

    dev = lambda a: torch.from_numpy(a).cuda()
    rowptr, col, val = dev(g.rowptr), dev(g.col), dev(g.val)
    Hd, dYd = dev(H), dev(dY)
    torch.cuda.synchronize()
    t_pre = time.time()
    gr = maxk.maxk_graph_create(rowptr, col, val)
    torch.cuda.synchronize()
    t_pre = time.time() - t_pre
    t_res = time.time()
    kmax = max(max(cfg.ks), k0)
    bwd_modes = {"auto": maxk.BWD_AUTO, "pull": maxk.BWD_PULL_CSC, "push": maxk.BWD_PUSH_CSR,
                 "expand": maxk.BWD_EXPAND_REDUCE, "slab": maxk.BWD_SLAB_PULL, "tiled": maxk.BWD_TILED}
    gr.set_bwd_mode(bwd_modes[args.bwd_mode])
    gr.reserve(dim, kmax)
    for kk in sorted(set(cfg.ks) | {k0}):
        gr.reserve(dim, kk)  # builds whatever the backward kernel chosen for this k needs
    torch.cuda.synchronize()
    t_res = time.time() - t_res
    Y = torch.empty((N, dim), device="cuda")
    idt = maxk.index_dtype(ib)

    def buffers(k):
        return (torch.empty((N, k), device="cuda"), torch.empty((N, k), dtype=idt, device="cuda"),
                torch.empty((N, k), device="cuda"))

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---------------------------------------------------------------- headline: K whole steps
    sp_data, sp_index, dXs = buffers(k0)

    def step(marks=None):
        if marks is not None:
            marks[0].record()
        maxk.maxk_topk_cbsr(Hd, k0, sp_data, sp_index)
        if marks is not None:
            marks[1].record()
        maxk.maxk_spgemm_fwd(gr, sp_data, sp_index, dim, Y)
        if marks is not None:
            marks[2].record()
        maxk.maxk_sspmm_bwd(gr, dYd, sp_index, dXs)
        if marks is not None:
            marks[3].record()

    for _ in range(args.warmup):
        step()
    marks = [[ev() for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(marks[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    t_topk = float(np.mean(_event_ms([(m[0], m[1]) for m in marks])))
    t_fwd = float(np.mean(_event_ms([(m[1], m[2]) for m in marks])))
    t_bwd = float(np.mean(_event_ms([(m[2], m[3]) for m in marks])))
    value = 2.0 * nnz * k0 / (ms_per_step * 1e-3)

    ab = algorithmic_bytes(N, nnz, dim, k0, ib)
    dom_name, dom_ms, dom_bytes = max((("maxk_spgemm_fwd", t_fwd, ab["fwd"]), ("maxk_sspmm_bwd", t_bwd, ab["bwd"])),
                                      key=lambda t: t[1])
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    dom_kernel = gr.bwd_choice(dim, k0) if "bwd" in dom_name else "rmw"
    tr = measured_traffic(cfg.name, k0, dom_name, dom_kernel)
    roofline = {"bound": "hbm", "kernel": dom_name, "device_kernel": dom_kernel, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": None if tr is None else tr["bytes"], "traffic_source": None if tr is None else tr["source"],
                # measured L2<->fabric bytes per call / this run's time per call: how close the call is to the memory
                # system's own limit, whatever the algorithmic count says
                "traffic_rate_GBs": None if tr is None else round(tr["bytes"] / (dom_ms * 1e-3) / 1e9, 1),
                "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": round(dom_ms, 4)}

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)  # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # the kernel to look for in the counter trace: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---------------------------------------------------------------- per-k table
    def timeit(fn, reps, warm=3):
        for _ in range(warm):
            fn()
        pairs = []
        for _ in range(reps):
            a, b = ev(), ev()
            a.record()
            fn()
            b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        ms = _event_ms(pairs)
        return float(np.mean(ms)), float(np.median(ms))

    per_k = []
    spmm_ms = None
    if not args.no_sweep:
        spmm_ms, _ = timeit(lambda: maxk.spmm_baseline(gr, Hd, Y), max(3, args.sweep_reps // 4), warm=1)
        for k in cfg.ks:
            sd, si, dx = buffers(k)
            b = algorithmic_bytes(N, nnz, dim, k, ib)
            tk, _ = timeit(lambda: maxk.maxk_topk_cbsr(Hd, k, sd, si), args.sweep_reps)
            tf, tf_med = timeit(lambda: maxk.maxk_spgemm_fwd(gr, sd, si, dim, Y), args.sweep_reps)
            row = {"k": k, "topk_ms": round(tk, 4), "fwd_ms": round(tf, 4), "fwd_ms_median": round(tf_med, 4),
                   "fwd_edges_k_per_s": nnz * k / (tf * 1e-3), "fwd_hbm_frac": round(b["fwd"] / (tf * 1e-3) / 8e12, 4),
                   "fwd_speedup_vs_spmm": round(spmm_ms / tf, 2)}
            # the same forward pass with the CBSR values stored in 2 bytes (fp32 accumulation; not the headline)
            b16 = algorithmic_bytes(N, nnz, dim, k, ib, value_bytes=2)
            for name, dt in (("bf16", torch.bfloat16), ("f16", torch.float16)):
                sd16 = torch.empty((N, k), dtype=dt, device="cuda")
                maxk.maxk_topk_cbsr_narrow(Hd, k, sd16, si)
                t16, _ = timeit(lambda: maxk.maxk_spgemm_fwd_narrow(gr, sd16, si, dim, Y), args.sweep_reps)
                row.update({f"fwd_{name}_values_ms": round(t16, 4),
                            f"fwd_{name}_values_hbm_frac": round(b16["fwd"] / (t16 * 1e-3) / 8e12, 4)})
                del sd16
            for mode, tag in ((maxk.BWD_PUSH_CSR, "bwd_push"), (maxk.BWD_PULL_CSC, "bwd_pull"),
                              (maxk.BWD_EXPAND_REDUCE, "bwd_expand_reduce"), (maxk.BWD_SLAB_PULL, "bwd_slab_pull"),
                              (maxk.BWD_TILED, "bwd_tiled")):
                gr.set_bwd_mode(mode)
                reps = max(3, args.sweep_reps // 4)
                tb, tb_med = timeit(lambda: maxk.maxk_sspmm_bwd(gr, dYd, si, dx), reps, warm=1)
                row.update({f"{tag}_ms": round(tb, 4), f"{tag}_edges_k_per_s": nnz * k / (tb * 1e-3),
                            f"{tag}_hbm_frac": round(b["bwd"] / (tb * 1e-3) / 8e12, 4),
                            f"{tag}_speedup_vs_spmm": round(spmm_ms / tb, 2)})
            gr.set_bwd_mode(maxk.BWD_AUTO)
            # the same backward pass reading dY stored as bf16 (fp32 products and sums; not the headline)
            dY16 = dYd.to(torch.bfloat16)
            t16, _ = timeit(lambda: maxk.maxk_sspmm_bwd_narrow(gr, dY16, si, dx), max(3, args.sweep_reps // 2), warm=1)
            row.update({"bwd_bf16_dY_ms": round(t16, 4)})
            del dY16
            tb, _ = timeit(lambda: maxk.maxk_sspmm_bwd(gr, dYd, si, dx), args.sweep_reps, warm=1)
            row.update({"bwd_auto_kernel": gr.bwd_choice(dim, k),
                        "bwd_ms": round(tb, 4), "bwd_edges_k_per_s": nnz * k / (tb * 1e-3),
                        "bwd_hbm_frac": round(b["bwd"] / (tb * 1e-3) / 8e12, 4),
                        "bwd_speedup_vs_spmm": round(spmm_ms / tb, 2),
                        "fwd_bwd_edges_k_per_s": 2.0 * nnz * k / ((tf + tb) * 1e-3)})
            # What binds the backward kernels below the HBM roofline: the slab-pull forms fetch whole 128-byte lines
            # of dY rows from L2 into the vector L1 (the lines that k columns touch; all of a row once k >= dim/8),
            # and that path moves 64 bytes per clock per CU.  The time that ceiling allows, and the share reached:
            ln = dim / 32.0 if 8 * k >= dim else lines_touched(dim, k)
            ceil_ms = nnz * ln * 128.0 / (L2_TO_L1_BYTES_PER_CLK_PER_CU * N_CU * CLOCK_HZ) * 1e3
            row.update({"bwd_slab_pull_lines_per_entry": round(ln, 2), "bwd_slab_pull_l1_fill_ceiling_ms": round(ceil_ms, 3),
                        "bwd_slab_pull_share_of_l1_fill_ceiling": round(ceil_ms / row["bwd_slab_pull_ms"], 3)})
            # a fraction above 1 means the gathered table sits in the Infinity Cache, not that HBM ran past its peak
            cbsr_bytes, dy_bytes = N * k * (4 + ib), 4 * N * dim
            row["note"] = ("CBSR %.0f MB and dY %.0f MB; gathers of a table that fits the %.0f MB Infinity Cache are not "
                           "bound by HBM" % (cbsr_bytes / 1e6, dy_bytes / 1e6, INFINITY_CACHE_BYTES / 1e6))
            per_k.append(row)
            del sd, si, dx

    # ---------------------------------------------------------------- CPU oracle on a bounded sample
    cpu = None
    if not args.no_cpu:
        import oracle
        rd, ri = oracle.topk_cbsr(H, k0)  # oracle inputs come from the oracle, never from the GPU
        budget_s = 8.0
        probe = min(N, 2000)
        t = time.perf_counter()
        oracle.spgemm_fwd(g.rowptr, g.col, g.val, rd, ri, dim, rows=np.arange(probe, dtype=np.int64))
        oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, ri, src_range=(0, probe))
        t_probe = max(time.perf_counter() - t, 1e-4)
        probe_edges = int(g.rowptr[probe])
        want_edges = probe_edges * (2 * budget_s / t_probe)
        R = int(min(N, max(probe, np.searchsorted(g.rowptr, want_edges))))
        edges = int(g.rowptr[R])
        t = time.perf_counter()
        oracle.spgemm_fwd(g.rowptr, g.col, g.val, rd, ri, dim, rows=np.arange(R, dtype=np.int64))
        tf_cpu = time.perf_counter() - t
        t = time.perf_counter()
        oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, ri, src_range=(0, R))
        tb_cpu = time.perf_counter() - t
        cpu = {"value": 2.0 * edges * k0 / (tf_cpu + tb_cpu), "unit": "edge*k/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"fp64 correctness oracle (not a tuned CPU code): forward over the first {R} rows and backward "
                         f"over the same source rows of the {cfg.name} workload ({edges} stored entries, k={k0}); "
                         f"fwd {tf_cpu:.2f}s bwd {tb_cpu:.2f}s",
               "fwd_edges_k_per_s": edges * k0 / tf_cpu, "bwd_edges_k_per_s": edges * k0 / tb_cpu}

    out = {
        "metric": "fwd SpGEMM + bwd SSpMM edges*k/s (whole step: top-k/CBSR + forward + backward)",
        "value": value, "unit": "edge*k/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: R-MAT graph N={N} nnz={nnz} (stands for: {cfg.stands_for}), "
                               f"dim={dim}, k={k0}, uint{8 * ib} sp_index, GCN weights, H,dY~N(0,1)",
                   "N": N, "nnz": nnz, "dim": dim, "k": k0, "max_degree": g.meta.get("max_degree"),
                   "bwd_mode": args.bwd_mode, "bwd_kernel": gr.bwd_choice(dim, k0),
                   "graph_handle": gr.info()},
        "step_breakdown_ms": {"topk_cbsr": round(t_topk, 4), "spgemm_fwd": round(t_fwd, 4),
                              "sspmm_bwd": round(t_bwd, 4)},
        "hbm_frac_by_algorithmic_bytes": {"fwd": round(ab["fwd"] / (t_fwd * 1e-3) / 8e12, 4),
                                          "bwd": round(ab["bwd"] / (t_bwd * 1e-3) / 8e12, 4),
                                          "topk": round(ab["topk"] / (t_topk * 1e-3) / 8e12, 4)},
        "target": "forward and backward EACH at >= 0.5 of the HBM roofline by algorithmic bytes, per k (see per_k)",
        "spmm_baseline_ms": None if spmm_ms is None else round(spmm_ms, 4),
        "per_k": per_k,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "untimed": {"input_generation_s": round(t_gen, 2), "graph_preprocessing_s": round(t_pre, 3),
                    "workspace_reserve_s": round(t_res, 3)},
        "paper_context": "A100 80GB, Reddit, dim 256, k=32 (Table 3): SpMM 44.98 ms, SpGEMM 15.49 ms, SSpMM 15.07 ms, "
                         "MaxK 0.261 ms; whole-training speedup 3.22x over DGL (cuSPARSE) and 4.24x over GNNAdvisor, GraphSAGE on Reddit at "
                         "k=16 (abstract, Sec. 5.4); other hardware and the real dataset, context only",
    }
    gr.destroy()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
