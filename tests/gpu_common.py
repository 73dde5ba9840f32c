"""Plumbing shared by the GPU parity tests: device copies, one full pass through the
C-ABI, and the comparisons against the CPU oracle (the oracle never sees GPU output)."""
import time

import numpy as np
import torch

import oracle
import paper_2312_08656_amd as maxk
from helpers import check_topk_properties, within_bound

_NP_IDX = {1: np.uint8, 2: np.uint16, 4: np.int32}


def say(*a):
    print(*a, flush=True)


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class DeviceGraph:
    def __init__(self, g):
        self.host = g
        self.rowptr, self.col, self.val = to_dev(g.rowptr), to_dev(g.col), to_dev(g.val)
        self.handle = maxk.maxk_graph_create(self.rowptr, self.col, self.val)

    def close(self):
        self.handle.destroy()


def gpu_topk(H_dev, k, index_bytes):
    N, _ = H_dev.shape
    sp_data = torch.empty((N, k), dtype=torch.float32, device="cuda")
    sp_index = torch.empty((N, k), dtype=maxk.index_dtype(index_bytes), device="cuda")
    if N * k:
        sp_data.fill_(float("nan"))  # anything left unwritten shows up
    maxk.maxk_topk_cbsr(H_dev, k, sp_data, sp_index)
    torch.cuda.synchronize()
    return sp_data, sp_index


def index_to_numpy(sp_index_dev):
    if sp_index_dev.dtype == torch.uint16:
        return sp_index_dev.view(torch.int16).cpu().numpy().view(np.uint16).astype(np.int32)
    return sp_index_dev.cpu().numpy().astype(np.int32)


def check_topk(H, k, sp_data_dev, sp_index_dev, ref=None, property_rows=20000):
    """Bit-exact against the oracle CBSR; plus the oracle-free characterisation on a row sample."""
    d = sp_data_dev.cpu().numpy()
    i = index_to_numpy(sp_index_dev)
    if ref is None:
        ref = oracle.topk_cbsr(H, k)
    assert np.array_equal(i, ref[1]), "sp_index differs from the oracle"
    assert np.array_equal(d.view(np.uint32), ref[0].view(np.uint32)), "sp_data bits differ from the oracle"
    N = H.shape[0]
    if N:
        rows = np.unique(np.linspace(0, N - 1, min(N, property_rows)).astype(np.int64))
        check_topk_properties(H[rows], k, d[rows], i[rows])
    return ref


def sample_rows(g, n_random, seed, include_longest=8):
    """Rows to check at full size: the longest rows (hub rows, split over work items),
    rows just around the chunk boundary, empty-ish rows, and a random sample."""
    deg = np.diff(g.rowptr)
    rng = np.random.default_rng(seed)
    picks = [np.argsort(deg)[-include_longest:], np.argsort(deg)[:4], rng.integers(0, g.N, n_random)]
    for target in (1023, 1024, 1025, 2047, 2048, 2049, 4096, 4097, 64, 65):
        near = np.nonzero(deg == target)[0][:2]
        picks.append(near)
    return np.unique(np.concatenate(picks)).astype(np.int64)


def slab_range_edge_nodes(g, dim, slab_kb=3584, val_bytes=4):
    """Destinations at the seams of the slab-pull kernels' work split.  A launch covers one slab of source rows; its
    (slab, destination) visits, in destination order, are dealt to wavefronts in groups and the groups are cut into
    eight contiguous ranges, one per XCD.  Returns, for the first, a middle and the last slab and for every group size
    the kernels use, the first and the last destination of each range (the group size depends on k and on which of
    the two kernel forms runs, so all of them are taken)."""
    slab_rows = max(slab_kb * 1024 // (dim * val_bytes), 64)
    n_slabs = (g.N + slab_rows - 1) // slab_rows
    picks = []
    for sl in sorted({0, n_slabs // 2, n_slabs - 1}):
        lo, hi = sl * slab_rows, min(g.N, (sl + 1) * slab_rows)
        dests = np.unique(g.col[g.rowptr[lo]:g.rowptr[hi]])  # the slab's visits, in the order the kernel lists them
        nv = dests.shape[0]
        if nv == 0:
            continue
        for group in (1, 2, 4, 8, 16, 32, 64):
            tasks = (nv + group - 1) // group
            per_xcd = (tasks + 7) // 8
            for x in range(8):
                first, last = x * per_xcd * group, min(nv, (x + 1) * per_xcd * group) - 1
                if first < nv:
                    picks += [dests[first], dests[max(first, last)]]
    return np.unique(np.asarray(picks, dtype=np.int64))


def check_forward(dg, ref_cbsr, sp_data_dev, sp_index_dev, dim, rows=None):
    g = dg.host
    Y = torch.full((g.N, dim), float("nan"), dtype=torch.float32, device="cuda")
    maxk.maxk_spgemm_fwd(dg.handle, sp_data_dev, sp_index_dev, dim, Y)
    torch.cuda.synchronize()
    ref, refabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, ref_cbsr[0], ref_cbsr[1], dim, rows=rows)
    got = Y.cpu().numpy() if rows is None else Y[torch.from_numpy(rows).cuda()].cpu().numpy()
    ok, ratio = within_bound(got, ref, refabs)
    assert ok, f"forward outside the bound (worst err/bound = {ratio:.3f})"
    assert bool(torch.isfinite(Y).all()), "forward left non-finite / unwritten output"
    return Y, ratio


def check_backward(dg, ref_cbsr, dY, dY_dev, sp_index_dev, mode, nodes=None):
    g = dg.host
    k = sp_index_dev.shape[1]
    dg.handle.set_bwd_mode(mode)
    dXs = torch.full((g.N, k), float("nan"), dtype=torch.float32, device="cuda")
    maxk.maxk_sspmm_bwd(dg.handle, dY_dev, sp_index_dev, dXs)
    torch.cuda.synchronize()
    dg.handle.set_bwd_mode(maxk.BWD_AUTO)
    ref, refabs = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, ref_cbsr[1], nodes=nodes)
    got = dXs.cpu().numpy() if nodes is None else dXs[torch.from_numpy(nodes).cuda()].cpu().numpy()
    ok, ratio = within_bound(got, ref, refabs)
    assert ok, f"backward (mode {mode}) outside the bound (worst err/bound = {ratio:.3f})"
    assert bool(torch.isfinite(dXs).all()), "backward left non-finite / unwritten output"
    return dXs, ratio


def check_spmm(dg, H, H_dev, rows=None):
    g = dg.host
    dim = H.shape[1]
    Y = torch.full((g.N, dim), float("nan"), dtype=torch.float32, device="cuda")
    maxk.spmm_baseline(dg.handle, H_dev, Y)
    torch.cuda.synchronize()
    ref, refabs = oracle.spmm(g.rowptr, g.col, g.val, H, rows=rows)
    got = Y.cpu().numpy() if rows is None else Y[torch.from_numpy(rows).cuda()].cpu().numpy()
    ok, ratio = within_bound(got, ref, refabs)
    assert ok, f"dense SpMM outside the bound (worst err/bound = {ratio:.3f})"
    return ratio


_NARROW = {"bf16": (torch.bfloat16, 2.0 ** -8), "f16": (torch.float16, 2.0 ** -11)}


def _bits_to_dev(bits, dtype):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(dtype)


def check_narrow(dg, H_dev, dY, k, index_bytes, ref_cbsr, dim, rows=None):
    """16-bit CBSR values: top-k writes the oracle's rounding of the fp32 values bit for bit (same indices);
    the forward pass on them meets the usual bound against the oracle run on the widened values, and stays
    within the format's rounding error of the fp32 result.  16-bit dY: every backward kernel meets the usual
    bound against the oracle run on the widened dY."""
    g = dg.host
    N = g.N
    ref32, refabs32 = oracle.spgemm_fwd(g.rowptr, g.col, g.val, ref_cbsr[0], ref_cbsr[1], dim, rows=rows)
    worst = {}
    for vt, (dtype, half_ulp) in _NARROW.items():
        sp_data = torch.empty((N, k), dtype=dtype, device="cuda")
        sp_index = torch.empty((N, k), dtype=maxk.index_dtype(index_bytes), device="cuda")
        if N * k:
            sp_data.fill_(float("nan"))
        maxk.maxk_topk_cbsr_narrow(H_dev, k, sp_data, sp_index)
        torch.cuda.synchronize()
        assert np.array_equal(index_to_numpy(sp_index), ref_cbsr[1]), f"{vt}: sp_index differs from the oracle"
        bits = sp_data.view(torch.int16).cpu().numpy().view(np.uint16)
        want = oracle.narrow(ref_cbsr[0], vt)
        assert np.array_equal(bits, want), f"{vt}: stored values differ from the oracle's rounding"
        Y = torch.full((N, dim), float("nan"), dtype=torch.float32, device="cuda")
        maxk.maxk_spgemm_fwd_narrow(dg.handle, sp_data, sp_index, dim, Y)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(Y).all()), f"{vt}: forward left non-finite / unwritten output"
        got = Y.cpu().numpy() if rows is None else Y[torch.from_numpy(rows).cuda()].cpu().numpy()
        ref, refabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, oracle.widen(want, vt), ref_cbsr[1], dim, rows=rows)
        ok, ratio = within_bound(got, ref, refabs)
        assert ok, f"{vt}: forward outside the bound (worst err/bound = {ratio:.3f})"
        # against the fp32 definition: each term is off by at most half a unit in the last kept place
        drift = np.abs(got.astype(np.float64) - ref32)
        assert np.all(drift <= (half_ulp + 1e-5) * refabs32 + 2e-6), f"{vt}: forward drifts from fp32 by more than rounding"
        worst[vt] = ratio
        # backward pass reading dY in this format (the rounding of dY is the oracle's, done on the CPU)
        dY_bits = oracle.narrow(dY, vt)
        dY16 = _bits_to_dev(dY_bits, dtype)
        refb, refbabs = oracle.sspmm_bwd(g.rowptr, g.col, g.val, oracle.widen(dY_bits, vt), ref_cbsr[1], nodes=rows)
        sp_index32 = sp_index
        for mode in (maxk.BWD_PULL_CSC, maxk.BWD_PUSH_CSR, maxk.BWD_EXPAND_REDUCE, maxk.BWD_SLAB_PULL, maxk.BWD_TILED,
                     maxk.BWD_AUTO):  # (the tiled kernel takes fp32 dY only: these calls run its slab-pull fallback)
            dg.handle.set_bwd_mode(mode)
            dXs = torch.full((N, k), float("nan"), dtype=torch.float32, device="cuda")
            maxk.maxk_sspmm_bwd_narrow(dg.handle, dY16, sp_index32, dXs)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(dXs).all()), f"{vt}: backward (mode {mode}) left non-finite / unwritten output"
            gotb = dXs.cpu().numpy() if rows is None else dXs[torch.from_numpy(rows).cuda()].cpu().numpy()
            ok, rb = within_bound(gotb, refb, refbabs)
            assert ok, f"{vt}: backward (mode {mode}) outside the bound (worst err/bound = {rb:.3f})"
            worst[vt] = max(worst[vt], rb)
        dg.handle.set_bwd_mode(maxk.BWD_AUTO)
    return worst


def check_adjoint(Y_dev, dY_dev, sp_data_dev, dXs_dev, rel=1e-4):
    """<A X, dY> = <X, A^T dY> on the GPU outputs (holds at any size; fp64 reduction)."""
    lhs = float((Y_dev.double() * dY_dev.double()).sum())
    rhs = float((sp_data_dev.double() * dXs_dev.double()).sum())
    scale = float((Y_dev.double().abs() * dY_dev.double().abs()).sum())
    assert abs(lhs - rhs) <= rel * scale, f"adjoint identity violated: {lhs} vs {rhs} (scale {scale})"


def full_pass(dg, H, dY, k, index_bytes, sampled, seed=0, n_random=1500, spmm=True, narrow=True):
    """top-k -> forward -> backward (both kernels) -> dense SpMM, each checked against the oracle."""
    g = dg.host
    dim = H.shape[1]
    t0 = time.time()
    H_dev, dY_dev = to_dev(H), to_dev(dY)
    sp_data, sp_index = gpu_topk(H_dev, k, index_bytes)
    ref = check_topk(H, k, sp_data, sp_index)
    say(f"    top-k ok ({time.time() - t0:.1f}s)")
    rows = sample_rows(g, n_random, seed) if sampled else None
    if sampled:
        rows = np.unique(np.concatenate([rows, slab_range_edge_nodes(g, dim)]))
    Y, rf = check_forward(dg, ref, sp_data, sp_index, dim, rows)
    say(f"    forward ok, worst err/bound {rf:.3f} ({time.time() - t0:.1f}s)")
    dX_pull, rb1 = check_backward(dg, ref, dY, dY_dev, sp_index, maxk.BWD_PULL_CSC, rows)
    dX_push, rb2 = check_backward(dg, ref, dY, dY_dev, sp_index, maxk.BWD_PUSH_CSR, rows)
    dX_er, rb3 = check_backward(dg, ref, dY, dY_dev, sp_index, maxk.BWD_EXPAND_REDUCE, rows)
    dX_auto, rb4 = check_backward(dg, ref, dY, dY_dev, sp_index, maxk.BWD_AUTO, rows)
    dX_slab, rb5 = check_backward(dg, ref, dY, dY_dev, sp_index, maxk.BWD_SLAB_PULL, rows)
    dX_tiled, rb6 = check_backward(dg, ref, dY, dY_dev, sp_index, maxk.BWD_TILED, rows)
    say(f"    backward ok, worst err/bound pull {rb1:.3f} push {rb2:.3f} expand/reduce {rb3:.3f} auto {rb4:.3f} "
        f"slab {rb5:.3f} tiled {rb6:.3f} ({time.time() - t0:.1f}s)")
    for dX in (dX_pull, dX_push, dX_er, dX_auto, dX_slab, dX_tiled):
        check_adjoint(Y, dY_dev, sp_data, dX)
    if spmm:
        rs = check_spmm(dg, H, H_dev, rows)
        say(f"    dense SpMM ok, worst err/bound {rs:.3f} ({time.time() - t0:.1f}s)")
    if narrow:
        rn = check_narrow(dg, H_dev, dY, k, index_bytes, ref, dim, rows)
        say(f"    16-bit values ok, worst err/bound {rn} ({time.time() - t0:.1f}s)")
