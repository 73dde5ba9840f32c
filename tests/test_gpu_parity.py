"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs -- element by element at sizes the oracle finishes in seconds, and on
sampled outputs (plus size-independent properties) at the full benchmark sizes.
Bars: sp_index / sp_data bit-exact; fp32 outputs within 1e-5 * sum|terms| + 1e-6."""
import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import csr_from_coo, read_golden

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2312_08656_amd as maxk
    from gpu_common import (DeviceGraph, check_backward, check_forward, check_spmm, check_topk, full_pass, gpu_topk,
                            index_to_numpy, say, to_dev)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    maxk.load_library()  # fails loudly if libmaxk.so is missing: there is no fallback
    # small slabs, so that the L2-tiled backward kernel sweeps several slabs even on these small graphs
    import os
    old = os.environ.get("MAXK_SLAB_KB")
    os.environ["MAXK_SLAB_KB"] = "64"
    yield
    if old is None:
        os.environ.pop("MAXK_SLAB_KB", None)
    else:
        os.environ["MAXK_SLAB_KB"] = old


# ------------------------------------------------------------------ small, element by element


def test_golden_example_on_gpu():
    g = read_golden("fig5_fig6_shape_example.txt")
    N, dim, k = (int(r[1]) for r in g["dims"])
    rowptr, col, val = csr_from_coo(N, [(int(a), int(b), float(c)) for a, b, c in g["A_coo"]])
    H = np.array(g["H"], dtype=np.float32)
    dY = np.array(g["dY"], dtype=np.float32)
    for ib in (1, 2, 4):
        sp_data, sp_index = gpu_topk(to_dev(H), k, ib)
        assert np.array_equal(index_to_numpy(sp_index), np.array(g["sp_index"], dtype=np.int32))
        assert np.array_equal(sp_data.cpu().numpy().view(np.uint32), np.array(g["sp_data"], np.float32).view(np.uint32))
        gr = maxk.maxk_graph_create(to_dev(rowptr), to_dev(col), to_dev(val))
        Y = torch.empty((N, dim), device="cuda")
        maxk.maxk_spgemm_fwd(gr, sp_data, sp_index, dim, Y)
        assert np.array_equal(Y.cpu().numpy(), np.array(g["Y"], dtype=np.float32))  # small integers: exact
        for mode in (maxk.BWD_PULL_CSC, maxk.BWD_PUSH_CSR, maxk.BWD_EXPAND_REDUCE, maxk.BWD_SLAB_PULL, maxk.BWD_TILED,
                     maxk.BWD_AUTO):
            gr.set_bwd_mode(mode)
            dXs = torch.empty((N, k), device="cuda")
            maxk.maxk_sspmm_bwd(gr, to_dev(dY), sp_index, dXs)
            assert np.array_equal(dXs.cpu().numpy(), np.array(g["dXs"], dtype=np.float32))
        gr.destroy()


@pytest.mark.parametrize("name", ["tiny", "tiny_directed"])
def test_tiny_configs_full_compare(name):
    cfg = synth.CONFIGS[name]
    dg = DeviceGraph(synth.graph(name))
    H, dY = synth.features(name, "H"), synth.features(name, "dY")
    for k in (8, 1, 3, 64, 20):
        say(f"  {name} k={k}")
        full_pass(dg, H, dY, k, 1, sampled=False)
    full_pass(dg, H, dY, 8, 4, sampled=False)
    dg.close()


@pytest.mark.parametrize("dim,k,ib", [(6, 3, 1), (37, 5, 1), (100, 100, 2), (256, 255, 1), (384, 96, 2), (512, 7, 4),
                                       (1024, 128, 2), (64, 64, 1), (130, 33, 1), (1024, 3, 2), (768, 40, 2), (96, 24, 1), (512, 200, 2), (1024, 300, 2), (260, 100, 2)])
def test_odd_shapes_and_index_widths(dim, k, ib):
    # signed general weights on a directed graph: exercises the transpose and cancellation
    # ((1024, 3): too many private output-row copies for LDS, the forward takes its single-copy fallback)
    g = synth.make_graph(700, 9000, 10, (0.5, 0.2, 0.2), directed=True, self_loops=False, seed=dim + k,
                         weights="normal")
    dg = DeviceGraph(g)
    H, dY = synth.normal_matrix(g.N, dim, 3), synth.normal_matrix(g.N, dim, 4)
    full_pass(dg, H, dY, k, ib, sampled=False)
    dg.close()


@pytest.mark.parametrize("dim,k,ib", [(64, 8, 1), (64, 20, 1), (256, 32, 1), (384, 96, 2), (128, 5, 4)])
def test_small_dense_graph_with_long_slab_visits(dim, k, ib):
    # average degree ~170 on 400 nodes: with the small test slabs many (slab, destination) visits hold more
    # than 32 entries, which the slab kernel hands to whole wavefronts; rows also exceed one 64-entry batch
    g = synth.make_graph(400, 34000, 0, directed=True, self_loops=True, seed=dim + k, weights="normal")
    dg = DeviceGraph(g)
    H, dY = synth.normal_matrix(g.N, dim, 5), synth.normal_matrix(g.N, dim, 6)
    full_pass(dg, H, dY, k, ib, sampled=False)
    dg.close()


def test_topk_ties_signed_zero_and_infinities():
    H = synth.normal_matrix(5000, 384, seed=5)
    synth.add_tie_rows(H, seed=5, percent=40, pool=16, const_every=8)
    H[7, :10] = [-0.0, 0.0, -0.0, 0.0, np.inf, -np.inf, np.inf, 0.0, -0.0, 1.0]
    H[8, :] = -np.inf
    H[9, :] = np.float32(-0.0)
    H[9, 5] = 0.0
    Hd = to_dev(H)
    for k in (1, 2, 32, 96, 192, 383, 384):
        sp_data, sp_index = gpu_topk(Hd, k, 2)
        check_topk(H, k, sp_data, sp_index)
    H256 = np.ascontiguousarray(H[:, :256])
    for k in (31, 32, 128, 256):
        sp_data, sp_index = gpu_topk(to_dev(H256), k, 1)
        check_topk(H256, k, sp_data, sp_index)
    # every register layout of the kernel (values per lane x vector width): widths 96..1000
    for dim in (96, 128, 130, 320, 640, 768, 1000):
        Hw = synth.normal_matrix(1500, dim, seed=dim)
        synth.add_tie_rows(Hw, seed=dim, percent=40, pool=16, const_every=8)
        Hw[3, :] = np.float32(0.25)
        for k in (1, dim // 3, dim - 1, dim):
            sp_data, sp_index = gpu_topk(to_dev(Hw), k, 2)
            check_topk(Hw, k, sp_data, sp_index)


@pytest.mark.parametrize("N", [1, 3, 8191, 8192 * 2 + 5, 8192 * 3 + 1, 8192 * 5 - 1, 8192 * 8 + 13, 70001])
def test_topk_row_pipeline_edges_and_value_ranges(N):
    """The top-k kernel gives a wavefront 1..8 consecutive rows (by N) and loads two rows ahead: sizes around every
    rows-per-wavefront step with a ragged last wavefront, and rows whose values make the pivot bisection work hard
    (huge and tiny magnitudes in one row, all-positive and all-negative rows, one outlier, nearly equal values)."""
    rng = np.random.default_rng(N)
    for dim, k, ib in ((256, 32, 1), (100, 7, 1), (384, 96, 2)):
        H = synth.normal_matrix(N, dim, seed=N + dim)
        n = min(N, 64)
        rows = rng.choice(N, size=n, replace=False)
        for i, r in enumerate(rows):
            m = i % 8
            if m == 0:
                H[r] = np.abs(H[r]) + np.float32(1e-3)                 # all positive: the pivot never needs the lower half
            elif m == 1:
                H[r] = -np.abs(H[r]) - np.float32(1e-3)                # all negative
            elif m == 2:
                H[r] *= np.float32(1e-30)                              # tiny magnitudes
                H[r, 0] = np.float32(3e38)                             # ... next to one huge outlier
            elif m == 3:
                H[r] = np.float32(1.0) + H[r] * np.float32(1e-6)       # nearly equal values (few distinct floats: ties)
            elif m == 4:
                H[r] = np.float32(1e-42) * rng.integers(-50, 50, dim).astype(np.float32)  # subnormals with ties
            elif m == 5:
                H[r] = np.float32(-3e38) + np.abs(H[r]) * np.float32(1e31)                # near -FLT_MAX
            elif m == 6:
                H[r] = np.exp(H[r] * np.float32(20.0)).astype(np.float32)                 # 17 orders of magnitude
            else:
                H[r] = np.float32(0.0)
                H[r, dim - 1] = np.float32(-1.0)                       # zeros and one negative
        sp_data, sp_index = gpu_topk(to_dev(H), k, ib)
        check_topk(H, k, sp_data, sp_index)


@pytest.mark.parametrize("dim,k,ib", [(256, 32, 1), (1024, 96, 2), (100, 7, 1)])
def test_topk_neighbouring_rows_far_apart(dim, k, ib):
    """A wavefront starts the pivot search of a row at the pivot of the row before it: here every row has another
    scale and offset than its neighbours (factors of 1e-20..1e20, offsets of either sign, all-zero and constant rows
    in between), so every such start is far from where the row's own pivot lies, in either direction."""
    N = 8192 * 8 + 77
    rng = np.random.default_rng(dim + k)
    H = synth.normal_matrix(N, dim, seed=dim * 7 + k)
    scale = np.float32(10.0) ** rng.integers(-20, 21, size=N).astype(np.float32)
    offset = rng.choice(np.array([0, 0, 1, -1, 50, -50, 1e4, -1e4], np.float32), size=N)
    H *= scale[:, None]
    H += (offset * scale)[:, None]
    H[rng.choice(N, 500, replace=False)] = np.float32(0.0)
    H[rng.choice(N, 500, replace=False)] = np.float32(-7.5)
    assert np.isfinite(H).all()
    sp_data, sp_index = gpu_topk(to_dev(H), k, ib)
    check_topk(H, k, sp_data, sp_index)


def test_empty_graph_empty_rows_duplicates_unsorted_columns():
    # N == 0
    z32 = torch.zeros(1, dtype=torch.int32, device="cuda")
    g0 = maxk.maxk_graph_create(z32, torch.empty(0, dtype=torch.int32, device="cuda"), torch.empty(0, device="cuda"))
    maxk.maxk_spgemm_fwd(g0, torch.empty((0, 4), device="cuda"), torch.empty((0, 4), dtype=torch.uint8, device="cuda"),
                         8, torch.empty((0, 8), device="cuda"))
    g0.destroy()
    maxk.maxk_topk_cbsr(torch.empty((0, 8), device="cuda"), 4, torch.empty((0, 4), device="cuda"),
                        torch.empty((0, 4), dtype=torch.uint8, device="cuda"))
    # a graph with no entries at all: outputs must be overwritten with zeros
    N, dim, k = 50, 16, 4
    H, dY = synth.normal_matrix(N, dim, 1), synth.normal_matrix(N, dim, 2)
    ge = synth.Graph(N, np.zeros(N + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    dg = DeviceGraph(ge)
    full_pass(dg, H, dY, k, 1, sampled=False)
    dg.close()
    # empty rows, empty columns, duplicate entries, columns in descending order within rows
    rng = np.random.default_rng(3)
    triples = []
    for i in range(N):
        if i % 5 == 0:
            continue  # empty row
        cols = rng.integers(0, N - 7, size=rng.integers(1, 200))  # last columns never referenced; repeats likely
        triples += [(i, int(c), float(rng.standard_normal())) for c in cols]
    rowptr, col, val = csr_from_coo(N, triples)
    for i in range(N):  # reverse each row: unsorted columns
        col[rowptr[i]:rowptr[i + 1]] = col[rowptr[i]:rowptr[i + 1]][::-1].copy()
        val[rowptr[i]:rowptr[i + 1]] = val[rowptr[i]:rowptr[i + 1]][::-1].copy()
    dg = DeviceGraph(synth.Graph(N, rowptr, col, val))
    full_pass(dg, H, dY, k, 1, sampled=False)
    dg.close()


def test_misaligned_views_take_the_scalar_paths():
    g = synth.graph("tiny_directed")
    dim, k = 64, 8
    H, dY = synth.features("tiny_directed", "H"), synth.features("tiny_directed", "dY")
    dg = DeviceGraph(g)
    ref = oracle.topk_cbsr(H, k)
    # H, sp_data and sp_index each start 4 (resp. 1) bytes off a 16-byte boundary
    Hbuf = torch.empty(g.N * dim + 1, device="cuda")
    Hd = Hbuf[1:].view(g.N, dim)
    Hd.copy_(to_dev(H))
    dbuf = torch.empty(g.N * k + 1, device="cuda")
    ibuf = torch.empty(g.N * k + 1, dtype=torch.uint8, device="cuda")
    sp_data, sp_index = dbuf[1:].view(g.N, k), ibuf[1:].view(g.N, k)
    maxk.maxk_topk_cbsr(Hd, k, sp_data, sp_index)
    check_topk(H, k, sp_data, sp_index, ref)
    check_forward(dg, ref, sp_data, sp_index, dim)
    check_backward(dg, ref, dY, to_dev(dY), sp_index, maxk.BWD_PUSH_CSR)
    check_backward(dg, ref, dY, to_dev(dY), sp_index, maxk.BWD_PULL_CSC)
    check_backward(dg, ref, dY, to_dev(dY), sp_index, maxk.BWD_EXPAND_REDUCE)
    check_backward(dg, ref, dY, to_dev(dY), sp_index, maxk.BWD_SLAB_PULL)
    check_backward(dg, ref, dY, to_dev(dY), sp_index, maxk.BWD_TILED)  # sp_index off by one byte: runs slab pull
    dxbuf = torch.empty(g.N * k + 1, device="cuda")  # misaligned dXs: the reduce phase takes its scalar path
    dg.handle.set_bwd_mode(maxk.BWD_EXPAND_REDUCE)
    maxk.maxk_sspmm_bwd(dg.handle, to_dev(dY), sp_index, dxbuf[1:].view(g.N, k))
    dref, dabs = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, ref[1])
    assert (np.abs(dxbuf[1:].view(g.N, k).cpu().numpy() - dref) <= 1e-5 * dabs + 1e-6).all()
    dg.handle.set_bwd_mode(maxk.BWD_AUTO)
    check_spmm(dg, H, Hd)
    # Y itself 4 bytes off a 16-byte boundary: forward (two-array, repacked, 16-bit values) and dense SpMM write
    # their rows with 4-byte stores then, whatever the hidden width
    fref, fabs_ = oracle.spgemm_fwd(g.rowptr, g.col, g.val, ref[0], ref[1], dim)
    sref, sabs = oracle.spmm(g.rowptr, g.col, g.val, H)
    ybuf = torch.full((g.N * dim + 1,), float("nan"), device="cuda")
    Yoff = ybuf[1:].view(g.N, dim)
    assert Yoff.data_ptr() % 16 == 4
    al_d, al_i = gpu_topk(to_dev(H), k, 1)
    for sd, si in ((sp_data, sp_index), (al_d, al_i)):
        Yoff.fill_(float("nan"))
        maxk.maxk_spgemm_fwd(dg.handle, sd, si, dim, Yoff)
        assert (np.abs(Yoff.cpu().numpy() - fref) <= 1e-5 * fabs_ + 1e-6).all(), "forward into a misaligned Y"
    Yoff.fill_(float("nan"))
    maxk.maxk_spgemm_fwd_noalloc(dg.handle, al_d, al_i, dim, Yoff)
    assert (np.abs(Yoff.cpu().numpy() - fref) <= 1e-5 * fabs_ + 1e-6).all(), "no-alloc forward into a misaligned Y"
    Yoff.fill_(float("nan"))
    maxk.spmm_baseline(dg.handle, to_dev(H), Yoff)
    assert (np.abs(Yoff.cpu().numpy() - sref) <= 1e-5 * sabs + 1e-6).all(), "dense SpMM into a misaligned Y"
    assert bool(torch.isnan(ybuf[0]))  # the element before the view was not touched
    dg.close()


def test_outputs_are_overwritten_and_calls_repeat():
    g = synth.graph("tiny")
    dg = DeviceGraph(g)
    H, dY = synth.features("tiny", "H"), synth.features("tiny", "dY")
    Hd, dYd = to_dev(H), to_dev(dY)
    sp_data, sp_index = gpu_topk(Hd, 8, 1)
    Y1 = torch.full((g.N, 64), 123.0, device="cuda")
    maxk.maxk_spgemm_fwd(dg.handle, sp_data, sp_index, 64, Y1)
    ref, refabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, *oracle.topk_cbsr(H, 8), 64)
    assert np.abs(Y1.cpu().numpy() - ref).max() < 1e-4
    for mode in (maxk.BWD_PULL_CSC, maxk.BWD_PUSH_CSR, maxk.BWD_EXPAND_REDUCE, maxk.BWD_SLAB_PULL, maxk.BWD_TILED):
        dg.handle.set_bwd_mode(mode)
        a = torch.full((g.N, 8), 55.0, device="cuda")
        b = torch.full((g.N, 8), -7.0, device="cuda")
        maxk.maxk_sspmm_bwd(dg.handle, dYd, sp_index, a)
        maxk.maxk_sspmm_bwd(dg.handle, dYd, sp_index, b)
        assert (a - b).abs().max().item() < 1e-5
    dg.close()


def test_tables_are_built_once_per_shape_and_reserve_builds_them_ahead():
    """Alternating hidden widths, k and dY formats on one handle never rebuilds a regrouping of A^T; after
    maxk_graph_reserve* the compute call for that shape adds none either."""
    g = synth.make_graph(500, 30000, 0, directed=True, self_loops=True, seed=77, weights="normal")
    dg = DeviceGraph(g)
    h = dg.handle

    def bwd(dim, k, mode, dtype=torch.float32):
        h.set_bwd_mode(mode)
        dY = to_dev(synth.normal_matrix(g.N, dim, dim + k)).to(dtype)
        H = synth.normal_matrix(g.N, dim, 3)
        _, si = gpu_topk(to_dev(H), k, 2)
        out = torch.empty((g.N, k), device="cuda")
        maxk.maxk_sspmm_bwd_narrow(h, dY, si, out)
        torch.cuda.synchronize()
        ref, refabs = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY.float().cpu().numpy(), oracle.topk_cbsr(H, k)[1])
        assert (np.abs(out.cpu().numpy() - ref) <= 1e-5 * refabs + 1e-6).all()

    assert h.cached_tables() == (0, 0)
    h.set_bwd_mode(maxk.BWD_SLAB_PULL)
    h.reserve(256, 32)
    h.reserve(384, 32)
    h.reserve(256, 32, torch.bfloat16)  # 16-bit rows: a slab height of their own
    n_slab = h.cached_tables()[0]
    assert 2 <= n_slab <= 3 and h.cached_tables()[1] == 0  # (two widths may share a slab height)
    h.set_bwd_mode(maxk.BWD_TILED)
    h.reserve(256, 8)
    h.reserve(256, 32)
    assert h.cached_tables() == (n_slab, 2)
    for _ in range(3):  # alternate shapes, formats and kernels: nothing new is built
        bwd(256, 32, maxk.BWD_SLAB_PULL)
        bwd(384, 32, maxk.BWD_SLAB_PULL)
        bwd(256, 32, maxk.BWD_SLAB_PULL, torch.bfloat16)
        bwd(256, 8, maxk.BWD_TILED)
        bwd(256, 32, maxk.BWD_TILED)
        assert h.cached_tables() == (n_slab, 2)
    bwd(128, 16, maxk.BWD_TILED)  # a shape nobody reserved: built by the call, once
    bwd(128, 16, maxk.BWD_TILED)
    assert h.cached_tables()[1] == 3
    h.set_bwd_mode(maxk.BWD_AUTO)
    dg.close()


# ------------------------------------------------------------------ mid size, element by element


@pytest.mark.parametrize("aggregator", ["mean", "gin_sum"])
def test_other_aggregators_as_edge_weights(aggregator):
    # "A could have different expressions according to aggregator type" (Sec. 3.2): GraphSAGE's mean
    # aggregator is val = 1/d_i (a non-symmetric matrix on a symmetric structure), a GIN-style sum is
    # val = 1 with (1 + eps) on the diagonal (unnormalised magnitudes against the error bound)
    g0 = synth.graph("sparse_mid")
    if aggregator == "mean":
        val = synth.make_weights(g0, "mean")
    else:
        val = np.ones(g0.nnz, dtype=np.float32)
        rows = np.repeat(np.arange(g0.N, dtype=np.int64), np.diff(g0.rowptr))
        val[rows == g0.col] = np.float32(1.0 + 0.1)
    g = synth.Graph(g0.N, g0.rowptr, g0.col, val, dict(g0.meta))
    dg = DeviceGraph(g)
    H, dY = synth.features("sparse_mid", "H"), synth.features("sparse_mid", "dY")
    full_pass(dg, H, dY, 32, 1, sampled=False, spmm=True)
    dg.close()



def test_sparse_mid_full_compare():
    name = "sparse_mid"
    cfg = synth.CONFIGS[name]
    g = synth.graph(name)
    say(f"  {name}: {g.meta}")
    dg = DeviceGraph(g)
    say(f"  handle: {dg.handle.info()}")
    H, dY = synth.features(name, "H"), synth.features(name, "dY")
    for k in cfg.ks:
        say(f"  {name} k={k}")
        full_pass(dg, H, dY, k, cfg.index_bytes, sampled=False, spmm=(k == cfg.ks[0]))
    dg.close()


# ------------------------------------------------------------------ MaxK backward scatter and autograd glue


@pytest.mark.parametrize("dim,k,ib", [(64, 8, 1), (384, 96, 2), (37, 5, 4), (256, 256, 1)])
def test_cbsr_scatter_is_exact(dim, k, ib):
    N = 3001
    H = synth.normal_matrix(N, dim, 12)
    vals = synth.normal_matrix(N, k, 13)
    _, ri = oracle.topk_cbsr(H, k)
    idx_np = ri.astype({1: np.uint8, 2: np.uint16, 4: np.int32}[ib])
    idx_dev = torch.from_numpy(idx_np.view(np.int16) if ib == 2 else idx_np).cuda()
    if ib == 2:
        idx_dev = idx_dev.view(torch.uint16)
    dense = torch.full((N, dim), float("nan"), device="cuda")
    maxk.maxk_cbsr_scatter(to_dev(vals), idx_dev, dense)
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), oracle.cbsr_scatter(vals, ri, dim).view(np.uint32))


def test_autograd_function_matches_the_oracle_chain():
    name = "tiny_directed"
    g = synth.graph(name)
    cfg = synth.CONFIGS[name]
    H, dY = synth.features(name, "H"), synth.features(name, "dY")
    dg = DeviceGraph(g)
    for k in (8, 20):
        Hd = to_dev(H).requires_grad_(True)
        Y = maxk.maxk_aggregate(Hd, dg.handle, k)
        Y.backward(to_dev(dY))
        rd, ri = oracle.topk_cbsr(H, k)
        ref, refabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, rd, ri, cfg.dim)
        assert (np.abs(Y.detach().cpu().numpy() - ref) <= 1e-5 * refabs + 1e-6).all()
        D, Dabs = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dY, ri)
        want = oracle.cbsr_scatter(D.astype(np.float32), ri, cfg.dim)
        bound = oracle.cbsr_scatter((1e-5 * Dabs + 1e-6).astype(np.float32), ri, cfg.dim) + 1e-7
        got = Hd.grad.cpu().numpy()
        assert (np.abs(got - want) <= bound).all()
        assert ((got != 0).sum(axis=1) <= k).all()
    dg.close()


# ------------------------------------------------------------------ HIP graph capture of a whole step


def test_step_captured_in_a_hip_graph_replays_correctly():
    # a serving / training loop may capture top-k -> forward -> backward once and replay it: after
    # maxk_graph_reserve the calls allocate nothing, synchronise nothing and record no memset nodes.
    # Every replay (fresh inputs in the same buffers, eager work and synchronisations in between) must
    # reproduce the eager result of the same inputs.
    name = "tiny_directed"
    g = synth.graph(name)
    dim, k = synth.CONFIGS[name].dim, 8
    dg = DeviceGraph(g)
    for mode in (maxk.BWD_TILED, maxk.BWD_SLAB_PULL, maxk.BWD_EXPAND_REDUCE, maxk.BWD_PULL_CSC, maxk.BWD_PUSH_CSR):
        dg.handle.set_bwd_mode(mode)
        dg.handle.reserve(dim, k)
        Hs = torch.empty((g.N, dim), device="cuda")
        dYs = torch.empty((g.N, dim), device="cuda")
        sp_data = torch.empty((g.N, k), device="cuda")
        sp_index = torch.empty((g.N, k), dtype=torch.uint8, device="cuda")
        Y = torch.empty((g.N, dim), device="cuda")
        dXs = torch.empty((g.N, k), device="cuda")

        def step():
            maxk.maxk_topk_cbsr(Hs, k, sp_data, sp_index)
            maxk.maxk_spgemm_fwd(dg.handle, sp_data, sp_index, dim, Y)
            maxk.maxk_sspmm_bwd(dg.handle, dYs, sp_index, dXs)

        Hs.copy_(to_dev(synth.normal_matrix(g.N, dim, 100)))
        dYs.copy_(to_dev(synth.normal_matrix(g.N, dim, 200)))
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()  # warm-up outside capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for rep in range(4):
            Hn, dYn = synth.normal_matrix(g.N, dim, 300 + rep), synth.normal_matrix(g.N, dim, 400 + rep)
            Hs.copy_(to_dev(Hn))
            dYs.copy_(to_dev(dYn))
            Y.fill_(float("nan"))
            dXs.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            rd, ri = oracle.topk_cbsr(Hn, k)
            assert np.array_equal(sp_index.cpu().numpy().astype(np.int32), ri), f"replay {rep}: sp_index"
            ref, refabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, rd, ri, dim)
            assert (np.abs(Y.cpu().numpy() - ref) <= 1e-5 * refabs + 1e-6).all(), f"replay {rep}: forward"
            ref, refabs = oracle.sspmm_bwd(g.rowptr, g.col, g.val, dYn, ri)
            assert (np.abs(dXs.cpu().numpy() - ref) <= 1e-5 * refabs + 1e-6).all(), f"replay {rep}: backward"
            (Y.sum() + dXs.sum()).item()  # eager work between replays
        del graph
    dg.handle.set_bwd_mode(maxk.BWD_AUTO)
    dg.close()


@pytest.mark.parametrize("vt,dtype", [("bf16", "bfloat16"), ("f16", "float16")])
def test_narrow_values_round_like_the_oracle_on_special_values(vt, dtype):
    """Halfway cases, the fp16 subnormal range, overflow to infinity, signed zeros: with k = dim the
    top-k call stores every value of the row, so the stored bits are the rounding of the whole input."""
    rng = np.random.default_rng(11)
    base = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 2049.0, 2051.0, 65504.0,
                     65519.0, 65520.0, 1e6, -1e6, 3.3e38, -3.3e38, 2.0 ** -14, 2.0 ** -15, 2.0 ** -24, 2.0 ** -25,
                     3 * 2.0 ** -25, 2.0 ** -26, 1e-30, -1e-30, 0.0, -0.0, 0.1, -0.1, np.inf, -np.inf], np.float32)
    dim = 64
    rows = [np.resize(base, dim), np.resize(-base, dim)]
    rows += [(rng.standard_normal(dim) * np.exp2(rng.integers(-30, 18, dim))).astype(np.float32) for _ in range(200)]
    bits = rng.integers(0, 2 ** 32, (400, dim), dtype=np.uint64).astype(np.uint32).view(np.float32)
    bits[~np.isfinite(bits)] = 1.0
    H = np.ascontiguousarray(np.vstack(rows + [bits]), dtype=np.float32)
    N = H.shape[0]
    sp_data = torch.empty((N, dim), dtype=getattr(torch, dtype), device="cuda")
    sp_index = torch.empty((N, dim), dtype=torch.uint8, device="cuda")
    maxk.maxk_topk_cbsr_narrow(to_dev(H), dim, sp_data, sp_index)
    torch.cuda.synchronize()
    assert np.array_equal(sp_index.cpu().numpy(), np.tile(np.arange(dim, dtype=np.uint8), (N, 1)))
    got = sp_data.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, oracle.narrow(H, vt))


def test_narrow_entry_points_with_fp32_values_are_the_plain_calls():
    cfg = synth.CONFIGS["tiny_directed"]
    g = synth.graph("tiny_directed")
    dg = DeviceGraph(g)
    H = synth.features("tiny_directed", "H")
    k = cfg.ks[0]
    a_d, a_i = gpu_topk(to_dev(H), k, 1)
    b_d = torch.empty_like(a_d)
    b_i = torch.empty_like(a_i)
    maxk.maxk_topk_cbsr_narrow(to_dev(H), k, b_d, b_i)
    assert torch.equal(a_d.view(torch.int32), b_d.view(torch.int32)) and torch.equal(a_i, b_i)
    Y1 = torch.empty((g.N, cfg.dim), device="cuda")
    Y2 = torch.empty_like(Y1)
    maxk.maxk_spgemm_fwd(dg.handle, a_d, a_i, cfg.dim, Y1)
    maxk.maxk_spgemm_fwd_narrow(dg.handle, b_d, b_i, cfg.dim, Y2)
    ref, refabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, *oracle.topk_cbsr(H, k), cfg.dim)
    for Y in (Y1, Y2):
        assert (np.abs(Y.cpu().numpy() - ref) <= 1e-5 * refabs + 1e-6).all()
    dg.close()


def test_graph_create_rejects_bad_structure():
    """Column ids outside [0, N), a rowptr that does not start at 0 / end at nnz / decreases: the handle is not
    created and nothing is read through the bad ids (the column check is a bounded histogram)."""
    rowptr = np.array([0, 2, 3, 5], np.int32)
    col = np.array([0, 2, 1, 0, 1], np.int32)
    val = np.ones(5, np.float32)
    ok = maxk.maxk_graph_create(to_dev(rowptr), to_dev(col), to_dev(val))
    ok.destroy()
    for bad_col in (3, -1, 2 ** 31 - 1):
        c = col.copy()
        c[3] = bad_col
        with pytest.raises(maxk.MaxKError):
            maxk.maxk_graph_create(to_dev(rowptr), to_dev(c), to_dev(val))
    for bad_ptr in ([1, 2, 3, 5], [0, 2, 3, 4], [0, 3, 2, 5]):
        with pytest.raises(maxk.MaxKError):
            maxk.maxk_graph_create(to_dev(np.array(bad_ptr, np.int32)), to_dev(col), to_dev(val))
    # the library is still usable afterwards
    g2 = maxk.maxk_graph_create(to_dev(rowptr), to_dev(col), to_dev(val))
    Y = torch.empty((3, 4), device="cuda")
    H = to_dev(np.arange(12, dtype=np.float32).reshape(3, 4))
    maxk.spmm_baseline(g2, H, Y)
    want = np.array([[0 + 8, 1 + 9, 2 + 10, 3 + 11], [4, 5, 6, 7], [0 + 4, 1 + 5, 2 + 6, 3 + 7]], np.float32)
    assert np.array_equal(Y.cpu().numpy(), want)
    g2.destroy()


@pytest.mark.parametrize("seed", [1, 2])
def test_random_shapes_sweep(seed):
    """Seeded random (N, density, dim, k, index width) cases through every kernel: catches the shape-dependent paths
    (vector widths, register layouts, packed records, both slab-pull forms, tails) the fixed lists may miss."""
    rng = np.random.default_rng(seed)
    for case in range(16):
        N = int(rng.integers(1, 2500))
        dim = int(rng.choice([4, 8, 20, 64, 100, 128, 256, 260, 384, 512, 768, 1024, int(rng.integers(1, 1025))]))
        k = int(rng.integers(1, dim + 1))
        if rng.random() < 0.3:
            k = max(1, dim // int(rng.choice([2, 4, 8, 16])))
        ib = 1 if dim <= 256 and rng.random() < 0.5 else (2 if rng.random() < 0.7 else 4)
        avg_deg = float(rng.choice([0.5, 2, 8, 40, 150]))
        directed = bool(rng.random() < 0.7)
        M = int(min(0.4 * N * (N - 1) if N > 1 else 0, max(0, N * avg_deg)))
        if not directed:
            M //= 2
        say(f"  case {case}: N={N} M={M} dim={dim} k={k} ib={ib} directed={directed}")
        g = synth.make_graph(N, M, 0, directed=directed, self_loops=bool(rng.random() < 0.5), seed=1000 * seed + case,
                             weights="normal")
        dg = DeviceGraph(g)
        H, dY = synth.normal_matrix(g.N, dim, 7000 + case), synth.normal_matrix(g.N, dim, 8000 + case)
        if rng.random() < 0.3:
            synth.add_tie_rows(H, seed=case, percent=30, pool=8, const_every=4)
        full_pass(dg, H, dY, k, ib, sampled=False, spmm=bool(rng.random() < 0.3))
        dg.close()
