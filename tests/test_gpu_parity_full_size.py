"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times:
CBSR compared bit-exactly on every row; forward / backward / dense SpMM compared on every
element where the oracle finishes in seconds (the headline workload at three k, the two
smaller dense-neighbourhood graphs), else on sampled outputs the oracle computes one by one
(hub rows, rows at the chunk boundaries, destinations at the seams of the slab kernels' work
split, random rows), plus the adjoint identity over the whole output."""
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2312_08656_amd as maxk
    from gpu_common import (DeviceGraph, check_adjoint, check_backward, check_forward, check_topk, full_pass, gpu_topk,
                            say, to_dev)

_cache = {}


def _setup(name):
    if name not in _cache:
        _cache.clear()  # one big configuration resident at a time
        g = synth.graph(name)
        say(f"  {name}: {g.meta}")
        dg = DeviceGraph(g)
        say(f"  handle: {dg.handle.info()}")
        _cache[name] = (dg, synth.features(name, "H"), synth.features(name, "dY"))
    return _cache[name]


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    maxk.load_library()
    yield
    for dg, _, _ in _cache.values():
        dg.close()
    _cache.clear()


def test_dense_graph_builds():
    dg, H, dY = _setup("dense")
    info = dg.handle.info()
    assert info["nnz"] == synth.CONFIGS["dense"].nnz == 114_848_855
    assert 15_000 <= info["max_degree"] <= 25_000
    # dense neighbourhoods: the library's own choice is the LDS-tiled kernel at small k and the L2-tiled pull above
    want = {8: "tiled", 16: "tiled", 32: "tiled", 64: "slab_pull", 96: "slab_pull", 128: "slab_pull"}
    assert {k: dg.handle.bwd_choice(256, k) for k in synth.CONFIGS["dense"].ks} == want


@pytest.mark.parametrize("k", synth.CONFIGS["dense"].ks)
def test_dense_sampled(k):
    dg, H, dY = _setup("dense")
    say(f"  dense k={k}")
    full_pass(dg, H, dY, k, 1, sampled=True, seed=k, n_random=600, spmm=(k == 32))


@pytest.mark.parametrize("k", [8, 32, 128])
def test_dense_every_element(k):
    """The headline workload compared on EVERY element of Y and dXs (the oracle needs a few seconds per k on the
    box's cores): forward, and every backward kernel the library's own choice can fall on here."""
    dg, H, dY = _setup("dense")
    say(f"  dense k={k}, every element")
    H_dev, dY_dev = to_dev(H), to_dev(dY)
    sp_data, sp_index = gpu_topk(H_dev, k, 1)
    ref = check_topk(H, k, sp_data, sp_index)
    Y, rf = check_forward(dg, ref, sp_data, sp_index, 256)
    worst = {"fwd": round(rf, 3)}
    for mode, name in ((maxk.BWD_AUTO, "auto"), (maxk.BWD_SLAB_PULL, "slab"), (maxk.BWD_TILED, "tiled")):
        dX, rb = check_backward(dg, ref, dY, dY_dev, sp_index, mode)
        check_adjoint(Y, dY_dev, sp_data, dX)
        worst[name] = round(rb, 3)
    say(f"    every element within the bound; worst err/bound {worst}")


@pytest.mark.parametrize("k", [2, 4, 192])
def test_dense_sampled_rest_of_the_papers_k_sweep(k):
    # the evaluation sweeps k over {2, 4, 8, ..., 192} at hidden width 256 (Sec. 5.1); the benchmark
    # configuration lists 8..128, these are the remaining ones
    dg, H, dY = _setup("dense")
    say(f"  dense k={k}")
    full_pass(dg, H, dY, k, 1, sampled=True, seed=k, n_random=300, spmm=False)


def test_wide_hidden_graph_builds():
    dg, H, dY = _setup("wide_hidden")
    assert dg.handle.info()["nnz"] == 14_671_666
    # sparse graph, hidden 384: expand/reduce at small k, plain pull once k is a large share of dim
    assert dg.handle.bwd_choice(384, 32) == "expand_reduce" and dg.handle.bwd_choice(384, 192) == "pull"


@pytest.mark.parametrize("k", synth.CONFIGS["wide_hidden"].ks)
def test_wide_hidden_sampled(k):
    dg, H, dY = _setup("wide_hidden")
    say(f"  wide_hidden k={k}")
    full_pass(dg, H, dY, k, 2, sampled=True, seed=k, n_random=1500, spmm=(k == 32))


def test_large_sparse_graph_builds():
    dg, H, dY = _setup("large_sparse")
    assert dg.handle.info()["nnz"] == 126_167_309


def test_large_sparse_sampled():
    dg, H, dY = _setup("large_sparse")
    say("  large_sparse k=64")
    full_pass(dg, H, dY, 64, 1, sampled=True, seed=64, n_random=1500, spmm=True)


# three more degree profiles from the kernel evaluation's average-degree > 50 group (Sec. 5.2; Table 1 sizes)


def test_ddi_like_every_element():
    dg, H, dY = _setup("ddi_like")
    assert dg.handle.info()["nnz"] == synth.CONFIGS["ddi_like"].nnz == 2_140_089
    say(f"  ddi_like: library's backward choice per k: "
        f"{ {k: dg.handle.bwd_choice(256, k) for k in synth.CONFIGS['ddi_like'].ks} }")
    for k in synth.CONFIGS["ddi_like"].ks:
        say(f"  ddi_like k={k}")
        full_pass(dg, H, dY, k, 1, sampled=False, spmm=(k == 32))


@pytest.mark.parametrize("k", [8, 32])
def test_proteins_like_every_element(k):
    dg, H, dY = _setup("proteins_like")
    assert dg.handle.info()["nnz"] == synth.CONFIGS["proteins_like"].nnz == 79_255_038
    say(f"  proteins_like k={k}: library's backward choice {dg.handle.bwd_choice(256, k)}")
    assert dg.handle.bwd_choice(256, k) == "tiled"  # the faster kernel by measurement at both k
    full_pass(dg, H, dY, k, 1, sampled=False, spmm=(k == 32), narrow=False)


@pytest.mark.parametrize("k", [16, 64])
def test_ppa_like_sampled(k):
    dg, H, dY = _setup("ppa_like")
    assert dg.handle.info()["nnz"] == synth.CONFIGS["ppa_like"].nnz == 43_040_151
    say(f"  ppa_like k={k}: library's backward choice {dg.handle.bwd_choice(256, k)}")
    full_pass(dg, H, dY, k, 1, sampled=True, seed=k, n_random=1500, spmm=(k == 16), narrow=(k == 16))
