"""The forward entry point that allocates nothing (its scratch memory is a fixed device array inside the library):
called through the C ABI, compared with maxk_spgemm_fwd and with the CPU oracle, on two calls in a row, the second
with a smaller input, plus the rejection of an input whose split rows do not fit the array."""
import os

import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2312_08656_amd as maxk
    from gpu_common import to_dev


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    maxk.load_library()
    old = os.environ.get("MAXK_CHUNK")
    os.environ["MAXK_CHUNK"] = "64"  # rows longer than 64 entries are split: partial rows go through the scratch array
    yield
    if old is None:
        os.environ.pop("MAXK_CHUNK", None)
    else:
        os.environ["MAXK_CHUNK"] = old


def _case(N, M, dim, k, ib, seed):
    g = synth.make_graph(N, M, 0, directed=True, self_loops=True, seed=seed, weights="normal")
    H = synth.normal_matrix(g.N, dim, seed + 1)
    gr = maxk.maxk_graph_create(to_dev(g.rowptr), to_dev(g.col), to_dev(g.val))
    assert gr.info()["n_split_rows"] > 0, "the case is meant to use partial rows"
    sp_data = torch.empty((g.N, k), device="cuda")
    sp_index = torch.empty((g.N, k), dtype=maxk.index_dtype(ib), device="cuda")
    maxk.maxk_topk_cbsr(to_dev(H), k, sp_data, sp_index)
    return g, H, gr, sp_data, sp_index


def _check(g, H, gr, sp_data, sp_index, dim, k):
    Y_ref = torch.full((g.N, dim), float("nan"), device="cuda")
    Y_new = torch.full((g.N, dim), float("nan"), device="cuda")
    maxk.maxk_spgemm_fwd(gr, sp_data, sp_index, dim, Y_ref)
    maxk.maxk_spgemm_fwd_noalloc(gr, sp_data, sp_index, dim, Y_new)
    torch.cuda.synchronize()
    ref, refabs = oracle.spgemm_fwd(g.rowptr, g.col, g.val, *oracle.topk_cbsr(H, k), dim)
    bound = 1e-5 * refabs + 1e-6
    got_ref, got_new = Y_ref.cpu().numpy(), Y_new.cpu().numpy()
    assert np.isfinite(got_new).all(), "the no-alloc call left output unwritten"
    assert (np.abs(got_new - ref) <= bound).all(), "no-alloc forward outside the bound against the oracle"
    assert (np.abs(got_ref - ref) <= bound).all()
    assert (np.abs(got_new.astype(np.float64) - got_ref) <= bound).all(), "no-alloc forward differs from maxk_spgemm_fwd"


def test_no_alloc_forward_matches_the_allocating_entry_point_twice_in_a_row():
    # first call: 3000 nodes, ~120 entries per row (every row split in two), hidden 256, k = 8 (repacked CBSR + partial rows)
    big = _case(3000, 360_000, 256, 8, 1, seed=31)
    _check(*big, 256, 8)
    # second call, smaller input (fewer nodes, narrower rows, other k): must not see anything of the first in the array
    small = _case(700, 60_000, 96, 24, 2, seed=32)
    _check(*small, 96, 24)
    # and the first one again, the array now holding the small case's leftovers
    _check(*big, 256, 8)
    big[2].destroy()
    small[2].destroy()


def test_no_alloc_forward_rejects_what_does_not_fit():
    # ~9400 partial rows of 1024 floats = 38 MB > the 32 MiB array: refused with its own status, nothing launched
    g, H, gr, sp_data, sp_index = _case(3000, 600_000, 1024, 16, 2, seed=33)
    Y = torch.zeros((g.N, 1024), device="cuda")
    with pytest.raises(maxk.MaxKError, match="scratch"):
        maxk.maxk_spgemm_fwd_noalloc(gr, sp_data, sp_index, 1024, Y)
    torch.cuda.synchronize()
    assert float(Y.abs().sum()) == 0.0
    maxk.maxk_spgemm_fwd(gr, sp_data, sp_index, 1024, Y)  # the allocating entry point takes it
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Y).all())
    gr.destroy()
