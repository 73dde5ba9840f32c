"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def lib():
    from paper_2312_08656_amd import binding
    if not binding.lib_path().exists():
        from paper_2312_08656_amd import build
        build.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    declared = []
    for h in sorted((ROOT / "include").glob("*.h")):
        names = re.findall(r"MAXK_API\s+[\w\s\*]+?\b(\w+)\s*\(", h.read_text())
        for name in names:
            assert hasattr(lib, name), f"{name} declared in {h.name} but not exported"
        declared += names
    assert len(declared) >= 12
    from paper_2312_08656_amd.binding import EXPORTS
    assert sorted(declared) == sorted(EXPORTS)


def test_status_strings_and_version(lib):
    assert lib.maxk_version() >= 100
    assert lib.maxk_status_string(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert lib.maxk_status_string(code) not in (b"ok", b"unknown status")
    assert lib.maxk_status_string(-99) == b"unknown status"


def test_invalid_arguments_are_rejected_without_touching_the_device(lib):
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1002)
    INVALID, UNSUPPORTED = -1, -2
    # top-k: k out of range, dim < 1, N < 0, bad index width, index width too small for dim, dim too large
    assert lib.maxk_topk_cbsr(fake, 10, 64, 0, fake, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr(fake, 10, 64, 65, fake, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr(fake, 10, 0, 1, fake, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr(fake, -1, 64, 8, fake, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr(fake, 10, 64, 8, fake, fake, 3, None) == INVALID
    assert lib.maxk_topk_cbsr(fake, 10, 384, 8, fake, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr(fake, 10, 4096, 8, fake, fake, 2, None) == UNSUPPORTED
    assert lib.maxk_topk_cbsr(None, 10, 64, 8, fake, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr(odd, 10, 64, 8, fake, fake, 1, None) == INVALID  # misaligned fp32 pointer
    assert lib.maxk_topk_cbsr(None, 0, 64, 8, None, None, 1, None) == 0  # N == 0 is a no-op
    # 16-bit value formats: unknown format, value pointer not aligned to its width, null handle
    odd1 = ctypes.c_void_p(0x1001)
    assert lib.maxk_topk_cbsr_narrow(fake, 10, 64, 8, fake, 3, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr_narrow(fake, 10, 64, 8, fake, -1, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr_narrow(fake, 10, 64, 8, odd1, 1, fake, 1, None) == INVALID
    assert lib.maxk_topk_cbsr_narrow(fake, 10, 64, 8, odd, 0, fake, 1, None) == INVALID  # fp32 values need 4
    assert lib.maxk_topk_cbsr_narrow(None, 0, 64, 8, None, 2, None, 1, None) == 0
    assert lib.maxk_spgemm_fwd_narrow(None, fake, 1, fake, 1, 64, 8, fake, None) == INVALID
    assert lib.maxk_sspmm_bwd_narrow(None, fake, 1, fake, 1, 64, 8, fake, None) == INVALID
    # graph handle: null outputs / handles
    assert lib.maxk_graph_create(None, 1, 1, fake, fake, fake, None) == INVALID
    h = ctypes.c_void_p()
    assert lib.maxk_graph_create(ctypes.byref(h), -1, 0, fake, fake, fake, None) == INVALID
    assert lib.maxk_graph_create(ctypes.byref(h), 4, 4, None, fake, fake, None) == INVALID
    assert not h
    assert lib.maxk_graph_destroy(None) == 0
    assert lib.maxk_spgemm_fwd(None, fake, fake, 1, 64, 8, fake, None) == INVALID
    assert lib.maxk_spgemm_fwd_noalloc(None, fake, fake, 1, 64, 8, fake, None) == INVALID  # null handle
    assert lib.maxk_sspmm_bwd(None, fake, fake, 1, 64, 8, fake, None) == INVALID
    assert lib.spmm_baseline(None, fake, 64, fake, None) == INVALID
    assert lib.maxk_graph_reserve(None, 64, 8) == INVALID
    assert lib.maxk_graph_set_bwd_mode(None, 1) == INVALID


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2312_08656_amd as maxk
    H = torch.zeros(4, 8)
    with pytest.raises(maxk.MaxKError):
        maxk.maxk_topk_cbsr(H, 2, torch.zeros(4, 2), torch.zeros(4, 2, dtype=torch.uint8))


def test_forward_private_copies_never_collide(lib):
    # The forward kernel walks flat units u = entry * k + position, 64 per wave instruction (aligned to
    # multiples of 64 within a batch of 64 entries), and lets entry e accumulate into copy e % NB without
    # atomics.  That is only safe if the entries sharing one instruction always map to distinct copies.
    for k in list(range(1, 200)) + [255, 256, 257, 384, 512, 1000, 1024]:
        nb = lib.maxk_fwd_private_copies(k)
        assert nb >= 1
        for u0 in range(0, 64 * k, 64):
            entries = sorted({u // k for u in range(u0, u0 + 64)})
            copies = [e % nb for e in entries]
            assert len(set(copies)) == len(copies), (k, nb, u0)
    assert lib.maxk_fwd_private_copies(0) < 0
    # and it is not wasteful for the benchmark's k values
    assert [lib.maxk_fwd_private_copies(k) for k in (8, 16, 32, 64, 96, 128, 192)] == [8, 4, 2, 1, 2, 1, 1]


def test_every_kernel_source_is_in_the_build():
    """A .hip file that the build script does not list would silently drop its kernels from libmaxk.so."""
    from pathlib import Path

    from paper_2312_08656_amd import build
    on_disk = sorted(p.name for p in (Path(build.__file__).parent / "csrc").glob("*.hip"))
    assert on_disk == sorted(build.SOURCES)
