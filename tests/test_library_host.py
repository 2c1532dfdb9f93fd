"""CPU-side checks of the HIP library: it loads, exports every symbol declared
in include/gs.h, and its host-only functions (workspace sizing) behave.  No
kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2407_15452_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_lib()
    return binding.lib()


def test_header_symbols_are_exported(lib):
    from paper_2407_15452_amd import binding
    header = open(os.path.join(ROOT, "include", "gs.h")).read()
    declared = set(re.findall(r"\b(gs_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_workspace_queries(lib):
    assert lib.gs_sgns_step_workspace_bytes(C.c_int64(0), C.c_int64(10), C.c_int32(5), C.c_int32(128), C.c_int32(0)) > 0
    small = lib.gs_sgns_step_workspace_bytes(C.c_int64(1000), C.c_int64(10), C.c_int32(5), C.c_int32(128), C.c_int32(0))
    big = lib.gs_sgns_step_workspace_bytes(C.c_int64(2000), C.c_int64(10), C.c_int32(5), C.c_int32(128), C.c_int32(0))
    assert 0 < small < big and small % 256 == 0
    assert lib.gs_csr_build_workspace_bytes(C.c_int64(1000), C.c_int64(10), C.c_uint32(1)) > \
        lib.gs_csr_build_workspace_bytes(C.c_int64(1000), C.c_int64(10), C.c_uint32(0))
    assert lib.gs_make_pairs_workspace_bytes(C.c_int64(10)) >= 256
    assert lib.gs_alias_build_workspace_bytes(C.c_int64(3), C.c_int64(100)) >= 16 * 100
    assert lib.gs_last_hip_error() == 0


def test_missing_library_is_an_error(monkeypatch):
    from paper_2407_15452_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libgs.so")
    with pytest.raises(RuntimeError):
        binding.lib()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_inputs_are_deterministic():
    import torch
    from paper_2407_15452_amd import inputs
    wl = inputs.WORKLOADS[0]
    a = inputs.edge_list(wl)
    b = inputs.edge_list(wl)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and a[0].numel() == wl.num_edges
    assert inputs.pairs_per_full_walk(20, 5) == 170 and inputs.pairs_per_full_walk(80, 10) == 1490
    w_in, w_out = inputs.init_tables(100, 64, 5)
    assert float(w_in.abs().max()) <= 0.5 / 64 and float(w_out.abs().max()) == 0


def test_argument_checks_that_need_no_gpu(lib):
    """Rejected on the host before anything is enqueued (no device pointer is touched)."""
    fake = C.c_void_p(256)                       # non-null, aligned; never dereferenced
    # one alias segment longer than a 32-bit position
    rc = lib.gs_alias_build(fake, C.c_int32(64), C.c_int64(1), C.c_int64(1 << 31), fake, fake, fake,
                            fake, C.c_size_t(1 << 62), None)
    assert rc == -3
    # 32-bit offsets cannot hold the symmetrised capacity
    rc = lib.gs_csr_build(fake, fake, None, C.c_int64((1 << 30) + 1), C.c_int64(10), C.c_uint32(1),
                          C.c_int32(32), fake, fake, None, fake, fake, C.c_size_t(1 << 62), None)
    assert rc == -3
    # dim not a multiple of the 16-byte piece; k beyond the limit; one table on both sides
    step = lambda w_in, w_out, dim, k: lib.gs_sgns_step(  # noqa: E731
        w_in, w_out, C.c_int64(10), C.c_int32(dim), C.c_int32(0), fake, fake, fake, C.c_int64(4),
        C.c_int32(k), C.c_float(0.1), fake, fake, C.c_size_t(1 << 62), None)
    other = C.c_void_p(512)
    assert step(fake, other, 6, 2) == -1
    assert step(fake, other, 8, 61) == -1
    assert step(fake, fake, 8, 2) == -1
    assert lib.gs_unique_ids_workspace_bytes(C.c_int64(1000), C.c_int64(100)) < \
        lib.gs_unique_ids_workspace_bytes(C.c_int64(1000), C.c_int64(10**9))
    assert lib.gs_sgns_step_fused_workspace_bytes(C.c_int64(1000), C.c_int64(10), C.c_int32(5), C.c_int32(128), C.c_int32(0)) > \
        lib.gs_sgns_step_workspace_bytes(C.c_int64(1000), C.c_int64(10), C.c_int32(5), C.c_int32(128), C.c_int32(0))


def test_static_step_rejects_oversized_batches_on_the_host(lib):
    """gs_sgns_step_static checks its limits before it asks for the scratch array's address."""
    fake, other = C.c_void_p(256), C.c_void_p(512)
    call = lambda pairs, k, dim: lib.gs_sgns_step_static(  # noqa: E731
        fake, other, C.c_int64(10), C.c_int32(dim), C.c_int32(0), fake, fake, fake, C.c_int64(pairs),
        C.c_int32(k), C.c_float(0.1), fake, None)
    assert call(4097, 5, 128) == -2
    assert call(4096, 16, 128) == -2            # 4096 * 17 terms > 65536
    assert call(1024, 5, 260) == -2
