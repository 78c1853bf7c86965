"""CPU-only checks of the boundary: the C-ABI library loads and exports every
symbol include/moe.h declares, argument validation and error codes, page
geometry, and the host packer (dense -> pages -> dense is the identity, the page
image has the documented layout).  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

import paper_2411_11217_amd as M
from paper_2411_11217_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "moe.h")).read()
    declared = set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(M.library_path() if os.path.exists(M.library_path()) else B._build.build())
    for name in sorted(declared):
        assert hasattr(lib, name), "missing export: " + name
    assert declared == set(M.EXPORTED_SYMBOLS)


def test_no_torch_types_in_the_abi():
    header = open(os.path.join(ROOT, "include", "moe.h")).read()
    assert "torch" not in header.lower() and "at::" not in header and "std::" not in header
    assert 'extern "C"' in header


@pytest.mark.parametrize("kw,code", [
    (dict(), 0),
    (dict(T=0), 0),
    (dict(T=-1), B.ERR_INVALID_ARG),
    (dict(k=0), B.ERR_INVALID_ARG),
    (dict(k=9), B.ERR_INVALID_ARG),
    (dict(E=65, k=2), B.ERR_INVALID_ARG),
    (dict(H=200), B.ERR_INVALID_ARG),
    (dict(F=64), B.ERR_INVALID_ARG),
    (dict(page_bytes=0), B.ERR_INVALID_ARG),
    (dict(page_bytes=16384 * 3 + 512), B.ERR_INVALID_ARG),
    (dict(dtype=7), B.ERR_UNSUPPORTED_DTYPE),
])
def test_shape_validation(kw, code):
    base = dict(T=64, H=256, F=512, E=8, k=2, dtype=1, page_bytes=65536)
    base.update(kw)
    s = B.MoEShape(base["T"], base["H"], base["F"], base["E"], base["k"], base["dtype"], base["page_bytes"])
    assert M.validate_shape(s) == code


def test_status_strings():
    lib = B._lib()
    assert lib.moe_status_string(0) == b"ok"
    assert lib.moe_status_string(B.ERR_PAGE_NOT_RESIDENT) == b"page not resident"
    assert b"unknown" in lib.moe_status_string(-99)


@pytest.mark.parametrize("dtype,H,F,page,gu,d", [
    ("f32", 256, 512, 64 * 1024, 16, 8),                 # tiny workload: 24 pages per expert
    ("bf16", 4096, 14336, 2 << 20, 112, 56),             # Mixtral-8x7B shape
    ("bf16", 6144, 16384, 4 << 20, 96, 48),              # Mixtral-8x22B shape
    ("bf16", 6144, 10752, 4 << 20, 63, 32),              # DBRX shape: the W2 group is 31.5 pages, padded to 32
])
def test_page_geometry(dtype, H, F, page, gu, d):
    s = M.make_shape(16, H, F, 8, 2, dtype, page)
    assert M.pages_required(s) == (gu, d)
    assert M.tile_bytes(s) == 128 * 64 * (2 if dtype == "bf16" else 4)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pack_unpack_round_trip_and_layout(dtype):
    E, H, F = 3, 256, 384
    s = M.make_shape(8, H, F, E, 1, dtype, 3 * M.tile_bytes(M.make_shape(8, H, F, E, 1, dtype, 1 << 20)))
    tdt = s.torch_dtype
    g = torch.Generator().manual_seed(5)
    W1 = torch.randn((E, F, H), generator=g).to(tdt)
    W3 = torch.randn((E, F, H), generator=g).to(tdt)
    W2 = torch.randn((E, H, F), generator=g).to(tdt)
    pw = M.PagedWeights(s, W1, W3, W2, order=torch.Generator().manual_seed(1), extra_pages=5)
    assert len(set(pw.table_host.reshape(-1).tolist())) == E * pw.ppe
    U1, U3, U2 = pw.unpack()
    assert torch.equal(U1, W1) and torch.equal(U3, W3) and torch.equal(U2, W2)

    # documented layout: tile (f/128, w, h/64) of group GU; inside a tile the 16-byte chunk c of row n sits
    # (f32)  in row n of 256 bytes at position (c & 8) | ((c & 7) ^ ((n >> 1) & 7)),
    # (bf16) in half-tile c >> 2 (8 KiB each), row n of 64 bytes, at position (c & 3) ^ ((n >> 2) & 2)
    esz = 2 if dtype == "bf16" else 4

    def chunk_offset(n, c):
        if dtype == "bf16":
            return (c >> 2) * 8192 + n * 64 + (((c & 3) ^ ((n >> 2) & 2)) << 4)
        return n * 256 + (((c & 8) | ((c & 7) ^ ((n >> 1) & 7))) << 4)

    tb = M.tile_bytes(s)
    tpp = s.page_bytes // tb
    e, ft, w, kt, n, c = 2, 1, 1, 3, 77, 5
    ti = (ft * 2 + w) * (H // 64) + kt
    slot = int(pw.table_host[e, ti // tpp])
    off = (ti % tpp) * tb + chunk_offset(n, c)
    got = pw.pages_host[slot, off:off + 16]
    src = W3[e, ft * 128 + n, kt * 64 + c * (16 // esz): kt * 64 + (c + 1) * (16 // esz)].contiguous()
    assert torch.equal(got, src.view(torch.uint8))
    # group D: tile (d/128, f/64) of W2 after the GU pages
    dtile, kt2, n, c = 1, 4, 9, 2
    ti = dtile * (F // 64) + kt2
    slot = int(pw.table_host[e, pw.pages_gu + ti // tpp])
    off = (ti % tpp) * tb + chunk_offset(n, c)
    src = W2[e, dtile * 128 + n, kt2 * 64 + c * (16 // esz): kt2 * 64 + (c + 1) * (16 // esz)].contiguous()
    assert torch.equal(pw.pages_host[slot, off:off + 16], src.view(torch.uint8))


def test_packed_pages_do_not_depend_on_slot_order():
    E, H, F = 2, 128, 256
    s = M.make_shape(8, H, F, E, 1, "bf16", 32768)
    g = torch.Generator().manual_seed(2)
    W1, W3, W2 = (torch.randn(sh, generator=g).to(torch.bfloat16) for sh in ((E, F, H), (E, F, H), (E, H, F)))
    a = M.PagedWeights(s, W1, W3, W2)
    b = M.PagedWeights(s, W1, W3, W2, order=torch.Generator().manual_seed(9), extra_pages=3)
    for e in range(E):
        for p in range(a.ppe):
            assert torch.equal(a.pages_host[int(a.table_host[e, p])], b.pages_host[int(b.table_host[e, p])])


def test_page_table_validation_and_pack_errors():
    s = M.make_shape(8, 128, 128, 2, 1, "bf16", 16384)
    gu, d = M.pages_required(s)
    table = torch.arange(2 * (gu + d), dtype=torch.int32).reshape(2, gu + d)
    M.page_table_validate(s, table, 2 * (gu + d))
    bad = table.clone()
    bad[1, 0] = -1
    with pytest.raises(M.MoEError) as ei:
        M.page_table_validate(s, bad, 2 * (gu + d))
    assert ei.value.status == B.ERR_PAGE_NOT_RESIDENT
    with pytest.raises(M.MoEError) as ei:
        M.page_table_validate(s, table, 2 * (gu + d) - 1)      # last slot outside the pool
    assert ei.value.status == B.ERR_PAGE_NOT_RESIDENT
    W = torch.zeros((2, 128, 128), dtype=torch.bfloat16)
    dup = table.clone()
    dup[1, 0] = dup[0, 0]
    with pytest.raises(M.MoEError) as ei:
        M.pack_weights(s, W, W, W, dup, 2 * (gu + d))
    assert ei.value.status == B.ERR_INVALID_ARG


def test_workspace_layout_is_ordered_and_aligned():
    s = M.make_shape(4096, 4096, 14336, 8, 2, "bf16", 2 << 20)
    L = M.workspace_layout(s)
    names = ["status", "topk_ids", "topk_w", "counts", "offsets", "row_src", "row_of", "row_w", "scan", "x_perm", "h", "out"]
    offs = [getattr(L, n) for n in names]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    R = s.R
    assert L.x_perm - L.scan >= L.permute_bytes
    assert L.h - L.x_perm >= R * s.H * 2 and L.out - L.h >= R * s.F * 2 and L.total - L.out >= R * s.H * 4


def test_null_and_small_workspace_errors_without_gpu():
    # argument errors are detected on the host before anything is enqueued
    lib = B._lib()
    s = M.make_shape(8, 128, 128, 2, 1, "bf16", 16384)
    assert lib.moe_route(ctypes.byref(s), None, None, None, None, None, None, None) == B.ERR_INVALID_ARG
    assert lib.moe_combine(ctypes.byref(s), None, None, None, None, None) == B.ERR_INVALID_ARG
    assert lib.moe_layer(ctypes.byref(s), None, None, None, None, None, 1, None, None, 0, None) == B.ERR_INVALID_ARG
    fake = ctypes.c_void_p(256)     # never dereferenced: the size check comes first
    assert lib.moe_layer(ctypes.byref(s), fake, fake, None, fake, fake, 1, fake, fake, 16, None) == B.ERR_WORKSPACE_TOO_SMALL
    assert lib.moe_permute(ctypes.byref(s), fake, None, None, fake, fake, fake, fake, None, None, fake, 0, None) \
        == B.ERR_WORKSPACE_TOO_SMALL
    s0 = M.make_shape(0, 128, 128, 2, 1, "bf16", 16384)
    assert lib.moe_route(ctypes.byref(s0), None, None, None, None, None, None, None) == 0   # T == 0: nothing to do
    assert lib.moe_set_option(b"no_such_option", 1) == B.ERR_INVALID_ARG
    assert M.get_option("xcd_remap") in (0, 1)


def test_pipeline_pool_size_and_argument_errors_without_gpu():
    # pool = every layer's resident pages + a double buffer for one layer's streamed pages
    s = M.make_shape(8, 256, 384, 3, 1, "bf16", 3 * 16384)
    gu, d = M.pages_required(s)
    ppe = gu + d
    assert M.pipeline_pool_pages(s, 4, 0) == 2 * 3 * ppe
    assert M.pipeline_pool_pages(s, 4, ppe) == 4 * 3 * ppe
    assert M.pipeline_pool_pages(s, 4, 5) == 4 * 3 * 5 + 2 * 3 * (ppe - 5)
    lib = B._lib()
    out = ctypes.c_int64(0)
    assert lib.moe_pipeline_pool_pages(ctypes.byref(s), 0, 0, ctypes.byref(out)) == B.ERR_INVALID_ARG
    assert lib.moe_pipeline_pool_pages(ctypes.byref(s), 1, ppe + 1, ctypes.byref(out)) == B.ERR_INVALID_ARG
    assert lib.moe_pipeline_pool_pages(ctypes.byref(s), 1, 0, None) == B.ERR_INVALID_ARG
    handle = ctypes.c_void_p(0)
    assert lib.moe_pipeline_create(ctypes.byref(s), 2, 4, None, None, None, 0, None, 0, None, ctypes.byref(handle)) \
        == B.ERR_INVALID_ARG
    assert lib.moe_pipeline_run(None, 1, None, None, None, None, None, None, 0, None, None) == B.ERR_INVALID_ARG
    assert lib.moe_pipeline_destroy(None) == B.ERR_INVALID_ARG


def test_host_packer_and_oracle_under_the_host_sanitizers(tmp_path):
    """The host-only translation unit of the library (csrc/moe_host.cpp: shape checks, page geometry, packer) and the C
    oracle, built with the host compiler's address and undefined-behaviour sanitizers and run on exact-size heap
    buffers (tests/sanitize_driver.cpp): an access outside a buffer, a signed overflow or a misaligned access in
    either ends the program with a report."""
    import shutil
    import subprocess
    if not (shutil.which("gcc") and shutil.which("g++")):
        pytest.skip("no host compiler")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2411_11217_amd", "csrc")]
    objs = []
    for cc, std, src in (("gcc", "-std=c11", os.path.join(ROOT, "oracle", "moe_oracle.c")),
                         ("g++", "-std=c++17", os.path.join(ROOT, "paper_2411_11217_amd", "csrc", "moe_host.cpp")),
                         ("g++", "-std=c++17", os.path.join(ROOT, "tests", "sanitize_driver.cpp"))):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        r = subprocess.run([cc, std, "-fopenmp", "-pthread"] + san + ["-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-4000:]
        objs.append(obj)
    exe = str(tmp_path / "sanitize_driver")
    r = subprocess.run(["g++", "-fopenmp", "-pthread"] + san + objs + ["-o", exe, "-lm"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "all ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
