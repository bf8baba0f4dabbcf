"""Boundary checks that need no GPU: the library loads, exports every symbol the header declares,
and rejects bad host-visible arguments with the documented status codes before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2605_27740_amd import binding
from paper_2605_27740_amd.binding import CacheDesc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return binding.load()


def good_desc(**over):
    # pointers only need to be non-NULL and aligned for validation; nothing dereferences them on the host
    d = dict(dtype=1, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16, batch=2,
             max_pages_per_seq=64, max_seq_len_hint=0, num_phys_pages=128, k_cache=0x1000, v_cache=0x2000,
             page_stats=0x3000, page_table=0x5000, seq_lens=0x6000, stats_dtype=0, force_recent_pages=0, kv_page_stride=0, kv_head_stride=0, min_seq_len_hint=0, reserved0=0)
    d.update(over)
    return CacheDesc(**d)


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "unique.h")).read()
    declared = set(re.findall(r"\b(unique_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib.c, name)
    assert lib.version().startswith("unique-gfx950")
    assert lib.status_string(0) == "ok" and "unknown" in lib.status_string(99)
    assert lib.page_stats_record_bytes(good_desc()) == 8 * 128 * 4 + 128
    assert lib.page_stats_record_bytes(good_desc(stats_dtype=1)) == 8 * 128 * 2 + 128
    assert lib.c.unique_page_stats_record_bytes(None) == 0 and lib.page_stats_record_bytes(good_desc(stats_dtype=5)) == 0


def test_debug_exports_live_in_the_profiling_build_only(lib):
    """The product library exports nothing but what include/unique.h declares; the stamps and the two ceiling probes
    exist only in the profiling build that bench.py's analysis modes load."""
    import subprocess
    from paper_2605_27740_amd import build
    def exported(path):
        out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
        return {ln.split()[-1] for ln in out.splitlines() if ln.split()[-1].startswith("unique_")}
    assert exported(build.LIB_PATH) == set(binding.EXPORTS)
    debug = {"unique_debug_dec_stamps", "unique_debug_gather_probe", "unique_debug_record_probe"}
    assert exported(build.build_profiling_library()) == set(binding.EXPORTS) | debug


def test_workspace_bytes(lib):
    n = lib.workspace_bytes(good_desc(), 16)
    assert n > 0 and n % 256 == 0
    # needs dimensions only
    assert lib.workspace_bytes(good_desc(k_cache=0, v_cache=0, page_stats=0, page_table=0, seq_lens=0), 16) == n
    # grows with the batch, covers score rows
    assert lib.workspace_bytes(good_desc(batch=64), 16) > n
    big = lib.workspace_bytes(good_desc(batch=1, max_pages_per_seq=16384), 256)
    assert big >= 8 * 16384 * 4
    out = C.c_size_t(0)
    assert lib.c.unique_workspace_bytes(C.byref(good_desc()), 0, C.byref(out)) == binding.ERR_INVALID_ARG
    assert lib.c.unique_workspace_bytes(None, 4, C.byref(out)) == binding.ERR_INVALID_ARG
    assert lib.c.unique_workspace_bytes(C.byref(good_desc()), 4, None) == binding.ERR_INVALID_ARG


@pytest.mark.parametrize("over,code", [
    (dict(dtype=2), binding.ERR_INVALID_ARG),
    (dict(batch=0), binding.ERR_INVALID_ARG),
    (dict(num_q_heads=30), binding.ERR_INVALID_ARG),          # not a multiple of num_kv_heads
    (dict(head_dim=96), binding.ERR_UNSUPPORTED),
    (dict(page_size=12), binding.ERR_UNSUPPORTED),
    (dict(num_q_heads=24, num_kv_heads=8), binding.ERR_UNSUPPORTED),   # G = 3
    (dict(num_q_heads=12, num_kv_heads=12), binding.ERR_UNSUPPORTED),  # Hkv = 12
    (dict(num_q_heads=64, num_kv_heads=64), binding.ERR_UNSUPPORTED),  # Hkv = 64
    (dict(k_cache=0), binding.ERR_INVALID_ARG),
    (dict(page_table=0), binding.ERR_INVALID_ARG),
    (dict(k_cache=0x1004), binding.ERR_INVALID_ARG),          # misaligned
    (dict(max_seq_len_hint=-1), binding.ERR_INVALID_ARG),
    (dict(min_seq_len_hint=-1), binding.ERR_INVALID_ARG),
    (dict(max_seq_len_hint=512, min_seq_len_hint=513), binding.ERR_INVALID_ARG),  # lower bound above the upper one
    (dict(stats_dtype=3), binding.ERR_INVALID_ARG),
    (dict(force_recent_pages=-1), binding.ERR_INVALID_ARG),
    (dict(max_pages_per_seq=2 ** 27, page_size=8, num_q_heads=32, num_kv_heads=32), binding.ERR_UNSUPPORTED),  # item index overflow
    (dict(page_stats=0x3010), binding.ERR_INVALID_ARG),       # needs 128-byte alignment
    (dict(kv_head_stride=1024), binding.ERR_INVALID_ARG),     # smaller than one S*D tile (2048)
    (dict(kv_head_stride=4096, kv_page_stride=4096 * 7), binding.ERR_INVALID_ARG),  # pages would overlap
    (dict(kv_head_stride=2052), binding.ERR_INVALID_ARG),     # not a multiple of 16 bytes
])
def test_descriptor_validation(lib, over, code):
    rc = lib.c.unique_dense_paged_decode(C.byref(good_desc(**over)), 0x7000, 0.0, 0x8000, None, 0x10000, 1 << 30, None)
    assert rc == code
    assert lib.last_error() != ""
    rc = lib.c.unique_update_page_stats(C.byref(good_desc(**over)), None, None, 0, None)
    assert rc == code


def test_call_argument_validation(lib):
    d = good_desc()
    ws, nws = 0x10000, 1 << 30
    c = lib.c
    # stats
    assert c.unique_update_page_stats(None, None, None, 0, None) == binding.ERR_INVALID_ARG
    assert c.unique_update_page_stats(C.byref(good_desc(page_stats=0)), None, None, 0, None) == binding.ERR_INVALID_ARG
    assert c.unique_update_page_stats(C.byref(d), 0x100, None, 1, None) == binding.ERR_INVALID_ARG
    assert c.unique_update_page_stats(C.byref(d), 0x100, 0x200, -1, None) == binding.ERR_INVALID_ARG
    # score + select
    f = c.unique_score_select_topk
    assert f(C.byref(d), None, 4, 0.5, 0x100, 0x200, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert f(C.byref(d), 0x7000, 0, 0.5, 0x100, 0x200, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert f(C.byref(d), 0x7000, 4, -1.0, 0x100, 0x200, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert f(C.byref(d), 0x7000, 4, float("nan"), 0x100, 0x200, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert f(C.byref(d), 0x7000, 4, 0.5, None, 0x200, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert f(C.byref(d), 0x7000, 4, 0.5, 0x100, 0x200, None, None, nws, None) == binding.ERR_WORKSPACE
    assert f(C.byref(d), 0x7000, 4, 0.5, 0x100, 0x200, None, ws, 16, None) == binding.ERR_WORKSPACE
    assert "too small" in lib.last_error()
    assert f(C.byref(d), 0x7000, 4, 0.5, 0x100, 0x200, None, ws + 8, nws, None) == binding.ERR_WORKSPACE
    assert f(C.byref(good_desc(page_stats=0)), 0x7000, 4, 0.5, 0x100, 0x200, None, ws, nws, None) == binding.ERR_INVALID_ARG
    # the two halves on their own
    ps, st = c.unique_page_scores, c.unique_select_topk
    assert ps(C.byref(d), 0x7000, 0.5, None, 64, None) == binding.ERR_INVALID_ARG
    assert ps(C.byref(d), 0x7000, 0.5, 0x9000, 60, None) == binding.ERR_INVALID_ARG     # stride < pages
    assert ps(C.byref(d), 0x7000, 0.5, 0x9000, 66, None) == binding.ERR_INVALID_ARG     # not a multiple of 4
    assert ps(C.byref(d), 0x7000, 0.5, 0x9004, 64, None) == binding.ERR_INVALID_ARG     # misaligned
    assert st(C.byref(d), None, 64, 4, 0x100, 0x200, None) == binding.ERR_INVALID_ARG
    assert st(C.byref(d), 0x9000, 64, 0, 0x100, 0x200, None) == binding.ERR_INVALID_ARG
    assert st(C.byref(d), 0x9000, 32, 4, 0x100, 0x200, None) == binding.ERR_INVALID_ARG
    # sparse decode
    g = c.unique_sparse_paged_decode
    assert g(C.byref(d), 0x7000, None, 0x200, 4, 0.0, 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert g(C.byref(d), 0x7000, 0x100, 0x200, 0, 0.0, 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert g(C.byref(d), 0x7000, 0x100, 0x200, 4, float("nan"), 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert g(C.byref(d), 0x7004, 0x100, 0x200, 4, 0.0, 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert g(C.byref(d), 0x7000, 0x100, 0x200, 4, 0.0, 0x8000, None, ws, 0, None) == binding.ERR_WORKSPACE
    assert g(C.byref(good_desc(v_cache=0)), 0x7000, 0x100, 0x200, 4, 0.0, 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    # fused step
    ds = c.unique_decode_step
    assert ds(C.byref(d), None, 4, 0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert ds(C.byref(d), 0x7000, 0, 0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert ds(C.byref(d), 0x7000, 4, -0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert ds(C.byref(d), 0x7000, 4, 0.5, 0.0, 1, 0x100, 0x200, None, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert ds(C.byref(d), 0x7000, 4, 0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, ws, 64, None) == binding.ERR_WORKSPACE
    assert ds(C.byref(good_desc(page_stats=0)), 0x7000, 4, 0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, ws, nws, None) == binding.ERR_INVALID_ARG
    # the step on the built-in scratch: same validation, and a step that does not fit is refused before any device call
    dss = c.unique_decode_step_static
    assert dss(C.byref(d), None, 4, 0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, None) == binding.ERR_INVALID_ARG
    assert dss(C.byref(d), 0x7000, 0, 0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, None) == binding.ERR_INVALID_ARG
    assert dss(C.byref(d), 0x7000, 4, 0.5, 0.0, 1, None, 0x200, 0x8000, None, None) == binding.ERR_INVALID_ARG
    assert dss(C.byref(good_desc(page_stats=0)), 0x7000, 4, 0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, None) == binding.ERR_INVALID_ARG
    too_big = good_desc(batch=64, max_pages_per_seq=16384)        # 64 x 8 score rows of 16384 floats = 32 MiB
    assert lib.workspace_bytes(too_big, 4) > binding.STATIC_SCRATCH_BYTES
    assert dss(C.byref(too_big), 0x7000, 4, 0.5, 0.0, 1, 0x100, 0x200, 0x8000, None, None) == binding.ERR_WORKSPACE
    assert "built-in scratch" in lib.last_error()
    # dense decode
    h = c.unique_dense_paged_decode
    assert h(C.byref(d), 0x7000, 0.0, None, None, ws, nws, None) == binding.ERR_INVALID_ARG
    assert h(C.byref(d), 0x7000, 0.0, 0x8000, None, None, 0, None) == binding.ERR_WORKSPACE


def test_binding_raises_with_detail(lib):
    with pytest.raises(binding.UniqueError) as e:
        lib.workspace_bytes(good_desc(head_dim=80), 4)
    assert e.value.code == binding.ERR_UNSUPPORTED and "head_dim=80" in str(e.value)


def test_header_is_plain_c_and_the_library_links_from_c(lib, tmp_path):
    """include/unique.h compiles as strict C99 and a C program linked against the library gets version, status
    strings and host-side validation errors without a GPU (tests/c_abi/abi_check.c)."""
    import subprocess
    from paper_2605_27740_amd import build as B
    exe = str(tmp_path / "abi_check")
    libdir = os.path.dirname(B.LIB_PATH)
    libname = os.path.basename(B.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi", "abi_check.c"), "-o", exe, "-L", libdir, f"-l:{libname}",
           f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "unique-gfx950" in r.stdout


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message: the path is measured on one GPU only."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU only" in r.stderr and r.stdout.strip() == ""
