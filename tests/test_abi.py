"""The C ABI: the built library loads without a GPU, exports every function that
include/okt.h declares, the Python binding mirrors the header, and argument
errors are caught on the host before anything is launched."""
import ctypes
import os
import re
import shutil
import subprocess

import numpy as np
import pytest

from oracle import okt_oracle as orc

import paper_2201_07598_amd as okt
from paper_2201_07598_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "okt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(okt_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    lib = okt.load_library()
    names = declared_functions()
    assert {"okt_residual_accumulate", "okt_topk_threshold_exact", "okt_threshold_select",
            "okt_region_partition", "okt_sparse_reduce"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_binding_mirrors_the_header():
    assert sorted(binding.SIGNATURES) == declared_functions()
    for name in binding.SIGNATURES:
        assert callable(getattr(okt, name)), name


def test_status_strings_and_version():
    assert okt.okt_version() >= 100
    assert okt.okt_status_string(0) == "ok"
    for code in (-1, -2, -3, -99):
        assert okt.okt_status_string(code)


def test_workspace_sizes_are_monotone_and_aligned():
    sizes = [okt.okt_workspace_bytes(n, 16) for n in (1, 1 << 20, 25_557_032, 336_000_000)]
    assert sizes == sorted(sizes) and all(s % 256 == 0 and s > 0 for s in sizes)
    assert okt.okt_workspace_bytes(1 << 20, 256) >= okt.okt_workspace_bytes(1 << 20, 4)
    assert okt.okt_sparse_reduce_batch_workspace_bytes(8, 16, 100_000) >= \
        8 * (okt.okt_sparse_reduce_batch_workspace_bytes(1, 16, 100_000) - 256)


def test_argument_errors_are_found_on_the_host():
    lib = okt.load_library()
    INVALID, WORKSPACE = -1, -2
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x1000)          # aligned, never dereferenced on these paths
    odd = ctypes.c_void_p(0x1004)           # not 16-byte aligned
    assert lib.okt_residual_accumulate(null, null, 1.0, 0, null) == 0          # n = 0: no-op
    assert lib.okt_residual_accumulate(null, fake, 1.0, 8, null) == INVALID
    assert lib.okt_residual_accumulate(fake, odd, 1.0, 8, null) == INVALID
    assert lib.okt_residual_accumulate(fake, fake, 1.0, 1 << 32, null) == INVALID
    assert lib.okt_topk_threshold_exact(fake, 10, 0, fake, fake, fake, 1 << 20, null) == INVALID   # k = 0
    assert lib.okt_topk_threshold_exact(fake, 10, 11, fake, fake, fake, 1 << 20, null) == INVALID  # k > n
    assert lib.okt_topk_threshold_exact(fake, 10, 5, fake, fake, fake, 4096, null) == WORKSPACE
    assert lib.okt_topk_threshold_exact(fake, 10, 5, fake, fake, null, 1 << 20, null) == WORKSPACE
    assert lib.okt_threshold_select(fake, 10, null, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_threshold_select(fake, 1 << 20, fake, fake, fake, 4, fake, fake, 8, null) == WORKSPACE
    assert lib.okt_region_partition(fake, fake, 0, 4, fake, fake, null) == INVALID          # n = 0
    assert lib.okt_region_partition(fake, fake, 100, 0, fake, fake, null) == INVALID        # R = 0
    assert lib.okt_sparse_reduce(fake, fake, fake, 0, 0, 10, fake, fake, 4, fake, null, fake, 1 << 20, null) == INVALID
    assert lib.okt_sparse_reduce(fake, fake, fake, 4, 20, 10, fake, fake, 4, fake, null, fake, 1 << 20, null) == INVALID
    assert lib.okt_sparse_reduce(fake, fake, fake, 4, 0, 1 << 20, fake, fake, 4, fake, null, fake, 64, null) == WORKSPACE
    assert lib.okt_coo_threshold_select(fake, odd, fake, 10, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_coo_threshold_select(fake, fake, null, 10, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_coo_threshold_select(fake, fake, fake, 1 << 32, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_coo_threshold_select(fake, fake, fake, 1 << 20, fake, fake, fake, 4, fake, fake, 8, null) == WORKSPACE
    assert lib.okt_index_intersect_restore(null, 100, fake, fake, fake, 10, fake, fake, 10, null, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_index_intersect_restore(fake, 100, fake, fake, fake, 10, null, fake, 10, null, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_index_intersect_restore(fake, 100, fake, fake, fake, 10, fake, fake, 10, null, null, fake, 1 << 20, null) == INVALID
    assert lib.okt_index_intersect_restore(fake, 100, fake, fake, fake, 1 << 20, fake, fake, 10, null, fake, fake, 8, null) == WORKSPACE
    # the entry point on the library's own scan state checks its arguments first, too
    assert lib.okt_threshold_select_noalloc(fake, 10, null, fake, fake, 4, fake, null) == INVALID
    assert lib.okt_threshold_select_noalloc(odd, 10, fake, fake, fake, 4, fake, null) == INVALID
    assert lib.okt_threshold_select_noalloc(fake, 1 << 32, fake, fake, fake, 4, fake, null) == INVALID
    assert lib.okt_threshold_select_noalloc(fake, 10, fake, null, fake, 4, fake, null) == INVALID
    assert lib.okt_threshold_select_copy(odd, 10, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_threshold_select_copy(fake, 1 << 20, fake, fake, fake, 4, fake, fake, 8, null) == WORKSPACE
    assert lib.okt_index_intersect_zero(null, 100, fake, fake, 10, fake, fake, 10, null, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_index_intersect_zero(fake, 100, fake, fake, 1 << 20, fake, fake, 10, null, fake, fake, 8, null) == WORKSPACE
    assert lib.okt_sparse_reduce_segments(fake, fake, fake, null, 4, 0, 10, fake, fake, 4, fake, null, fake, 1 << 20, null) == INVALID
    assert lib.okt_sparse_reduce_segments(fake, fake, fake, fake, 4, 20, 10, fake, fake, 4, fake, null, fake, 1 << 20, null) == INVALID
    assert lib.okt_sparse_reduce_segments(fake, fake, fake, fake, 4, 0, 1 << 20, fake, fake, 4, fake, null, fake, 64, null) == WORKSPACE
    # okt_accumulate_topk_select(grad, res, lr, n, k, th, cnt, idx, val, capacity, nnz, ws, ws_bytes, stream)
    assert lib.okt_accumulate_topk_select(fake, ctypes.c_void_p(0x2000), 1.0, 10, 0, fake, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID   # k = 0
    assert lib.okt_accumulate_topk_select(fake, ctypes.c_void_p(0x2000), 1.0, 10, 11, fake, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID  # k > n
    assert lib.okt_accumulate_topk_select(fake, ctypes.c_void_p(0x2000), 1.0, 0, 1, fake, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID    # n = 0
    assert lib.okt_accumulate_topk_select(fake, fake, 1.0, 10, 5, fake, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID                      # grad is the residual
    assert lib.okt_accumulate_topk_select(fake, odd, 1.0, 10, 5, fake, fake, fake, fake, 4, fake, fake, 1 << 20, null) == INVALID
    assert lib.okt_accumulate_topk_select(fake, ctypes.c_void_p(0x2000), 1.0, 10, 5, fake, fake, null, fake, 4, fake, fake, 1 << 20, null) == INVALID   # capacity without idx_out
    assert lib.okt_accumulate_topk_select(fake, ctypes.c_void_p(0x2000), 1.0, 10, 5, fake, fake, fake, fake, 4, fake, fake, 4096, null) == WORKSPACE
    assert lib.okt_accumulate_topk_select(fake, ctypes.c_void_p(0x2000), 1.0, 10, 5, fake, fake, fake, fake, 4, fake, null, 1 << 20, null) == WORKSPACE
    assert lib.okt_stream_copy(null, null, 0, null) == 0                                 # n = 0: no-op
    assert lib.okt_stream_copy(fake, odd, 8, null) == INVALID
    assert lib.okt_stream_copy(fake, fake, 1 << 32, null) == INVALID
    assert lib.okt_stream_sum(fake, 8, null, null) == INVALID
    assert lib.okt_stream_sum(odd, 8, fake, null) == INVALID
    with pytest.raises(TypeError):
        okt.okt_residual_accumulate(None, None, 1.0)


def test_header_is_plain_c(tmp_path):
    """include/okt.h is a C header: it compiles as C99 and as C++ without a warning,
    and a C program can name every declared function."""
    import shutil
    import subprocess
    names = declared_functions()
    src = tmp_path / "use_okt.c"
    body = "\n".join(f"    p[{i}] = (fn)&{name};" for i, name in enumerate(names))
    src.write_text('#include "okt.h"\ntypedef void (*fn)(void);\nint main(void) {\n'
                   f'    fn p[{len(names)}];\n{body}\n'
                   '    okt_chunk c = {0, 0, 0, 0, 0};\n'
                   f'    return p[{len(names) - 1}] == 0 || c.count != 0 || OKT_ERR_HIP == 0;\n'
                   '}\n')
    inc = os.path.join(ROOT, "include")
    for compiler, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        if shutil.which(compiler) is None:
            pytest.skip(f"{compiler} not installed")
        cmd = [compiler, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc,
               "-x", "c" if compiler == "gcc" else "c++", str(src)]
        done = subprocess.run(cmd, capture_output=True, text=True)
        assert done.returncode == 0, done.stderr


def test_cabi_host_program_builds_and_links(tmp_path):
    """tests/cabi/cabi_smoke.cpp, the torch-free caller of the C ABI, compiles for
    gfx950 and links against the built library (it runs on the GPU machine, from smoke())."""
    import subprocess
    from paper_2201_07598_amd import build as okt_build
    out = okt_build.build_cabi_smoke(verbose=False, out=str(tmp_path / "cabi_smoke.bin"))
    listing = subprocess.run(["ldd", out], capture_output=True, text=True).stdout
    assert "libokt.so" in listing and "not found" not in listing.split("libokt.so")[1].splitlines()[0]


def test_balance_plan_library_matches_the_oracle():
    # host logic of the library (no GPU involved) against the oracle
    rng = np.random.default_rng(92)
    cases = [[10_000] + [0] * 7, [0] * 7 + [10_000], [3, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 1],
             [5, 5, 5, 5, 5], [0] * 6, [2 ** 32 - 1] + [1] * 9]
    for P in (5, 9, 16, 64, 200):
        for _ in range(20):
            s = rng.integers(0, 30, P)
            s[rng.integers(0, P)] = rng.integers(100, 5000)
            cases.append([int(x) for x in s])
    for sizes in cases:
        want = orc.balance_plan(sizes)
        got = okt.okt_balance_plan(sizes)
        assert got[0] == want[0], sizes
        assert [tuple(int(x) for x in c) for c in got[1]] == [tuple(c) for c in want[1]], sizes


def test_index_searches_match_std_lower_bound(tmp_path):
    """The searches behind the reduce's boundary tables (bisection, and the one that
    starts from a guess) are plain functions a host compiler can build: checked
    here against std::lower_bound on random lists, ranges and guesses."""
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = tmp_path / "search_check"
    subprocess.run([gxx, "-O2", "-std=c++17", "-Wall", "-Werror", "-I",
                    os.path.join(ROOT, "paper_2201_07598_amd", "csrc"),
                    os.path.join(ROOT, "tests", "cabi", "search_check.cpp"), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout
    assert "0 disagreements" in out.stdout


def test_workspace_plans_hold_on_any_device(tmp_path):
    """The workspace layouts are host arithmetic (okt_sizes.h): for lengths up to
    2^32 - 1 and devices of 1 to 1024 compute units the parts of the three-pass
    select's workspace lie in order without overlap, cover every tile, and fit the
    size a caller is told; both select forms' launches cover the vector."""
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = tmp_path / "sizes_check"
    subprocess.run([gxx, "-O2", "-std=c++17", "-Wall", "-Werror", "-I",
                    os.path.join(ROOT, "paper_2201_07598_amd", "csrc"),
                    os.path.join(ROOT, "tests", "cabi", "sizes_check.cpp"), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout
    assert "0 violations" in out.stdout
