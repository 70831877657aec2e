"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, sizes its workspace sensibly and rejects bad arguments
before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "ebsp_zipline.h"), os.path.join(ROOT, "include", "ebsp_zipline_bench.h")]
ORACLE_HEADER = os.path.join(ROOT, "include", "ebsp_zipline_oracle.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2001_01347_amd import build, zipline
    if not os.path.exists(zipline.LIB_PATH):
        build.build()
    return zipline.load()


def declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ebsp_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    from paper_2001_01347_amd import zipline
    names = declared_functions()
    assert len(names) >= 7
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    assert sorted(zipline.EXPORTS) == names


def test_headers_are_plain_c(tmp_path):
    # the boundary is a C ABI: every header must compile as C11 on its own, and a C program that uses it must link
    import subprocess
    for h in HEADERS + [ORACLE_HEADER]:
        src = tmp_path / (os.path.basename(h) + ".c")
        src.write_text(f'#include "{h}"\nint main(void) {{ return 0; }}\n')
        subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Wpedantic", "-Werror", "-fsyntax-only", str(src)], check=True)
    # a C caller of the oracle's entry point, linked against the oracle library
    import oracle
    lib_path = oracle.build()
    prog = tmp_path / "call_oracle.c"
    prog.write_text(f"""#include "{ORACLE_HEADER}"
#include <stdio.h>
int main(void) {{
    const int64_t ts[2 * 3] = {{10, 20, 30, 14, 29, 44}};
    int64_t barrier = 0, wait = 0; int32_t iters[2] = {{0, 0}};
    int rc = ebsp_zipline_oracle(ts, 1, 2, 3, &barrier, iters, &wait, 1);
    printf("%d %lld %lld %d %d\\n", rc, (long long)barrier, (long long)wait, iters[0], iters[1]);
    return 0;
}}
""")
    exe = tmp_path / "call_oracle"
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", str(prog), lib_path, "-fopenmp", f"-Wl,-rpath,{os.path.dirname(lib_path)}",
                    "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out == ["0", "30", "1", "3", "2"]        # the two-worker example worked by hand in tests/golden/worked_examples.json


def test_oracle_library_exports_its_header(oracle):
    text = re.sub(r"/\*.*?\*/", "", open(ORACLE_HEADER).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(ebsp_[a-z_]+)\s*\(", text)))
    assert names == ["ebsp_zipline_oracle"]
    lib = ctypes.CDLL(oracle.build())
    assert hasattr(lib, "ebsp_zipline_oracle")


def test_kernel_names(lib):
    from paper_2001_01347_amd import zipline
    names = zipline.ebsp_zipline_kernel_names()
    assert len(names) == lib.ebsp_zipline_kernel_count() >= 5
    assert all(n.startswith("zl_") for n in names)
    assert lib.ebsp_zipline_kernel_name(-1) is None
    assert lib.ebsp_zipline_kernel_name(len(names)) is None


def test_workspace_bytes(lib):
    from paper_2001_01347_amd import zipline
    ws = zipline.ebsp_zipline_workspace_bytes
    # one workgroup per instance needs no scratch
    assert ws(1, 4, 8) == 0 and ws(4096, 16, 64) == 0 and ws(16384, 64, 256) == 0
    # larger instances: crossing indices dominate, 4 bytes per (row, bin)
    big = ws(64, 1024, 4096)
    assert big > 64 * 1024 * 2048 * 4 and big % 256 == 0
    assert ws(1, 1, 16385) > 0
    assert ws(2, 256, 1024) > ws(1, 256, 1024)
    # invalid shapes
    assert ws(-1, 4, 8) == 0 and ws(1, 0, 8) == 0 and ws(1, 4, 0) == 0
    assert ws(1, 1 << 16, 1 << 15) == 0          # P*R >= 2^31


def test_argument_errors_are_reported_without_a_device(lib):
    from paper_2001_01347_amd import zipline
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)   # never dereferenced: every call below fails validation first
    assert lib.ebsp_zipline_batch(one, -1, 4, 8, one, one, one, null, null, 0, null) == -2
    assert "shape" in zipline.ebsp_last_error()
    assert lib.ebsp_zipline_batch(one, 1, 0, 8, one, one, one, null, null, 0, null) == -2
    assert lib.ebsp_zipline_batch(one, 1, 4, 0, one, one, one, null, null, 0, null) == -2
    assert lib.ebsp_zipline_batch(one, 1, 1 << 16, 1 << 15, one, one, one, null, null, 0, null) == -2
    assert lib.ebsp_zipline_batch(null, 1, 4, 8, one, one, one, null, null, 0, null) == -1
    assert lib.ebsp_zipline_batch(one, 1, 4, 8, null, one, one, null, null, 0, null) == -1
    assert lib.ebsp_zipline_batch(one, 1, 4, 8, one, null, one, null, null, 0, null) == -1
    assert lib.ebsp_zipline_batch(one, 1, 4, 8, one, one, null, null, null, 0, null) == -1
    # B == 0 is a no-op even with NULL data
    assert lib.ebsp_zipline_batch(null, 0, 4, 8, null, null, null, null, null, 0, null) == 0
    # multi-window shapes need a workspace that is present, large enough and aligned
    need = zipline.ebsp_zipline_workspace_bytes(2, 256, 1024)
    assert lib.ebsp_zipline_batch(one, 2, 256, 1024, one, one, one, null, null, 0, null) == -1
    assert lib.ebsp_zipline_batch(one, 2, 256, 1024, one, one, one, null, one, need - 1, null) == -3
    assert lib.ebsp_zipline_batch(one, 2, 256, 1024, one, one, one, null,
                                  ctypes.c_void_p(264), need, null) == -3
    assert lib.ebsp_zipline_profile_end(None, None) == -2     # no profile open
    assert lib.ebsp_zipline_profile_begin(0) == -2


def test_simulation_argument_errors(lib):
    from paper_2001_01347_amd import zipline
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)   # never dereferenced: every call below fails validation first
    sim = lib.ebsp_simulate_supersteps
    # (last_end0, interval, sync_cost, S, B, P, R, barrier, iters, wait, status, workspace, bytes, stream)
    assert sim(one, one, 0, -1, 1, 4, 8, one, one, one, null, one, 1 << 20, null) == -2
    assert sim(one, one, -1, 2, 1, 4, 8, one, one, one, null, one, 1 << 20, null) == -2
    assert "sync_cost" in zipline.ebsp_last_error()
    assert sim(one, one, 0, 2, 1, 0, 8, one, one, one, null, one, 1 << 20, null) == -2
    assert sim(null, one, 0, 2, 1, 4, 8, one, one, one, null, one, 1 << 20, null) == -1
    assert sim(one, null, 0, 2, 1, 4, 8, one, one, one, null, one, 1 << 20, null) == -1
    assert sim(one, one, 0, 2, 1, 4, 8, one, null, one, null, one, 1 << 20, null) == -1
    assert sim(one, one, 0, 2, 1, 4, 8, one, one, one, null, null, 0, null) == -1       # the start times need a workspace
    assert sim(one, one, 0, 2, 1, 4, 8, one, one, one, null, ctypes.c_void_p(264), 1 << 20, null) == -3
    need = zipline.ebsp_simulate_workspace_bytes(3, 600, 240)
    assert need >= zipline.ebsp_zipline_workspace_bytes(3, 600, 240) + 3 * 600 * 8
    assert zipline.ebsp_simulate_workspace_bytes(5, 16, 64) == 5 * 16 * 8 + (-5 * 16 * 8) % 256
    assert sim(one, one, 0, 2, 3, 600, 240, one, one, one, null, one, need - 256, null) == -3
    # no supersteps or no instances: nothing to do, whatever the pointers
    assert sim(null, null, 0, 0, 3, 4, 8, null, null, null, null, null, 0, null) == 0
    assert sim(null, null, 0, 5, 0, 4, 8, null, null, null, null, null, 0, null) == 0


def test_a_valid_call_without_a_gfx950_fails_loudly(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2001_01347_amd import zipline
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)   # never dereferenced: the device check comes before any launch
    assert lib.ebsp_zipline_batch(one, 1, 4, 8, one, one, one, null, null, 0, null) == -5
    assert "device" in zipline.ebsp_last_error()
    assert lib.ebsp_zipline_range_batch(one, 1, 4, 8, one, one, one, null, null, 0, null) == -5
    assert lib.ebsp_predict_zipline_batch(one, one, 1, 4, 8, one, one, one, null, null, 0, null) == -5


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2001_01347_amd import zipline
    with pytest.raises(ValueError):
        zipline.ebsp_zipline_batch(torch.zeros((1, 2, 3), dtype=torch.int64))


def test_binding_checks_the_buffers_it_is_given():
    # device, dtype, shape and contiguity of every caller-supplied output, and the workspace, are checked before
    # their addresses go to the library (a wrong buffer would be written out of bounds by a kernel)
    import torch
    from paper_2001_01347_amd import zipline
    check = zipline._check_buffer
    dev = torch.device("cpu")
    good = torch.zeros((3, 4), dtype=torch.int32)
    check("iters", good, dev, torch.int32, (3, 4))
    for bad in (torch.zeros((3, 4), dtype=torch.int64), torch.zeros((4, 3), dtype=torch.int32),
                torch.zeros((3, 8), dtype=torch.int32)[:, ::2], torch.zeros(12, dtype=torch.int32)):
        with pytest.raises(ValueError):
            check("iters", bad, dev, torch.int32, (3, 4))
    with pytest.raises(ValueError):
        check("iters", good, torch.device("meta"), torch.int32, (3, 4))
    ws = zipline._check_workspace
    raw = torch.zeros(2048, dtype=torch.uint8)
    skew = (-raw.data_ptr()) % 256
    ws(raw[skew:skew + 1024], dev, 1000)
    with pytest.raises(ValueError):
        ws(raw[skew + 8:skew + 1032], dev, 1000)        # not 256-byte aligned
    ws(None, dev, 0)
    for bad, need in ((raw[skew:skew + 512], 1000), (torch.zeros(1024, dtype=torch.int32), 16),
                      (None, 1), (torch.zeros(2048, dtype=torch.uint8)[::2], 16)):
        with pytest.raises(ValueError):
            ws(bad, dev, need)


def test_plan_of_a_shape_and_the_tuning_knobs(lib):
    """Host logic of the multi-window plan: shape_info, the knobs' limits and their effect on the sizes."""
    from paper_2001_01347_amd import zipline
    info = zipline.ebsp_zipline_shape_info
    tune = zipline.ebsp_zipline_tune
    try:
        tune(0, 0, 0)
        assert info(4096, 16, 64) == {"multi": 0, "window_cap": 0, "bins": 0, "max_windows": 0, "window_fill": 0, "slices": 0}
        big = info(64, 1024, 4096)              # many workers: 8192-record windows, filled to the brim
        assert big["multi"] == 1 and big["window_cap"] == 8192 and big["window_fill"] == 8192
        assert big["bins"] == 1024 * 4096 // 1024            # fine bins of window_cap / 8 keys on average
        # any two neighbouring windows hold more than window_fill keys: at most 2n/fill + 3 windows, an even number
        assert big["max_windows"] % 2 == 0 and 2 * 1024 * 4096 // 8192 + 3 <= big["max_windows"] <= 2 * 1024 * 4096 // 8192 + 4
        few = info(1024, 256, 1024)             # fewer than 512 workers: 4096-record windows
        assert few["window_cap"] == 4096 and few["window_fill"] == 4096 and few["bins"] == 256 * 1024 // 512
        # the knobs: limits
        for bad in [(1000, 0, 0), (0, -1, 0), (0, 16385, 0), (0, 0, 100), (0, 0, -5)]:
            with pytest.raises(zipline.ZipLineError):
                tune(*bad)
        # a smaller fill means more windows and more scratch; a fill above the capacity is capped
        base = zipline.ebsp_zipline_workspace_bytes(64, 1024, 4096)
        tune(0, 0, 2048)
        half = info(64, 1024, 4096)
        assert half["window_fill"] == 2048 and half["max_windows"] > big["max_windows"]
        assert zipline.ebsp_zipline_workspace_bytes(64, 1024, 4096) > base
        tune(0, 0, 1 << 20)
        assert info(64, 1024, 4096)["window_fill"] == 8192
        # the capacity and the single-workgroup limit
        tune(16384, 0, 0)
        assert info(64, 1024, 4096)["window_cap"] == 16384
        tune(0, 4096, 0)
        assert info(16384, 64, 256)["multi"] == 1 and zipline.ebsp_zipline_workspace_bytes(16384, 64, 256) > 0
        # the range objective leaves room for its short list and cuts instances above 8192 entries
        tune(0, 0, 0)
        assert zipline.ebsp_zipline_range_workspace_bytes(16384, 64, 256) > 0
        assert zipline.ebsp_zipline_range_workspace_bytes(4096, 16, 64) == 0
        assert zipline.ebsp_zipline_range_workspace_bytes(64, 1024, 4096) > base     # more, smaller windows
    finally:
        tune(0, 0, 0)
