"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, rejects bad arguments before touching the GPU, and its host
planning code (magic division, tile choice, workspace plan) is self-consistent."""
import ctypes
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "convnet_hotpath.h")


@pytest.fixture(scope="module")
def lib():
    from paper_1312_5853_amd import binding, build
    if build.is_stale():
        build.build()
    return binding.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", " ".join(l for l in text.splitlines() if not l.startswith("#")))))


def test_every_declared_symbol_is_exported(lib):
    from paper_1312_5853_amd import binding
    names = declared_functions()
    assert {"conv_fwd", "conv_bwd_data", "conv_bwd_filter", "conv_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(names)


def test_status_strings(lib):
    seen = set()
    for code in range(0, -8, -1):
        s = lib.conv_status_string(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert lib.conv_status_string(-99).decode() == "unknown status"
    assert lib.conv_last_hip_error().decode() == ""


GOOD = dict(N=2, C=16, H=13, W=13, K=32, R=3, S=3, stride=1, pad=1)
PTR = 0x10000          # never dereferenced: every call below fails a host-side check first


def call(lib, fn, ws=PTR, ws_bytes=1 << 30, a=PTR, b=PTR, out=PTR, dtype=0, **over):
    d = dict(GOOD, **over)
    return getattr(lib, fn)(a, b, out, d["N"], d["C"], d["H"], d["W"], d["K"], d["R"], d["S"], d["stride"], d["pad"],
                            dtype, ws, ws_bytes, None)


@pytest.mark.parametrize("fn", ["conv_fwd", "conv_bwd_data", "conv_bwd_filter"])
def test_argument_checks_run_before_any_gpu_call(lib, fn):
    from paper_1312_5853_amd import binding as b
    assert call(lib, fn, a=None) == b.ERR_INVALID_ARG
    assert call(lib, fn, b=None) == b.ERR_INVALID_ARG
    assert call(lib, fn, out=None) == b.ERR_INVALID_ARG
    for key in ("N", "C", "H", "W", "K", "R", "S", "stride"):
        assert call(lib, fn, **{key: 0}) == b.ERR_INVALID_ARG, key
        assert call(lib, fn, **{key: -3}) == b.ERR_INVALID_ARG, key
    assert call(lib, fn, pad=-1) == b.ERR_INVALID_ARG
    assert call(lib, fn, R=16, pad=1) == b.ERR_INVALID_ARG          # empty output (P <= 0)
    assert call(lib, fn, dtype=3) == b.ERR_BAD_DTYPE and call(lib, fn, dtype=-1) == b.ERR_BAD_DTYPE
    assert call(lib, fn, N=2048, C=64, H=64, W=64) == b.ERR_TOO_LARGE
    assert call(lib, fn, a=PTR + 4) == b.ERR_MISALIGNED
    assert call(lib, fn, out=PTR + 8) == b.ERR_MISALIGNED
    assert call(lib, fn, ws=PTR + 16) == b.ERR_MISALIGNED
    need = lib.conv_workspace_bytes({"conv_fwd": 0, "conv_bwd_data": 1, "conv_bwd_filter": 2}[fn],
                                    *[GOOD[k] for k in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad")], 0)
    assert need > 0
    assert call(lib, fn, ws=None, ws_bytes=0) == b.ERR_WORKSPACE
    assert call(lib, fn, ws_bytes=need - 1) == b.ERR_WORKSPACE


def test_batch_stride_checks(lib):
    from paper_1312_5853_amd import binding as b
    d = GOOD
    args = [PTR, PTR, PTR] + [d[k] for k in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad")]
    sample_x, sample_y = 16 * 169, 32 * 169
    assert lib.conv_fwd_ex(*args, sample_x - 1, 0, 0, PTR, 1 << 30, None) == b.ERR_INVALID_ARG
    assert lib.conv_fwd_ex(*args, 0, sample_y - 1, 0, PTR, 1 << 30, None) == b.ERR_INVALID_ARG
    assert lib.conv_fwd_ex(*args, 1 << 40, 0, 0, PTR, 1 << 30, None) == b.ERR_TOO_LARGE


def test_workspace_bytes(lib):
    dims = [128, 256, 13, 13, 384, 3, 3, 1, 1]
    a = lib.conv_workspace_bytes(0, *dims, 0)
    assert a == lib.conv_workspace_bytes(0, *dims, 0) and a >= 384 * 2304 * 4
    assert lib.conv_workspace_bytes(2, *dims, 0) >= 384 * 2304 * 4
    # bf16 backward-data (direct-to-LDS kernel): tap table, re-laid filters, and the channel-blocked copy of the
    # output gradient with its zero padding in place (15 x 15 positions of 32 bytes per plane and 16-channel block);
    # no partial sums
    xb = 128 * (384 // 16) * 15 * 15 * 32
    assert xb < lib.conv_workspace_bytes(1, *dims, 1) <= xb + 256 * 3456 * 4 + 65536
    # bf16 outputs: written by the bf16 kernels themselves, nothing extra
    for op in (0, 1, 2):
        assert lib.conv_workspace_bytes(op, *dims, 2) == lib.conv_workspace_bytes(op, *dims, 1)
    odd = [4, 3, 32, 32, 20, 5, 5, 2, 1]            # 3 -> 20 channels: no bf16 kernel
    up = lambda v: -(-v // 256) * 256                                       # regions are 256-byte aligned
    ws = lambda op, dt: lib.conv_workspace_bytes(op, *odd, dt)
    # forward (few-channel kernel reads bf16 itself): only the filters are widened; bf16 output written directly
    assert ws(0, 1) - ws(0, 0) == up(20 * 3 * 25 * 4) and ws(0, 2) == ws(0, 1)
    # backward-data: both inputs widened to fp32 copies, a bf16 output staged in fp32 first
    assert ws(1, 1) - ws(1, 0) == up(4 * 20 * 15 * 15 * 4) + up(20 * 3 * 25 * 4)
    assert ws(1, 2) - ws(1, 1) == up(4 * 3 * 32 * 32 * 4)
    # backward-filter (tap-table kernel reads bf16 itself): nothing extra; its output is fp32 in every mode
    assert ws(2, 1) == ws(2, 0) == ws(2, 2)
    assert lib.conv_workspace_bytes(3, *dims, 0) == 0
    assert lib.conv_workspace_bytes(0, 0, 256, 13, 13, 384, 3, 3, 1, 1, 0) == 0


def test_glue_argument_checks(lib):
    from paper_1312_5853_amd import binding as b
    assert lib.relu_fwd(None, PTR, 4, 0, None) == b.ERR_INVALID_ARG
    assert lib.relu_fwd(PTR, PTR, -1, 0, None) == b.ERR_INVALID_ARG
    assert lib.relu_fwd(PTR, PTR, 0, 0, None) == b.OK
    assert lib.relu_fwd(PTR, PTR, 4, 3, None) == b.ERR_BAD_DTYPE
    assert lib.relu_bwd(PTR, PTR + 2, PTR, 4, 0, None) == b.ERR_MISALIGNED      # fp32 needs 4-byte alignment
    assert lib.relu_bwd(PTR, PTR + 1, PTR, 4, 1, None) == b.ERR_MISALIGNED      # bf16 needs 2-byte alignment
    for fn in (lib.maxpool3x3s2_fwd, lib.relu_maxpool3x3s2_fwd):
        assert fn(PTR, PTR, 4, 2, 5, 0, None) == b.ERR_INVALID_ARG         # plane smaller than the window
        assert fn(PTR, PTR, 0, 5, 5, 0, None) == b.ERR_INVALID_ARG
        assert fn(None, PTR, 1, 5, 5, 0, None) == b.ERR_INVALID_ARG
        assert fn(PTR, PTR, 1, 5, 5, 7, None) == b.ERR_BAD_DTYPE
    for fn in (lib.maxpool3x3s2_bwd, lib.relu_maxpool3x3s2_bwd):
        assert fn(PTR, None, PTR, 1, 5, 5, 0, None) == b.ERR_INVALID_ARG
        assert fn(PTR, PTR, PTR + 1, 1, 5, 5, 0, None) == b.ERR_MISALIGNED
        assert fn(PTR, PTR, PTR + 1, 1, 5, 5, 2, None) == b.ERR_MISALIGNED
        assert fn(PTR, PTR, PTR, 1, 5, 5, -1, None) == b.ERR_BAD_DTYPE


def test_binding_fails_loudly_without_the_library(tmp_path):
    import sys
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_1312_5853_amd import binding\n"
            "binding.LIB_PATH = %r\n"
            "try:\n    binding.lib()\nexcept RuntimeError as e:\n    print('raised'); sys.exit(0)\nsys.exit(1)\n"
            % (ROOT, str(tmp_path / "missing.so")))
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True)
    assert out.returncode == 0 and "raised" in out.stdout


def test_product_never_imports_the_oracle():
    import sys
    code = ("import sys; sys.path.insert(0, %r)\n"
            "import paper_1312_5853_amd.binding, paper_1312_5853_amd.stack, paper_1312_5853_amd.synth\n"
            "sys.exit(1 if any(m == 'oracle' or m.startswith('oracle.') for m in sys.modules) else 0)\n" % ROOT)
    assert subprocess.run([sys.executable, "-c", code]).returncode == 0
    for name in ("binding.py", "stack.py", "synth.py", "build.py", "__init__.py"):
        text = open(os.path.join(ROOT, "paper_1312_5853_amd", name)).read()
        assert "import oracle" not in text and "from oracle" not in text
    for name in os.listdir(os.path.join(ROOT, "paper_1312_5853_amd", "csrc")):
        if not name.endswith((".h", ".hip", ".cpp", ".c")):
            continue
        assert "oracle" not in open(os.path.join(ROOT, "paper_1312_5853_amd", "csrc", name)).read().lower()


def test_host_planning_selftest(tmp_path):
    exe = str(tmp_path / "host_selftest")
    src = os.path.join(ROOT, "tests", "host_selftest.cpp")
    subprocess.run(["g++", "-O2", "-std=c++17", "-o", exe, src], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout
    assert "0 failures" in out.stdout


SAN_FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
# leak checking off (the OpenMP runtime keeps its thread pool); the link-order check is off because the test
# harness may preload a library of its own ahead of the sanitizer runtime
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")


def test_oracle_runs_clean_under_address_and_ub_sanitizers(tmp_path):
    """The C oracle built with AddressSanitizer + UndefinedBehaviorSanitizer: all entry points on exactly-sized heap
    tensors (padding beyond the filter, strides that leave rows unread, 1x1 outputs), checked by closed forms."""
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-std=c99", "-fopenmp", "-Wall", "-Wextra"] + SAN_FLAGS +
                   ["-o", exe, os.path.join(ROOT, "tests", "oracle_sanitizer_main.c"),
                    os.path.join(ROOT, "oracle", "conv_oracle.c"), "-lm"], check=True)
    out = subprocess.run([exe], capture_output=True, text=True, env=SAN_ENV)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "0 failures" in out.stdout and "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr


def test_host_planning_runs_clean_under_sanitizers(tmp_path):
    """The host-side planning header (argument checks, extents, tile and split choice, workspace layout, magic
    division) under the same sanitizers: signed overflow in the size arithmetic would stop the run."""
    exe = str(tmp_path / "host_selftest_san")
    subprocess.run(["g++", "-std=c++17"] + SAN_FLAGS + ["-o", exe, os.path.join(ROOT, "tests", "host_selftest.cpp")],
                   check=True)
    out = subprocess.run([exe], capture_output=True, text=True, env=SAN_ENV)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "0 failures" in out.stdout and "runtime error" not in out.stderr


def test_noalloc_entry_point_checks_before_any_gpu_call(lib):
    """conv_bwd_filter_noalloc: the ordinary argument checks, and a pass that needs more scratch than the built-in
    buffer is refused with its own status -- all on the host (no GPU here)."""
    from paper_1312_5853_amd import binding as b
    f = lib.conv_bwd_filter_noalloc
    good = (2, 16, 13, 13, 32, 3, 3, 1, 1)
    assert f(None, PTR, PTR, *good, 0, None) == b.ERR_INVALID_ARG
    assert f(PTR, PTR, None, *good, 0, None) == b.ERR_INVALID_ARG
    assert f(PTR, PTR, PTR, 0, 16, 13, 13, 32, 3, 3, 1, 1, 0, None) == b.ERR_INVALID_ARG
    assert f(PTR, PTR, PTR, *good, 9, None) == b.ERR_BAD_DTYPE
    assert f(PTR + 4, PTR, PTR, *good, 0, None) == b.ERR_MISALIGNED
    # bf16 second layer at N = 256: about 100 MB of packed copies and partial sums
    big = (256, 48, 27, 27, 128, 5, 5, 1, 2)
    assert lib.conv_workspace_bytes(b.OP_BWD_FILTER, *big, 1) > b.NOALLOC_SCRATCH_BYTES
    assert f(PTR, PTR, PTR, *big, 1, None) == b.ERR_SCRATCH_LIMIT
    # fp32: every layer of the stack fits at every batch size of the workload list
    from paper_1312_5853_amd import synth
    for N in (64, 128, 256):
        for name, L in synth.LAYERS.items():
            dims = (N, L["C"], L["H"], L["W"], L["K"], L["R"], L["S"], L["stride"], L["pad"])
            assert lib.conv_workspace_bytes(b.OP_BWD_FILTER, *dims, 0) <= b.NOALLOC_SCRATCH_BYTES, (N, name)
    header = open(HEADER).read()
    assert "#define CONV_NOALLOC_SCRATCH_BYTES (48u << 20)" in header


def test_convert_argument_checks(lib):
    from paper_1312_5853_amd import binding as b
    assert lib.convert_f32_to_bf16(None, PTR, 8, None) == b.ERR_INVALID_ARG
    assert lib.convert_f32_to_bf16(PTR, None, 8, None) == b.ERR_INVALID_ARG
    assert lib.convert_f32_to_bf16(PTR, PTR, -1, None) == b.ERR_INVALID_ARG
    assert lib.convert_f32_to_bf16(PTR + 2, PTR, 8, None) == b.ERR_MISALIGNED
    assert lib.convert_f32_to_bf16(PTR, PTR + 1, 8, None) == b.ERR_MISALIGNED
    assert lib.convert_f32_to_bf16(PTR, PTR, 0, None) == b.OK


def test_grouped_argument_checks(lib):
    from paper_1312_5853_amd import binding as b
    dims = [4, 96, 27, 27, 256, 5, 5, 1, 2]
    for fn in (lib.conv_fwd_grouped, lib.conv_bwd_data_grouped, lib.conv_bwd_filter_grouped):
        assert fn(PTR, PTR, PTR, *dims, 0, 0, PTR, 1 << 30, None) == b.ERR_INVALID_ARG        # no groups
        assert fn(PTR, PTR, PTR, *dims, 5, 0, PTR, 1 << 30, None) == b.ERR_INVALID_ARG        # 96 % 5
        assert fn(PTR, PTR, PTR, *dims, 3, 0, PTR, 1 << 30, None) == b.ERR_INVALID_ARG        # 256 % 3
        assert fn(None, PTR, PTR, *dims, 2, 0, PTR, 1 << 30, None) == b.ERR_INVALID_ARG
        assert fn(PTR, PTR, PTR, *dims, 2, 9, PTR, 1 << 30, None) == b.ERR_BAD_DTYPE
        assert fn(PTR, PTR, PTR, *dims, 2, 0, None, 0, None) == b.ERR_WORKSPACE
        assert fn(PTR, PTR + 4, PTR, *dims, 2, 0, PTR, 1 << 30, None) == b.ERR_MISALIGNED
    # columns in one launch hold one filter copy / one set of partial sums per column
    for op in (0, 1, 2):
        two = lib.conv_workspace_bytes_grouped(op, *dims, 2, 0)
        one = lib.conv_workspace_bytes(op, 4, 48, 27, 27, 128, 5, 5, 1, 2, 0)
        assert two > one and lib.conv_workspace_bytes_grouped(op, *dims, 1, 0) == lib.conv_workspace_bytes(op, *dims, 0)
    assert lib.conv_workspace_bytes_grouped(0, *dims, 7, 0) == 0


def test_bias_argument_checks(lib):
    from paper_1312_5853_amd import binding as b
    assert lib.bias_fwd(None, PTR, 2, 3, 4, 0, None) == b.ERR_INVALID_ARG
    assert lib.bias_fwd(PTR, PTR, 0, 3, 4, 0, None) == b.ERR_INVALID_ARG
    assert lib.bias_fwd(PTR, PTR, 2, 3, 4, 5, None) == b.ERR_BAD_DTYPE
    assert lib.bias_fwd(PTR + 2, PTR, 2, 3, 4, 0, None) == b.ERR_MISALIGNED
    assert lib.bias_fwd(PTR, PTR, 1 << 15, 1 << 10, 1 << 7, 0, None) == b.ERR_TOO_LARGE
    need = lib.bias_bwd_workspace_bytes(128, 96)
    assert need == 96 * 21 * 4 and lib.bias_bwd_workspace_bytes(0, 96) == 0
    assert lib.bias_bwd(PTR, PTR, 128, 96, 3025, 0, PTR, need - 1, None) == b.ERR_WORKSPACE
    assert lib.bias_bwd(PTR, PTR, 128, 96, 3025, 0, None, need, None) == b.ERR_WORKSPACE
    assert lib.bias_bwd(PTR, None, 128, 96, 3025, 0, PTR, need, None) == b.ERR_INVALID_ARG
    assert lib.bias_bwd(PTR, PTR, 128, 96, 3025, 0, PTR + 16, need, None) == b.ERR_MISALIGNED


def test_fused_epilogue_argument_checks(lib):
    from paper_1312_5853_amd import binding as b
    dims = (2, 16, 8, 8, 16, 3, 3, 1, 1)
    need = lib.conv_workspace_bytes(b.OP_FWD, *dims, 0)
    assert lib.conv_fwd_bias_relu(PTR, PTR, None, None, *dims, 1, 0, PTR, need, None) == b.ERR_INVALID_ARG
    assert lib.conv_fwd_bias_relu(PTR, PTR, None, PTR, *dims, 2, 0, PTR, need, None) == b.ERR_INVALID_ARG   # relu flag
    assert lib.conv_fwd_bias_relu(PTR, PTR, PTR + 2, PTR, *dims, 1, 0, PTR, need, None) == b.ERR_MISALIGNED  # bias
    assert lib.conv_fwd_bias_relu(PTR, PTR, None, PTR, *dims, 1, 9, PTR, need, None) == b.ERR_BAD_DTYPE
    assert lib.conv_fwd_bias_relu(PTR, PTR, None, PTR, *dims, 1, 0, None, 0, None) == b.ERR_WORKSPACE
    need = lib.conv_workspace_bytes(b.OP_BWD_DATA, *dims, 0)
    assert lib.conv_bwd_data_relu(PTR, PTR, None, PTR, *dims, 0, PTR, need, None) == b.ERR_INVALID_ARG      # no mask
    assert lib.conv_bwd_data_relu(PTR, PTR, PTR + 2, PTR, *dims, 0, PTR, need, None) == b.ERR_MISALIGNED
    assert lib.conv_bwd_data_relu(PTR, PTR, PTR, PTR, *dims, 0, None, 0, None) == b.ERR_WORKSPACE


def test_fc_and_sgd_argument_checks(lib):
    from paper_1312_5853_amd import binding as b
    # workspace: the partial sums of a split reduction, nothing when the reduction is not split
    assert lib.fc_workspace_bytes(b.OP_FWD, 128, 9216, 4096, 0) == 16 * 128 * 4096 * 4
    assert lib.fc_workspace_bytes(b.OP_BWD_FILTER, 128, 9216, 4096, 0) == 0
    assert lib.fc_workspace_bytes(b.OP_FWD, 128, 9214, 4096, 0) == 0                 # invalid: I % 4
    assert lib.fc_workspace_bytes(7, 128, 9216, 4096, 0) == 0
    assert lib.fc_fwd(PTR, PTR, None, PTR, 4, 6, 8, 0, 0, None, 0, None) == b.ERR_INVALID_ARG
    assert lib.fc_fwd(PTR, PTR, None, PTR, 4, 8, 6, 0, 0, None, 0, None) == b.ERR_INVALID_ARG
    assert lib.fc_fwd(None, PTR, None, PTR, 4, 8, 8, 0, 0, None, 0, None) == b.ERR_INVALID_ARG
    assert lib.fc_fwd(PTR, PTR, None, PTR, 4, 8, 8, 2, 0, None, 0, None) == b.ERR_INVALID_ARG
    assert lib.fc_fwd(PTR, PTR, None, PTR, 4, 8, 8, 0, 1, None, 0, None) == b.ERR_BAD_DTYPE
    assert lib.fc_fwd(PTR + 4, PTR, None, PTR, 4, 8, 8, 0, 0, None, 0, None) == b.ERR_MISALIGNED
    assert lib.fc_fwd(PTR, PTR, None, PTR, 1 << 16, 1 << 15, 8, 0, 0, None, 0, None) == b.ERR_TOO_LARGE
    assert lib.fc_fwd(PTR, PTR, None, PTR, 128, 9216, 4096, 0, 0, None, 0, None) == b.ERR_WORKSPACE
    assert lib.fc_bwd_data(PTR, PTR, PTR, 0, 8, 8, 0, None, 0, None) == b.ERR_INVALID_ARG
    assert lib.fc_bwd_filter(PTR, None, PTR, 4, 8, 8, 0, None, 0, None) == b.ERR_INVALID_ARG
    f = ctypes.c_float
    assert lib.sgd_update(None, PTR, PTR, 4, f(0.1), f(0), f(0), f(1), None) == b.ERR_INVALID_ARG
    assert lib.sgd_update(PTR, PTR, PTR, -1, f(0.1), f(0), f(0), f(1), None) == b.ERR_INVALID_ARG
    assert lib.sgd_update(PTR, PTR + 2, PTR, 4, f(0.1), f(0), f(0), f(1), None) == b.ERR_MISALIGNED
    assert lib.sgd_update(None, None, None, 0, f(0.1), f(0), f(0), f(1), None) == b.OK
    ptrs = (ctypes.c_void_p * 2)(PTR, PTR)
    odd = (ctypes.c_void_p * 2)(PTR, PTR + 2)
    nul = (ctypes.c_void_p * 2)(PTR, None)
    cnt = (ctypes.c_int64 * 2)(8, 8)
    neg = (ctypes.c_int64 * 2)(8, -1)
    assert lib.sgd_update_multi(ptrs, ptrs, nul, cnt, 2, f(0.1), f(0), f(0), f(1), None) == b.ERR_INVALID_ARG
    assert lib.sgd_update_multi(ptrs, ptrs, ptrs, neg, 2, f(0.1), f(0), f(0), f(1), None) == b.ERR_INVALID_ARG
    assert lib.sgd_update_multi(ptrs, odd, ptrs, cnt, 2, f(0.1), f(0), f(0), f(1), None) == b.ERR_MISALIGNED
    assert lib.sgd_update_multi(None, None, None, None, 0, f(0.1), f(0), f(0), f(1), None) == b.OK
