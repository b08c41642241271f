"""Host-side checks of the C ABI (no GPU needed): the library loads, exports every symbol the header
declares, and every argument error is reported before any device is touched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2210_03858_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_library()
    return binding.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "bcq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bcq_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = _declared_functions()
    assert {"bcq_quantize", "bcq_pack", "bcq_unpack", "bcq_linear_fwd", "bcq_linear_bwd_input",
            "bcq_linear_bwd_alpha", "bcq_workspace_bytes", "bcq_status_string"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    from paper_2210_03858_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_status_strings(lib):
    seen = set()
    for code in range(8):
        s = lib.bcq_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert lib.bcq_abi_version() >= 2


A = 0x1000  # a fake, aligned, never dereferenced pointer


def test_workspace_bytes_validation(lib):
    out = ctypes.c_size_t(123)
    assert lib.bcq_workspace_bytes(1, 8, 64, 64, 3, 1, None) == 1
    assert lib.bcq_workspace_bytes(9, 8, 64, 64, 3, 1, ctypes.byref(out)) == 3
    assert lib.bcq_workspace_bytes(1, 8, 64, 48, 3, 1, ctypes.byref(out)) == 2
    assert lib.bcq_workspace_bytes(1, 8, 64, 64, 9, 1, ctypes.byref(out)) == 2
    assert lib.bcq_workspace_bytes(1, 8, 64, 64, 3, 7, ctypes.byref(out)) == 3
    assert lib.bcq_workspace_bytes(0, 0, 64, 64, 3, 0, ctypes.byref(out)) == 0  # T ignored for quantize
    assert out.value >= 16


def test_argument_errors_before_device(lib):
    q, N, K, T = 3, 64, 64, 8
    # NULL
    assert lib.bcq_quantize(None, N, K, q, A, A, None, None, 0, None) == 1
    assert lib.bcq_pack(None, N, K, q, A, None) == 1
    assert lib.bcq_unpack(A, N, K, q, None, None) == 1
    assert lib.bcq_pack_transposed(A, N, K, q, None, None) == 1
    assert lib.bcq_linear_fwd(A, None, A, 1, T, N, K, q, A, None, 0, None) == 1
    assert lib.bcq_linear_bwd_input(A, None, A, None, 1, T, N, K, q, A, None, 0, None) == 1
    assert lib.bcq_linear_bwd_alpha(A, A, A, 1, T, N, K, q, q, 1.0, None, None, 0, None) == 1
    # shape
    assert lib.bcq_quantize(A, N, 40, q, A, A, None, None, 0, None) == 2
    assert lib.bcq_quantize(A, N, 16384 + 32, q, A, A, None, None, 0, None) == 2
    assert lib.bcq_pack(A, 0, K, q, A, None) == 2
    assert lib.bcq_linear_fwd(A, A, A, 1, 0, N, K, q, A, None, 0, None) == 2
    assert lib.bcq_linear_fwd(A, A, A, 1, T, N, K, 0, A, None, 0, None) == 2
    assert lib.bcq_linear_bwd_input(A, A, A, A, 1, T, 48, K, q, A, None, 0, None) == 2  # twin needs N % 32 == 0
    assert lib.bcq_pack_transposed(A, 48, K, q, A, None) == 2
    assert lib.bcq_linear_bwd_alpha(A, A, A, 1, T, N, K, q, q + 1, 1.0, A, None, 0, None) == 2
    assert lib.bcq_linear_bwd_alpha(A, A, A, 1, T, N, K, q, 0, 1.0, A, None, 0, None) == 2
    # dtype
    assert lib.bcq_linear_fwd(A, A, A, 2, T, N, K, q, A, None, 0, None) == 3
    assert lib.bcq_linear_bwd_input(A, None, A, A, -1, T, N, K, q, A, None, 0, None) == 3
    # alignment
    assert lib.bcq_linear_fwd(A + 4, A, A, 1, T, N, K, q, A, None, 0, None) == 4
    assert lib.bcq_linear_fwd(A, A, A, 1, T, N, K, q, A, A + 8, 1 << 20, None) == 4
    assert lib.bcq_quantize(A, N, K, q, A, A, A + 1, None, 0, None) == 4
    # workspace too small
    assert lib.bcq_quantize(A, N, K, q, A, A, None, A, 4, None) == 5


def test_group_size_errors_before_device(lib):
    """g must be a multiple of 32 in [32, K] that divides K; everything else is as for the row-wise calls."""
    q, N, K, T = 3, 64, 192, 8
    out = ctypes.c_size_t(0)
    i64 = ctypes.c_int64
    for g in (0, 16, 48, 128, 384, -64):
        assert lib.bcq_workspace_bytes_grouped(1, T, N, K, i64(g), q, 1, ctypes.byref(out)) == 2, g
        assert lib.bcq_quantize_grouped(A, N, K, i64(g), q, A, A, None, None, 0, None) == 2, g
        assert lib.bcq_linear_fwd_grouped(A, A, A, 1, T, N, K, i64(g), q, A, None, 0, None) == 2, g
        assert lib.bcq_linear_bwd_input_grouped(A, None, A, A, 1, T, N, K, i64(g), q, A, None, 0, None) == 2, g
        assert lib.bcq_linear_bwd_alpha_grouped(A, A, A, 1, T, N, K, i64(g), q, q, 1.0, A, None, 0, None) == 2, g
    for g in (32, 64, 96, 192):
        assert lib.bcq_workspace_bytes_grouped(3, 64, N, K, i64(g), q, 1, ctypes.byref(out)) == 0, g
    assert lib.bcq_linear_fwd_grouped(None, A, A, 1, T, N, K, i64(64), q, A, None, 0, None) == 1
    assert lib.bcq_linear_bwd_alpha_grouped(A, A, A, 1, T, N, K, i64(64), q, q + 1, 1.0, A, None, 0, None) == 2
    assert lib.bcq_linear_fwd_grouped(A, A + 4, A, 1, T, N, K, i64(64), q, A, None, 0, None) == 4
    # a group-wise dalpha workspace with per-32-column partials is larger than the row-wise one
    rw, gw = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert lib.bcq_workspace_bytes(3, 512, 256, 512, q, 1, ctypes.byref(rw)) == 0
    assert lib.bcq_workspace_bytes_grouped(3, 512, 256, 512, i64(64), q, 1, ctypes.byref(gw)) == 0
    assert gw.value > rw.value


def test_decode_layout_errors_before_device(lib):
    q, N, K, T = 3, 100, 1056, 8
    i64 = ctypes.c_int64
    out = ctypes.c_size_t(0)
    assert lib.bcq_decode_layout_bytes(N, K, q, ctypes.byref(out)) == 0
    assert out.value == 7 * 3 * q * 1024  # ceil(100 / 16) row tiles x ceil(1056 / 512) segments x q KiB
    assert lib.bcq_decode_layout_bytes(N, 40, q, ctypes.byref(out)) == 2
    assert lib.bcq_decode_layout_bytes(N, K, q, None) == 1
    assert lib.bcq_pack_decode(A, N, K, q, None, None) == 1
    assert lib.bcq_pack_decode(A, N, K, 9, A, None) == 2
    assert lib.bcq_pack_decode(A + 4, N, K, q, A, None) == 4
    ws = 1 << 24
    assert lib.bcq_linear_fwd_decode(A, A, A, 1, T, N, K, i64(K), q, A, None, 0, None) == 1       # workspace required
    assert lib.bcq_linear_fwd_decode(A, A, A, 0, T, N, K, i64(K), q, A, A, ws, None) == 3         # bf16 only
    assert lib.bcq_linear_fwd_decode(A, A, A, 1, 81, N, K, i64(K), q, A, A, ws, None) == 2        # at most 80 tokens
    assert lib.bcq_linear_fwd_decode(A, A, A, 1, T, N, K, i64(96), q, A, A, ws, None) == 2        # g % 512 != 0
    assert lib.bcq_linear_fwd_decode(A, A, A, 1, T, N, K, i64(K), q, A, A, 16, None) == 5         # workspace too small
    assert lib.bcq_linear_fwd_decode(A, A, A + 2, 1, T, N, K, i64(K), q, A, A, ws, None) == 4


def test_fwd_lut_errors_before_device(lib):
    q, N, K, T = 3, 64, 1024, 2
    assert lib.bcq_linear_fwd_lut(A, A, A, 1, T, N, K, q, None, None) == 1
    assert lib.bcq_linear_fwd_lut(A, A, A, 1, 5, N, K, q, A, None) == 2          # at most 4 tokens
    assert lib.bcq_linear_fwd_lut(A, A, A, 1, 4, N, 4096 + 32, q, A, None) == 2  # tables beyond 128 KiB of LDS
    assert lib.bcq_linear_fwd_lut(A, A, A, 1, 1, N, 16384 + 32, q, A, None) == 2
    assert lib.bcq_linear_fwd_lut(A, A, A, 1, T, N, 1000, q, A, None) == 2
    assert lib.bcq_linear_fwd_lut(A, A, A, 0, T, N, K, q, A, None) == 3          # bf16 only
    assert lib.bcq_linear_fwd_lut(A, A, A + 4, 1, T, N, K, q, A, None) == 4
    import torch
    if not torch.cuda.is_available():
        assert lib.bcq_linear_fwd_lut(A, A, A, 1, 1, N, 16384, q, A, None) == 7   # fits; no device here


def test_fwd_static_errors_before_device(lib):
    q, N, K, T = 3, 64, 1024, 8
    assert lib.bcq_linear_fwd_static(A, A, A, 1, T, N, K, q, None, None) == 1
    assert lib.bcq_linear_fwd_static(A, A, A, 1, 81, N, K, q, A, None) == 2       # at most 80 tokens
    assert lib.bcq_linear_fwd_static(A, A, A, 1, T, N, 1000, q, A, None) == 2
    assert lib.bcq_linear_fwd_static(A, A, A, 0, T, N, K, q, A, None) == 3        # bf16 only
    assert lib.bcq_linear_fwd_static(A, A + 8, A, 1, T, N, K, q, A, None) == 4
    assert lib.bcq_linear_fwd_static(A, A, A, 1, 80, N, 12800, q, A, None) == 5   # 2112000 bytes of scratch > 2 MiB
    assert lib.bcq_linear_fwd_static(A, A, A, 1, 16, N, 63488 + 512, q, A, None) == 5
    import torch
    if not torch.cuda.is_available():
        assert lib.bcq_linear_fwd_static(A, A, A, 1, 80, N, 12288, q, A, None) == 7  # fits; no device here


def test_batch_plan_errors_and_layout_before_device(lib):
    from paper_2210_03858_amd.binding import BatchLayer
    sz = ctypes.c_size_t
    tb, wb = sz(0), sz(0)
    L = (BatchLayer * 2)()
    for l, (N, K) in zip(L, ((2560, 2560), (1280, 5120))):
        l.tiled = l.tiled_t = l.alpha = l.x = l.dy = l.y = l.dx = l.dalpha = A
        l.N, l.K = N, K
    T, q = 8, 4
    assert lib.bcq_batch_sizes(1, L, 2, T, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 0
    # plan: 128-byte header + 128 bytes per layer + 8 bytes per pre-kernel block (5 + 10 segments) + 16 bytes per piece
    # (the piece size is chosen per batch; 160 + 80 row tiles give between 2 and 60 pieces), rounded up to 256;
    # workspace: (4 x 2048 + 256) bytes per segment at up to 8 tokens
    fixed = 128 + 2 * 128 + 8 * 15
    assert tb.value % 256 == 0 and fixed + 16 * 2 <= tb.value <= fixed + 16 * 60 + 255
    assert wb.value == 15 * (4 * 2048 + 256)
    assert lib.bcq_batch_sizes(2, L, 2, 16, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 0
    assert wb.value == q * 2 * (5 + 3) * (4 * 2048 + 256)  # one set per plane, two operand halves, N / 512 rounded up
    assert lib.bcq_batch_sizes(1, None, 2, T, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 1
    assert lib.bcq_batch_sizes(1, L, 2, T, q, q, 1, None, ctypes.byref(wb)) == 1
    assert lib.bcq_batch_sizes(0, L, 2, T, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 3     # not a batched op
    assert lib.bcq_batch_sizes(1, L, 0, T, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 2
    assert lib.bcq_batch_sizes(1, L, 2, 17, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 2    # at most 16 tokens
    assert lib.bcq_batch_sizes(1, L, 2, T, 5, 5, 1, ctypes.byref(tb), ctypes.byref(wb)) == 2     # at most 4 planes
    assert lib.bcq_batch_sizes(1, L, 2, T, q, q, 0, ctypes.byref(tb), ctypes.byref(wb)) == 3     # bf16 only
    L[1].K = 5120 + 16
    assert lib.bcq_batch_sizes(1, L, 2, T, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 2  # K % 32 != 0
    L[1].K, L[1].N = 5120, 1280 + 16
    assert lib.bcq_batch_sizes(1, L, 2, T, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 0
    assert lib.bcq_batch_sizes(2, L, 2, T, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 2  # dx: the twin needs N % 32 == 0
    assert lib.bcq_batch_sizes(3, L, 2, T, q, 0, 1, ctypes.byref(tb), ctypes.byref(wb)) == 2  # q_train outside [1, q]
    L[1].N = 1280
    assert lib.bcq_batch_sizes(1, L, 2, T, q, q, 1, ctypes.byref(tb), ctypes.byref(wb)) == 0
    buf = ctypes.create_string_buffer(tb.value)
    assert lib.bcq_batch_plan(1, L, 2, T, q, q, 1.0, 1, buf, tb.value - 1) == 5
    assert lib.bcq_batch_plan(1, L, 2, T, q, q, 1.0, 1, None, tb.value) == 1
    assert lib.bcq_batch_plan(3, L, 2, T, q, 0, 1.0, 1, buf, tb.value) == 2                   # q_train outside [1, q]
    L[0].y = None
    assert lib.bcq_batch_plan(1, L, 2, T, q, q, 1.0, 1, buf, tb.value) == 1
    assert lib.bcq_batch_plan(3, L, 2, T, q, q, 1.0, 1, buf, tb.value) == 0                   # dalpha does not read y
    L[0].y = A + 4
    assert lib.bcq_batch_plan(1, L, 2, T, q, q, 1.0, 1, buf, tb.value) == 4
    L[0].y = A
    assert lib.bcq_batch_plan(1, L, 2, T, q, q, 1.0, 1, buf, tb.value) == 0
    # run: checks that need no device come first
    assert lib.bcq_linear_batched(buf, None, tb.value, A, 1 << 30, None) == 1
    assert lib.bcq_linear_batched(buf, A, tb.value, A, 16, None) == 5                          # workspace too small
    assert lib.bcq_linear_batched(buf, A + 8, tb.value, A, 1 << 30, None) == 4
    junk = ctypes.create_string_buffer(tb.value)
    assert lib.bcq_linear_batched(junk, A, tb.value, A, 1 << 30, None) == 3                    # not a plan
    import torch
    if not torch.cuda.is_available():
        assert lib.bcq_linear_batched(buf, A, tb.value, A, 1 << 30, None) == 7


def test_prepare_errors_before_device(lib):
    i64 = ctypes.c_int64
    assert lib.bcq_prepare(9, 8, 64, 64, i64(64), 3, 1) == 3
    assert lib.bcq_prepare(1, 8, 64, 48, i64(48), 3, 1) == 2
    assert lib.bcq_prepare(1, 8, 64, 64, i64(48), 3, 1) == 2      # group size must divide K
    assert lib.bcq_prepare(1, 8, 64, 64, i64(64), 3, 5) == 3
    assert lib.bcq_batch_prepare(None, 1024) == 1
    junk = ctypes.create_string_buffer(1024)
    assert lib.bcq_batch_prepare(junk, 1024) == 3                  # not a plan
    import torch
    if not torch.cuda.is_available():
        assert lib.bcq_prepare(1, 8, 64, 64, i64(64), 3, 1) == 7


def test_no_device_is_reported(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    assert lib.bcq_linear_fwd(A, A, A, 1, 8, 64, 64, 3, A, None, 0, None) == 7


def test_binding_fails_loudly_without_library(monkeypatch):
    from paper_2210_03858_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libbcq_hip.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: --gpus 2 must exit with a message before anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
