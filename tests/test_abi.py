"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2510_10467_amd import build as hip_build
    if hip_build.is_stale():
        hip_build.build()
    import paper_2510_10467_amd as bcq
    return bcq.lib()


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(bcq_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"bcq_pack", "bcq_unpack", "bcq_gemv", "bcq_gemm_mixed", "bcq_gemv_offset", "bcq_gemm_mixed_offset", "bcq_gemv_multi",
            "bcq_quantize", "bcq_bench_stream_read", "bcq_bench_fp16_gemv", "bcq_bench_issue_probe", "bcq_strerror", "bcq_select_kernel", "bcq_select_dequant_shape", "bcq_last_kernel"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"


def test_strerror_covers_all_codes(lib):
    seen = set()
    for code in range(0, -7, -1):
        msg = lib.bcq_strerror(code).decode()
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 7
    assert lib.bcq_strerror(-99).decode() == "unknown status"


def test_argument_validation_without_device(lib):
    # pointers are never dereferenced on an error path, so fake aligned addresses are enough
    P, S, X, Y = 0x1000, 0x2000, 0x3000, 0x4000
    gemv = lib.bcq_gemv
    assert gemv(None, S, 2, X, Y, 16, 128, 1, 128, None) == -1
    assert gemv(P, S, 0, X, Y, 16, 128, 1, 128, None) == -2
    assert gemv(P, S, 9, X, Y, 16, 128, 1, 128, None) == -2
    assert gemv(P, S, 2, X, Y, 0, 128, 1, 128, None) == -3
    assert gemv(P, S, 2, X, Y, 16, 192, 1, 128, None) == -3      # n % group != 0
    assert gemv(P, S, 2, X, Y, 16, 128, 1, 48, None) == -3       # group % 32 != 0
    assert gemv(P, S, 2, X, Y, 16, 64, 1, 128, None) == -3       # n < group
    assert gemv(P, S, 2, X, Y, 16, 128, -1, 128, None) == -3
    assert gemv(P + 4, S, 2, X, Y, 16, 128, 1, 128, None) == -4
    assert gemv(P, S, 2, X + 2, Y, 16, 128, 1, 128, None) == -4
    assert gemv(P, S, 2, X, Y + 1, 16, 128, 1, 128, None) == -4
    assert gemv(P, S, 2, X, Y, 16, 128, 0, 128, None) == 0       # empty batch: no-op
    ptrs = (ctypes.c_void_p * 5)(None, None, S, None, None)
    mixed = lib.bcq_gemm_mixed
    assert mixed(P, ptrs, None, 4, X, Y, 16, 128, 1, 128, None) == -1
    assert mixed(P, ptrs, 0x5000, 0, X, Y, 16, 128, 1, 128, None) == -2
    assert mixed(P, ptrs, 0x5000, 4, X, Y, 16, 100, 1, 128, None) == -3
    assert mixed(P, ptrs, 0x5000, 4, X, Y, 16, 128, 0, 128, None) == 0
    none = (ctypes.c_void_p * 5)()
    assert mixed(P, none, 0x5000, 4, X, Y, 16, 128, 1, 128, None) == -1
    # asymmetric entry points: same checks, the offset set may be absent but not misaligned
    Z = 0x6000
    goff = lib.bcq_gemv_offset
    assert goff(P, None, Z, 2, X, Y, 16, 128, 1, 128, None) == -1
    assert goff(P, S, Z, 9, X, Y, 16, 128, 1, 128, None) == -2
    assert goff(P, S, Z, 2, X, Y, 16, 192, 1, 128, None) == -3
    assert goff(P, S, Z + 2, 2, X, Y, 16, 128, 1, 128, None) == -4
    assert goff(P, S, Z, 2, X, Y, 16, 128, 0, 128, None) == 0
    assert goff(P, S, None, 2, X, Y, 16, 128, 0, 128, None) == 0
    moff = lib.bcq_gemm_mixed_offset
    zptrs = (ctypes.c_void_p * 5)(None, None, Z, None, None)
    assert moff(P, ptrs, zptrs, None, 4, X, Y, 16, 128, 1, 128, None) == -1
    assert moff(P, ptrs, zptrs, 0x5000, 4, X, Y, 16, 128, 0, 128, None) == 0
    assert moff(P, ptrs, None, 0x5000, 4, X, Y, 16, 128, 0, 128, None) == 0
    bad = (ctypes.c_void_p * 5)(None, None, Z + 8, None, None)
    assert moff(P, ptrs, bad, 0x5000, 4, X, Y, 16, 128, 1, 128, None) == -4
    # several matrices in one call
    multi = lib.bcq_gemv_multi
    pp = (ctypes.c_void_p * 2)(P, P + 0x100)
    sp = (ctypes.c_void_p * 2)(S, S + 0x100)
    yp = (ctypes.c_void_p * 2)(Y, Y + 0x100)
    mm = (ctypes.c_int64 * 2)(16, 32)
    assert multi(0, pp, sp, mm, yp, 2, X, 128, 1, 128, None) == -3
    assert multi(5, pp, sp, mm, yp, 2, X, 128, 1, 128, None) == -3
    assert multi(2, None, sp, mm, yp, 2, X, 128, 1, 128, None) == -1
    assert multi(2, pp, sp, mm, yp, 0, X, 128, 1, 128, None) == -2
    assert multi(2, pp, sp, mm, yp, 2, X, 192, 1, 128, None) == -3
    assert multi(2, pp, sp, (ctypes.c_int64 * 2)(16, 0), yp, 2, X, 128, 1, 128, None) == -3
    assert multi(2, (ctypes.c_void_p * 2)(P, None), sp, mm, yp, 2, X, 128, 1, 128, None) == -1
    assert multi(2, (ctypes.c_void_p * 2)(P, P + 4), sp, mm, yp, 2, X, 128, 1, 128, None) == -4
    assert multi(2, pp, sp, mm, yp, 2, X, 128, 0, 128, None) == 0
    # the quantiser
    quant = lib.bcq_quantize
    W = 0x7000
    sets = (ctypes.c_void_p * 5)(None, None, S, S + 0x100, S + 0x200)
    assert quant(None, 2, 4, 20, P, sets, None, 16, 128, 128, None) == -1
    assert quant(W, 2, 4, 20, P, None, None, 16, 128, 128, None) == -1
    assert quant(W, 0, 4, 20, P, sets, None, 16, 128, 128, None) == -2
    assert quant(W, 3, 2, 20, P, sets, None, 16, 128, 128, None) == -2
    assert quant(W, 2, 5, 20, P, sets, None, 16, 128, 128, None) == -2
    assert quant(W, 2, 4, 0, P, sets, None, 16, 128, 128, None) == -2       # expansion needs a cycle
    assert quant(W, 2, 2, -1, P, sets, None, 16, 128, 128, None) == -2
    assert quant(W, 2, 4, 20, P, sets, None, 16, 192, 128, None) == -3
    assert quant(W, 2, 4, 20, P, sets, None, 16, 192, 96, None) == -3       # group not 32/64/128/256
    assert quant(W, 2, 4, 20, P, sets, None, 0, 128, 128, None) == -3
    assert quant(W + 2, 2, 4, 20, P, sets, None, 16, 128, 128, None) == -4
    assert quant(W, 2, 4, 20, P, (ctypes.c_void_p * 5)(None, None, S, None, S), None, 16, 128, 128, None) == -1
    assert quant(W, 2, 4, 20, P, sets, (ctypes.c_void_p * 5)(None, None, Z, Z, None), 16, 128, 128, None) == -1
    assert quant(W, 2, 4, 20, P, (ctypes.c_void_p * 5)(None, None, S + 1, S, S), None, 16, 128, 128, None) == -4
    # benchmark reference kernels
    assert lib.bcq_bench_stream_read(None, 1024, 0x2000, None) == -1
    assert lib.bcq_bench_stream_read(0x1000, 1000, 0x2000, None) == -3
    assert lib.bcq_bench_stream_read(0x1008, 1024, 0x2000, None) == -3
    assert lib.bcq_bench_fp16_gemv(0x1000, 0x2000, None, 4, 64, None) == -1
    assert lib.bcq_bench_fp16_gemv(0x1000, 0x2000, 0x3000, 4, 60, None) == -3
    assert lib.bcq_bench_fp16_gemv(0x1002, 0x2000, 0x3000, 4, 64, None) == -4
    assert lib.bcq_bench_issue_probe(0, 8, 4, 100, None, 0x2000, None) == -1
    assert lib.bcq_bench_issue_probe(0, 8, 17, 100, 0x1000, 0x2000, None) == -3
    assert lib.bcq_bench_issue_probe(3, 8, 4, 100, 0x1000, 0x2000, None) == -3
    assert lib.bcq_bench_issue_probe(0, 5, 4, 100, 0x1000, 0x2000, None) == -3
    assert lib.bcq_pack(0x1000, 0x2000, 4, 8, 48, None) == -3
    assert lib.bcq_pack(0x1000, 0x2000, 0, 8, 64, None) == -2
    assert lib.bcq_unpack(None, 0x2000, 4, 8, 64, None) == -1
    assert lib.bcq_select_dequant_shape(3, 4) == -6
    assert lib.bcq_select_dequant_shape(2, 2) == 0
    assert lib.bcq_select_dequant_shape(0, 4) == 0
    assert lib.bcq_select_dequant_shape(32, 2) == 0
    assert lib.bcq_select_dequant_shape(0, 8) == 0
    assert lib.bcq_select_dequant_shape(1, 8) == -6
    assert lib.bcq_select_dequant_shape(4, 40) == 0
    assert lib.bcq_select_dequant_shape(4, 8) == 0
    assert lib.bcq_select_dequant_shape(2, 8) == 0
    assert lib.bcq_select_dequant_shape(2, 40) == -6
    assert lib.bcq_select_dequant_shape(16, 2) == -6
    assert lib.bcq_select_dequant_shape(0, 3) == -6
    assert lib.bcq_select_dequant_shape(-1, 4) == -6
    assert lib.bcq_select_dequant_shape(0, 0) == 0
    assert lib.bcq_select_kernel(17) == -6
    assert lib.bcq_select_kernel(5) == 0            # the table look-up kernel is the last variant
    assert lib.bcq_select_kernel(6) == -6
    assert lib.bcq_select_kernel(0) == 0


def test_binding_refuses_cpu_tensors():
    import torch

    import paper_2510_10467_amd as bcq
    planes = torch.zeros((2, 4, 4), dtype=torch.int32)
    scales = torch.zeros((2, 4, 1), dtype=torch.float16)
    x = torch.zeros((1, 128), dtype=torch.float16)
    with pytest.raises(TypeError):
        bcq.bcq_gemv(planes, scales, 2, x)


def test_test_knobs_are_per_thread(lib):
    """One thread forcing a kernel variant or a workgroup shape leaves the other threads' dispatch alone."""
    import threading
    lib.bcq_selected_kernel.restype = ctypes.c_int
    assert lib.bcq_select_kernel(0) == 0
    seen = {}
    forced = threading.Event()
    checked = threading.Event()

    def forcing():
        assert lib.bcq_select_kernel(2) == 0
        seen["forcing"] = lib.bcq_selected_kernel()
        forced.set()
        checked.wait(10)
        seen["forcing_after"] = lib.bcq_selected_kernel()

    def watching():
        forced.wait(10)
        seen["watching"] = lib.bcq_selected_kernel()
        seen["watching_last"] = lib.bcq_last_kernel()
        checked.set()

    threads = [threading.Thread(target=forcing), threading.Thread(target=watching)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(20)
    assert seen["forcing"] == 2 and seen["forcing_after"] == 2
    assert seen["watching"] == 0, "a variant forced by one thread changed another thread's choice"
    assert lib.bcq_selected_kernel() == 0


def test_pack_rejects_what_one_grid_cannot_hold(lib):
    """More plane words than 2^31 - 1 workgroups of 256 threads cover: an error before any launch."""
    C, P = 0x1000, 0x2000
    assert lib.bcq_pack(C, P, 4, ctypes.c_int64(1 << 33), ctypes.c_int64(4096), None) == -3
    assert lib.bcq_unpack(P, C, 8, ctypes.c_int64(1 << 36), ctypes.c_int64(32), None) == -3
    assert lib.bcq_pack(C, P, 1, ctypes.c_int64(1 << 41), ctypes.c_int64(32), None) == -3
