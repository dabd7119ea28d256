"""ctypes binding of the C ABI in ``include/bcq.h``.

Argument marshalling only: every step of the product runs in the HIP kernels.
PyTorch supplies device memory and the current stream.  There is no CPU
fallback: if the shared library is missing the import of this module's
functions raises, and every call checks that its tensors live on the GPU.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbcq_hip.so")
_lib = None

BCQ_MAX_PLANES = 8
KERNEL_AUTO, KERNEL_SIGN_SELECT, KERNEL_PLANE_MFMA, KERNEL_DEQUANT_MFMA = 0, 1, 2, 3
KERNEL_IDS = {"auto": 0, "sign_select": 1, "plane_mfma": 2, "dequant_mfma": 3, "plane_f16": 4, "lut": 5}


class BcqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().bcq_strerror(status).decode()} (status {status})")


def lib() -> ctypes.CDLL:
    """Load ``libbcq_hip.so`` (built in-tree by ``build.py``); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                "or `python paper_2510_10467_amd/build.py`")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.bcq_strerror.restype = ctypes.c_char_p
        L.bcq_strerror.argtypes = [i32]
        L.bcq_select_kernel.argtypes = [i32]
        L.bcq_select_dequant_shape.argtypes = [i32, i32]
        L.bcq_select_dequant_shape.restype = i32
        L.bcq_last_kernel.restype = ctypes.c_char_p
        L.bcq_pack.argtypes = [vp, vp, i32, i64, i64, vp]
        L.bcq_unpack.argtypes = [vp, vp, i32, i64, i64, vp]
        L.bcq_gemv.argtypes = [vp, vp, i32, vp, vp, i64, i64, i32, i32, vp]
        L.bcq_gemm_mixed.argtypes = [vp, vp, vp, i32, vp, vp, i64, i64, i32, i32, vp]
        L.bcq_gemv_multi.argtypes = [i32, vp, vp, vp, vp, i32, vp, i64, i32, i32, vp]
        L.bcq_gemv_multi.restype = i32
        L.bcq_gemv_offset.argtypes = [vp, vp, vp, i32, vp, vp, i64, i64, i32, i32, vp]
        L.bcq_gemm_mixed_offset.argtypes = [vp, vp, vp, vp, i32, vp, vp, i64, i64, i32, i32, vp]
        L.bcq_quantize.argtypes = [vp, i32, i32, i32, vp, vp, vp, i64, i64, i32, vp]
        L.bcq_quantize.restype = i32
        L.bcq_quantize_form.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, i64, i64, i32, vp]
        L.bcq_quantize_form.restype = i32
        L.bcq_bench_stream_read.argtypes = [vp, i64, vp, vp]
        L.bcq_bench_stream_read.restype = i32
        L.bcq_bench_fp16_gemv.argtypes = [vp, vp, vp, i64, i64, vp]
        L.bcq_bench_fp16_gemv.restype = i32
        L.bcq_bench_issue_probe.argtypes = [i32, i32, i32, i32, vp, vp, vp]
        L.bcq_bench_issue_probe.restype = i32
        for f in (L.bcq_select_kernel, L.bcq_pack, L.bcq_unpack, L.bcq_gemv, L.bcq_gemm_mixed, L.bcq_gemv_offset,
                  L.bcq_gemm_mixed_offset):
            f.restype = i32
        _lib = L
    return _lib


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor (there is no CPU path)")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise BcqError(status, where)


def select_kernel(variant) -> None:
    """Force a kernel variant by name or id ('auto' restores the default choice)."""
    vid = KERNEL_IDS[variant] if isinstance(variant, str) else int(variant)
    _check(lib().bcq_select_kernel(vid), "bcq_select_kernel")


def select_dequant_shape(request_tiles: int = 0, row_blocks: int = 0) -> None:
    """Benchmarks and tests: force the workgroup shape of the large-batch kernel ((0, 0) = automatic)."""
    _check(lib().bcq_select_dequant_shape(int(request_tiles), int(row_blocks)), "bcq_select_dequant_shape")


def last_kernel() -> str:
    return lib().bcq_last_kernel().decode()


def bcq_pack(codes: torch.Tensor, planes: torch.Tensor | None = None) -> torch.Tensor:
    """int8 codes [P][m][n] (>0 is +1) -> int32-typed planes [P][m][n/32] holding the uint32 words."""
    P, m, n = codes.shape
    if planes is None:
        planes = torch.empty((P, m, n // 32), dtype=torch.int32, device=codes.device)
    _check(lib().bcq_pack(_dev(codes, torch.int8, "codes"), _dev(planes, torch.int32, "planes"), P, m, n, _stream()),
           "bcq_pack")
    return planes


def bcq_unpack(planes: torch.Tensor, codes: torch.Tensor | None = None) -> torch.Tensor:
    """planes [P][m][n/32] -> int8 codes [P][m][n] in {-1,+1}."""
    P, m, words = planes.shape
    if codes is None:
        codes = torch.empty((P, m, words * 32), dtype=torch.int8, device=planes.device)
    _check(lib().bcq_unpack(_dev(planes, torch.int32, "planes"), _dev(codes, torch.int8, "codes"), P, m, words * 32,
                            _stream()), "bcq_unpack")
    return codes


def bcq_gemv(planes: torch.Tensor, scales_p: torch.Tensor, p: int, x: torch.Tensor,
             y: torch.Tensor | None = None, group: int = 128, offsets: torch.Tensor | None = None) -> torch.Tensor:
    """Uniform precision: y[b][r] = sum_{i<p} sum_j scales_p[i][r][j/group] * B_i[r][j] * x[b][j];
    with ``offsets`` (float16 [m][n/group], asymmetric scheme) plus sum_j offsets[r][j/group] * x[b][j]."""
    _, m, words = planes.shape
    n = words * 32
    batch = x.shape[0]
    if x.shape != (batch, n) or scales_p.shape != (p, m, n // group) or planes.shape[0] < p:
        raise ValueError("bcq_gemv: inconsistent shapes")
    if y is None:
        y = torch.empty((batch, m), dtype=torch.float16, device=x.device)
    elif y.shape != (batch, m):
        raise ValueError("bcq_gemv: y has the wrong shape")
    if offsets is not None:
        if offsets.shape != (m, n // group):
            raise ValueError("bcq_gemv: offsets have the wrong shape")
        _check(lib().bcq_gemv_offset(_dev(planes, torch.int32, "planes"), _dev(scales_p, torch.float16, "scales_p"),
                                     _dev(offsets, torch.float16, "offsets"), p, _dev(x, torch.float16, "x"),
                                     _dev(y, torch.float16, "y"), m, n, batch, group, _stream()), "bcq_gemv_offset")
        return y
    _check(lib().bcq_gemv(_dev(planes, torch.int32, "planes"), _dev(scales_p, torch.float16, "scales_p"), p,
                          _dev(x, torch.float16, "x"), _dev(y, torch.float16, "y"), m, n, batch, group, _stream()),
           "bcq_gemv")
    return y


def bcq_gemv_multi(planes: list, scales_p: list, p: int, x: torch.Tensor, ys: list | None = None, group: int = 128) -> list:
    """Several matrices (same n and precision) applied to the same activations in one call: the q/k/v or
    gate/up projections of a decoder layer.  Returns the list of outputs (those of bcq_gemv within the tolerance both are held
    to; bit for bit wherever the same kernel form serves both)."""
    count = len(planes)
    batch, n = x.shape
    if len(scales_p) != count or (ys is not None and len(ys) != count):
        raise ValueError("bcq_gemv_multi: lists of different lengths")
    ms = []
    for k in range(count):
        _, m, words = planes[k].shape
        if words * 32 != n or scales_p[k].shape != (p, m, n // group) or planes[k].shape[0] < p:
            raise ValueError(f"bcq_gemv_multi: inconsistent shapes for matrix {k}")
        ms.append(m)
    if ys is None:
        ys = [torch.empty((batch, m), dtype=torch.float16, device=x.device) for m in ms]
    pp = (ctypes.c_void_p * count)(*[_dev(t, torch.int32, f"planes[{k}]") for k, t in enumerate(planes)])
    sp = (ctypes.c_void_p * count)(*[_dev(t, torch.float16, f"scales_p[{k}]") for k, t in enumerate(scales_p)])
    yp = (ctypes.c_void_p * count)(*[_dev(t, torch.float16, f"ys[{k}]") for k, t in enumerate(ys)])
    mp = (ctypes.c_int64 * count)(*ms)
    for k in range(count):
        if ys[k].shape != (batch, ms[k]):
            raise ValueError(f"bcq_gemv_multi: ys[{k}] has the wrong shape")
    _check(lib().bcq_gemv_multi(count, ctypes.cast(pp, ctypes.c_void_p), ctypes.cast(sp, ctypes.c_void_p),
                                ctypes.cast(mp, ctypes.c_void_p), ctypes.cast(yp, ctypes.c_void_p), p,
                                _dev(x, torch.float16, "x"), n, batch, group, _stream()), "bcq_gemv_multi")
    return ys


def bcq_gemm_mixed(planes: torch.Tensor, scales_by_p: dict, p_req: torch.Tensor, x: torch.Tensor,
                   y: torch.Tensor | None = None, group: int = 128, offsets_by_p: dict | None = None) -> torch.Tensor:
    """Per-request precision: request b uses planes 0..p_req[b]-1 and scale set scales_by_p[p_req[b]]
    (and the offset set offsets_by_p[p_req[b]] if there is one)."""
    p_max, m, words = planes.shape
    n = words * 32
    batch = x.shape[0]
    if x.shape != (batch, n) or p_req.shape != (batch,):
        raise ValueError("bcq_gemm_mixed: inconsistent shapes")
    ptrs = (ctypes.c_void_p * (p_max + 1))()
    for q, s in scales_by_p.items():
        if not 1 <= q <= p_max or s.shape != (q, m, n // group):
            raise ValueError(f"bcq_gemm_mixed: bad scale set for precision {q}")
        ptrs[q] = _dev(s, torch.float16, f"scales_by_p[{q}]")
    if y is None:
        y = torch.empty((batch, m), dtype=torch.float16, device=x.device)
    elif y.shape != (batch, m):
        raise ValueError("bcq_gemm_mixed: y has the wrong shape")
    if offsets_by_p:
        optrs = (ctypes.c_void_p * (p_max + 1))()
        for q, z in offsets_by_p.items():
            if not 1 <= q <= p_max or z.shape != (m, n // group):
                raise ValueError(f"bcq_gemm_mixed: bad offset set for precision {q}")
            optrs[q] = _dev(z, torch.float16, f"offsets_by_p[{q}]")
        _check(lib().bcq_gemm_mixed_offset(_dev(planes, torch.int32, "planes"), ctypes.cast(ptrs, ctypes.c_void_p),
                                           ctypes.cast(optrs, ctypes.c_void_p), _dev(p_req, torch.int32, "p_req"), p_max,
                                           _dev(x, torch.float16, "x"), _dev(y, torch.float16, "y"), m, n, batch, group,
                                           _stream()), "bcq_gemm_mixed_offset")
        return y
    _check(lib().bcq_gemm_mixed(_dev(planes, torch.int32, "planes"), ctypes.cast(ptrs, ctypes.c_void_p),
                                _dev(p_req, torch.int32, "p_req"), p_max, _dev(x, torch.float16, "x"),
                                _dev(y, torch.float16, "y"), m, n, batch, group, _stream()), "bcq_gemm_mixed")
    return y


def bcq_quantize(w: torch.Tensor, p_low: int, p_high: int, cycles: int, group: int = 128, with_offset: bool = False,
                 planes: torch.Tensor | None = None, scales_by_p: dict | None = None, offsets_by_p: dict | None = None,
                 listing_residual: bool = False):
    """Algorithm 1 on float16 weights [m][n]: returns ``(planes int32 [p_high][m][n/32], {p: scales float16
    [p][m][n/group]}, {p: offsets float16 [m][n/group]} or None)`` for p = p_low..p_high.  ``listing_residual``
    selects the expansion residual as the algorithm's listing prints it (``bcq_quantize_form``)."""
    m, n = w.shape
    if n % 32 or n % group:
        raise ValueError("bcq_quantize: n must be a multiple of 32 and of group")
    dev = w.device
    if planes is None:
        planes = torch.empty((p_high, m, n // 32), dtype=torch.int32, device=dev)
    elif planes.shape != (p_high, m, n // 32):
        raise ValueError("bcq_quantize: planes has the wrong shape")
    rng = range(max(p_low, 1), min(p_high, BCQ_MAX_PLANES) + 1)
    if scales_by_p is None:
        scales_by_p = {p: torch.empty((p, m, n // group), dtype=torch.float16, device=dev) for p in rng}
    if with_offset and offsets_by_p is None:
        offsets_by_p = {p: torch.empty((m, n // group), dtype=torch.float16, device=dev) for p in rng}
    size = max(p_high, 0) + 1
    sp = (ctypes.c_void_p * size)()
    op = (ctypes.c_void_p * size)()
    for p in rng:
        if scales_by_p[p].shape != (p, m, n // group):
            raise ValueError(f"bcq_quantize: bad scale set for precision {p}")
        sp[p] = _dev(scales_by_p[p], torch.float16, f"scales_by_p[{p}]")
        if offsets_by_p is not None:
            if offsets_by_p[p].shape != (m, n // group):
                raise ValueError(f"bcq_quantize: bad offset set for precision {p}")
            op[p] = _dev(offsets_by_p[p], torch.float16, f"offsets_by_p[{p}]")
    _check(lib().bcq_quantize_form(_dev(w, torch.float16, "w"), p_low, p_high, cycles, 1 if listing_residual else 0,
                                   _dev(planes, torch.int32, "planes"), ctypes.cast(sp, ctypes.c_void_p),
                                   ctypes.cast(op, ctypes.c_void_p) if offsets_by_p is not None else None,
                                   m, n, group, _stream()), "bcq_quantize")
    return planes, scales_by_p, offsets_by_p


def bench_stream_read(buf: torch.Tensor, sink: torch.Tensor) -> None:
    """Benchmark reference: stream ``buf`` (any dtype, a multiple of 16 bytes) through 128-bit loads."""
    if not buf.is_cuda or not buf.is_contiguous():
        raise TypeError("buf must be a contiguous GPU tensor")
    _check(lib().bcq_bench_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), _dev(sink, torch.int32, "sink"), _stream()),
           "bcq_bench_stream_read")


def bench_fp16_gemv(w: torch.Tensor, x: torch.Tensor, y: torch.Tensor) -> torch.Tensor:
    """Benchmark reference: y = w @ x in binary16 with fp32 accumulation, one wavefront per row."""
    m, n = w.shape
    if x.shape != (n,) or y.shape != (m,):
        raise ValueError("bench_fp16_gemv: inconsistent shapes")
    _check(lib().bcq_bench_fp16_gemv(_dev(w, torch.float16, "w"), _dev(x, torch.float16, "x"), _dev(y, torch.float16, "y"), m, n,
                                     _stream()), "bcq_bench_fp16_gemv")
    return y


def bench_issue_probe(kind: int, valu: int, waves: int, iters: int, ticks: torch.Tensor, sink: torch.Tensor) -> torch.Tensor:
    """Benchmark reference: one workgroup of ``waves`` wavefronts alternates matrix instructions of ``kind`` with ``valu``
    vector FMAs; ``ticks`` (int64[32]) receives per wavefront the shader-clock and the 100 MHz ticks of its loop."""
    if ticks.numel() < 32 or sink.numel() < 1024:
        raise ValueError("bench_issue_probe: ticks needs 32 values, sink 1024")
    _check(lib().bcq_bench_issue_probe(int(kind), int(valu), int(waves), int(iters), _dev(ticks, torch.int64, "ticks"),
                                       _dev(sink, torch.float32, "sink"), _stream()), "bcq_bench_issue_probe")
    return ticks
