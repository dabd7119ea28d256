"""Helpers for the GPU parity tests: host->device marshalling, guard bands around outputs, and the oracle
comparison.  check_gemv and check_mixed, which nearly every parity test goes through, hand the kernels an output
tensor with 4 KiB of sentinel either side and assert the sentinels untouched."""
import numpy as np
import torch

import oracle
import paper_2510_10467_amd as bcq

DEV = torch.device("cuda:0")


def to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


class DeviceLayer:
    def __init__(self, layer):
        self.layer = layer
        self.planes = to_dev(layer.planes)
        self.scales = {p: to_dev(s) for p, s in layer.scales.items()}


GUARD_BYTES = 4096
_SENTINEL = {torch.float16: 0x7A5C, torch.int32: 0x5A5AC3C3, torch.int8: 0x5B}


class Guarded:
    """An output tensor with 4 KiB of sentinel either side, so that a store past either end shows."""

    def __init__(self, shape, dtype=torch.float16):
        self.dtype = dtype
        size = int(np.prod(shape))
        item = torch.empty((), dtype=dtype).element_size()
        self.guard = GUARD_BYTES // item
        raw_dtype = {2: torch.int16, 4: torch.int32, 1: torch.int8}[item]
        self.raw = torch.full((self.guard + size + self.guard,), _SENTINEL[dtype], dtype=raw_dtype, device=DEV)
        self.t = self.raw[self.guard:self.guard + size].view(dtype).view(*shape)
        assert self.t.is_contiguous() and self.t.data_ptr() % 16 == 0

    def check(self, what: str):
        torch.cuda.synchronize()
        lo, hi = self.raw[:self.guard], self.raw[-self.guard:]
        ok = bool((lo == _SENTINEL[self.dtype]).all()) and bool((hi == _SENTINEL[self.dtype]).all())
        assert ok, f"{what}: a store landed outside the output tensor"
        return self.t


def assert_within_tolerance(y_gpu: torch.Tensor, y_ref: np.ndarray, a_ref: np.ndarray, what: str):
    """|y - y_ref| <= 4e-3 * sum_j |W_p[r,j] x_j| + one binary16 ulp at y_ref, element by element."""
    y = y_gpu.detach().cpu().numpy().astype(np.float64)
    assert y.shape == y_ref.shape, what
    err = np.abs(y - y_ref)
    tol = oracle.tolerance(y_ref, a_ref)
    bad = np.argwhere(~(err <= tol))
    if bad.size:
        b, r = bad[0]
        raise AssertionError(f"{what}: {len(bad)} of {y.size} outside tolerance; first at [b={b}, r={r}] "
                             f"gpu={y[b, r]!r} ref={y_ref[b, r]!r} err={err[b, r]:.3e} tol={tol[b, r]:.3e}")
    return float(np.max(err / tol))


def check_gemv(dl: DeviceLayer, p: int, x: np.ndarray, kernel: str, group: int = 128, offsets: np.ndarray | None = None):
    bcq.select_kernel(kernel)
    try:
        out = Guarded((x.shape[0], dl.layer.m))
        bcq.bcq_gemv(dl.planes, dl.scales[p], p, to_dev(x), y=out.t, group=group,
                     offsets=None if offsets is None else to_dev(offsets))
        used = bcq.last_kernel()
        y = out.check(f"bcq_gemv[{kernel} -> {used}] m={dl.layer.m} n={dl.layer.n} p={p} batch={x.shape[0]}")
    finally:
        bcq.select_kernel("auto")
    y_ref, a_ref = oracle.gemv(dl.layer.planes, dl.layer.scales[p], x, group, offsets=offsets)
    worst = assert_within_tolerance(y, y_ref, a_ref, f"bcq_gemv[{kernel}] m={dl.layer.m} n={dl.layer.n} p={p} batch={x.shape[0]}"
                                                     f"{'' if offsets is None else ' with offsets'}")
    return used, worst


def check_mixed(dl: DeviceLayer, p_req: np.ndarray, x: np.ndarray, kernel: str, group: int = 128, offsets_by_p: dict | None = None):
    bcq.select_kernel(kernel)
    try:
        out = Guarded((x.shape[0], dl.layer.m))
        bcq.bcq_gemm_mixed(dl.planes, dl.scales, to_dev(p_req.astype(np.int32)), to_dev(x), y=out.t, group=group,
                           offsets_by_p=None if not offsets_by_p else {q: to_dev(z) for q, z in offsets_by_p.items()})
        used = bcq.last_kernel()
        y = out.check(f"bcq_gemm_mixed[{kernel} -> {used}] m={dl.layer.m} n={dl.layer.n} batch={x.shape[0]}")
    finally:
        bcq.select_kernel("auto")
    y_ref, a_ref = oracle.gemm_mixed(dl.layer.planes, dl.layer.scales, p_req, x, group, offsets_by_p=offsets_by_p)
    worst = assert_within_tolerance(y, y_ref, a_ref, f"bcq_gemm_mixed[{kernel}] m={dl.layer.m} n={dl.layer.n} batch={x.shape[0]}")
    return used, worst
