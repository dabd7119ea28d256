"""Helpers for the GPU parity tests: host->device marshalling and the oracle comparison."""
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
        y = bcq.bcq_gemv(dl.planes, dl.scales[p], p, to_dev(x), group=group,
                         offsets=None if offsets is None else to_dev(offsets))
        torch.cuda.synchronize()
        used = bcq.last_kernel()
    finally:
        bcq.select_kernel("auto")
    y_ref, a_ref = oracle.gemv(dl.layer.planes, dl.layer.scales[p], x, group, offsets=offsets)
    worst = assert_within_tolerance(y, y_ref, a_ref, f"bcq_gemv[{kernel}] m={dl.layer.m} n={dl.layer.n} p={p} batch={x.shape[0]}"
                                                     f"{'' if offsets is None else ' with offsets'}")
    return used, worst


def check_mixed(dl: DeviceLayer, p_req: np.ndarray, x: np.ndarray, kernel: str, group: int = 128, offsets_by_p: dict | None = None):
    bcq.select_kernel(kernel)
    try:
        y = bcq.bcq_gemm_mixed(dl.planes, dl.scales, to_dev(p_req.astype(np.int32)), to_dev(x), group=group,
                               offsets_by_p=None if not offsets_by_p else {q: to_dev(z) for q, z in offsets_by_p.items()})
        torch.cuda.synchronize()
        used = bcq.last_kernel()
    finally:
        bcq.select_kernel("auto")
    y_ref, a_ref = oracle.gemm_mixed(dl.layer.planes, dl.layer.scales, p_req, x, group, offsets_by_p=offsets_by_p)
    worst = assert_within_tolerance(y, y_ref, a_ref, f"bcq_gemm_mixed[{kernel}] m={dl.layer.m} n={dl.layer.n} batch={x.shape[0]}")
    return used, worst
