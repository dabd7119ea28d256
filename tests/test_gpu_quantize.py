"""GPU parity of bcq_quantize against the quantiser oracle.

Codes are integers decided by floating point: both sides decide them in IEEE double, where every
sum over a group of binary16 weights is exact, so planes are compared bit for bit and scales /
offsets bit for bit after the single rounding to binary16.  The quantised layer is then run through
bcq_gemv, and the product is checked against the float64 product of the ORIGINAL weights within the
quantisation error the oracle's model predicts.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_10467_amd as bcq
import synthetic_inputs as syn
from tests.gpu_util import Guarded, to_dev

pytestmark = pytest.mark.gpu


def run_gpu(w, p_low, p_high, cycles, group=128, with_offset=False, listing=False):
    # every output sits between 4 KiB bands of sentinel values: a store past either end fails the test
    m, n = w.shape
    g_planes = Guarded((p_high, m, n // 32), torch.int32)
    g_scales = {p: Guarded((p, m, n // group)) for p in range(p_low, p_high + 1)}
    g_offsets = {p: Guarded((m, n // group)) for p in range(p_low, p_high + 1)} if with_offset else None
    planes, scales, offsets = bcq.bcq_quantize(to_dev(w), p_low, p_high, cycles, group=group, with_offset=with_offset,
                                               planes=g_planes.t, scales_by_p={p: g.t for p, g in g_scales.items()},
                                               offsets_by_p=None if g_offsets is None else {p: g.t for p, g in g_offsets.items()},
                                               listing_residual=listing)
    torch.cuda.synchronize()
    assert bcq.last_kernel() == "quantize"
    what = f"bcq_quantize m={m} n={n} p={p_low}..{p_high} g={group}"
    g_planes.check(what + " planes")
    for p, g in g_scales.items():
        g.check(what + f" scale set {p}")
    for p, g in (g_offsets or {}).items():
        g.check(what + f" offset set {p}")
    planes = planes.cpu().numpy().view(np.uint32)
    scales = {p: s.cpu().numpy() for p, s in scales.items()}
    offsets = None if offsets is None else {p: z.cpu().numpy() for p, z in offsets.items()}
    return planes, scales, offsets


def compare(w, p_low, p_high, cycles, group=128, with_offset=False, listing=False):
    print(f"quantize m={w.shape[0]} n={w.shape[1]} p={p_low}..{p_high} T={cycles} g={group} offset={with_offset} listing={listing}", flush=True)
    planes, scales, offsets = run_gpu(w, p_low, p_high, cycles, group, with_offset, listing)
    q = oracle.quantize(w, p_low, p_high, cycles, group=group, with_offset=with_offset, literal_residual=listing)
    ref_planes = oracle.pack(q["codes"])
    diff = np.count_nonzero(planes != ref_planes)
    assert diff == 0, f"{diff} of {planes.size} plane words differ"
    for p in range(p_low, p_high + 1):
        ref = q["scales"][p].astype(np.float16)
        assert np.array_equal(scales[p].view(np.uint16), ref.view(np.uint16)), f"scale set {p} differs"
        if with_offset:
            refz = q["offsets"][p].astype(np.float16)
            assert np.array_equal(offsets[p].view(np.uint16), refz.view(np.uint16)), f"offset set {p} differs"
    return planes, scales, offsets


@pytest.mark.parametrize("m,n", [(64, 1024), (37, 1280), (5, 128), (300, 4096)])
def test_paper_setting(m, n):
    """p_L = 2, p_H = 4, T = 20, g = 128 (sections 3.2 and 4.1), several tiles and a ragged tail of words."""
    compare(syn.make_weights(m, n, seed=(91, m)), 2, 4, 20)


@pytest.mark.parametrize("p_low,p_high,cycles", [(1, 1, 0), (1, 4, 3), (2, 2, 0), (3, 4, 5), (4, 4, 7), (2, 3, 1)])
def test_precision_ranges(p_low, p_high, cycles):
    compare(syn.make_weights(48, 512, seed=(92, p_low * 10 + p_high)), p_low, p_high, cycles)


@pytest.mark.parametrize("group", [32, 64, 256])
def test_group_sizes(group):
    compare(syn.make_weights(24, 1024, seed=(93, group)), 2, 4, 6, group=group)


@pytest.mark.parametrize("group", [64, 128])
def test_asymmetric(group):
    w = syn.make_weights(40, 1024, seed=(94, group))
    w = (w.astype(np.float32) + 0.03).astype(np.float16)
    compare(w, 2, 4, 8, group=group, with_offset=True)


def test_degenerate_groups():
    """Zero groups, constant groups, a group with a single non-zero, negative zeros."""
    w = syn.make_weights(8, 512, seed=(95, 0))
    w[0, :] = 0
    w[1, :128] = 0.375
    w[1, 128:256] = -0.375
    w[2, :128] = 0
    w[2, 5] = 1.0
    w[3, 256:384] = -0.0
    w[4, ::2] = 0
    compare(w, 2, 4, 5)
    compare(w, 2, 4, 5, with_offset=True)


def test_quantised_layer_runs_through_the_product():
    """Quantise, then y = W_p x on the GPU from the planes and scale sets just written: within the
    product's tolerance of the oracle product for those planes, and close to the product with the
    original weights, closer with every added plane."""
    m, n = 256, 2048
    w = syn.make_weights(m, n, seed=(96, 0), heavy_tail=False)
    x = syn.make_x(3, n, seed=(96, 0))
    planes, scales, _ = compare(w, 2, 4, 20)
    exact = x.astype(np.float64) @ w.astype(np.float64).T
    rel = []
    for p in (2, 3, 4):
        y = bcq.bcq_gemv(to_dev(planes), to_dev(scales[p]), p, to_dev(x))
        torch.cuda.synchronize()
        y_ref, a_ref = oracle.gemv(planes, scales[p], x)
        yy = y.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(yy - y_ref) <= oracle.tolerance(y_ref, a_ref))
        rel.append(np.linalg.norm(yy - exact) / np.linalg.norm(exact))
    assert rel[0] > rel[1] > rel[2]
    assert rel[0] < 0.45 and rel[2] < 0.16


@pytest.mark.parametrize("m,n", [(64, 1024), (37, 1280)])
@pytest.mark.parametrize("with_offset", [False, True])
def test_listing_residual_form(m, n, with_offset):
    """The expansion residual as Algorithm 1 prints it (all p planes subtracted): bit-exact against the oracle's
    literal form at the paper's setting and at few cycles, other group sizes, and different from the default form."""
    w = syn.make_weights(m, n, seed=(98, m))
    if with_offset:
        w = (w.astype(np.float32) + 0.03).astype(np.float16)
    planes_l, scales_l, _ = compare(w, 2, 4, 20, with_offset=with_offset, listing=True)
    compare(w, 2, 4, 2, with_offset=with_offset, listing=True)
    compare(w, 1, 3, 3, group=64, with_offset=with_offset, listing=True)
    compare(w, 3, 4, 4, group=256 if n % 256 == 0 else 32, with_offset=with_offset, listing=True)
    planes_d, _, _ = run_gpu(w, 2, 4, 20, 128, with_offset)
    assert np.array_equal(planes_l[:2], planes_d[:2]) and not np.array_equal(planes_l[2:], planes_d[2:])


@pytest.mark.parametrize("m,n,with_offset,listing", [(14336, 4096, False, False), (4096, 14336, True, False), (14336, 4096, False, True)])
def test_full_size_layers_sampled_rows(m, n, with_offset, listing):
    """The benchmark's shapes and settings (p 2..4, T = 20); groups are independent, so the oracle runs on a
    sample of rows and every plane word, scale and offset of those rows must match bit for bit."""
    w = syn.make_weights(m, n, seed=(97, m))
    print(f"quantize full size m={m} n={n} offset={with_offset}", flush=True)
    planes, scales, offsets = run_gpu(w, 2, 4, 20, 128, with_offset, listing)
    rng = np.random.default_rng([syn.BASE_SEED, 97, m])
    rows = np.unique(np.concatenate([[0, 1, m - 1], rng.integers(0, m, size=45)]))
    q = oracle.quantize(np.ascontiguousarray(w[rows]), 2, 4, 20, with_offset=with_offset, literal_residual=listing)
    assert np.array_equal(planes[:, rows, :], oracle.pack(q["codes"]))
    for p in (2, 3, 4):
        assert np.array_equal(scales[p][:, rows, :].view(np.uint16), q["scales"][p].astype(np.float16).view(np.uint16))
        if with_offset:
            assert np.array_equal(offsets[p][rows, :].view(np.uint16), q["offsets"][p].astype(np.float16).view(np.uint16))
