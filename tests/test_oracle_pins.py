"""Pins for the CPU oracle: it is checked against things other than itself.

Each test states what it pins.  Sources: the worked example of section 3.1
(Fig. 2), the 0 -> -1 convention of the Fig. 1 caption, the BCQ definition of
section 2.2, the q = 1 special case of section 2.2, the memory-footprint table
of section 1, exact rational brute force on tiny inputs, closed forms, and the
numpy library matmul on a matrix rebuilt with numpy's own bit unpacking.
The asymmetric offset (section 4.1) is pinned by the identity "an offset is one
more all-(+1) plane whose scale is the offset", which reduces it to the
symmetric path pinned above, by rational brute force and by closed forms.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import synthetic_inputs as syn

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# helpers written from the definition, independent of the oracle's C code
# ----------------------------------------------------------------------------
def bit_of(planes, i, r, j):
    """Bit of column j in plane i, row r (word j>>5, bit j&31), pure Python."""
    return (int(planes[i, r, j >> 5]) >> (j & 31)) & 1


def brute_force(planes, scale_sets, p_req, x, group, offset_sets=None):
    """Exact rational y[b][r] and sum of |terms| from the definition, pure Python loops."""
    _, m, words = planes.shape
    n = words * 32
    batch = x.shape[0]
    y = [[Fraction(0)] * m for _ in range(batch)]
    a = [[Fraction(0)] * m for _ in range(batch)]
    for b in range(batch):
        p = int(p_req[b])
        s = scale_sets[p]
        for r in range(m):
            acc = Fraction(0)
            aacc = Fraction(0)
            for j in range(n):
                w = Fraction(0)
                for i in range(p):
                    alpha = Fraction(float(s[i, r, j // group]))
                    w += alpha if bit_of(planes, i, r, j) else -alpha
                if offset_sets is not None and offset_sets.get(p) is not None:
                    w += Fraction(float(offset_sets[p][r, j // group]))
                t = w * Fraction(float(x[b, j]))
                acc += t
                aacc += abs(t)
            y[b][r] = acc
            a[b][r] = aacc
    return y, a


def numpy_dense(planes, scales_p, group):
    """W_p rebuilt with numpy's own bit unpacking (library routine), float64."""
    p = scales_p.shape[0]
    _, m, words = planes.shape
    n = words * 32
    # little-endian bytes of each uint32, LSB-first bits => column order
    bits = np.unpackbits(planes[:p].astype("<u4").view(np.uint8).reshape(p, m, words * 4), axis=2, bitorder="little")
    signs = bits.astype(np.float64) * 2.0 - 1.0
    alpha = np.repeat(scales_p.astype(np.float64), group, axis=2)
    assert alpha.shape == (p, m, n)
    return (alpha * signs).sum(axis=0)


# ----------------------------------------------------------------------------
# P1: worked example of section 3.1 and the 0 -> -1 convention
# ----------------------------------------------------------------------------
def read_worked_example():
    rows = []
    with open(os.path.join(GOLDEN, "worked_example_3bit.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            level, bits, signs = line.split()
            rows.append((int(level), [int(b) for b in bits.split(",")], [int(s) for s in signs.split(",")]))
    return rows


def test_worked_example_values(oracle):
    rows = read_worked_example()
    assert [r[0] for r in rows] == [1, 2, 3]
    n, group = 128, 128
    full_bits = rows[-1][1]                       # (0, 0, 1)
    planes = syn.make_planes(1, n, p_max=3, seed=(11, 0))
    col = 37                                       # an arbitrary column inside the group
    for i, b in enumerate(full_bits):
        w, k = col >> 5, col & 31
        planes[i, 0, w] = (planes[i, 0, w] & ~np.uint32(1 << k)) | np.uint32(b << k)
    # three distinct scale sets, exact binary fractions so the sums are exact
    sets = {
        1: np.array([[[0.75]]], dtype=np.float16),
        2: np.array([[[0.5]], [[0.1875]]], dtype=np.float16),
        3: np.array([[[0.625]], [[0.25]], [[0.09375]]], dtype=np.float16),
    }
    for level, bits, signs in rows:
        assert bits == full_bits[:level]
        w = oracle.dequant(planes, sets[level], group)
        expect = sum(s * float(sets[level][i, 0, 0]) for i, s in enumerate(signs))
        assert w[0, col] == expect
    # the headline case written out: -a1 - a2 + a3
    a1, a2, a3 = (float(v) for v in sets[3][:, 0, 0])
    assert oracle.dequant(planes, sets[3], group)[0, col] == -a1 - a2 + a3


def test_zero_bit_is_minus_one_and_one_hot_readout(oracle):
    # x = e_j reads W_p[r, j] back through the product; power-of-two scales keep it exact.
    m, n, group, p = 3, 256, 128, 2
    planes = syn.make_planes(m, n, p_max=2, seed=(12, 0))
    s = np.empty((p, m, n // group), dtype=np.float16)
    s[0] = [[1.0, 2.0]] * m
    s[1] = [[0.25, 0.5]] * m
    for j in (0, 31, 32, 127, 128, 255):
        x = np.zeros((1, n), dtype=np.float16)
        x[0, j] = 1.0
        y, a = oracle.gemv(planes, s, x, group)
        for r in range(m):
            expect = sum(float(s[i, r, j // group]) * (1.0 if bit_of(planes, i, r, j) else -1.0) for i in range(p))
            assert y[0, r] == expect
            assert a[0, r] == abs(expect)


# ----------------------------------------------------------------------------
# P2: exact rational brute force on tiny inputs (uniform and per-request)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,group,p_max,batch,seed", [
    (1, 128, 128, 1, 1, 0),
    (3, 128, 128, 3, 2, 1),
    (4, 256, 128, 4, 3, 2),
    (2, 256, 64, 4, 2, 3),
    (2, 96, 32, 2, 1, 4),
])
def test_brute_force_rational(oracle, m, n, group, p_max, batch, seed):
    layer = syn.make_layer(m, n, p_max=p_max, group=group, seed=(20, seed), signed=True)
    x = syn.make_x(batch, n, seed=(20, seed))
    for p in range(1, p_max + 1):
        y, a = oracle.gemv(layer.planes, layer.scales[p], x, group)
        ye, ae = brute_force(layer.planes, layer.scales, [p] * batch, x, group)
        for b in range(batch):
            for r in range(m):
                assert abs(Fraction(y[b, r]) - ye[b][r]) <= Fraction(1, 10 ** 13) * ae[b][r] + Fraction(1, 10 ** 300)
                assert abs(Fraction(a[b, r]) - ae[b][r]) <= Fraction(1, 10 ** 13) * ae[b][r] + Fraction(1, 10 ** 300)
    p_req = syn.make_p_req(batch, 1, p_max, seed=(20, seed))
    y, a = oracle.gemm_mixed(layer.planes, layer.scales, p_req, x, group)
    ye, ae = brute_force(layer.planes, layer.scales, p_req, x, group)
    for b in range(batch):
        for r in range(m):
            assert abs(Fraction(y[b, r]) - ye[b][r]) <= Fraction(1, 10 ** 13) * ae[b][r] + Fraction(1, 10 ** 300)


# ----------------------------------------------------------------------------
# P3: all-(+1) planes => sum(alpha) * sum(x) per group; all-zero bits => its negative
# ----------------------------------------------------------------------------
def test_all_plus_one_planes_closed_form(oracle):
    m, n, group, p = 5, 512, 128, 3
    s = syn.make_scales(p, m, n, group, seed=(30, 0))
    x = syn.make_x(2, n, seed=(30, 0))
    ones = np.full((p, m, n // 32), 0xFFFFFFFF, dtype=np.uint32)
    zeros = np.zeros_like(ones)
    xs = x.astype(np.float64).reshape(2, n // group, group).sum(axis=2)          # [batch][G]
    alpha_sum = s.astype(np.float64).sum(axis=0)                                   # [m][G]
    expect = np.einsum("rg,bg->br", alpha_sum, xs)
    y1, _ = oracle.gemv(ones, s, x, group)
    y0, _ = oracle.gemv(zeros, s, x, group)
    scale = np.abs(alpha_sum).sum(axis=1)[None, :] * np.abs(x.astype(np.float64)).sum(axis=1)[:, None]
    assert np.all(np.abs(y1 - expect) <= 1e-13 * scale)
    assert np.all(np.abs(y0 + expect) <= 1e-13 * scale)


# ----------------------------------------------------------------------------
# P4: q = 1 (section 2.2): a sign-matrix product; with alpha = x = 1 it is 2*popcount - n
# ----------------------------------------------------------------------------
def test_one_bit_popcount_identity(oracle):
    m, n, group = 7, 1024, 128
    planes = syn.make_planes(m, n, p_max=1, seed=(40, 0))
    s = np.ones((1, m, n // group), dtype=np.float16)
    x = np.ones((1, n), dtype=np.float16)
    y, a = oracle.gemv(planes, s, x, group)
    pop = np.array([sum(bin(int(w)).count("1") for w in planes[0, r]) for r in range(m)])
    assert np.array_equal(y[0], (2 * pop - n).astype(np.float64))
    assert np.array_equal(a[0], np.full(m, float(n)))


def test_one_bit_sign_matrix_product(oracle):
    m, n, group = 6, 384, 128
    planes = syn.make_planes(m, n, p_max=1, seed=(41, 0))
    x = syn.make_x(2, n, seed=(41, 0))
    s = np.ones((1, m, n // group), dtype=np.float16)
    sign = np.array([[1.0 if bit_of(planes, 0, r, j) else -1.0 for j in range(n)] for r in range(m)])
    y, _ = oracle.gemv(planes, s, x, group)
    ref = x.astype(np.float64) @ sign.T
    assert np.allclose(y, ref, rtol=0, atol=1e-12 * n)


# ----------------------------------------------------------------------------
# P5: library matmul on a matrix rebuilt with numpy's own unpackbits
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,group", [(33, 1024, 128), (16, 4096, 128), (5, 640, 64)])
def test_against_numpy_matmul(oracle, m, n, group):
    layer = syn.make_layer(m, n, group=group, seed=(50, m))
    x = syn.make_x(3, n, seed=(50, m))
    for p in (1, 2, 3, 4):
        w = numpy_dense(layer.planes, layer.scales[p], group)
        assert np.array_equal(oracle.dequant(layer.planes, layer.scales[p], group), w)
        y, a = oracle.gemv(layer.planes, layer.scales[p], x, group)
        xr = x.astype(np.float64)
        ref = xr @ w.T
        aref = np.abs(xr) @ np.abs(w).T
        assert np.all(np.abs(y - ref) <= 1e-12 * aref)
        assert np.all(np.abs(a - aref) <= 1e-12 * aref)


def test_half_widening_all_bit_patterns(oracle):
    # every binary16 pattern used as a scale with an all-(+1) plane reads back its own value
    m, n, group = 65536, 32, 32
    s = np.arange(65536, dtype=np.uint16).view(np.float16).reshape(1, m, 1)
    ones = np.full((1, m, 1), 0xFFFFFFFF, dtype=np.uint32)
    w = oracle.dequant(ones, s, group)[:, 0]
    ref = s.reshape(-1).astype(np.float64)
    finite = np.isfinite(ref)
    assert np.array_equal(w[finite], ref[finite])
    assert np.array_equal(np.isnan(w), np.isnan(ref))
    assert np.array_equal(np.isinf(w), np.isinf(ref))


# ----------------------------------------------------------------------------
# P6: storage accounting against the memory-footprint table of section 1
# ----------------------------------------------------------------------------
def test_memory_table_ratios():
    table = {}
    with open(os.path.join(GOLDEN, "memory_footprint_llama31_8b.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            table[parts[0]] = [float(v) for v in parts[1:]]
    layer = syn.make_layer(64, 1024, seed=(60, 0))
    plane_bytes = layer.planes.nbytes / layer.planes.shape[0]
    for p, key in ((2, "BCQ2"), (3, "BCQ3"), (4, "BCQ4")):
        scale_b, binary_b = layer.scales[p].nbytes, plane_bytes * p
        assert binary_b / scale_b == 8.0                      # fp16 scale per 128 one-bit codes
        assert abs(table[key][0] / table[key][1] - scale_b / binary_b) < 0.005   # printed to 2 decimals
        assert abs(table[key][1] / table["BCQ2"][1] - p / 2) < 0.01            # bytes proportional to p
    ours = sum(layer.scales[p].nbytes for p in (2, 3, 4)) + plane_bytes * 4
    separate = sum(layer.scales[p].nbytes + plane_bytes * p for p in (2, 3, 4))
    assert abs(ours / separate - table["Proposed"][2] / table["Multi-model"][2]) < 0.005
    assert round(100 * (1 - table["Proposed"][2] / table["Multi-model"][2])) == table["reduction_percent"][0]
    # the byte formula used for the roofline matches the arrays it describes
    x_y = 1 * 1024 * 2 + 1 * 64 * 2
    assert syn.algorithmic_bytes(64, 1024, 3, 1) == int(plane_bytes * 3) + layer.scales[3].nbytes + x_y


# ----------------------------------------------------------------------------
# P7: packing round trips and single-bit probes
# ----------------------------------------------------------------------------
def test_pack_round_trip_and_bit_order(oracle):
    codes = syn.make_codes(3, 5, 96, seed=(70, 0))
    planes = oracle.pack(codes)
    assert planes.shape == (3, 5, 3) and planes.dtype == np.uint32
    assert np.array_equal(oracle.unpack(planes), codes)
    raw = syn.make_planes(4, 64, p_max=2, seed=(70, 1))
    assert np.array_equal(oracle.pack(oracle.unpack(raw)), raw)
    # numpy's own packer agrees (little-endian bytes, LSB-first bits)
    lib = np.packbits((codes > 0).astype(np.uint8), axis=2, bitorder="little").view("<u4")
    assert np.array_equal(lib.reshape(planes.shape), planes)
    for k in range(64):
        c = -np.ones((1, 1, 64), dtype=np.int8)
        c[0, 0, k] = 1
        w = oracle.pack(c)[0, 0]
        assert int(w[k >> 5]) == 1 << (k & 31) and int(w[1 - (k >> 5)]) == 0
    # zero and negative codes both mean -1
    c = np.array([[[0, -1, -128, 1, 127] + [1] * 27]], dtype=np.int8)
    assert int(oracle.pack(c)[0, 0, 0]) == 0xFFFFFFFF & ~0b00111


# ----------------------------------------------------------------------------
# P9 / P10: symmetries and prefix invariance
# ----------------------------------------------------------------------------
def test_symmetries_and_prefix_invariance(oracle):
    m, n, group = 9, 768, 128
    layer = syn.make_layer(m, n, seed=(90, 0))
    x = syn.make_x(2, n, seed=(90, 0))
    for p in (1, 2, 3, 4):
        y, a = oracle.gemv(layer.planes, layer.scales[p], x, group)
        yn, an = oracle.gemv(layer.planes, layer.scales[p], -x, group)
        assert np.array_equal(yn, -y) and np.array_equal(an, a)
        yc, ac = oracle.gemv(~layer.planes, layer.scales[p], x, group)
        assert np.array_equal(yc, -y) and np.array_equal(ac, a)
        scrambled = layer.planes.copy()
        scrambled[p:] = syn.make_planes(m, n, seed=(90, 1))[p:]
        ys, _ = oracle.gemv(scrambled, layer.scales[p], x, group)
        assert np.array_equal(ys, y)
        # permuting requests permutes output rows
        yp, _ = oracle.gemv(layer.planes, layer.scales[p], x[::-1].copy(), group)
        assert np.array_equal(yp, y[::-1])
    # scale sets of different precisions are distinct objects: the wrong set gives another answer
    y3, _ = oracle.gemv(layer.planes, layer.scales[3], x, group)
    y3_wrong, _ = oracle.gemv(layer.planes, layer.scales[4][:3].copy(), x, group)
    assert not np.allclose(y3, y3_wrong)


def test_mixed_rows_equal_uniform_rows(oracle):
    m, n, group = 8, 512, 128
    layer = syn.make_layer(m, n, seed=(91, 0))
    x = syn.make_x(6, n, seed=(91, 0))
    p_req = np.array([2, 4, 3, 3, 1, 4], dtype=np.int32)
    ym, am = oracle.gemm_mixed(layer.planes, layer.scales, p_req, x, group)
    for b, p in enumerate(p_req):
        yu, au = oracle.gemv(layer.planes, layer.scales[int(p)], x[b:b + 1], group)
        assert np.array_equal(ym[b], yu[0]) and np.array_equal(am[b], au[0])


def test_tolerance_definition(oracle):
    # one binary16 ulp: spacing of binary16 at |y_ref|, never below 2^-24
    assert oracle.ulp16(1.0) == 2.0 ** -10
    assert oracle.ulp16(1.9999) == 2.0 ** -10
    assert oracle.ulp16(2.0) == 2.0 ** -9
    assert oracle.ulp16(0.0) == 2.0 ** -24
    assert oracle.ulp16(-3e-6) == 2.0 ** -24
    assert oracle.ulp16(1000.0) == float(np.spacing(np.float16(1000.0)))
    assert np.allclose(oracle.tolerance(np.array([1.0]), np.array([10.0])), 4e-3 * 10 + 2.0 ** -10)


def test_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.pack(np.zeros((1, 1, 33), dtype=np.int8))
    layer = syn.make_layer(2, 128, seed=(99, 0))
    with pytest.raises(ValueError):
        oracle.gemm_mixed(layer.planes, layer.scales, [5], syn.make_x(1, 128), 128)


# ----------------------------------------------------------------------------
# P11: asymmetric offset (section 4.1).  z[r][g] is one more plane of all +1 with scale z:
#      checked against the SYMMETRIC oracle path (pinned above) on such an extended layer,
#      against exact rational brute force, and against closed forms.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,group,p_max,batch,seed", [(3, 256, 128, 3, 2, 0), (5, 384, 64, 4, 3, 1), (2, 1024, 128, 2, 1, 2)])
def test_offset_is_an_extra_all_ones_plane(oracle, m, n, group, p_max, batch, seed):
    layer = syn.make_layer(m, n, p_max=p_max, group=group, seed=(110, seed), signed=True)
    x = syn.make_x(batch, n, seed=(110, seed))
    for p in range(1, p_max + 1):
        z = syn.make_offsets(p, m, n, group, seed=(110, seed))
        y, a = oracle.gemv(layer.planes, layer.scales[p], x, group, offsets=z)
        planes_ext = np.concatenate([layer.planes[:p], np.full((1, m, n // 32), 0xFFFFFFFF, dtype=np.uint32)])
        scales_ext = np.concatenate([layer.scales[p], z[None]])
        y2, a2 = oracle.gemv(planes_ext, scales_ext, x, group)
        scale = a2 + 1e-300
        assert np.all(np.abs(y - y2) <= 1e-13 * scale)
        assert np.all(np.abs(a - a2) <= 1e-13 * scale)
        w = oracle.dequant(layer.planes, layer.scales[p], group, offsets=z)
        w2 = oracle.dequant(planes_ext, scales_ext, group)
        assert np.array_equal(w, w2) or np.all(np.abs(w - w2) <= 1e-15 * np.abs(w2).max())


def test_offset_brute_force_and_closed_forms(oracle):
    m, n, group, p_max, batch = 3, 256, 128, 3, 3
    layer = syn.make_layer(m, n, p_max=p_max, group=group, seed=(111, 0), signed=True)
    x = syn.make_x(batch, n, seed=(111, 0))
    zs = {p: syn.make_offsets(p, m, n, group, seed=(111, 0)) for p in range(1, p_max + 1)}
    p_req = syn.make_p_req(batch, 1, p_max, seed=(111, 0))
    y, a = oracle.gemm_mixed(layer.planes, layer.scales, p_req, x, group, offsets_by_p=zs)
    ye, ae = brute_force(layer.planes, layer.scales, p_req, x, group, offset_sets=zs)
    for b in range(batch):
        for r in range(m):
            assert abs(Fraction(y[b, r]) - ye[b][r]) <= Fraction(1, 10 ** 13) * ae[b][r] + Fraction(1, 10 ** 300)
            assert abs(Fraction(a[b, r]) - ae[b][r]) <= Fraction(1, 10 ** 13) * ae[b][r] + Fraction(1, 10 ** 300)
    # a precision without an offset set in the dictionary is the symmetric product
    only2 = {2: zs[2]}
    y2, _ = oracle.gemm_mixed(layer.planes, layer.scales, np.array([1, 2, 3], dtype=np.int32), x, group, offsets_by_p=only2)
    y1s, _ = oracle.gemv(layer.planes, layer.scales[1], x[:1], group)
    y3s, _ = oracle.gemv(layer.planes, layer.scales[3], x[2:], group)
    y2o, _ = oracle.gemv(layer.planes, layer.scales[2], x[1:2], group, offsets=zs[2])
    assert np.array_equal(y2[0], y1s[0]) and np.array_equal(y2[2], y3s[0]) and np.array_equal(y2[1], y2o[0])
    # closed form: zero scales leave y[b][r] = sum_g z[r][g] * sum_{j in g} x[b][j]
    zero_scales = np.zeros_like(layer.scales[2])
    y0, a0 = oracle.gemv(layer.planes, zero_scales, x, group, offsets=zs[2])
    xs = x.astype(np.float64).reshape(batch, n // group, group).sum(axis=2)
    expect = np.einsum("rg,bg->br", zs[2].astype(np.float64), xs)
    bound = 1e-13 * (np.abs(zs[2].astype(np.float64)).sum(axis=1)[None, :] * np.abs(x.astype(np.float64)).sum(axis=1)[:, None])
    assert np.all(np.abs(y0 - expect) <= bound)
    # linearity in the offset: y(z) - y(0) is that same closed form
    ysym, _ = oracle.gemv(layer.planes, layer.scales[2], x, group)
    yoff, _ = oracle.gemv(layer.planes, layer.scales[2], x, group, offsets=zs[2])
    assert np.all(np.abs((yoff - ysym) - expect) <= 1e-12 * (np.abs(ysym) + np.abs(expect) + 1e-300))
    # a dropped offset must be visible at the acceptance tolerance (the pin would catch a no-op)
    assert np.any(np.abs(yoff - ysym) > oracle.tolerance(yoff, a0 + np.abs(ysym)))
