"""GPU checks that hold at any size: full-size layers in the launch configuration the benchmark
times (sampled rows against the oracle), invariants of the method, edge cases of the ABI."""
import numpy as np
import pytest

import synthetic_inputs as syn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from tests import gpu_util
    return gpu_util


def sampled_rows_check(gpu, oracle, layer, dl, p, x, rows, y_gpu, what):
    """Oracle on a subset of rows (the product is independent per output row)."""
    sub_planes = np.ascontiguousarray(layer.planes[:, rows, :])
    sub_scales = np.ascontiguousarray(layer.scales[p][:, rows, :])
    y_ref, a_ref = oracle.gemv(sub_planes, sub_scales, x)
    y = y_gpu.cpu().numpy().astype(np.float64)[:, rows]
    err = np.abs(y - y_ref)
    tol = oracle.tolerance(y_ref, a_ref)
    assert np.all(err <= tol), f"{what}: max err/tol {np.max(err / tol):.3f}"


@pytest.mark.parametrize("name,m,n", [("gate_proj", 14336, 4096), ("down_proj", 4096, 14336), ("q_proj", 4096, 4096),
                                       ("k_proj", 1024, 4096), ("llama70b_up", 28672, 8192), ("llama70b_down", 8192, 28672),
                                       ("phi4_attn", 5120, 5120), ("phi4_up", 17920, 5120), ("phi4_down", 5120, 17920)])
def test_full_size_layers_sampled_rows(gpu, oracle, name, m, n):
    import torch

    import paper_2510_10467_amd as bcq
    layer = syn.make_layer(m, n, seed=(200, m, n))
    dl = gpu.DeviceLayer(layer)
    rng = np.random.default_rng([syn.BASE_SEED, 200, m])
    rows = np.unique(np.concatenate([[0, 15, 16, m - 17, m - 1], rng.integers(0, m, size=120)]))
    # (256 and 512 requests: the shapes with eight waves on a 256-request tile, 64 rows on gate_proj at 256, 128 rows otherwise)
    batches = {"gate_proj": (1, 3, 16, 80, 256, 512), "llama70b_down": (1, 3, 16, 80, 256), "q_proj": (1, 3, 16, 80, 256),
               "llama70b_up": (1, 3, 16, 80, 256)}.get(name, (1, 3, 16, 80))
    for batch in batches:
        x = syn.make_x(batch, n, seed=(200, batch))
        xd = gpu.to_dev(x)
        for p in (2, 3, 4):
            out = gpu.Guarded((batch, m))
            bcq.bcq_gemv(dl.planes, dl.scales[p], p, xd, y=out.t)
            y = out.check(f"{name} p={p} batch={batch} ({bcq.last_kernel()})")
            sampled_rows_check(gpu, oracle, layer, dl, p, x, rows, y, f"{name} p={p} batch={batch} ({bcq.last_kernel()})")


@pytest.mark.parametrize("m,n,p,batches,kernels", [
    # two planes of just under 2 GiB each (16 K slices in four chunks per wave; 32-bit offsets inside a plane at their limit)
    (262144 - 11, 65536, 2, (1, 3, 16, 80), {"plane_mfma", "plane_f16", "dequant_mfma"}),
    # one plane of more than 2 GiB: past what the tuned kernels address, the table look-up kernel takes every batch
    (262144 + 5, 65536, 1, (1, 3), {"lut"}),
])
def test_planes_at_the_limit_of_32_bit_offsets(gpu, oracle, m, n, p, batches, kernels):
    """Maximum sizes: byte offsets inside one plane are 32-bit in the tuned kernels, which take planes below 2 GiB; a
    larger plane goes to the table look-up kernel, which indexes in 64 bits.  Sampled rows (first, last, the rows around 2^31
    bytes into a plane) against the oracle, every output guarded."""
    import paper_2510_10467_amd as bcq
    layer = syn.make_layer(m, n, p_max=p, seed=(280, m, p), precisions=[p], signed=True)
    dl = gpu.DeviceLayer(layer)
    rng = np.random.default_rng([syn.BASE_SEED, 280, m])
    rows = np.unique(np.concatenate([[0, 15, 16, m - 17, m - 16, m - 2, m - 1, 262143 - 16, min(262143, m - 1), min(262144, m - 1)],
                                     rng.integers(0, m, size=60)]))
    seen = set()
    for batch in batches:
        x = syn.make_x(batch, n, seed=(280, batch))
        out = gpu.Guarded((batch, m))
        bcq.bcq_gemv(dl.planes, dl.scales[p], p, gpu.to_dev(x), y=out.t)
        used = bcq.last_kernel()
        seen.add(used)
        y = out.check(f"m={m} n={n} p={p} batch={batch} ({used})")
        sampled_rows_check(gpu, oracle, layer, dl, p, x, rows, y, f"m={m} n={n} p={p} batch={batch} ({used})")
    assert seen == kernels, seen


@pytest.mark.parametrize("m,n", [(12300, 4096), (12290, 5120), (12400, 6144), (12500, 7168), (12304, 8192), (10236, 4096), (8200, 4096),
                                 (14330, 4096), (14350, 8192), (14336, 5120)])
def test_row_streaming_form_sampled_rows(gpu, oracle, m, n):
    """Tall matrices with two to eight requests (and with one request at one or two planes) run the FP4 family in its
    row-streaming form (one operand image per four row blocks, chunks of 1024 columns prefetched one ahead): 4 to 8
    chunks per row, one and two request tiles, one and two waves per row block, a last workgroup with absent row blocks
    and a ragged last block; the shapes and batches it leaves to the other kernels are checked in the same loop."""
    import paper_2510_10467_amd as bcq
    layer = syn.make_layer(m, n, seed=(270, m, n), signed=True)
    dl = gpu.DeviceLayer(layer)
    rng = np.random.default_rng([syn.BASE_SEED, 270, m])
    rows = np.unique(np.concatenate([[0, 15, 16, 63, 64, m - 65, m - 64, m - 17, m - 16, m - 13, m - 2, m - 1], rng.integers(0, m, size=150)]))
    streamed = 0
    for batch in (1, 2, 3, 4, 5, 7, 8):
        x = syn.make_x(batch, n, seed=(270, batch))
        xd = gpu.to_dev(x)
        for p in (1, 2, 3, 4):
            out = gpu.Guarded((batch, m))
            bcq.bcq_gemv(dl.planes, dl.scales[p], p, xd, y=out.t)
            used = bcq.last_kernel()
            streamed += used == "plane_mfma_rows"
            y = out.check(f"m={m} n={n} p={p} batch={batch} ({used})")
            sampled_rows_check(gpu, oracle, layer, dl, p, x, rows, y, f"m={m} n={n} p={p} batch={batch} ({used})")
            if used == "plane_mfma_rows":
                again = bcq.bcq_gemv(dl.planes, dl.scales[p], p, xd)
                assert np.array_equal(again.cpu().numpy().view(np.uint16), y.cpu().numpy().view(np.uint16)), "not deterministic"
    # two to four requests at every width from 640 row blocks on, five to eight at 4096 columns from 512 row blocks on, one
    # request at one or two planes from 896 row blocks on with 4096 or 8192 columns
    single = 2 if m > 895 * 16 and n in (4096, 8192) else 0
    assert streamed == (0 if m < 10225 else 12) + (12 if n == 4096 else 0) + single, streamed


@pytest.mark.parametrize("m", [12300, 8200])
def test_row_streaming_form_per_request_precision(gpu, oracle, m):
    """Per-request precision on the row-streaming form (4096 columns): a lane reports one request per tile of four and
    reads that request's own scale set.  Sampled rows against the oracle; each request bit for bit what the uniform call
    at its precision gives; precisions outside 1 .. p_max clamped; a precision without a scale set, or none with one,
    gives zeros; planes beyond the deepest precision present may hold anything."""
    import torch

    import paper_2510_10467_amd as bcq
    n = 4096
    layer = syn.make_layer(m, n, seed=(272, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    rng = np.random.default_rng([syn.BASE_SEED, 272, m])
    rows = np.unique(np.concatenate([[0, 15, 16, 63, 64, m - 17, m - 16, m - 9, m - 1], rng.integers(0, m, size=120)]))
    sub_planes = np.ascontiguousarray(layer.planes[:, rows, :])
    sub_scales = {p: np.ascontiguousarray(sc[:, rows, :]) for p, sc in layer.scales.items()}
    for batch in (2, 3, 4, 5, 8):
        streams = batch > 4 or m >= 10240
        x = syn.make_x(batch, n, seed=(272, batch))
        xd = gpu.to_dev(x)
        draws = [rng.integers(1, 5, size=batch).astype(np.int32), np.full(batch, 2, dtype=np.int32),
                 np.array([4, 3, 2, 1, 1, 2, 3, 4][:batch], dtype=np.int32)]
        for p_req in draws:
            out = gpu.Guarded((batch, m))
            bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(p_req), xd, y=out.t)
            used = bcq.last_kernel()
            assert used == ("plane_mfma_rows" if streams else "plane_mfma"), (batch, used)
            y = out.check(f"mixed m={m} batch={batch} p_req={p_req.tolist()}")
            y_ref, a_ref = oracle.gemm_mixed(sub_planes, sub_scales, p_req, x)
            err = np.abs(y.cpu().numpy().astype(np.float64)[:, rows] - y_ref)
            assert np.all(err <= oracle.tolerance(y_ref, a_ref)), f"m={m} batch={batch} p_req={p_req.tolist()}"
            if streams:
                for p in sorted(set(p_req.tolist())):
                    yu = bcq.bcq_gemv(dl.planes, dl.scales[p], p, xd)
                    assert bcq.last_kernel() == "plane_mfma_rows"
                    sel = torch.from_numpy(p_req == p).to(y.device)
                    assert torch.equal(y[sel], yu[sel]), f"request at p={p} differs from the uniform call (batch {batch})"
        if not streams:
            continue
        # clamping, a missing set, no set at all, garbage in the planes nobody uses
        wild = np.array([0, -3, 9, 2, 3, 77, 1, 4][:batch], dtype=np.int32)
        clamped = np.clip(wild, 1, 4).astype(np.int32)
        y_wild = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(wild), xd)
        y_ok = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(clamped), xd)
        assert torch.equal(y_wild, y_ok)
        no3 = {p: sc for p, sc in dl.scales.items() if p != 3}
        p3 = np.array([3, 2, 3, 4, 1, 3, 2, 3][:batch], dtype=np.int32)
        y_no3 = bcq.bcq_gemm_mixed(dl.planes, no3, gpu.to_dev(p3), xd)
        y_all = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(p3), xd)
        is3 = torch.from_numpy(p3 == 3).to(y_all.device)
        assert torch.all(y_no3[is3] == 0) and torch.equal(y_no3[~is3], y_all[~is3])
        only3 = {3: dl.scales[3]}
        p12 = np.array([1, 2, 4, 2, 1, 4, 2, 1][:batch], dtype=np.int32)
        out = gpu.Guarded((batch, m))
        bcq.bcq_gemm_mixed(dl.planes, only3, gpu.to_dev(p12), xd, y=out.t)
        assert bcq.last_kernel() == "plane_mfma_rows"
        assert torch.all(out.check("no request has a scale set") == 0)
        scrambled = layer.planes.copy()
        scrambled[2:] = syn.make_planes(m, n, seed=(272, 99))[2:]
        p2 = np.array([2, 1, 2, 2, 1, 2, 1, 2][:batch], dtype=np.int32)
        ya = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(p2), xd)
        yb = bcq.bcq_gemm_mixed(gpu.to_dev(scrambled), dl.scales, gpu.to_dev(p2), xd)
        assert torch.equal(ya, yb), "planes beyond the deepest precision present influenced the result"
    torch.cuda.synchronize()


@pytest.mark.parametrize("ms,n", [((6400, 6400), 4096), ((12300, 1000, 20), 4096), ((14336, 14336), 4096), ((5000, 3000, 2000, 300), 8192)])
def test_row_streaming_form_several_matrices(gpu, oracle, ms, n):
    """bcq_gemv_multi on the row-streaming form: the matrices are taken together when all their rows make a matrix tall
    enough (each of them may be too short on its own); a matrix's last workgroup may hold absent row blocks.  Sampled
    rows against the oracle, and bit for bit the separate calls wherever those run the same form."""
    import torch

    import paper_2510_10467_amd as bcq
    layers = [syn.make_layer(m, n, seed=(273, k, m), signed=True) for k, m in enumerate(ms)]
    dls = [gpu.DeviceLayer(L) for L in layers]
    rng = np.random.default_rng([syn.BASE_SEED, 273, len(ms)])
    for batch in (1, 2, 4, 7):
        x = syn.make_x(batch, n, seed=(273, batch))
        xd = gpu.to_dev(x)
        for p in (2, 4):
            if batch > 4 and n != 4096:
                continue                    # (five to eight requests stream at 4096 columns only)
            outs = [gpu.Guarded((batch, m)) for m in ms]
            bcq.bcq_gemv_multi([d.planes for d in dls], [d.scales[p] for d in dls], p, xd, ys=[o.t for o in outs])
            # (one request streams at one or two planes only, from 896 row blocks in all on)
            single = p <= 2 and sum(ms) > 895 * 16
            assert bcq.last_kernel() == ("plane_mfma_rows" if batch > 1 or single else "plane_mfma"), (ms, batch, p, bcq.last_kernel())
            for k, (L, d, o) in enumerate(zip(layers, dls, outs)):
                y = o.check(f"multi matrix {k} of {ms} batch={batch} p={p}")
                m = L.m
                rows = np.unique(np.concatenate([[0, min(15, m - 1), m - 1, max(m - 17, 0)], rng.integers(0, m, size=40)]))
                sampled_rows_check(gpu, oracle, L, d, p, x, rows, y, f"multi matrix {k} of {ms} batch={batch} p={p}")
                alone = bcq.bcq_gemv(d.planes, d.scales[p], p, xd)
                if bcq.last_kernel() == "plane_mfma_rows":
                    assert torch.equal(alone, y), f"matrix {k} of {ms}: differs from the separate call on the same form"


def test_row_streaming_form_reads_every_binary16_activation_exactly(gpu):
    """The row-streaming form builds its operand image with code of its own: every finite binary16 value, alone in its
    scale group, against rows whose only non-zero scale (1.0, one plane) sits on that group, comes back bit for bit
    (one, two, four and eight requests: one and two request tiles, one and two waves per row block)."""
    import paper_2510_10467_amd as bcq
    values = np.arange(65536, dtype=np.uint16).view(np.float16)
    values = values[np.isfinite(values)]                              # 63488 values
    seen = set()
    for n, batch, launches, m in ((8192, 4, None, 12288), (8192, 2, 40, 12288), (4096, 8, 40, 12288), (8192, 1, 40, 14336), (4096, 1, 40, 14336)):
        groups = n // 128
        rng = np.random.default_rng([syn.BASE_SEED, 271, n])
        planes = rng.integers(0, 2 ** 32, size=(1, m, n // 32), dtype=np.uint32)
        group_of_row = np.arange(m) % groups                          # row r reads group r mod groups
        scales = np.zeros((1, m, groups), dtype=np.float16)
        scales[0, np.arange(m), group_of_row] = 1.0
        cols = np.arange(groups) * 128 + rng.integers(0, 128, size=groups)       # where in its group a value sits
        col_of_row = cols[group_of_row]
        bit = (planes[0, np.arange(m), col_of_row // 32] >> (col_of_row % 32).astype(np.uint32)) & 1
        sign = np.where(bit == 1, 1.0, -1.0)
        x = np.zeros((len(values) // groups, n), dtype=np.float16)
        x[:, cols] = values.reshape(-1, groups)
        planes_d, scales_d = gpu.to_dev(planes), gpu.to_dev(scales)
        for k, start in enumerate(range(0, x.shape[0], batch)):
            if launches is not None and k >= launches:
                break                                                 # two and eight requests only sample
            xb = x[start:start + batch]
            y = bcq.bcq_gemv(planes_d, scales_d, 1, gpu.to_dev(xb)).cpu().numpy()
            seen.add(bcq.last_kernel())
            want = (xb[:, col_of_row].astype(np.float64) * sign[None, :]).astype(np.float16)
            same = (y.view(np.uint16) == want.view(np.uint16)) | ((y == 0) & (want == 0))
            assert np.all(same), (f"n={n} batch {batch}: {np.count_nonzero(~same)} values not reproduced, first "
                                  f"{want[~same][0]!r} -> {y[~same][0]!r}")
    assert seen == {"plane_mfma_rows"}, seen


def test_prefix_invariance_and_determinism(gpu):
    """Only the first p planes are read (section 3.3): scrambling the others leaves y bit-identical;
    repeated launches give bit-identical results."""
    import torch

    import paper_2510_10467_amd as bcq
    m, n = 300, 4096
    layer = syn.make_layer(m, n, seed=(210, 0))
    x = gpu.to_dev(syn.make_x(2, n, seed=(210, 0)))
    for kernel in ("plane_mfma", "sign_select", "lut", "dequant_mfma", "plane_f16"):
        bcq.select_kernel(kernel)
        try:
            for p in (1, 2, 3):
                scrambled = layer.planes.copy()
                scrambled[p:] = syn.make_planes(m, n, seed=(210, p))[p:]
                sc = gpu.to_dev(layer.scales[p])
                y0 = bcq.bcq_gemv(gpu.to_dev(layer.planes), sc, p, x)
                y1 = bcq.bcq_gemv(gpu.to_dev(scrambled), sc, p, x)
                y2 = bcq.bcq_gemv(gpu.to_dev(layer.planes), sc, p, x)
                torch.cuda.synchronize()
                assert torch.equal(y0, y1), f"{kernel}: planes >= p influenced the result"
                assert torch.equal(y0, y2), f"{kernel}: not deterministic"
        finally:
            bcq.select_kernel("auto")


def test_one_hot_readout_and_symmetries(gpu, oracle):
    """x = e_j with power-of-two scales reads W_p[r, j] back exactly; y(-x) = -y(x); complementing
    every plane negates y (all exact in every kernel up to the final rounding)."""
    import torch

    import paper_2510_10467_amd as bcq
    m, n, p = 64, 2048, 3
    planes = syn.make_planes(m, n, seed=(220, 0))
    scales = np.empty((p, m, n // 128), dtype=np.float16)
    scales[0], scales[1], scales[2] = 1.0, 0.25, 0.0625
    w = oracle.dequant(planes, scales)                      # exact: multiples of 1/16 below 2
    cols = [0, 1, 2, 3, 31, 32, 63, 64, 127, 128, 1023, 1024, 1500, 2047]
    x = np.zeros((len(cols), n), dtype=np.float16)
    for b, j in enumerate(cols):
        x[b, j] = 1.0
    xr = syn.make_x(4, n, seed=(220, 1))
    for kernel in ("plane_mfma", "sign_select", "lut", "dequant_mfma", "plane_f16"):
        bcq.select_kernel(kernel)
        try:
            y = bcq.bcq_gemv(gpu.to_dev(planes), gpu.to_dev(scales), p, gpu.to_dev(x)).cpu().numpy().astype(np.float64)
            assert np.array_equal(y, w[:, cols].T), f"{kernel}: one-hot read-out differs"
            ya = bcq.bcq_gemv(gpu.to_dev(planes), gpu.to_dev(scales), p, gpu.to_dev(xr))
            yn = bcq.bcq_gemv(gpu.to_dev(planes), gpu.to_dev(scales), p, gpu.to_dev(-xr))
            yc = bcq.bcq_gemv(gpu.to_dev(~planes), gpu.to_dev(scales), p, gpu.to_dev(xr))
            torch.cuda.synchronize()
            assert torch.equal(yn, -ya), f"{kernel}: y(-x) != -y(x)"
            assert torch.equal(yc, -ya), f"{kernel}: complemented planes do not negate y"
        finally:
            bcq.select_kernel("auto")


@pytest.mark.parametrize("m,n,batch", [(14336, 4096, 16), (14336, 4096, 96), (4096, 14336, 200), (14336, 4096, 400)])
def test_full_size_mixed_precision_sampled_rows(gpu, oracle, m, n, batch):
    """Per-request precision at the benchmark's shapes: the paper-sized batch on the plane-wise fp16 kernel,
    serving-sized ones on the dequantising kernel."""
    import torch

    import paper_2510_10467_amd as bcq
    layer = syn.make_layer(m, n, seed=(231, m, n))
    dl = gpu.DeviceLayer(layer)
    x = syn.make_x(batch, n, seed=(231, batch))
    p_req = syn.make_p_req(batch, 2, 4, seed=(231, batch))
    y = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(p_req), gpu.to_dev(x))
    torch.cuda.synchronize()
    assert bcq.last_kernel() == {16: "plane_f16", 96: "dequant_mfma", 200: "dequant_mfma", 400: "dequant_mfma"}[batch]
    rng = np.random.default_rng([syn.BASE_SEED, 231, m])
    rows = np.unique(np.concatenate([[0, 15, 16, m - 1], rng.integers(0, m, size=60)]))
    sub = {p: np.ascontiguousarray(s[:, rows, :]) for p, s in layer.scales.items()}
    y_ref, a_ref = oracle.gemm_mixed(np.ascontiguousarray(layer.planes[:, rows, :]), sub, p_req, x)
    err = np.abs(y.cpu().numpy().astype(np.float64)[:, rows] - y_ref)
    assert np.all(err <= oracle.tolerance(y_ref, a_ref))


def test_mixed_equals_uniform_per_request_and_request_permutation(gpu):
    import torch

    import paper_2510_10467_amd as bcq
    m, n = 200, 4096
    layer = syn.make_layer(m, n, seed=(230, 0))
    dl = gpu.DeviceLayer(layer)
    batch = 9
    x = syn.make_x(batch, n, seed=(230, 1))
    p_req = np.array([2, 4, 3, 1, 4, 2, 3, 3, 1], dtype=np.int32)
    ym = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(p_req), gpu.to_dev(x))
    for b in range(batch):
        yu = bcq.bcq_gemv(dl.planes, dl.scales[int(p_req[b])], int(p_req[b]), gpu.to_dev(x[b:b + 1]))
        assert torch.equal(ym[b], yu[0]), f"request {b}: mixed result differs from the uniform-precision call"
    perm = np.array([3, 0, 8, 1, 7, 2, 6, 4, 5])
    yp = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(p_req[perm]), gpu.to_dev(np.ascontiguousarray(x[perm])))
    torch.cuda.synchronize()
    assert torch.equal(yp, ym[torch.from_numpy(perm).to(ym.device)])


def test_p_req_is_clamped_and_missing_scale_set_gives_zeros(gpu, oracle):
    import torch

    import paper_2510_10467_amd as bcq
    m, n = 48, 1024
    layer = syn.make_layer(m, n, seed=(240, 0))
    dl = gpu.DeviceLayer(layer)
    x = syn.make_x(4, n, seed=(240, 1))
    for kernel in ("plane_mfma", "sign_select", "lut"):
        bcq.select_kernel(kernel)
        try:
            y = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(np.array([0, 9, -3, 4], dtype=np.int32)), gpu.to_dev(x))
            y_ref, a_ref = oracle.gemm_mixed(layer.planes, layer.scales, [1, 4, 1, 4], x)
            gpu.assert_within_tolerance(y, y_ref, a_ref, f"{kernel}: clamped p_req")
            partial = {2: dl.scales[2], 4: dl.scales[4]}                     # no set for precision 3
            y = bcq.bcq_gemm_mixed(dl.planes, partial, gpu.to_dev(np.array([2, 3, 4, 3], dtype=np.int32)), gpu.to_dev(x))
            torch.cuda.synchronize()
            y_ref, a_ref = oracle.gemm_mixed(layer.planes, layer.scales, [2, 2, 4, 2], x)
            y_ref[[1, 3]] = 0.0
            a_ref[[1, 3]] = 0.0
            gpu.assert_within_tolerance(y, y_ref, a_ref, f"{kernel}: missing scale set")
            assert torch.count_nonzero(y[1]) == 0 and torch.count_nonzero(y[3]) == 0
        finally:
            bcq.select_kernel("auto")


ALL_FAMILIES = ("plane_mfma", "sign_select", "lut", "dequant_mfma", "plane_f16")


def test_extreme_activation_magnitudes(gpu, oracle):
    """Large, tiny and subnormal binary16 activations: every kernel family meets the stated tolerance alone (the
    split of an activation into E5M2 terms is exact over the whole binary16 range)."""
    m, n = 40, 2048
    layer = syn.make_layer(m, n, seed=(250, 0), signed=True)
    dl = gpu.DeviceLayer(layer)
    rng = np.random.default_rng([syn.BASE_SEED, 250])
    x = np.empty((4, n), dtype=np.float16)
    x[0] = (rng.normal(size=n) * 4.0e3).clip(-65504, 65504).astype(np.float16)      # large, products still fit binary16
    x[1] = (rng.normal(size=n) * 1e-2).astype(np.float16)
    x[2] = (rng.normal(size=n) * 3e-6).astype(np.float16)                             # mostly subnormal
    x[3] = 0.0
    x[3, ::16] = np.where(rng.random(n // 16) < 0.5, 65504.0, -65504.0)               # the largest finite binary16 values
    for kernel in ALL_FAMILIES:
        gpu.check_gemv(dl, 3, x, kernel)
        for b in range(4):
            gpu.check_gemv(dl, 3, x[b:b + 1], kernel)


@pytest.mark.parametrize("m,n", [(131, 4096), (50, 28672)])
def test_small_and_mixed_magnitude_activations(gpu, oracle, m, n):
    """Activations N(0, sigma^2) for sigma down to the subnormal range, and vectors that mix magnitudes of 1e4 and
    1e-5, at batches 1, 2, 4 and 7 and every precision, with each kernel family forced."""
    layer = syn.make_layer(m, n, seed=(251, m))
    dl = gpu.DeviceLayer(layer)
    rng = np.random.default_rng([syn.BASE_SEED, 251, m])
    vectors = [syn.make_x(1, n, seed=(251, k), scale=sigma)[0] for k, sigma in enumerate((1e-2, 1e-3, 1e-4, 3e-6))]
    big = rng.random(n) < 0.5
    large = 1e4 if n <= 4096 else 2.5e3            # so that the results of the long rows still fit binary16
    vectors.append(np.where(big, rng.normal(size=n) * large, rng.normal(size=n) * 1e-5).astype(np.float16))
    mostly_small = rng.random(n) < 1.0 / 64.0                                          # a few large values per group
    vectors.append(np.where(mostly_small, rng.normal(size=n) * 1e4, rng.normal(size=n) * 1e-5).astype(np.float16))
    vectors.append(syn.make_x(1, n, seed=(251, 9))[0])
    x_all = np.stack(vectors)                                                          # 7 requests
    for kernel in ALL_FAMILIES:
        for p in (1, 2, 3, 4):
            for batch in (1, 2, 4, 7):
                for start in range(0, 7, batch):
                    xb = x_all[start:start + batch]
                    if len(xb) == batch or batch == 7:
                        gpu.check_gemv(dl, p, xb, kernel)
    # per-request precision on the same vectors
    p_req = np.array([1, 2, 3, 4, 4, 2, 3], dtype=np.int32)
    for kernel in ALL_FAMILIES:
        gpu.check_mixed(dl, p_req, x_all, kernel)
        gpu.check_mixed(dl, p_req[:3], x_all[:3], kernel)


@pytest.mark.parametrize("kernel", ALL_FAMILIES)
def test_every_binary16_activation_is_read_exactly(gpu, kernel):
    """Every finite binary16 value as an activation, alone in its scale group, against a row whose only non-zero
    scale (1.0, one plane) sits on that group: y must be the value itself or its negative, bit for bit."""
    import torch

    import paper_2510_10467_amd as bcq
    groups = 256                                   # values per request
    n, m = groups * 128, groups
    rng = np.random.default_rng([syn.BASE_SEED, 252])
    planes = rng.integers(0, 2 ** 32, size=(1, m, n // 32), dtype=np.uint32)
    scales = np.zeros((1, m, groups), dtype=np.float16)
    scales[0, np.arange(m), np.arange(m)] = 1.0    # row r reads group r
    pos = rng.integers(0, 128, size=groups)        # where in its group a value sits
    cols = np.arange(groups) * 128 + pos
    bit = (planes[0, np.arange(m), cols // 32] >> (cols % 32).astype(np.uint32)) & 1
    sign = np.where(bit == 1, 1.0, -1.0)
    patterns = np.arange(65536, dtype=np.uint16)
    values = patterns.view(np.float16)
    values = values[np.isfinite(values)]           # 63488 values = 248 requests of 256
    assert len(values) % groups == 0
    x = np.zeros((len(values) // groups, n), dtype=np.float16)
    x[:, cols] = values.reshape(-1, groups)
    planes_d, scales_d = gpu.to_dev(planes), gpu.to_dev(scales)
    expect = (values.reshape(-1, groups).astype(np.float64) * sign[None, :]).astype(np.float16)
    bcq.select_kernel(kernel)
    try:
        for batch in (1, 2, 4, 7, 31):
            for start in range(0, x.shape[0], batch):
                xb = x[start:start + batch]
                y = bcq.bcq_gemv(planes_d, scales_d, 1, gpu.to_dev(xb)).cpu().numpy()
                want = expect[start:start + batch]
                same = (y.view(np.uint16) == want.view(np.uint16)) | ((y == 0) & (want == 0))
                assert np.all(same), (f"{kernel} batch {batch}: {np.count_nonzero(~same)} values not reproduced, first "
                                      f"{want[~same][0]!r} -> {y[~same][0]!r}")
                if batch in (7, 31) and start > 3 * batch:
                    break                           # the larger batches only sample
    finally:
        bcq.select_kernel("auto")
    torch.cuda.synchronize()


def test_graph_replay_matches_eager(gpu):
    """The launches are capturable; several replays with eager work in between stay bit-identical."""
    import torch

    import paper_2510_10467_amd as bcq
    m, n = 512, 4096
    layer = syn.make_layer(m, n, seed=(260, 0))
    dl = gpu.DeviceLayer(layer)
    x = gpu.to_dev(syn.make_x(2, n, seed=(260, 1)))
    p_req = gpu.to_dev(np.array([3, 2], dtype=np.int32))
    y1 = torch.empty((2, m), dtype=torch.float16, device=x.device)
    y2 = torch.empty_like(y1)
    eager1 = bcq.bcq_gemv(dl.planes, dl.scales[4], 4, x).clone()
    eager2 = bcq.bcq_gemm_mixed(dl.planes, dl.scales, p_req, x).clone()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        bcq.bcq_gemv(dl.planes, dl.scales[4], 4, x, y1)
        bcq.bcq_gemm_mixed(dl.planes, dl.scales, p_req, x, y2)
    for _ in range(3):
        y1.zero_()
        y2.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y1, eager1) and torch.equal(y2, eager2)
        _ = bcq.bcq_gemv(dl.planes, dl.scales[2], 2, x)          # eager work between replays
        torch.cuda.synchronize()


def test_large_pack_round_trip(gpu, oracle):
    import paper_2510_10467_amd as bcq
    raw = syn.make_planes(4096, 4096, seed=(270, 0))
    codes = bcq.bcq_unpack(gpu.to_dev(raw))
    again = bcq.bcq_pack(codes)
    assert np.array_equal(again.cpu().numpy().view(np.uint32), raw)
    sample = codes[:, :8, :].cpu().numpy()
    assert np.array_equal(sample, oracle.unpack(np.ascontiguousarray(raw[:, :8, :])))
