"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element,
on the same seeded inputs.  Integer work (packing) is bit-exact; products must satisfy
|y - y_ref| <= 4e-3 * sum_j |W_p[r,j] x_j| + one binary16 ulp."""
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


def test_pack_unpack_bit_exact(gpu, oracle):
    import torch

    import paper_2510_10467_amd as bcq
    for (P, m, n, seed) in [(4, 37, 4096, 0), (1, 1, 32, 1), (3, 130, 224, 2), (8, 5, 1024, 3)]:
        codes = syn.make_codes(P, m, n, seed=(100, seed))
        if seed == 2:
            codes[0, 0, :8] = [0, -5, 127, -128, 1, 2, 0, 0]      # zero / negative mean -1, any positive means +1
        planes = bcq.bcq_pack(gpu.to_dev(codes))
        torch.cuda.synchronize()
        host = oracle.pack(codes)
        assert np.array_equal(planes.cpu().numpy().view(np.uint32), host), f"pack P={P} m={m} n={n}"
        back = bcq.bcq_unpack(planes)
        assert np.array_equal(back.cpu().numpy(), oracle.unpack(host))
        raw = syn.make_planes(m, n, p_max=P, seed=(100, seed))
        again = bcq.bcq_pack(bcq.bcq_unpack(gpu.to_dev(raw)))
        assert np.array_equal(again.cpu().numpy().view(np.uint32), raw), "pack(unpack(w)) != w"


SMALL_SHAPES = [
    # m, n, group: several tiles plus ragged tails in m, odd group counts in n
    (1, 128, 128), (16, 1024, 128), (37, 2048, 128), (131, 4096, 128), (70, 1536, 128), (33, 640, 128),
    (19, 256, 64), (8, 96, 32), (40, 5120, 128),
]


GENERIC_KERNELS = ("sign_select", "lut")      # the two kernels that take every legal shape


@pytest.mark.parametrize("kernel", GENERIC_KERNELS)
@pytest.mark.parametrize("m,n,group", SMALL_SHAPES + [(200, 6240, 96), (67, 2080, 32), (129, 4096, 128)])
def test_generic_kernels_uniform(gpu, m, n, group, kernel):
    """(with the table look-ups: one and several table tiles of 2048 columns, a ragged last tile, more and fewer rows
    than a workgroup's 64, one and two request tiles of four)"""
    layer = syn.make_layer(m, n, group=group, seed=(110, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (1, 3, 5):
        x = syn.make_x(batch, n, seed=(110, batch))
        for p in (1, 2, 3, 4):
            used, _ = gpu.check_gemv(dl, p, x, kernel, group)
            assert used == kernel


@pytest.mark.parametrize("kernel", GENERIC_KERNELS)
@pytest.mark.parametrize("m,n,group", [(37, 2048, 128), (16, 1024, 128), (19, 256, 64), (70, 4160, 32)])
def test_generic_kernels_mixed(gpu, m, n, group, kernel):
    layer = syn.make_layer(m, n, group=group, seed=(120, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (1, 6, 16):
        x = syn.make_x(batch, n, seed=(120, batch))
        p_req = syn.make_p_req(batch, 1, 4, seed=(120, batch))
        gpu.check_mixed(dl, p_req, x, kernel, group)


@pytest.mark.parametrize("kernel", GENERIC_KERNELS + ("auto",))
@pytest.mark.parametrize("m,n,group", [(70, 4224, 128), (9, 256, 64), (300, 2048, 128)])
def test_five_to_eight_planes(gpu, m, n, group, kernel):
    """The ABI takes up to eight planes; beyond four they run on the table look-ups (the default) or the per-bit kernel:
    uniform precision 5 to 8, and per-request precision drawn from 1 to 8 with planes stored to 8."""
    layer = syn.make_layer(m, n, p_max=8, group=group, seed=(125, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (1, 3):
        x = syn.make_x(batch, n, seed=(125, batch))
        for p in (5, 6, 7, 8):
            used, _ = gpu.check_gemv(dl, p, x, kernel, group)
            assert used == ("lut" if kernel == "auto" else kernel)
        p_req = syn.make_p_req(batch, 1, 8, seed=(125, batch))
        p_req[0] = 8
        used, _ = gpu.check_mixed(dl, p_req, x, kernel, group)
        assert used == ("lut" if kernel == "auto" else kernel)


@pytest.fixture
def forced_shape():
    """Force a workgroup shape of the large-batch kernel ("tiles,row blocks") for one test."""
    import paper_2510_10467_amd as bcq

    def force(shape):
        tiles, rows = (int(v) for v in shape.split(","))
        bcq.select_dequant_shape(tiles, rows)
    yield force
    bcq.select_dequant_shape(0, 0)


PLANE_MFMA_SHAPES = [
    # m, n: one and several K slices of 1024 columns, ragged row tails, chunked K (n = 28672),
    # short last slices of 2, 6, 1+... groups (n a multiple of 256 but not of 1024; 17920 is the Phi-4 width)
    (16, 1024), (37, 2048), (131, 4096), (40, 5120), (75, 14336), (50, 28672), (1, 1024), (530, 3072),
    (37, 1280), (33, 1792), (16, 2304), (20, 17920), (17, 3840),
]


@pytest.mark.parametrize("m,n", PLANE_MFMA_SHAPES)
def test_plane_mfma_uniform(gpu, m, n):
    layer = syn.make_layer(m, n, seed=(130, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (1, 2, 3, 4, 7):
        x = syn.make_x(batch, n, seed=(130, batch))
        for p in (1, 2, 3, 4):
            used, _ = gpu.check_gemv(dl, p, x, "plane_mfma")
            assert used == "plane_mfma"


@pytest.mark.parametrize("m,n", [(37, 2048), (131, 4096), (75, 14336), (37, 1280), (20, 17920)])
def test_plane_mfma_mixed(gpu, m, n):
    layer = syn.make_layer(m, n, seed=(140, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (1, 4, 6, 16):
        x = syn.make_x(batch, n, seed=(140, batch))
        p_req = syn.make_p_req(batch, 1, 4, seed=(140, batch))
        gpu.check_mixed(dl, p_req, x, "plane_mfma")


@pytest.mark.parametrize("kernel", ["dequant_mfma", "plane_f16"])
@pytest.mark.parametrize("m,n", [(37, 2048), (131, 4096), (70, 1536), (64, 640), (200, 8192)])
def test_dequant_mfma_uniform(gpu, m, n, kernel):
    """Both large-batch variants: weights rebuilt in fp16 (dequant_mfma), or the +-1 planes multiplied
    themselves and the group sums scaled in fp32 (plane_f16)."""
    layer = syn.make_layer(m, n, seed=(150, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (1, 17, 64, 100, 256):
        x = syn.make_x(batch, n, seed=(150, batch))
        for p in (1, 2, 3, 4):
            used, _ = gpu.check_gemv(dl, p, x, kernel)
            assert used == kernel


@pytest.mark.parametrize("kernel", ["dequant_mfma", "plane_f16"])
@pytest.mark.parametrize("shape", ["0,4", "0,2", "0,1", "0,8", "32,4", "32,2", "32,1", "32,8", "1,4", "1,2", "1,1", "2,4", "2,2", "4,4", "4,8", "4,40", "2,8"])
def test_dequant_mfma_every_workgroup_shape(gpu, shape, forced_shape, kernel):
    """The kernel picks its workgroup shape (request tiles, row blocks) from m and the batch; small test
    matrices would only ever see one of them, so each is forced here (ragged rows, ragged request tiles;
    "0" is the tile of 16 requests, "32" that of 32; row-block code 8 is one row block with eight teams)."""
    forced_shape(shape)
    layer = syn.make_layer(200, 1536, seed=(151, 0), signed=True)
    dl = gpu.DeviceLayer(layer)
    offsets = syn.make_offsets(3, 200, 1536, seed=(151, 1))
    for batch in (3, 16, 32, 64, 100, 257):
        x = syn.make_x(batch, 1536, seed=(151, batch))
        for p in (2, 4):
            used, _ = gpu.check_gemv(dl, p, x, kernel)
            assert used == kernel
        gpu.check_gemv(dl, 3, x, kernel, offsets=offsets)


@pytest.mark.parametrize("m,n", [(37, 2048), (20, 1536), (33, 3584), (130, 4096)])
def test_plane_mfma_groups_of_256(gpu, m, n):
    """Scale groups of 256 columns: four scales per K slice, each serving two matrix instructions; 1536 and
    3584 end in a half slice."""
    layer = syn.make_layer(m, n, group=256, seed=(152, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    zs = {p: syn.make_offsets(p, m, n, 256, seed=(152, m)) for p in (2, 3)}
    for batch in (1, 2, 3, 9):
        x = syn.make_x(batch, n, seed=(152, batch))
        for p in (1, 2, 3, 4):
            used, _ = gpu.check_gemv(dl, p, x, "plane_mfma", 256)
            assert used == "plane_mfma"
        gpu.check_gemv(dl, 3, x, "plane_mfma", 256, offsets=zs[3])
        p_req = syn.make_p_req(batch, 1, 4, seed=(152, batch))
        gpu.check_mixed(dl, p_req, x, "plane_mfma", 256)
        gpu.check_mixed(dl, p_req, x, "plane_mfma", 256, offsets_by_p=zs)
    used, _ = gpu.check_gemv(dl, 2, syn.make_x(1, n, seed=(152, 99)), "auto", 256)
    assert used == "plane_mfma"


@pytest.mark.parametrize("m,n", [(37, 2048), (20, 1024), (130, 4096), (24, 9216)])
def test_plane_mfma_groups_of_64(gpu, m, n):
    """Scale groups of 64 columns: sixteen scales per K slice, one matrix instruction per half group.
    9216 columns run as two chunks of slices."""
    layer = syn.make_layer(m, n, group=64, seed=(156, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (1, 2, 3, 9):
        x = syn.make_x(batch, n, seed=(156, batch))
        for p in (1, 2, 3, 4):
            used, _ = gpu.check_gemv(dl, p, x, "plane_mfma", 64)
            assert used == "plane_mfma"
        p_req = syn.make_p_req(batch, 1, 4, seed=(156, batch))
        gpu.check_mixed(dl, p_req, x, "plane_mfma", 64)
    used, _ = gpu.check_gemv(dl, 2, syn.make_x(1, n, seed=(156, 99)), "auto", 64)
    assert used == "plane_mfma"
    # the asymmetric scheme: an offset per 64 columns times the sum of that half of a matrix instruction's columns
    zs = {p: syn.make_offsets(p, m, n, 64, seed=(156, p)) for p in (1, 2, 3, 4)}
    for batch in (1, 2, 4, 7):
        x = syn.make_x(batch, n, seed=(157, batch))
        for p in (1, 2, 4):
            used, _ = gpu.check_gemv(dl, p, x, "plane_mfma", 64, offsets=zs[p])
            assert used == "plane_mfma"
        p_req = syn.make_p_req(batch, 1, 4, seed=(157, batch))
        gpu.check_mixed(dl, p_req, x, "plane_mfma", 64, offsets_by_p=zs)
        gpu.check_mixed(dl, p_req, x, "plane_mfma", 64, offsets_by_p={2: zs[2], 4: zs[4]})   # precisions 1 and 3 have none
    used, _ = gpu.check_gemv(dl, 2, syn.make_x(1, n, seed=(156, 98)), "auto", 64, offsets=zs[2])
    assert used == "plane_mfma"


@pytest.mark.parametrize("kernel", ["dequant_mfma", "plane_f16"])
@pytest.mark.parametrize("group", [64, 256])
def test_dequant_mfma_other_group_sizes(gpu, group, kernel):
    import paper_2510_10467_amd as bcq
    layer = syn.make_layer(150, 1536, group=group, seed=(153, group), signed=True)
    dl = gpu.DeviceLayer(layer)
    if kernel == "plane_f16" and group == 64:
        # its matrix instruction sums over the 128 columns of a step, which would mix two groups of 64
        bcq.select_kernel(kernel)
        try:
            with pytest.raises(bcq.BcqError) as e:
                bcq.bcq_gemv(dl.planes, dl.scales[2], 2, gpu.to_dev(syn.make_x(5, 1536, seed=(153, 5))), group=64)
            assert e.value.status == -6
        finally:
            bcq.select_kernel("auto")
        return
    offsets = syn.make_offsets(2, 150, 1536, group, seed=(153, 1))
    for batch in (5, 64, 130):
        x = syn.make_x(batch, 1536, seed=(153, batch))
        for p in (1, 3, 4):
            used, _ = gpu.check_gemv(dl, p, x, kernel, group)
            assert used == kernel
        gpu.check_gemv(dl, 2, x, kernel, group, offsets=offsets)


@pytest.mark.parametrize("kernel", ["dequant_mfma", "plane_f16"])
@pytest.mark.parametrize("rows", ["1,4", "1,2", "1,1", "0,8", "32,2", "32,1", "32,8"])
def test_dequant_mfma_mixed(gpu, rows, forced_shape, kernel):
    """Per-request precision on the large-batch kernels (weights rebuilt per precision present, or the planes
    multiplied once and every request's own scales applied to the group sums): every workgroup shape, ragged
    rows and request tiles, tiles in which one, some or all precisions occur, a precision without a scale set
    (zeros), precisions outside [1, p_max] (clamped), offsets for some precisions only."""
    forced_shape(rows)
    m, n = 150, 1536
    layer = syn.make_layer(m, n, seed=(154, 0), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (5, 16, 32, 64, 130):
        x = syn.make_x(batch, n, seed=(154, batch))
        p_req = syn.make_p_req(batch, 1, 4, seed=(154, batch))
        used, _ = gpu.check_mixed(dl, p_req, x, kernel)
        assert used == kernel
        gpu.check_mixed(dl, np.full(batch, 3, dtype=np.int32), x, kernel)           # one precision only
        two = np.where(np.arange(batch) % 2 == 0, 2, 4).astype(np.int32)
        gpu.check_mixed(dl, two, x, kernel)
    zs = {p: syn.make_offsets(p, m, n, seed=(154, p)) for p in (2, 4)}
    x = syn.make_x(70, n, seed=(154, 70))
    p_req = syn.make_p_req(70, 1, 4, seed=(154, 71))
    gpu.check_mixed(dl, p_req, x, kernel, offsets_by_p=zs)
    if kernel == "plane_f16":
        wide = gpu.DeviceLayer(syn.make_layer(70, 2048, group=256, seed=(154, 9), signed=True))
        zw = {p: syn.make_offsets(p, 70, 2048, 256, seed=(154, p)) for p in (3,)}
        gpu.check_mixed(wide, syn.make_p_req(13, 1, 4, seed=(154, 13)), syn.make_x(13, 2048, seed=(154, 13)), kernel, 256, offsets_by_p=zw)


@pytest.mark.parametrize("kernel", ["dequant_mfma", "plane_f16"])
def test_dequant_mfma_mixed_clamps_and_missing_sets(gpu, kernel):
    import torch

    import paper_2510_10467_amd as bcq
    m, n, batch = 100, 1024, 40
    layer = syn.make_layer(m, n, seed=(155, 0))
    dl = gpu.DeviceLayer(layer)
    x = syn.make_x(batch, n, seed=(155, 1))
    wild = np.array([0, -3, 9, 2, 3] * 8, dtype=np.int32)                 # clamped to 1, 1, 4, 2, 3
    clamped = np.clip(wild, 1, 4).astype(np.int32)
    bcq.select_kernel(kernel)
    try:
        y_wild = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(wild), gpu.to_dev(x))
        y_ok = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(clamped), gpu.to_dev(x))
        some = {p: s for p, s in dl.scales.items() if p != 3}              # no scale set for precision 3
        y_some = bcq.bcq_gemm_mixed(dl.planes, some, gpu.to_dev(clamped), gpu.to_dev(x))
        torch.cuda.synchronize()
        assert bcq.last_kernel() == kernel
    finally:
        bcq.select_kernel("auto")
    assert torch.equal(y_wild, y_ok)
    is3 = torch.from_numpy(clamped == 3).to(y_ok.device)
    assert torch.all(y_some[is3] == 0) and torch.equal(y_some[~is3], y_ok[~is3])


@pytest.mark.parametrize("shape", ["1,4", "1,2", "1,1", "2,4", "2,2", "4,4", "4,8", "4,40", "2,8", None])
def test_per_request_precision_one_launch_per_precision(gpu, shape, forced_shape):
    """Beyond 64 requests `dequant_mfma` serves a batch with per-request precision by one launch of the uniform
    kernel per precision, each workgroup picking the requests of that precision out of the batch by rank:
    every workgroup shape of that path, ragged last tiles, precisions in runs and interleaved, a precision
    nobody has, everybody at one precision, more than 1024 requests (the ranking goes in blocks of 1024),
    clamped precisions, a precision without a scale set (zeros), offsets for some precisions only."""
    import torch

    import paper_2510_10467_amd as bcq
    if shape:
        forced_shape(shape)
    m, n = 150, 1536
    dl = gpu.DeviceLayer(syn.make_layer(m, n, seed=(158, 0), signed=True))
    for batch in (65, 130, 300, 1100):
        x = syn.make_x(batch, n, seed=(158, batch))
        drawn = syn.make_p_req(batch, 1, 4, seed=(158, batch))
        cases = [drawn, np.sort(drawn), np.full(batch, 2, dtype=np.int32), np.where(np.arange(batch) % 3 == 0, 4, 3).astype(np.int32)]
        for p_req in cases[:4 if batch <= 300 else 1]:
            used, _ = gpu.check_mixed(dl, p_req.astype(np.int32), x, "dequant_mfma")
            assert used == "dequant_mfma"
    zs = {p: syn.make_offsets(p, m, n, seed=(158, p)) for p in (1, 3)}
    x = syn.make_x(200, n, seed=(158, 200))
    gpu.check_mixed(dl, syn.make_p_req(200, 1, 4, seed=(158, 201)), x, "dequant_mfma", offsets_by_p=zs)
    wild = np.array([0, -3, 9, 2, 3] * 40, dtype=np.int32)                # clamped to 1, 1, 4, 2, 3
    clamped = np.clip(wild, 1, 4).astype(np.int32)
    bcq.select_kernel("dequant_mfma")
    try:
        y_wild = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(wild), gpu.to_dev(x))
        y_ok = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(clamped), gpu.to_dev(x))
        some = {p: s for p, s in dl.scales.items() if p != 3}              # no scale set for precision 3
        y_some = bcq.bcq_gemm_mixed(dl.planes, some, gpu.to_dev(clamped), gpu.to_dev(x), y=torch.full_like(y_ok, 7.0))
        torch.cuda.synchronize()
    finally:
        bcq.select_kernel("auto")
    assert torch.equal(y_wild, y_ok)
    is3 = torch.from_numpy(clamped == 3).to(y_ok.device)
    assert torch.all(y_some[is3] == 0) and torch.equal(y_some[~is3], y_ok[~is3])


def test_forced_variant_and_last_kernel_are_per_thread(gpu):
    """One thread forces the generic kernel; another, launching at the same time, keeps the default choice, and each
    reads its own last kernel."""
    import threading

    import torch

    import paper_2510_10467_amd as bcq
    layer = syn.make_layer(64, 2048, seed=(185, 0))
    dl = gpu.DeviceLayer(layer)
    x = gpu.to_dev(syn.make_x(1, 2048, seed=(185, 1)))
    seen, forced, done = {}, threading.Event(), threading.Event()

    def forcing():
        bcq.select_kernel("sign_select")
        forced.set()
        bcq.bcq_gemv(dl.planes, dl.scales[2], 2, x)
        done.wait(30)
        seen["forcing"] = bcq.last_kernel()
        bcq.select_kernel("auto")

    def default():
        forced.wait(30)
        bcq.bcq_gemv(dl.planes, dl.scales[2], 2, x)
        seen["default"] = bcq.last_kernel()
        done.set()

    threads = [threading.Thread(target=forcing), threading.Thread(target=default)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(60)
    torch.cuda.synchronize()
    assert seen == {"forcing": "sign_select", "default": "plane_mfma"}


def test_forced_variant_that_cannot_run_is_an_error(gpu):
    import paper_2510_10467_amd as bcq
    layer = syn.make_layer(16, 640, seed=(160, 0))            # n is shorter than one K slice
    dl = gpu.DeviceLayer(layer)
    x = gpu.to_dev(syn.make_x(1, 640, seed=(160, 0)))
    bcq.select_kernel("plane_mfma")
    try:
        with pytest.raises(bcq.BcqError) as e:
            bcq.bcq_gemv(dl.planes, dl.scales[2], 2, x)
        assert e.value.status == -6
    finally:
        bcq.select_kernel("auto")
    # the default choice falls back to a kernel that can
    gpu.check_gemv(dl, 2, syn.make_x(1, 640, seed=(160, 0)), "auto")


def test_auto_dispatch_by_batch(gpu):
    layer = syn.make_layer(96, 2048, seed=(170, 0))
    dl = gpu.DeviceLayer(layer)
    used, _ = gpu.check_gemv(dl, 3, syn.make_x(1, 2048, seed=(170, 1)), "auto")
    assert used == "plane_mfma"
    used, _ = gpu.check_gemv(dl, 3, syn.make_x(16, 2048, seed=(170, 2)), "auto")
    assert used == "plane_mfma"
    used, _ = gpu.check_gemv(dl, 3, syn.make_x(128, 2048, seed=(170, 3)), "auto")
    assert used == "plane_mfma"            # too few rows for the dequantising kernel to pay
    big = gpu.DeviceLayer(syn.make_layer(4096, 1024, seed=(171, 0)))
    used, _ = gpu.check_gemv(big, 3, syn.make_x(8, 1024, seed=(171, 1)), "auto")
    assert used == "plane_mfma"
    used, _ = gpu.check_gemv(big, 3, syn.make_x(9, 1024, seed=(171, 6)), "auto")      # 4096 rows: from 9 requests on,
    assert used == "plane_f16"                                                         # one tile of 16: planes multiplied as they are
    used, _ = gpu.check_gemv(big, 3, syn.make_x(64, 1024, seed=(171, 2)), "auto")
    assert used == "dequant_mfma"
    p_req = syn.make_p_req(40, 1, 4, seed=(170, 4))
    used, _ = gpu.check_mixed(dl, p_req, syn.make_x(40, 2048, seed=(170, 4)), "auto")
    assert used == "plane_mfma"            # 96 rows: too short for the dequantising kernel
    used, _ = gpu.check_mixed(big, p_req, syn.make_x(40, 1024, seed=(171, 4)), "auto")  # 40 requests: tiles of 16
    assert used == "plane_f16"
    p_many = syn.make_p_req(130, 1, 4, seed=(171, 7))
    used, _ = gpu.check_mixed(big, p_many, syn.make_x(130, 1024, seed=(171, 7)), "auto")
    assert used == "dequant_mfma"
    used, _ = gpu.check_mixed(big, p_many[:97], syn.make_x(97, 1024, seed=(171, 9)), "auto")   # beyond 96: one pass per precision
    assert used == "dequant_mfma"
    used, _ = gpu.check_mixed(big, p_many[:96], syn.make_x(96, 1024, seed=(171, 10)), "auto")
    assert used == "plane_f16"
    used, _ = gpu.check_mixed(big, p_req[:16], syn.make_x(16, 1024, seed=(171, 5)), "auto")
    assert used == "plane_f16"
    used, _ = gpu.check_mixed(big, p_req[:8], syn.make_x(8, 1024, seed=(171, 8)), "auto")
    assert used == "plane_mfma"
    short = gpu.DeviceLayer(syn.make_layer(2048, 1024, seed=(173, 0)))         # 2048 rows: the large-batch kernel from 40 requests on
    used, _ = gpu.check_gemv(short, 4, syn.make_x(32, 1024, seed=(173, 1)), "auto")
    assert used == "plane_mfma"
    used, _ = gpu.check_gemv(short, 4, syn.make_x(48, 1024, seed=(173, 2)), "auto")
    assert used == "dequant_mfma"
    used, _ = gpu.check_mixed(short, p_req[:30], syn.make_x(30, 1024, seed=(173, 3)), "auto")
    assert used == "plane_mfma"
    used, _ = gpu.check_mixed(short, p_req, syn.make_x(40, 1024, seed=(173, 4)), "auto")
    assert used == "plane_f16"
    tall = gpu.DeviceLayer(syn.make_layer(8192, 1024, seed=(172, 0)))          # 8192 rows: the crossover sits at 9 requests (5 for p <= 2)
    used, _ = gpu.check_gemv(tall, 3, syn.make_x(8, 1024, seed=(172, 1)), "auto")
    assert used == "plane_mfma"
    used, _ = gpu.check_gemv(tall, 3, syn.make_x(9, 1024, seed=(172, 2)), "auto")
    assert used == "plane_f16"
    used, _ = gpu.check_gemv(tall, 3, syn.make_x(17, 1024, seed=(172, 6)), "auto")      # one tile of 32
    assert used == "plane_f16"
    used, _ = gpu.check_gemv(tall, 3, syn.make_x(33, 1024, seed=(172, 9)), "auto")
    assert used == "dequant_mfma"
    used, _ = gpu.check_gemv(tall, 2, syn.make_x(4, 1024, seed=(172, 4)), "auto")
    assert used == "plane_mfma"
    used, _ = gpu.check_gemv(tall, 2, syn.make_x(5, 1024, seed=(172, 5)), "auto")
    assert used == "plane_f16"
    used, _ = gpu.check_mixed(tall, p_req[:30], syn.make_x(30, 1024, seed=(172, 3)), "auto")
    assert used == "plane_f16"
    used, _ = gpu.check_mixed(tall, p_many[:64], syn.make_x(64, 1024, seed=(172, 7)), "auto")    # tiles of 32 requests up to 64
    assert used == "plane_f16"
    used, _ = gpu.check_mixed(tall, p_many[:65], syn.make_x(65, 1024, seed=(172, 9)), "auto")    # beyond: one pass per precision
    assert used == "dequant_mfma"
    used, _ = gpu.check_mixed(tall, p_req[:8], syn.make_x(8, 1024, seed=(172, 8)), "auto")
    assert used == "plane_mfma"


# ----------------------------------------------------------------------------
# asymmetric scheme: offsets per (row, group) and precision, every kernel family
# ----------------------------------------------------------------------------
OFFSET_SHAPES = [(16, 1024), (37, 2048), (131, 4096), (20, 17920), (33, 1792), (50, 28672)]


@pytest.mark.parametrize("m,n", OFFSET_SHAPES)
def test_offsets_plane_mfma(gpu, m, n):
    layer = syn.make_layer(m, n, seed=(180, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    zs = {p: syn.make_offsets(p, m, n, seed=(180, m)) for p in (1, 2, 3, 4)}
    for batch in (1, 2, 4, 7):
        x = syn.make_x(batch, n, seed=(180, batch))
        for p in (1, 2, 3, 4):
            used, _ = gpu.check_gemv(dl, p, x, "plane_mfma", offsets=zs[p])
            assert used == "plane_mfma"
    for batch in (1, 6, 16):
        x = syn.make_x(batch, n, seed=(181, batch))
        p_req = syn.make_p_req(batch, 1, 4, seed=(181, batch))
        gpu.check_mixed(dl, p_req, x, "plane_mfma", offsets_by_p=zs)
        gpu.check_mixed(dl, p_req, x, "plane_mfma", offsets_by_p={2: zs[2], 4: zs[4]})   # precisions 1 and 3 have none


@pytest.mark.parametrize("kernel", GENERIC_KERNELS)
@pytest.mark.parametrize("m,n,group", [(37, 2048, 128), (33, 640, 128), (9, 512, 64), (5, 96, 32), (70, 4160, 64)])
def test_offsets_generic_kernels(gpu, m, n, group, kernel):
    layer = syn.make_layer(m, n, group=group, seed=(182, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    zs = {p: syn.make_offsets(p, m, n, group, seed=(182, m)) for p in (1, 2, 3, 4)}
    for batch in (1, 5):
        x = syn.make_x(batch, n, seed=(182, batch))
        for p in (1, 3, 4):
            gpu.check_gemv(dl, p, x, kernel, group, offsets=zs[p])
        p_req = syn.make_p_req(batch, 1, 4, seed=(182, batch))
        gpu.check_mixed(dl, p_req, x, kernel, group, offsets_by_p={1: zs[1], 3: zs[3]})


@pytest.mark.parametrize("m,n", [(37, 2048), (131, 4096), (64, 640)])
def test_offsets_dequant_mfma(gpu, m, n):
    layer = syn.make_layer(m, n, seed=(183, m), signed=True)
    dl = gpu.DeviceLayer(layer)
    for batch in (1, 64, 100, 256):
        x = syn.make_x(batch, n, seed=(183, batch))
        for p in (1, 2, 4):
            z = syn.make_offsets(p, m, n, seed=(183, m))
            used, _ = gpu.check_gemv(dl, p, x, "dequant_mfma", offsets=z)
            assert used == "dequant_mfma"


def test_offsets_change_the_result_and_null_is_symmetric(gpu):
    import torch

    import paper_2510_10467_amd as bcq
    layer = syn.make_layer(48, 2048, seed=(184, 0))
    dl = gpu.DeviceLayer(layer)
    x = gpu.to_dev(syn.make_x(3, 2048, seed=(184, 0)))
    z = gpu.to_dev(syn.make_offsets(3, 48, 2048, seed=(184, 0)))
    y_sym = bcq.bcq_gemv(dl.planes, dl.scales[3], 3, x)
    y_off = bcq.bcq_gemv(dl.planes, dl.scales[3], 3, x, offsets=z)
    y_zero = bcq.bcq_gemv(dl.planes, dl.scales[3], 3, x, offsets=torch.zeros_like(z))
    assert not torch.equal(y_sym, y_off)
    assert torch.equal(y_sym, y_zero)


# ----------------------------------------------------------------------------
# several matrices on the same activations in one call (q/k/v, gate/up)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("ms,n", [((64, 16, 16), 1024), ((37, 50), 2048), ((131, 16, 75, 1), 4096), ((40, 24), 17920), ((20,), 1024)])
def test_gemv_multi_equals_separate_calls(gpu, oracle, ms, n):
    import torch

    import paper_2510_10467_amd as bcq
    layers = [syn.make_layer(m, n, seed=(190, k, m), signed=True) for k, m in enumerate(ms)]
    dls = [gpu.DeviceLayer(layer) for layer in layers]
    for batch in (1, 3, 4, 9):
        xh = syn.make_x(batch, n, seed=(190, batch))
        x = gpu.to_dev(xh)
        for p in (1, 2, 3, 4):
            outs = [gpu.Guarded((batch, m)) for m in ms]
            bcq.bcq_gemv_multi([d.planes for d in dls], [d.scales[p] for d in dls], p, x, ys=[o.t for o in outs])
            ys = [o.check(f"bcq_gemv_multi ms={ms} n={n} p={p} batch={batch}, output {k}") for k, o in enumerate(outs)]
            assert bcq.last_kernel() == "plane_mfma"
            for d, y in zip(dls, ys):
                y_ref, a_ref = oracle.gemv(d.layer.planes, d.layer.scales[p], xh)
                gpu.assert_within_tolerance(y, y_ref, a_ref, f"bcq_gemv_multi ms={ms} n={n} p={p} batch={batch}")
                assert torch.equal(y, bcq.bcq_gemv(d.planes, d.scales[p], p, x)), "multi differs from the separate call"


@pytest.mark.parametrize("kernel", ["auto", "dequant_mfma", "plane_f16"])
def test_gemv_multi_on_the_large_batch_kernels(gpu, oracle, kernel, forced_shape):
    """Beyond the first kernel's batches the matrices of a multi call run as ONE launch of the large-batch kernels
    (the rows of workgroups of all matrices side by side, the shape chosen for the sum of their rows): ragged
    row counts, two to four matrices, matrices too short for those kernels on their own, every family forced
    and the automatic choice, a forced workgroup shape of every kind."""
    import torch

    import paper_2510_10467_amd as bcq
    n = 1536
    for ms, shape in (((4096, 1024, 1000), None), ((150, 70), "1,4"), ((150, 70, 33, 260), "0,1"), ((100, 300), "4,40"), ((4100, 90), "32,8")):
        if shape and kernel == "auto":
            continue
        if shape and kernel == "plane_f16" and not shape.startswith(("0,", "32,")):
            continue
        if shape and kernel == "dequant_mfma" and shape.startswith(("0,", "32,")):
            continue
        layers = [syn.make_layer(m, n, seed=(192, k, m), signed=True) for k, m in enumerate(ms)]
        dls = [gpu.DeviceLayer(layer) for layer in layers]
        if shape:
            forced_shape(shape)
        for batch in ((20, 70) if kernel != "plane_f16" else (12, 30)):
            xh = syn.make_x(batch, n, seed=(192, batch))
            x = gpu.to_dev(xh)
            for p in (2, 4):
                bcq.select_kernel(kernel)
                try:
                    ys = bcq.bcq_gemv_multi([d.planes for d in dls], [d.scales[p] for d in dls], p, x)
                    torch.cuda.synchronize()
                    used = bcq.last_kernel()
                finally:
                    bcq.select_kernel("auto")
                assert used == (kernel if kernel != "auto" else ("plane_f16" if batch <= 32 else "dequant_mfma")), used
                for d, y in zip(dls, ys):
                    y_ref, a_ref = oracle.gemv(d.layer.planes, d.layer.scales[p], xh)
                    gpu.assert_within_tolerance(y, y_ref, a_ref, f"bcq_gemv_multi[{kernel}] ms={ms} shape={shape} p={p} batch={batch}")
        bcq.select_dequant_shape(0, 0)


def test_gemv_multi_falls_back_to_separate_launches(gpu, oracle):
    import torch

    import paper_2510_10467_amd as bcq
    # n shorter than a K slice: the generic kernel runs, one launch per matrix
    layers = [syn.make_layer(m, 640, seed=(191, m)) for m in (16, 40)]
    dls = [gpu.DeviceLayer(layer) for layer in layers]
    xh = syn.make_x(2, 640, seed=(191, 0))
    ys = bcq.bcq_gemv_multi([d.planes for d in dls], [d.scales[3] for d in dls], 3, gpu.to_dev(xh))
    torch.cuda.synchronize()
    assert bcq.last_kernel() == "lut"
    for d, y in zip(dls, ys):
        y_ref, a_ref = oracle.gemv(d.layer.planes, d.layer.scales[3], xh)
        gpu.assert_within_tolerance(y, y_ref, a_ref, "bcq_gemv_multi fallback")


def test_benchmark_reference_kernels(gpu):
    """The plain binary16 matrix-vector kernel the benchmark compares against computes what it says, and
    the streaming-read kernel leaves its sink alone."""
    import torch

    import paper_2510_10467_amd as bcq
    rng = np.random.default_rng(5)
    w = (rng.standard_normal((77, 1096)) * 0.05).astype(np.float16)
    x = rng.standard_normal(1096).astype(np.float16)
    y = bcq.bench_fp16_gemv(gpu.to_dev(w), gpu.to_dev(x), torch.empty(77, dtype=torch.float16, device=gpu.DEV))
    ref = w.astype(np.float64) @ x.astype(np.float64)
    mag = np.abs(w.astype(np.float64)) @ np.abs(x.astype(np.float64))
    assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - ref) <= 1e-3 * mag + 1e-3)
    buf = gpu.to_dev(rng.integers(0, 2 ** 31, size=100_003 * 4, dtype=np.int64).astype(np.int32))
    sink = torch.zeros(64, dtype=torch.int32, device=gpu.DEV)
    bcq.bench_stream_read(buf, sink)
    torch.cuda.synchronize()
    assert int(sink.abs().sum()) == 0
    # the instruction-issue probe reports a positive tick count for every wave it ran, and more ticks with more vector work
    ticks = torch.zeros(32, dtype=torch.int64, device=gpu.DEV)
    scratch = torch.zeros(1024, dtype=torch.float32, device=gpu.DEV)
    per_kind = []
    for valu in (0, 16):
        bcq.bench_issue_probe(2, valu, 4, 500, ticks, scratch)
        torch.cuda.synchronize()
        t = ticks.cpu().numpy().reshape(16, 2)
        assert np.all(t[:4] > 0)
        per_kind.append(int(t[:4, 0].max()))
    assert per_kind[1] > per_kind[0]


@pytest.mark.parametrize("kernel", ["dequant_mfma", "plane_f16"])
@pytest.mark.parametrize("n", [128, 256, 384])
def test_large_batch_kernels_on_one_to_three_groups(gpu, kernel, n):
    """Fewer 128-column groups than teams in a workgroup: some teams have nothing to do but still take every
    barrier; uniform and per-request precision, offsets, all three batch regimes."""
    m = 50
    layer = syn.make_layer(m, n, seed=(157, n), signed=True)
    dl = gpu.DeviceLayer(layer)
    z = syn.make_offsets(3, m, n, seed=(157, 1))
    for batch in (1, 16, 70, 257):
        x = syn.make_x(batch, n, seed=(157, batch))
        for p in (1, 4):
            used, _ = gpu.check_gemv(dl, p, x, kernel)
            assert used == kernel
        gpu.check_gemv(dl, 3, x, kernel, offsets=z)
        used, _ = gpu.check_mixed(dl, syn.make_p_req(batch, 1, 4, seed=(157, batch)), x, kernel)
        assert used == kernel


def test_seeded_random_cases_against_the_oracle(gpu):
    """Eighty seeded random cases of bcq_gemm_mixed and bcq_gemv: shapes (ragged rows, one to 32 groups of columns,
    groups of 64 / 128 / 256), batches on both sides of every dispatch threshold, precisions drawn, sorted, all
    equal or outside [1, p_max], offsets for some precisions, automatic dispatch or a forced large-batch shape."""
    import torch

    import paper_2510_10467_amd as bcq
    rng = np.random.default_rng([syn.BASE_SEED, 910])
    shapes = ["1,4", "1,2", "1,1", "2,4", "2,2", "4,4", "4,8", "4,40", None, None, None, None]
    done = 0
    while done < 80:
        m = int(rng.choice([16, 37, 100, 150, 260, 700, 1100, 4100, 8200]))
        n = int(rng.choice([1024, 1536, 2048, 2304, 4096]))
        group = int(rng.choice([128, 128, 128, 256, 64])) if n % 256 == 0 else 128
        batch = int(rng.choice([1, 3, 8, 9, 16, 17, 33, 48, 49, 64, 65, 80, 97, 128, 129, 200, 257, 400, 1030]))
        if n % group or m * batch > 300000:
            continue
        layer = syn.make_layer(m, n, group=group, seed=(911, done), signed=bool(rng.integers(2)))
        dl = gpu.DeviceLayer(layer)
        x = syn.make_x(batch, n, seed=(912, done))
        kind = int(rng.integers(4))
        if kind == 0:
            p_req = syn.make_p_req(batch, 1, 4, seed=(913, done))
        elif kind == 1:
            p_req = np.sort(syn.make_p_req(batch, 2, 4, seed=(913, done)))
        elif kind == 2:
            p_req = np.full(batch, int(rng.integers(1, 5)), dtype=np.int32)
        else:
            p_req = rng.choice([1, 4, 4, 4, 7, -2], size=batch).astype(np.int32)
        zs = None
        if rng.integers(3) == 0:
            zs = {p: syn.make_offsets(p, m, n, group, seed=(914, done, p)) for p in (1, 2, 3, 4) if rng.integers(2)}
        kernel = str(rng.choice(["auto", "auto", "dequant_mfma"]))
        shape = shapes[int(rng.integers(len(shapes)))]
        what = f"case {done}: m={m} n={n} group={group} batch={batch} kind={kind} offsets={sorted(zs) if zs else None} kernel={kernel} shape={shape}"
        if shape and kernel != "auto":
            bcq.select_dequant_shape(*[int(v) for v in shape.split(",")])
        try:
            bcq.select_kernel(kernel)
            try:
                y = bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(p_req.astype(np.int32)), gpu.to_dev(x), group=group,
                                       offsets_by_p={q: gpu.to_dev(z) for q, z in zs.items()} if zs else None)
                torch.cuda.synchronize()
            finally:
                bcq.select_kernel("auto")
            y_ref, a_ref = gpu.oracle.gemm_mixed(layer.planes, layer.scales, np.clip(p_req, 1, 4).astype(np.int32), x, group, offsets_by_p=zs)
            gpu.assert_within_tolerance(y, y_ref, a_ref, what)
            p = int(rng.integers(1, 5))
            gpu.check_gemv(dl, p, x, "auto", group, offsets=zs[p] if zs and p in zs else None)
        finally:
            bcq.select_dequant_shape(0, 0)
        done += 1


def test_seeded_random_cases_on_the_table_look_up_kernel(gpu):
    """Forty seeded random cases forced onto the table look-ups: widths that are multiples of 32 only (one to four table
    tiles, ragged last tile), groups of 32 to 416 columns, planes stored to 3..8, ragged row counts on both sides of the
    4, 8 and 16 rows of a workgroup, one request (two tiles per stretch) and several, precisions uniform or per request,
    inside and outside [1, p_max], offsets for some precisions."""
    import torch

    import paper_2510_10467_amd as bcq
    rng = np.random.default_rng([syn.BASE_SEED, 920])
    done = 0
    while done < 40:
        group = int(rng.choice([32, 64, 96, 128, 160, 256, 416]))
        n = group * int(rng.integers(1, 1 + min(40, 8320 // group)))
        m = int(rng.choice([1, 3, 4, 5, 17, 63, 130, 2047, 2050, 8191, 8200]))
        batch = int(rng.choice([1, 1, 1, 2, 3, 5, 8, 9]))
        p_max = int(rng.integers(3, 9))
        if m * n > 24_000_000:
            continue
        layer = syn.make_layer(m, n, p_max=p_max, group=group, seed=(921, done), signed=bool(rng.integers(2)))
        dl = gpu.DeviceLayer(layer)
        x = syn.make_x(batch, n, seed=(922, done))
        kind = int(rng.integers(3))
        if kind == 0:
            p_req = syn.make_p_req(batch, 1, p_max, seed=(923, done))
        elif kind == 1:
            p_req = np.full(batch, int(rng.integers(1, p_max + 1)), dtype=np.int32)
        else:
            p_req = rng.choice([1, p_max, p_max, 11, -2], size=batch).astype(np.int32)
        zs = None
        if rng.integers(3) == 0:
            zs = {p: syn.make_offsets(p, m, n, group, seed=(924, done, p)) for p in range(1, p_max + 1) if rng.integers(2)}
        what = f"lut case {done}: m={m} n={n} group={group} batch={batch} p_max={p_max} kind={kind} offsets={sorted(zs) if zs else None}"
        bcq.select_kernel("lut")
        try:
            out = gpu.Guarded((batch, m))
            bcq.bcq_gemm_mixed(dl.planes, dl.scales, gpu.to_dev(p_req.astype(np.int32)), gpu.to_dev(x), y=out.t, group=group,
                               offsets_by_p={q: gpu.to_dev(z) for q, z in zs.items()} if zs else None)
            assert bcq.last_kernel() == "lut"
            y = out.check(what)
        finally:
            bcq.select_kernel("auto")
        y_ref, a_ref = gpu.oracle.gemm_mixed(layer.planes, layer.scales, np.clip(p_req, 1, p_max).astype(np.int32), x, group, offsets_by_p=zs)
        gpu.assert_within_tolerance(y, y_ref, a_ref, what)
        p = int(rng.integers(1, p_max + 1))
        used, _ = gpu.check_gemv(dl, p, x, "lut", group, offsets=zs[p] if zs and p in zs else None)
        assert used == "lut"
        done += 1


def test_auto_dispatch_on_widths_the_plane_wise_kernel_does_not_take(gpu):
    """n = 1152 (a multiple of 128, not of 256): with 1024 rows and more (2048 on wider matrices) the large-batch kernels take
    it from one request on (plane-wise fp16 up to 32 requests); shorter matrices go to the table look-ups at one request and to
    the large-batch kernels from two; groups of 32 always run on the table look-ups."""
    tall = gpu.DeviceLayer(syn.make_layer(4100, 1152, seed=(175, 0)))
    short = gpu.DeviceLayer(syn.make_layer(1000, 1152, seed=(175, 1)))
    fine = gpu.DeviceLayer(syn.make_layer(4100, 1152, group=32, seed=(175, 2)))
    mid = gpu.DeviceLayer(syn.make_layer(1100, 1152, seed=(175, 3)))
    for dl, batch, group, want in ((mid, 1, 128, "plane_f16"), (mid, 2, 128, "plane_f16"),
                                   (tall, 1, 128, "plane_f16"), (tall, 3, 128, "plane_f16"), (tall, 40, 128, "dequant_mfma"),
                                   (short, 1, 128, "lut"), (short, 3, 128, "lut"), (fine, 1, 32, "lut"), (fine, 5, 32, "lut")):
        for p in (2, 4):
            used, _ = gpu.check_gemv(dl, p, syn.make_x(batch, 1152, seed=(175, batch)), "auto", group)
            assert used == want, (dl.layer.m, batch, group, p, used)
