"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle.

Bar: max |gpu - oracle| / RMS(oracle) <= 1e-5 for each of y, dx, dC (exact
basis, fp32 arithmetic).  Small shapes are compared element by element; the
full-size workloads are compared, layer by layer on the GPU's own fp32 layer
inputs, on whole rows and whole coefficient slabs that reach every output tile.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_14852_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-5


def tol_for(degree):
    """The same 1e-5 at every degree: above degree 8 the kernels advance T_k in a difference form
    that keeps the basis error from growing with k^2 near u = +-1."""
    return TOL


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_layer(x, C, dy=None, family=0, need_dx=True, need_dC=True):
    """Run forward (+ backward when dy is given) on the GPU; returns numpy arrays."""
    B, I = x.shape
    _, O, K = C.shape
    d = K - 1
    prev = binding.chebykan_set_kernel_family(family)
    try:
        xd, Cd = _dev(x), _dev(C)
        ws = binding.alloc_workspace(B, I, O, d)
        y = torch.full((B, O), float("nan"), device="cuda")
        binding.chebykan_forward(xd, Cd, y, ws)
        out = [y.cpu().numpy()]
        if dy is not None:
            dyd = _dev(dy)
            dx = torch.full((B, I), float("nan"), device="cuda") if need_dx else None
            dC = torch.full((I, O, K), float("nan"), device="cuda") if need_dC else None
            binding.chebykan_backward(xd, Cd, dyd, dx, dC, ws)
            out += [None if dx is None else dx.cpu().numpy(), None if dC is None else dC.cpu().numpy()]
        torch.cuda.synchronize()
    finally:
        binding.chebykan_set_kernel_family(prev)
    return out


def _inputs(B, I, O, d, seed, x_mean=0.0, x_std=1.0):
    x = wl.make_x(B, I, seed, x_mean, x_std)
    C = wl.make_coeff(I, O, d, seed + 1)
    dy = wl.make_dy(B, O, seed + 2)
    return x, C, dy


def _check_full(x, C, dy, family, label):
    y, dx, dC = gpu_layer(x, C, dy, family)
    y_ref = oracle.forward(x, C)
    dx_ref, dC_ref = oracle.backward(x, C, dy)
    errs = {"y": oracle.rel_err(y, y_ref), "dx": oracle.rel_err(dx, dx_ref), "dC": oracle.rel_err(dC, dC_ref)}
    print("%s family=%d errs=%s" % (label, family, {k: "%.2e" % v for k, v in errs.items()}), flush=True)
    tol = tol_for(C.shape[2] - 1)
    for k, v in errs.items():
        assert np.isfinite(v) and v <= tol, (label, family, k, v)


# shapes spanning several tiles with ragged tails in every dimension; the
# degrees with specialised kernels and several without
SMALL_SHAPES = [
    (256, 64, 64, 4),      # the small configuration as is
    (300, 70, 150, 8),
    (513, 33, 129, 3),
    (260, 257, 65, 5),
    (1000, 8, 64, 6),
    (777, 64, 1, 6),
    (129, 130, 257, 6),
    (64, 40, 256, 8),
    (37, 5, 3, 2),
    (130, 20, 70, 7),
    (3, 1, 1, 1),
    (50, 17, 9, 0),
    (64, 24, 40, 15),
    (32, 16, 48, 24),
    (1, 64, 64, 4),
    # every column-block count of the input-gradient tiles (1..4) and odd feature counts
    (200, 5, 40, 6),
    (150, 16, 72, 6),
    (140, 21, 64, 3),
    (131, 10, 100, 3),
    (260, 12, 48, 5),
    (129, 7, 520, 8),      # contraction over more than 512 outputs (accumulator fold in dx)
    # the feature-per-lane input gradient past one fold block (both chunk widths, ragged last chunk) and at degree 2
    (200, 64, 530, 4),
    (150, 64, 600, 5),
    (300, 64, 40, 2),
    (1200, 70, 40, 8),     # more than 512 rows per batch slice and more than 14 feature chunks (folds in dC, forward)
    # 1..4 columns beyond a multiple of 128: the streamed tail (forward into y, coefficient gradient through its own
    # partials into a window of dC), with one and with several batch slices, beside the 64-wide tail tile (5 columns)
    (700, 40, 130, 5),
    (300, 24, 259, 4),
    (2200, 64, 132, 8),
    (900, 70, 257, 3),
    (520, 48, 133, 6),
    # feature counts just above a multiple of 32 with enough work for a second launch: the feature-per-lane
    # input gradient over the full tiles plus a packed-column launch for the last 1, 6 and 9 features (one and
    # two column blocks); 75 features at degree 6 do not fit two blocks and stay with one padded tile
    (4096, 65, 512, 5),
    (2048, 70, 1024, 3),
    (4096, 73, 512, 6),
    (4096, 75, 512, 6),
    # narrow outputs with every lane-group width and several feature groups
    (333, 8, 1, 6),
    (100, 20, 2, 3),
    (77, 70, 3, 8),
    (50, 300, 4, 5),
    (2000, 64, 1, 6),
    # the paper's operator shapes (Table 5) and other small batches whose forward contraction is split
    (128, 40, 256, 8),
    (64, 256, 512, 15),
    (32, 512, 1024, 24),
    (100, 600, 130, 2),
    (200, 130, 70, 7),
    # the highest degree the interface takes and one between the specialised ones
    (40, 9, 33, 32),
    (33, 12, 20, 11),
    # the widest layers the interface takes (16-bit widths), on the matrix-core and the streaming kernels
    (8, 65535, 8, 2),
    (8, 8, 65535, 2),
    (16, 65535, 3, 2),
    # one batch slice and enough tiles for the slice kernel to write dC itself, 128-wide tiles and a tail tile
    (100, 1000, 130, 3),
]


@pytest.mark.parametrize("shape", SMALL_SHAPES, ids=lambda s: "B%d_I%d_O%d_d%d" % s)
@pytest.mark.parametrize("family", [0, 1], ids=["auto", "generic"])
def test_small_shapes_elementwise(shape, family):
    B, I, O, d = shape
    x, C, dy = _inputs(B, I, O, d, seed=1000 + B + I + O + d)
    _check_full(x, C, dy, family, "small %s" % (shape,))


def test_audio_like_input_distribution_with_saturation():
    """x ~ N(-2, 1.5^2) plus a few saturating values (|x| > 9 gives u = +-1 in fp32)."""
    B, I, O, d = 400, 96, 80, 5
    x, C, dy = _inputs(B, I, O, d, seed=77, x_mean=-2.0, x_std=1.5)
    x[0, :8] = [12.0, -12.0, 30.0, -30.0, 9.5, -9.5, 0.0, -0.0]
    _check_full(x, C, dy, 0, "audio-like")


def test_degenerate_inputs():
    B, I, O, d = 130, 12, 20, 4
    x, C, dy = _inputs(B, I, O, d, seed=5)
    Cz = np.zeros_like(C)
    y, dx, dC = gpu_layer(x, Cz, dy)
    assert np.all(y == 0.0) and np.all(dx == 0.0)
    assert oracle.rel_err(dC, oracle.backward(x, Cz, dy, need_dx=False)[1]) <= TOL
    dyh = np.zeros_like(dy)
    dyh[7, 3] = 1.0
    y, dx, dC = gpu_layer(x, C, dyh)
    assert np.all(dx[np.arange(B) != 7] == 0.0)
    assert np.all(dC[:, np.arange(O) != 3, :] == 0.0)
    dx_ref, dC_ref = oracle.backward(x, C, dyh)
    assert np.max(np.abs(dx - dx_ref)) <= 1e-5 * max(1.0, np.max(np.abs(dx_ref)))
    assert np.max(np.abs(dC - dC_ref)) <= 1e-5


def test_skipping_one_gradient_gives_the_same_other():
    B, I, O, d = 200, 48, 72, 6
    x, C, dy = _inputs(B, I, O, d, seed=9)
    _, dx_a, dC_a = gpu_layer(x, C, dy)
    _, dx_b, none_c = gpu_layer(x, C, dy, need_dC=False)
    _, none_x, dC_b = gpu_layer(x, C, dy, need_dx=False)
    assert none_c is None and none_x is None
    assert np.array_equal(dx_a, dx_b) and np.array_equal(dC_a, dC_b)


def test_bitwise_reproducible():
    B, I, O, d = 2048, 64, 64, 6
    x, C, dy = _inputs(B, I, O, d, seed=13)
    a = gpu_layer(x, C, dy)
    b = gpu_layer(x, C, dy)
    for p, q in zip(a, b):
        assert np.array_equal(p, q)


def test_empty_batch_and_error_codes_on_device():
    I, O, d = 8, 4, 3
    C = _dev(wl.make_coeff(I, O, d, 1))
    x = torch.empty((0, I), device="cuda")
    y = torch.empty((0, O), device="cuda")
    binding.chebykan_forward(x, C, y, binding.alloc_workspace(0, I, O, d))
    dC = torch.full((I, O, d + 1), float("nan"), device="cuda")
    binding.chebykan_backward(x, C, y, torch.empty((0, I), device="cuda"), dC, binding.alloc_workspace(0, I, O, d))
    torch.cuda.synchronize()
    assert torch.all(dC == 0).item()
    with pytest.raises(binding.ChebykanError) as e:
        st = binding.raw_forward(None, C.data_ptr(), C.data_ptr(), 4, I, O, d)
        raise binding.ChebykanError(st, "chebykan_forward")
    assert e.value.status == binding.CHEBYKAN_ERR_NULL


def test_outputs_outside_the_tensor_are_untouched():
    """Outputs live inside larger poisoned buffers; the guard bands must survive."""
    B, I, O, d = 131, 67, 35, 5
    x, C, dy = _inputs(B, I, O, d, seed=21)
    xd, Cd, dyd = _dev(x), _dev(C), _dev(dy)
    pad = 1024
    sentinel = 12345.5

    def guarded(n):
        buf = torch.full((n + 2 * pad,), sentinel, device="cuda")
        return buf, buf[pad:pad + n]

    ybuf, yv = guarded(B * O)
    dxbuf, dxv = guarded(B * I)
    dCbuf, dCv = guarded(I * O * (d + 1))
    ws = binding.alloc_workspace(B, I, O, d)
    binding.chebykan_forward(xd, Cd, yv.view(B, O), ws)
    binding.chebykan_backward(xd, Cd, dyd, dxv.view(B, I), dCv.view(I, O, d + 1), ws)
    torch.cuda.synchronize()
    for buf, n in ((ybuf, B * O), (dxbuf, B * I), (dCbuf, I * O * (d + 1))):
        assert torch.all(buf[:pad] == sentinel).item() and torch.all(buf[pad + n:] == sentinel).item()
        assert not torch.any(buf[pad:pad + n] == sentinel).item()
    assert oracle.rel_err(yv.view(B, O).cpu().numpy(), oracle.forward(x, C)) <= TOL


def test_base_pointers_only_four_byte_aligned():
    """Every tensor starts one float past a 16-byte boundary: the vectorised paths must not be taken."""
    for (B, I, O, d) in [(300, 64, 64, 6), (200, 40, 136, 8), (150, 64, 1, 6)]:
        x, C, dy = _inputs(B, I, O, d, seed=41 + O)
        K = d + 1

        def shifted(a):
            buf = torch.zeros(a.size + 5, device="cuda")
            v = buf[1:1 + a.size]
            v.copy_(torch.from_numpy(a.reshape(-1)))
            assert v.data_ptr() % 16 == 4
            return buf, v.view(*a.shape)

        (_, xd), (_, Cd), (_, dyd) = shifted(x), shifted(C), shifted(dy)
        (_, y), (_, dx), (_, dC) = (shifted(np.zeros((B, O), np.float32)), shifted(np.zeros((B, I), np.float32)),
                                    shifted(np.zeros((I, O, K), np.float32)))
        ws = binding.alloc_workspace(B, I, O, d)
        binding.chebykan_forward(xd, Cd, y, ws)
        binding.chebykan_backward(xd, Cd, dyd, dx, dC, ws)
        torch.cuda.synchronize()
        dx_ref, dC_ref = oracle.backward(x, C, dy)
        assert oracle.rel_err(y.cpu().numpy(), oracle.forward(x, C)) <= TOL
        assert oracle.rel_err(dx.cpu().numpy(), dx_ref) <= TOL
        assert oracle.rel_err(dC.cpu().numpy(), dC_ref) <= TOL


def test_non_default_stream():
    B, I, O, d = 300, 64, 64, 4
    x, C, dy = _inputs(B, I, O, d, seed=31)
    xd, Cd = _dev(x), _dev(C)
    y = torch.empty((B, O), device="cuda")
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        binding.chebykan_forward(xd, Cd, y, binding.alloc_workspace(B, I, O, d), stream=s)
    s.synchronize()
    assert oracle.rel_err(y.cpu().numpy(), oracle.forward(x, C)) <= TOL


# ------------------------------------------------------- full-size workloads

def _tile_covering_rows(B):
    """One row out of every block of 128 consecutive rows, at an offset that walks through all 128 positions
    (so every 32-row block position and both edges of a tile occur), plus the first and last rows of the tensor."""
    tiles = np.arange((B + 127) // 128)
    rows = tiles * 128 + (tiles * 37 + 5) % 128
    rows = np.concatenate([rows[rows < B], [0, 127 % B, B - 1, max(B - 128, 0)]])
    return np.unique(rows)


def _tile_covering_features(I, degree):
    """One input feature out of every block of min(16, 128 // (degree+1)) features - no coefficient-gradient
    tile is wider than that - at a walking offset, plus the first and last feature."""
    step = max(1, min(16, 128 // (degree + 1)))
    blocks = np.arange((I + step - 1) // step)
    feats = blocks * step + (blocks * 5 + 3) % step
    return np.unique(np.concatenate([feats[feats < I], [0, I - 1]]))


def _covering_layer_check(x, C, dy, y, dx, dC, label):
    """A full-size layer against the oracle on whole rows and whole coefficient slabs chosen so that every
    output tile of y, dx and dC holds compared elements: y[b, :] and dx[b, :] for one row of every 128-row
    block, dC[i, :, :] for one feature of every feature block.  dC[i] needs only column i of x.
    Each tensor's error is normalised by the RMS of the oracle values compared."""
    B, I = x.shape
    _, O, K = C.shape
    rows = _tile_covering_rows(B)
    feats = _tile_covering_features(I, K - 1)
    xr, dyr = np.ascontiguousarray(x[rows]), np.ascontiguousarray(dy[rows])
    e_y = oracle.rel_err(y[rows], oracle.forward(xr, C))
    dx_ref, _ = oracle.backward(xr, C, dyr, need_dC=False)
    e_dx = oracle.rel_err(dx[rows], dx_ref)
    _, dC_ref = oracle.backward(np.ascontiguousarray(x[:, feats]), np.ascontiguousarray(C[feats]), dy, need_dx=False)
    e_dC = oracle.rel_err(dC[feats], dC_ref)
    print("%s rows=%d features=%d y=%.2e dx=%.2e dC=%.2e" % (label, rows.size, feats.size, e_y, e_dx, e_dC), flush=True)
    assert np.isfinite(y).all() and np.isfinite(dx).all() and np.isfinite(dC).all()
    assert e_y <= TOL and e_dx <= TOL and e_dC <= TOL, (label, e_y, e_dx, e_dC)


def test_full_size_row_block_elementwise():
    """Audio-shaped first layer at its real widths (257 -> 512, degree 5, x ~ N(-2, 1.5^2)): every
    element of y and dx for a block of rows that spans tiles and ends ragged, and all of dC."""
    w = wl.WORKLOADS["c4"]
    (I, O), d = w.layers[0], w.degree
    B = 1000 + 37
    x = wl.make_x(B, I, 4242, w.x_mean, w.x_std)
    C = wl.make_coeff(I, O, d, 4243)
    dy = wl.make_dy(B, O, 4244)
    _check_full(x, C, dy, 0, "c4 first layer, %d rows" % B)


@pytest.mark.parametrize("B", [16384, 16389], ids=["planes_16B_aligned", "planes_ragged"])
def test_forward_split_when_the_wide_launch_would_underfill(B):
    """About 16384 rows x 130 outputs: 128 wide tiles plus 128 tail tiles, each launch under one workgroup
    per compute unit, so the plan splits the contraction over 512 inputs into ranges (the workspace query
    says so) and sums the planes (streaming sum, with and without 16-byte accesses).  Every element of y
    against the oracle."""
    I, O, d = 512, 130, 3
    assert binding.chebykan_workspace_bytes(B, I, O, d, binding.CHEBYKAN_PASS_FORWARD) >= 2 * B * O * 4
    x = wl.make_x(B, I, 5151)
    C = wl.make_coeff(I, O, d, 5152)
    (y,) = gpu_layer(x, C)
    err = oracle.rel_err(y, oracle.forward(x, C))
    print("split forward with tail tile: y=%.2e" % err, flush=True)
    assert np.isfinite(y).all() and err <= TOL


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_full_size_workload_every_tile(name):
    """Whole stack at its real size through the single-layer calls.  Each layer is checked on the GPU's own
    fp32 inputs (x_l = y_{l-1}, dy_l = dx_{l+1}), on whole rows and coefficient slabs that reach every tile."""
    w = wl.WORKLOADS[name]
    x0, Cs, dy_last = wl.workload_inputs(w)
    xs = [x0]
    for C in Cs:
        (y,) = gpu_layer(xs[-1], C)
        xs.append(y)
    dys = [None] * len(Cs)
    dys[-1] = dy_last
    for l in reversed(range(len(Cs))):
        y, dx, dC = gpu_layer(xs[l], Cs[l], dys[l])
        assert np.array_equal(y, xs[l + 1])          # forward is reproducible
        _covering_layer_check(xs[l], Cs[l], dys[l], y, dx, dC, "%s layer %d %s" % (name, l, w.layers[l]))
        if l > 0:
            dys[l - 1] = dx


def test_calibration_entry_points():
    """The roofline calibration kernels: the copy copies, the MFMA loop reports its flop count and finishes."""
    src = torch.randn(1 << 20, device="cuda")
    dst = torch.zeros_like(src)
    assert binding.chebykan_calibrate_copy(dst, src) == src.numel() * 4
    sink = torch.full((8 * 256,), float("nan"), device="cuda")
    flops = binding.chebykan_calibrate_mfma(sink, 8, 10)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert flops == 8 * 4 * 10 * 32 * 4096.0
    assert bool(torch.isfinite(sink).all())
    lib = binding.load()
    assert lib.chebykan_calibrate_copy(dst.data_ptr(), src.data_ptr(), 3, None) == binding.CHEBYKAN_ERR_SHAPE
    assert lib.chebykan_calibrate_mfma(None, 8, 10, None, None) == binding.CHEBYKAN_ERR_NULL


def test_batch_whose_outputs_exceed_four_gib():
    """16.8 million rows of an 8->64 layer: y and dy are 4.3 GB each, so element offsets pass 2^32 bytes.
    Inputs are generated on the GPU from a fixed seed (no 8 GB host arrays); the oracle runs on sampled rows
    (forward and dx are independent per row) and on sampled dC entries with the two dy columns they need."""
    B, I, O, d = (1 << 24) + 77, 8, 64, 6
    gen = torch.Generator(device="cuda")
    gen.manual_seed(251114852)
    x = torch.randn((B, I), device="cuda", generator=gen)
    dy = torch.randn((B, O), device="cuda", generator=gen)
    C = _dev(wl.make_coeff(I, O, d, 9))
    y = torch.empty((B, O), device="cuda")
    dx = torch.empty((B, I), device="cuda")
    dC = torch.empty_like(C)
    ws = binding.alloc_workspace(B, I, O, d)
    binding.chebykan_forward(x, C, y, ws)
    binding.chebykan_backward(x, C, dy, dx, dC, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([np.arange(0, 130), np.arange(B - 140, B), rng.integers(0, B, 300),
                                     np.arange((1 << 24) - 70, (1 << 24) + 70)]))
    rows_t = torch.from_numpy(rows).cuda()
    xs, dys, Cn = x[rows_t].cpu().numpy(), dy[rows_t].cpu().numpy(), C.cpu().numpy()
    assert oracle.rel_err(y[rows_t].cpu().numpy(), oracle.forward(xs, Cn)) <= TOL
    dx_ref, _ = oracle.backward(xs, Cn, dys, need_dC=False)
    assert oracle.rel_err(dx[rows_t].cpu().numpy(), dx_ref) <= TOL
    cols = [5, 63]
    x_all = x.cpu().numpy()
    dy_cols = dy[:, cols].contiguous().cpu().numpy()
    is_, ks = rng.integers(0, I, 6), rng.integers(0, d + 1, 6)
    os_local = rng.integers(0, 2, 6)
    ref = oracle.dC_at(x_all, dy_cols, d, is_, os_local, ks)
    got = dC.cpu().numpy()[is_, np.array(cols)[os_local], ks]
    scale = float(np.sqrt(np.mean(dC.cpu().numpy().astype(np.float64) ** 2)))
    assert np.max(np.abs(got - ref)) / scale <= TOL


def test_narrow_layer_whose_input_exceeds_four_gib():
    """16.8 million rows of a 64->1 layer (the streaming kernels): x is 4.3 GB."""
    B, I, O, d = (1 << 24) + 5, 64, 1, 6
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20251114)
    x = torch.randn((B, I), device="cuda", generator=gen)
    dy = torch.randn((B, O), device="cuda", generator=gen)
    C = _dev(wl.make_coeff(I, O, d, 19))
    y = torch.empty((B, O), device="cuda")
    dx = torch.empty((B, I), device="cuda")
    dC = torch.empty_like(C)
    ws = binding.alloc_workspace(B, I, O, d)
    binding.chebykan_forward(x, C, y, ws)
    binding.chebykan_backward(x, C, dy, dx, dC, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    rows = np.unique(np.concatenate([np.arange(0, 70), np.arange(B - 70, B), rng.integers(0, B, 300),
                                     np.arange((1 << 24) - 40, (1 << 24) + 5)]))
    rows_t = torch.from_numpy(rows).cuda()
    xs, dys, Cn = x[rows_t].cpu().numpy(), dy[rows_t].cpu().numpy(), C.cpu().numpy()
    assert oracle.rel_err(y[rows_t].cpu().numpy(), oracle.forward(xs, Cn)) <= TOL
    dx_ref, _ = oracle.backward(xs, Cn, dys, need_dC=False)
    assert oracle.rel_err(dx[rows_t].cpu().numpy(), dx_ref) <= TOL
    feats = [0, 63]                                  # dC[i, :, :] depends on column i of x only
    x_cols = x[:, feats].contiguous().cpu().numpy()
    dy_all = dy.cpu().numpy()
    is_local, ks = rng.integers(0, 2, 6), rng.integers(0, d + 1, 6)
    ref = oracle.dC_at(x_cols, dy_all, d, is_local, np.zeros(6, dtype=np.int64), ks)
    got = dC.cpu().numpy()[np.array(feats)[is_local], 0, ks]
    scale = float(np.sqrt(np.mean(dC.cpu().numpy().astype(np.float64) ** 2)))
    assert np.max(np.abs(got - ref)) / scale <= TOL
