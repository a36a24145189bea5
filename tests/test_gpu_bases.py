"""GPU parity of the Legendre / Hermite / Fourier layers (paper Sec. 2.3, Sec. 6.3) against their fp64 oracle.

Same bar as the Chebyshev layer: max |gpu - oracle| / RMS(oracle) <= 1e-5 for y, dx and dC.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_14852_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-5
NAMES = {1: "legendre", 2: "hermite", 3: "fourier"}


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_layer_basis(kind, x, C, dy, family=0):
    B, I = x.shape
    _, O, K = C.shape
    prev = binding.chebykan_set_kernel_family(family)
    try:
        xd, Cd, dyd = _dev(x), _dev(C), _dev(dy)
        ws = binding.alloc_workspace(B, I, O, K - 1)
        y = torch.full((B, O), float("nan"), device="cuda")
        dx = torch.full((B, I), float("nan"), device="cuda")
        dC = torch.full((I, O, K), float("nan"), device="cuda")
        binding.chebykan_forward_basis(kind, xd, Cd, y, ws)
        binding.chebykan_backward_basis(kind, xd, Cd, dyd, dx, dC, ws)
        torch.cuda.synchronize()
    finally:
        binding.chebykan_set_kernel_family(prev)
    return y.cpu().numpy(), dx.cpu().numpy(), dC.cpu().numpy()


# (B, I, O, degree): every kernel family of the Chebyshev path; degrees with and without specialised kernels
SHAPES = [
    (256, 64, 64, 4),
    (300, 70, 150, 8),
    (513, 33, 129, 3),
    (260, 257, 65, 5),
    (1000, 8, 64, 6),
    (777, 64, 1, 6),
    (129, 130, 257, 6),
    (100, 20, 2, 4),
    (64, 40, 256, 8),
    (130, 20, 70, 7),
    (37, 5, 3, 2),
    (50, 17, 9, 10),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "B%d_I%d_O%d_d%d" % s)
@pytest.mark.parametrize("kind", [1, 2, 3], ids=lambda k: NAMES[k])
@pytest.mark.parametrize("family", [0, 1], ids=["auto", "generic"])
def test_small_shapes_elementwise(shape, kind, family):
    B, I, O, d = shape
    if kind == 3 and d % 2:
        d += 1                                   # the Fourier basis pairs cos and sin
    x = wl.make_x(B, I, 5000 + B + I + O + d)
    C = wl.make_coeff(I, O, d, 5001 + B + I + O + d)
    dy = wl.make_dy(B, O, 5002 + B + I + O + d)
    y, dx, dC = gpu_layer_basis(kind, x, C, dy, family)
    dx_ref, dC_ref = oracle.backward_basis(kind, x, C, dy)
    errs = (oracle.rel_err(y, oracle.forward_basis(kind, x, C)), oracle.rel_err(dx, dx_ref),
            oracle.rel_err(dC, dC_ref))
    print("%s %s family=%d errs y %.2e dx %.2e dC %.2e" % (NAMES[kind], (B, I, O, d), family, *errs), flush=True)
    assert all(np.isfinite(e) and e <= TOL for e in errs), errs


def test_chebyshev_kind_is_the_exact_path_and_errors():
    B, I, O, d = 130, 12, 20, 4
    x, C, dy = wl.make_x(B, I, 1), wl.make_coeff(I, O, d, 2), wl.make_dy(B, O, 3)
    y, dx, dC = gpu_layer_basis(0, x, C, dy)
    xd, Cd = _dev(x), _dev(C)
    y2 = torch.empty((B, O), device="cuda")
    binding.chebykan_forward(xd, Cd, y2, binding.alloc_workspace(B, I, O, d))
    torch.cuda.synchronize()
    assert np.array_equal(y, y2.cpu().numpy())
    lib = binding.load()
    st = lib.chebykan_forward_basis(3, xd.data_ptr(), Cd.data_ptr(), y2.data_ptr(), B, I, O, 5, None, 0, None)
    assert st == binding.CHEBYKAN_ERR_SHAPE      # odd Fourier degree
    st = lib.chebykan_forward_basis(7, xd.data_ptr(), Cd.data_ptr(), y2.data_ptr(), B, I, O, d, None, 0, None)
    assert st == binding.CHEBYKAN_ERR_SHAPE      # unknown basis
