"""Stack-level entry points and the autograd wrapper against the fp64 oracle (GPU)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_14852_amd import binding, workloads as wl
from paper_2511_14852_amd.autograd import ChebyKANStack, ChebyKANStackFunction

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _oracle_stack(x0, Cs, dy_last):
    """Layer by layer in fp64 on the oracle's own activations."""
    xs = [x0.astype(np.float64)]
    for C in Cs:
        xs.append(oracle.forward(xs[-1], C))
    grads, dCs = [None] * len(Cs) + [dy_last.astype(np.float64)], []
    for l in reversed(range(len(Cs))):
        dx, dC = oracle.backward(xs[l], Cs[l], grads[l + 1])
        grads[l] = dx
        dCs.insert(0, dC)
    return xs, grads, dCs


# the last four are large and narrow enough for the single-launch forward (all hidden widths <= 64,
# >= 32768 rows): ragged last row tile, a narrow and a matrix-core last layer, every fused degree
@pytest.mark.parametrize("widths,degree,B", [((8, 64, 64, 1), 6, 700), ((20, 33, 9), 5, 300), ((64, 64), 4, 256),
                                              ((12, 40, 24, 16, 5), 3, 130),
                                              ((8, 64, 64, 1), 6, 32768 + 77), ((70, 64, 32), 5, 32768),
                                              ((9, 16, 48, 3), 4, 33000), ((5, 64, 64, 64, 12), 3, 32800)])
def test_stack_calls_against_the_oracle(widths, degree, B):
    x0 = wl.make_x(B, widths[0], 11)
    Cs = [wl.make_coeff(i, o, degree, 20 + l) for l, (i, o) in enumerate(zip(widths[:-1], widths[1:]))]
    dy = wl.make_dy(B, widths[-1], 13)
    dev = lambda a: torch.from_numpy(a).cuda()
    Cd = [dev(c) for c in Cs]
    acts = [dev(x0)] + [torch.full((B, w), float("nan"), device="cuda") for w in widths[1:]]
    ws = binding.alloc_stack_workspace(B, widths, degree)
    binding.chebykan_stack_forward(Cd, acts, ws)
    grads = [torch.full((B, w), float("nan"), device="cuda") for w in widths[:-1]] + [dev(dy)]
    dCd = [torch.full_like(c, float("nan")) for c in Cd]
    binding.chebykan_stack_backward(Cd, acts, grads, dCd, ws)
    torch.cuda.synchronize()
    # per layer, on the GPU's own fp32 layer inputs (an end-to-end comparison would measure how the
    # network amplifies rounding differences of earlier layers, not the kernels)
    for l in range(len(Cs)):
        x_l, g_l = acts[l].cpu().numpy(), grads[l + 1].cpu().numpy()
        assert oracle.rel_err(acts[l + 1].cpu().numpy(), oracle.forward(x_l, Cs[l])) <= TOL
        dx_ref, dC_ref = oracle.backward(x_l, Cs[l], g_l)
        assert oracle.rel_err(grads[l].cpu().numpy(), dx_ref) <= TOL
        assert oracle.rel_err(dCd[l].cpu().numpy(), dC_ref) <= TOL
    # against the chained single-layer calls: bit for bit when the stack call issues the same launches,
    # within rounding when it runs the layers in one kernel (other chunking of the contraction)
    y = acts[0]
    for l, c in enumerate(Cd):
        out = torch.empty((B, widths[l + 1]), device="cuda")
        binding.chebykan_forward(y, c, out, binding.alloc_workspace(B, widths[l], widths[l + 1], degree))
        y = out
    torch.cuda.synchronize()
    if B < 32768:
        assert torch.equal(y, acts[-1])
    else:
        assert oracle.rel_err(acts[-1].cpu().numpy(), y.cpu().numpy().astype(np.float64)) <= TOL


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_full_size_workload_through_the_stack_calls(name):
    """Each workload at its real size through the two calls the benchmark times (for the tabular stack:
    the single-launch forward, the one-kernel first-layer backward and the shared slice-sum launch).
    Whole rows and coefficient slabs that reach every output tile of every layer against the oracle, on
    the GPU's own fp32 layer inputs."""
    from test_gpu_parity import _covering_layer_check
    w = wl.WORKLOADS[name]
    x0, Cs, dy_last = wl.workload_inputs(w)
    B, widths, degree = w.batch, list(w.widths), w.degree
    dev = lambda a: torch.from_numpy(a).cuda()
    Cd = [dev(c) for c in Cs]
    acts = [dev(x0)] + [torch.full((B, wd), float("nan"), device="cuda") for wd in widths[1:]]
    ws = binding.alloc_stack_workspace(B, widths, degree)
    binding.chebykan_stack_forward(Cd, acts, ws)
    grads = [torch.full((B, wd), float("nan"), device="cuda") for wd in widths[:-1]] + [dev(dy_last)]
    dCd = [torch.full_like(c, float("nan")) for c in Cd]
    binding.chebykan_stack_backward(Cd, acts, grads, dCd, ws)
    torch.cuda.synchronize()
    for l in range(len(Cs)):
        _covering_layer_check(acts[l].cpu().numpy(), Cs[l], grads[l + 1].cpu().numpy(), acts[l + 1].cpu().numpy(),
                              grads[l].cpu().numpy(), dCd[l].cpu().numpy(),
                              "%s stack calls, layer %d %s" % (name, l, w.layers[l]))


def test_stack_skips_and_errors():
    widths, degree, B = (8, 16, 4), 4, 64
    Cd = [torch.from_numpy(wl.make_coeff(i, o, degree, 5)).cuda() for i, o in zip(widths[:-1], widths[1:])]
    acts = [torch.randn(B, widths[0], device="cuda")] + [torch.empty(B, w, device="cuda") for w in widths[1:]]
    binding.chebykan_stack_forward(Cd, acts, binding.alloc_stack_workspace(B, widths, degree))
    grads = [None, torch.empty(B, widths[1], device="cuda"), torch.randn(B, widths[2], device="cuda")]
    dCs = [torch.empty_like(Cd[0]), None]
    binding.chebykan_stack_backward(Cd, acts, grads, dCs, binding.alloc_stack_workspace(B, widths, degree))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dCs[0]).all())
    with pytest.raises(binding.ChebykanError):       # first layer with neither output
        binding.chebykan_stack_backward(Cd, acts, grads, [None, None], binding.alloc_stack_workspace(B, widths, degree))
    lib = binding.load()
    assert lib.chebykan_stack_forward(0, None, degree, B, None, None, None, 0, None) == binding.CHEBYKAN_ERR_NULL


def test_autograd_wrapper_matches_the_oracle_gradients():
    widths, degree, B = (10, 48, 24, 3), 5, 200
    torch.manual_seed(0)
    model = ChebyKANStack(widths, degree)
    x = torch.randn(B, widths[0], device="cuda", requires_grad=True)
    y = model(x)
    w = torch.randn_like(y)
    (y * w).sum().backward()
    Cs = [p.detach().cpu().numpy() for p in model.coeffs]
    xs, g_ref, dC_ref = _oracle_stack(x.detach().cpu().numpy(), Cs, w.cpu().numpy())
    assert oracle.rel_err(y.detach().cpu().numpy(), xs[-1]) <= 3 * TOL
    assert oracle.rel_err(x.grad.cpu().numpy(), g_ref[0]) <= 6 * TOL
    for p, ref in zip(model.coeffs, dC_ref):
        assert oracle.rel_err(p.grad.cpu().numpy(), ref) <= 6 * TOL
    # no gradient for the input requested: dx of the first layer is skipped
    x2 = x.detach().clone()
    for p in model.coeffs:
        p.grad = None
    (ChebyKANStackFunction.apply(x2, *model.coeffs) * w).sum().backward()
    for p, ref in zip(model.coeffs, dC_ref):
        assert oracle.rel_err(p.grad.cpu().numpy(), ref) <= 6 * TOL
