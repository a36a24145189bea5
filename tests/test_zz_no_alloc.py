"""chebykan_backward_noalloc (the entry point for callers that cannot allocate: static device scratch
instead of a caller workspace) against chebykan_backward, through the C ABI.  Same kernels and plans,
so the results must be equal bit for bit - and within 1e-5 of the oracle like every exact-basis
result.  Two calls in a row share the scratch array; the second has the smaller input."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_14852_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def _run_both(B, I, O, d, seed, need_dx=True, need_dC=True):
    x = torch.from_numpy(wl.make_x(B, I, seed)).cuda()
    C = torch.from_numpy(wl.make_coeff(I, O, d, seed + 1)).cuda()
    dy = torch.from_numpy(wl.make_dy(B, O, seed + 2)).cuda()
    outs = []
    for static in (False, True):
        dx = torch.full((B, I), float("nan"), device="cuda") if need_dx else None
        dC = torch.full((I, O, d + 1), float("nan"), device="cuda") if need_dC else None
        if static:
            st = binding.raw_backward_noalloc(x.data_ptr(), C.data_ptr(), dy.data_ptr(),
                                              dx.data_ptr() if need_dx else None, dC.data_ptr() if need_dC else None,
                                              B, I, O, d, torch.cuda.current_stream().cuda_stream)
        else:
            ws = binding.alloc_workspace(B, I, O, d)
            st = binding.raw_backward(x.data_ptr(), C.data_ptr(), dy.data_ptr(),
                                      dx.data_ptr() if need_dx else None, dC.data_ptr() if need_dC else None,
                                      B, I, O, d, ws.data_ptr() if ws is not None else None,
                                      ws.numel() if ws is not None else 0, torch.cuda.current_stream().cuda_stream)
        assert st == binding.CHEBYKAN_OK, (static, binding.chebykan_status_string(st))
        torch.cuda.synchronize()
        outs.append((dx, dC))
    return x, C, dy, outs


def _compare(B, I, O, d, seed, check_oracle=True, **kw):
    x, C, dy, ((dx0, dC0), (dx1, dC1)) = _run_both(B, I, O, d, seed, **kw)
    if dx0 is not None:
        assert torch.equal(dx0, dx1), "dx differs between the workspace and the static-scratch call"
    if dC0 is not None:
        assert torch.equal(dC0, dC1), "dC differs between the workspace and the static-scratch call"
    if check_oracle:
        dx_ref, dC_ref = oracle.backward(x.cpu().numpy(), C.cpu().numpy(), dy.cpu().numpy())
        if dx1 is not None:
            assert oracle.rel_err(dx1.cpu().numpy(), dx_ref) <= 1e-5
        if dC1 is not None:
            assert oracle.rel_err(dC1.cpu().numpy(), dC_ref) <= 1e-5


def test_two_calls_in_a_row_second_smaller():
    binding.chebykan_init()
    # 29 batch slices of partial coefficient gradients (about 3 MiB of scratch), then a smaller layer
    # whose partials land on what the first call left behind
    assert 0 < binding.chebykan_workspace_bytes(30000, 64, 64, 6, binding.CHEBYKAN_PASS_BACKWARD) <= binding.CHEBYKAN_NOALLOC_SCRATCH_BYTES
    _compare(30000, 64, 64, 6, 901, check_oracle=False)
    _compare(700, 40, 72, 5, 911)


def test_split_input_gradient_and_narrow_layers_on_static_scratch():
    _compare(64, 40, 520, 8, 921)          # small batch: the dx contraction is split into planes in the scratch
    _compare(5000, 64, 1, 6, 931)          # streaming kernels: per-workgroup partials
    _compare(4096, 8, 64, 6, 941)          # both gradients from one kernel
    _compare(300, 20, 33, 11, 951)         # a degree without specialised kernels: no scratch at all
    _compare(900, 48, 80, 4, 961, need_dx=False)
    _compare(900, 48, 80, 4, 971, need_dC=False)


def test_shape_beyond_the_scratch_is_refused_and_nothing_runs():
    B, I, O, d = 16384, 1024, 1024, 8
    assert binding.chebykan_workspace_bytes(B, I, O, d, binding.CHEBYKAN_PASS_BACKWARD) > binding.CHEBYKAN_NOALLOC_SCRATCH_BYTES
    dC = torch.full((8,), 7.0, device="cuda")
    P = dC.data_ptr()     # never dereferenced: the call is refused before anything is enqueued
    st = binding.raw_backward_noalloc(P, P, P, P, P, B, I, O, d, None)
    assert st == binding.CHEBYKAN_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.all(dC == 7.0)


def test_argument_errors_match_the_workspace_entry_point():
    P = 4096
    assert binding.raw_backward_noalloc(P, P, None, P, P, 4, 4, 4, 2) == binding.CHEBYKAN_ERR_NULL
    assert binding.raw_backward_noalloc(P, P, P, None, None, 4, 4, 4, 2) == binding.CHEBYKAN_ERR_NULL
    assert binding.raw_backward_noalloc(P, P, P, P, P, 4, 4, -3, 2) == binding.CHEBYKAN_ERR_SHAPE
