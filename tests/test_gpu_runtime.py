"""GPU tests of the library's process-wide services: device preparation, calls from several
host threads, and the per-kernel timing that bench.py reports."""
import threading

import numpy as np
import pytest
import torch

import oracle
from paper_2511_14852_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def _layer(B, I, O, d, seed):
    x = torch.from_numpy(wl.make_x(B, I, seed)).cuda()
    C = torch.from_numpy(wl.make_coeff(I, O, d, seed + 1)).cuda()
    dy = torch.from_numpy(wl.make_dy(B, O, seed + 2)).cuda()
    return x, C, dy


def test_init_is_idempotent():
    binding.chebykan_init()
    binding.chebykan_init()


def test_kernel_timing_names_and_durations():
    B, I, O, d = 1024, 64, 64, 6
    x, C, dy = _layer(B, I, O, d, 31)
    y = torch.empty((B, O), device="cuda")
    dx = torch.empty((B, I), device="cuda")
    dC = torch.empty_like(C)
    ws = binding.alloc_workspace(B, I, O, d)
    binding.chebykan_forward(x, C, y, ws)                 # untimed
    binding.chebykan_trace_begin(16)
    binding.chebykan_forward(x, C, y, ws)
    binding.chebykan_backward(x, C, dy, dx, dC, ws)
    n, dropped = binding.chebykan_trace_end()
    binding.chebykan_backward(x, C, dy, dx, dC, ws)       # after the end: untimed
    torch.cuda.synchronize()
    recs = binding.chebykan_trace_records(n)
    binding.chebykan_trace_free()
    print(recs, flush=True)
    assert dropped == 0 and n >= 3
    names = [r[0] for r in recs]
    assert names[0].startswith("fwd_mfma_kernel<FwdCfg<6, 64")
    assert any(nm.startswith("dx2_mfma_kernel<") or nm.startswith("dx_mfma_kernel<") for nm in names)
    assert any(nm.startswith("dC_mfma_kernel<") for nm in names)
    for name, grid, block, layer, ops, share, layer2, ops2, us in recs:
        assert grid[0] >= 1 and block in (256, 1024) and 0.5 < us < 5000.0, (name, grid, block, us)
        assert layer == 0 and share == 1.0 and ops2 == 0
        if name.startswith("fwd_mfma_kernel"):
            assert ops == binding.OP_FORWARD
        if name.startswith("dx2_mfma_kernel") or name.startswith("dx_mfma_kernel"):
            assert ops == binding.OP_DX
        if name.startswith("dC_mfma_kernel"):
            assert ops == binding.OP_DC
        if name.startswith("dC_combine_kernel"):
            assert ops == binding.OP_DC | binding.OP_SUM
    # the timed calls computed what the untimed ones compute
    y_ref = oracle.forward(x.cpu().numpy(), C.cpu().numpy())
    assert oracle.rel_err(y.cpu().numpy(), y_ref) <= 1e-5


def test_timing_capacity_is_respected():
    x, C, dy = _layer(256, 16, 16, 4, 41)
    y = torch.empty((256, 16), device="cuda")
    ws = binding.alloc_workspace(256, 16, 16, 4)
    binding.chebykan_trace_begin(2)
    for _ in range(5):
        binding.chebykan_forward(x, C, y, ws)
    n, dropped = binding.chebykan_trace_end()
    torch.cuda.synchronize()
    assert n == 2 and dropped >= 3
    assert len(binding.chebykan_trace_records(n)) == 2
    binding.chebykan_trace_free()


def test_calls_from_two_host_threads():
    """Two threads, each on its own stream, run layers of different shapes at once; both match the oracle."""
    shapes = [(700, 40, 72, 6), (515, 33, 129, 3)]
    results = [None, None]

    def work(k):
        B, I, O, d = shapes[k]
        torch.cuda.set_device(0)
        s = torch.cuda.Stream()
        x, C, dy = _layer(B, I, O, d, 51 + 10 * k)
        y = torch.empty((B, O), device="cuda")
        dx = torch.empty((B, I), device="cuda")
        dC = torch.empty_like(C)
        ws = binding.alloc_workspace(B, I, O, d)
        torch.cuda.synchronize()
        for _ in range(20):
            binding.chebykan_forward(x, C, y, ws, s)
            binding.chebykan_backward(x, C, dy, dx, dC, ws, s)
        s.synchronize()
        results[k] = (x.cpu().numpy(), C.cpu().numpy(), dy.cpu().numpy(), y.cpu().numpy(), dx.cpu().numpy(), dC.cpu().numpy())

    threads = [threading.Thread(target=work, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for k in range(2):
        x, C, dy, y, dx, dC = results[k]
        dx_ref, dC_ref = oracle.backward(x, C, dy)
        errs = (oracle.rel_err(y, oracle.forward(x, C)), oracle.rel_err(dx, dx_ref), oracle.rel_err(dC, dC_ref))
        assert all(np.isfinite(e) and e <= 1e-5 for e in errs), (k, errs)
