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


def test_calls_captured_in_a_graph_replay_like_eager_calls():
    """A forward, a workspace backward and a static-scratch backward recorded into one HIP graph after
    chebykan_init(); three replays, with eager work of the library and synchronisations between them, each
    give what the eager calls give (the library enqueues kernels only: no memsets, no allocation, no
    function-attribute changes at launch time)."""
    binding.chebykan_init()
    B, I, O, d = 700, 40, 72, 6
    x, C, dy = _layer(B, I, O, d, 71)
    y = torch.empty((B, O), device="cuda")
    dx = torch.empty((B, I), device="cuda")
    dC = torch.empty_like(C)
    dx2 = torch.empty((B, I), device="cuda")
    dC2 = torch.empty_like(C)
    ws = binding.alloc_workspace(B, I, O, d)
    s = torch.cuda.Stream()

    def issue(stream):
        binding.chebykan_forward(x, C, y, ws, stream)
        binding.chebykan_backward(x, C, dy, dx, dC, ws, stream)
        st = binding.raw_backward_noalloc(x.data_ptr(), C.data_ptr(), dy.data_ptr(), dx2.data_ptr(), dC2.data_ptr(),
                                          B, I, O, d, stream.cuda_stream)
        assert st == binding.CHEBYKAN_OK

    issue(s)
    s.synchronize()
    eager = [t.clone() for t in (y, dx, dC, dx2, dC2)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        issue(s)
    other = _layer(300, 16, 16, 4, 81)
    y_o = torch.empty((300, 16), device="cuda")
    ws_o = binding.alloc_workspace(300, 16, 16, 4)
    for replay in range(3):
        for t in (y, dx, dC, dx2, dC2):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("y", "dx", "dC", "dx static", "dC static"), (y, dx, dC, dx2, dC2), eager):
            assert torch.equal(got, want), (replay, name)
        binding.chebykan_forward(other[0], other[1], y_o, ws_o)      # eager work between the replays
        torch.cuda.synchronize()
    y_ref = oracle.forward(x.cpu().numpy(), C.cpu().numpy())
    assert oracle.rel_err(y.cpu().numpy(), y_ref) <= 1e-5
