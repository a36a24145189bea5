"""Host-side checks of the C-ABI library that need no GPU: the library loads,
exports every symbol the public header declares, and rejects bad arguments
before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2511_14852_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(chebykan_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    declared = _declared_functions()
    assert set(binding.EXPORTS) == set(declared)
    for name in declared:
        assert hasattr(lib, name), name
        assert ctypes.cast(getattr(lib, name), ctypes.c_void_p).value


def test_version_and_status_strings():
    assert binding.chebykan_version() >= 1000
    seen = set()
    for code in (0, -1, -2, -3, -4, -5):
        s = binding.chebykan_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert "unknown" in binding.chebykan_status_string(-99)


def test_argument_validation_happens_before_any_device_use():
    P = 4096  # any non-null value: never dereferenced on these paths
    assert binding.raw_forward(None, P, P, 4, 4, 4, 2) == binding.CHEBYKAN_ERR_NULL
    assert binding.raw_forward(P, None, P, 4, 4, 4, 2) == binding.CHEBYKAN_ERR_NULL
    assert binding.raw_forward(P, P, None, 4, 4, 4, 2) == binding.CHEBYKAN_ERR_NULL
    assert binding.raw_forward(P, P, P, -1, 4, 4, 2) == binding.CHEBYKAN_ERR_SHAPE
    assert binding.raw_forward(P, P, P, 4, 0, 4, 2) == binding.CHEBYKAN_ERR_SHAPE
    assert binding.raw_forward(P, P, P, 4, 4, 0, 2) == binding.CHEBYKAN_ERR_SHAPE
    assert binding.raw_forward(P, P, P, 4, 4, 4, -1) == binding.CHEBYKAN_ERR_SHAPE
    assert binding.raw_forward(P, P, P, 4, 4, 4, binding.CHEBYKAN_MAX_DEGREE + 1) == binding.CHEBYKAN_ERR_SHAPE
    assert binding.raw_forward(P, P, P, 4, 70000, 70000, 8) == binding.CHEBYKAN_ERR_SHAPE
    assert binding.raw_backward(P, P, None, P, P, 4, 4, 4, 2) == binding.CHEBYKAN_ERR_NULL
    assert binding.raw_backward(P, P, P, None, None, 4, 4, 4, 2) == binding.CHEBYKAN_ERR_NULL
    assert binding.raw_backward(P, P, P, P, P, 4, 4, -3, 2) == binding.CHEBYKAN_ERR_SHAPE


def test_workspace_query_is_host_only_and_checked():
    P = 4096
    assert binding.chebykan_workspace_bytes(-1, 4, 4, 2, 0) == 0
    assert binding.chebykan_workspace_bytes(4, 4, 4, 2, 7) == 0
    for (B, I, O, d) in [(256, 64, 64, 4), (65536, 64, 64, 6), (16384, 1024, 1024, 8), (65536, 64, 1, 6)]:
        for which in (0, 1):
            n = binding.chebykan_workspace_bytes(B, I, O, d, which)
            assert 0 <= n < (2 << 30)
            if n > 0:
                if which == 0:
                    assert binding.raw_forward(P, P, P, B, I, O, d, None, 0) == binding.CHEBYKAN_ERR_WORKSPACE
                    assert binding.raw_forward(P, P, P, B, I, O, d, P, n - 1) == binding.CHEBYKAN_ERR_WORKSPACE
                else:
                    assert binding.raw_backward(P, P, P, P, P, B, I, O, d, None, 0) == binding.CHEBYKAN_ERR_WORKSPACE
                    assert binding.raw_backward(P, P, P, P, P, B, I, O, d, P, n - 1) == binding.CHEBYKAN_ERR_WORKSPACE


def test_workspace_matches_the_documented_partial_layout():
    """Backward workspace = slices x in x out x (degree+1) floats for some whole slice count."""
    for (B, I, O, d) in [(256, 64, 64, 4), (65536, 8, 64, 6), (65536, 64, 1, 6), (32768, 512, 256, 3),
                         (16000, 257, 512, 5), (16384, 1024, 1024, 8)]:
        n = binding.chebykan_workspace_bytes(B, I, O, d, binding.CHEBYKAN_PASS_BACKWARD)
        per_slice = I * O * (d + 1) * 4
        assert n > 0 and n % per_slice == 0
        assert 1 <= n // per_slice <= max(1, (B + 31) // 32)
        assert n <= (512 << 20) + per_slice
    # degrees without specialised kernels need no workspace
    assert binding.chebykan_workspace_bytes(1024, 64, 64, 11, binding.CHEBYKAN_PASS_BACKWARD) == 0
    assert binding.chebykan_workspace_bytes(1024, 64, 64, 11, binding.CHEBYKAN_PASS_FORWARD) == 0
    # forward: none when the batch alone fills the chip; whole [B,O] planes when the contraction is split
    assert binding.chebykan_workspace_bytes(65536, 64, 64, 6, binding.CHEBYKAN_PASS_FORWARD) == 0
    n = binding.chebykan_workspace_bytes(32, 512, 1024, 24, binding.CHEBYKAN_PASS_FORWARD)
    assert n > 0 and n % (32 * 1024 * 4) == 0 and 2 <= n // (32 * 1024 * 4) <= 64
    # a wide launch that would leave most compute units with one workgroup (250 + 125 tail) is split too
    n = binding.chebykan_workspace_bytes(16000, 512, 257, 5, binding.CHEBYKAN_PASS_FORWARD)
    assert n > 0 and n % (16000 * 257 * 4) == 0 and 2 <= n // (16000 * 257 * 4) <= 4
    assert binding.chebykan_workspace_bytes(16000, 512, 512, 5, binding.CHEBYKAN_PASS_FORWARD) == 0


def test_workspace_query_over_random_shapes():
    """The host-side plans behind the workspace query, over 400 seeded random shapes: a backward workspace is a
    whole number of partial tensors with at most one slice per 32 rows, a forward workspace a whole number
    (2..64) of output planes, and both stay under 2 GiB + one tensor."""
    rng = np.random.default_rng(20251114)
    for _ in range(400):
        B = int(rng.choice([1, 7, 32, 33, 64, 100, 255, 256, 1000, 4095, 4096, 16000, 65536, 300000]))
        I = int(rng.choice([1, 3, 8, 17, 64, 80, 257, 512, 1024, 3000]))
        O = int(rng.choice([1, 2, 4, 5, 33, 64, 65, 128, 129, 192, 257, 512, 1000]))
        d = int(rng.choice([0, 1, 2, 3, 4, 5, 6, 7, 8, 11, 15, 24, 32]))
        per_slice = I * O * (d + 1) * 4
        nb = binding.chebykan_workspace_bytes(B, I, O, d, binding.CHEBYKAN_PASS_BACKWARD)
        nf = binding.chebykan_workspace_bytes(B, I, O, d, binding.CHEBYKAN_PASS_FORWARD)
        assert nb >= 0 and nf >= 0
        if nb:
            # partial coefficient tensors, or (small batches) partial dx planes if those need more room
            planes = B * I * 4
            rem = O % 128
            if O > 128 and 1 <= rem <= 4 and I * rem * (d + 1) <= 16384 and nb % per_slice and nb % planes:
                # 1..4 columns beyond the 128-wide tiles are streamed: their per-workgroup partials
                # (in x tail columns x (degree+1) floats each) lie behind the partial tensors of the tiles
                unit = I * rem * (d + 1) * 4
                assert any((nb - t * unit) > 0 and (nb - t * unit) % per_slice == 0 for t in range(1, 2049)), (B, I, O, d, nb)
                continue
            assert nb % per_slice == 0 or nb % planes == 0, (B, I, O, d, nb)
            if nb % per_slice == 0 and nb // per_slice > 64:
                assert nb // per_slice <= (B + 31) // 32, (B, I, O, d, nb)
            assert nb <= (2 << 30) + per_slice + planes
        if nf:
            assert nf % (B * O * 4) == 0 and 2 <= nf // (B * O * 4) <= 64, (B, I, O, d, nf)


def test_kernel_family_switch_round_trips():
    prev = binding.chebykan_set_kernel_family(1)
    assert binding.chebykan_set_kernel_family(prev) == 1
    assert binding.chebykan_set_kernel_family(99) == prev   # invalid value ignored
    assert binding.chebykan_set_kernel_family(prev) == prev


def test_no_device_is_reported_not_faked():
    """Without a gfx950 device the library must refuse, not fall back to the CPU."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    P = 4096
    assert binding.raw_forward(P, P, P, 4, 4, 4, 2) == binding.CHEBYKAN_ERR_DEVICE


def test_host_table_builder_matches_the_oracle_table():
    """chebykan_lut_build runs on the host: its fp32 table against the oracle's fp64 construction."""
    import oracle
    for degree, n in [(0, 2), (1, 5), (6, 1025), (8, 2049), (24, 257)]:
        lut = binding.chebykan_lut_build(degree, n).numpy()
        want = oracle.lut_build(degree, n)
        assert lut.shape == want.shape
        assert np.array_equal(lut, want.astype(np.float32))
    lib = binding.load()
    assert lib.chebykan_lut_build(None, 3, 9) == binding.CHEBYKAN_ERR_NULL
    buf = np.zeros(16, dtype=np.float32)
    assert lib.chebykan_lut_build(buf.ctypes.data, 3, 1) == binding.CHEBYKAN_ERR_SHAPE
    assert lib.chebykan_lut_build(buf.ctypes.data, -1, 4) == binding.CHEBYKAN_ERR_SHAPE
