"""Kernel logic on the CPU: the library's HIP sources are compiled with a host
compiler against an emulation of the HIP runtime (tests/emu/shim), each
workgroup runs as a group of OS threads, and AddressSanitizer watches every
global and LDS access.  This checks tiling, indexing, barriers, ragged edges
and the batch-slice reduction of the MFMA kernels without a GPU; the result is
compared with the fp64 oracle.  The emulated MFMA encodes the assumed operand
layout, which only the GPU parity tests can confirm.
"""
import os
import shutil
import subprocess
import tempfile

import numpy as np
import pytest

import oracle
from lut_checks import dx_error
from paper_2511_14852_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EMU = os.path.join(ROOT, "tests", "emu")
CSRC = os.path.join(ROOT, "paper_2511_14852_amd", "csrc")
CLANG = "/opt/rocm/lib/llvm/bin/clang++"


@pytest.fixture(scope="module")
def emu_driver():
    if not os.path.exists(CLANG):
        pytest.skip("no host clang++ for the emulation build")
    out_dir = os.path.join(EMU, "_build")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "emu_driver")
    hip_srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))
    srcs = hip_srcs + [os.path.join(EMU, "emu_state.cpp"), os.path.join(EMU, "emu_driver.cpp"),
                       os.path.join(EMU, "emu_stack_driver.cpp")]
    deps = srcs + [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(EMU, "shim", "hip", "hip_runtime.h")]
    if not os.path.exists(exe) or os.path.getmtime(exe) < max(os.path.getmtime(p) for p in deps):
        from concurrent.futures import ThreadPoolExecutor
        flags = [CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fno-omit-frame-pointer", "-Wno-psabi",
                 "-DCHEBYKAN_TEST_HOOKS",
                 "-I", os.path.join(EMU, "shim"), "-x", "c++"]

        def compile_one(src):
            obj = os.path.join(out_dir, os.path.basename(src) + ".o")
            subprocess.run([*flags, "-c", src, "-o", obj], check=True, cwd=EMU)
            return obj

        with ThreadPoolExecutor(max_workers=8) as pool:
            objs = list(pool.map(compile_one, srcs))
        drivers = {"emu_driver": "emu_driver.cpp.o", "emu_stack_driver": "emu_stack_driver.cpp.o"}
        shared = [o for o in objs if os.path.basename(o) not in drivers.values()]
        for name, obj in drivers.items():
            out = os.path.join(out_dir, name)
            subprocess.run([CLANG, "-fsanitize=address", *shared, os.path.join(out_dir, obj), "-o", out + ".tmp",
                            "-lpthread"], check=True, cwd=EMU)
            os.replace(out + ".tmp", out)
    return exe


def _run(exe, B, I, O, d, family, seed=1, lut_size=0, basis=0, tune=None, deriv_table=False):
    x = wl.make_x(B, I, seed)
    C = wl.make_coeff(I, O, d, seed + 1)
    dy = wl.make_dy(B, O, seed + 2)
    td = tempfile.mkdtemp(prefix="emu_")
    try:
        x.tofile(os.path.join(td, "x.bin"))
        C.tofile(os.path.join(td, "C.bin"))
        dy.tofile(os.path.join(td, "dy.bin"))
        args = [exe, td, str(B), str(I), str(O), str(d), str(family)]
        if lut_size:
            lut = oracle.lut_build(d, lut_size).astype(np.float32)
            lut.tofile(os.path.join(td, "lut.bin"))
            args.append(str(lut_size))
            if deriv_table:
                dlut = oracle.lut_build_derivative(d, lut_size).astype(np.float32)
                dlut.tofile(os.path.join(td, "dlut.bin"))
                args.append("9")
        elif basis:
            args += ["0", str(basis)]
        env = dict(os.environ, CHEBYKAN_TEST_HOOKS=str(tune)) if tune is not None else None
        r = subprocess.run(args, capture_output=True, text=True, timeout=600, env=env)
        assert r.returncode == 0, (r.stdout[-1000:], r.stderr[-4000:])
        y = np.fromfile(os.path.join(td, "y.bin"), dtype=np.float32).reshape(B, O)
        dx = np.fromfile(os.path.join(td, "dx.bin"), dtype=np.float32).reshape(B, I)
        dC = np.fromfile(os.path.join(td, "dC.bin"), dtype=np.float32).reshape(I, O, d + 1)
    finally:
        shutil.rmtree(td, ignore_errors=True)
    if lut_size and deriv_table:
        _, dC_ref = oracle.backward_lut(x, C, dy, lut, need_dx=False)
        return (oracle.rel_err(y, oracle.forward_lut(x, C, lut)), oracle.rel_err(dx, oracle.dx_lut2(x, C, dy, dlut)),
                oracle.rel_err(dC, dC_ref))
    if lut_size:
        _, dC_ref = oracle.backward_lut(x, C, dy, lut, need_dx=False)
        return (oracle.rel_err(y, oracle.forward_lut(x, C, lut)), dx_error(dx, x, C, dy, lut),
                oracle.rel_err(dC, dC_ref))
    if basis:
        dx_ref, dC_ref = oracle.backward_basis(basis, x, C, dy)
        return (oracle.rel_err(y, oracle.forward_basis(basis, x, C)), oracle.rel_err(dx, dx_ref),
                oracle.rel_err(dC, dC_ref))
    dx_ref, dC_ref = oracle.backward(x, C, dy)
    return (oracle.rel_err(y, oracle.forward(x, C)), oracle.rel_err(dx, dx_ref), oracle.rel_err(dC, dC_ref))


# The default run takes one case per kernel family (QUICK); CHEBYKAN_EMU_FULL=1 runs every case
# (about a quarter of an hour on 8 cores).
FULL = os.environ.get("CHEBYKAN_EMU_FULL", "0") == "1"
QUICK = {
    (140, 7, 130, 6), (129, 5, 257, 8), (140, 40, 72, 6), (300, 64, 1, 6), (40, 12, 70, 15), (33, 6, 130, 24),
    (200, 8, 64, 6),
    (130, 9, 64, 4, 65), (300, 64, 1, 6, 65),                 # table variant
    (130, 9, 64, 4, 1), (129, 5, 130, 8, 3),                  # other bases
    (129, (5, 64, 12), 3),                                    # stack calls
}


def _select(cases):
    return [c if (FULL or c in QUICK) else pytest.param(c, marks=pytest.mark.skip(reason="set CHEBYKAN_EMU_FULL=1"))
            for c in cases]


# (B, I, O, degree): ragged in every dimension, both output-tile widths, aligned and
# unaligned coefficient slabs, several batch slices
CASES = [
    (130, 9, 70, 3),
    (130, 9, 64, 4),
    (150, 13, 33, 5),
    (140, 7, 130, 6),
    (129, 5, 257, 8),
    (600, 10, 12, 6),
    # enough input features for the feature-per-lane input-gradient kernel, ragged feature
    # tiles, both chunk widths, a contraction longer than one fold
    (140, 40, 72, 6),
    (131, 70, 36, 8),
    (130, 33, 20, 3),
    (129, 34, 530, 4),
    # very narrow outputs: the streaming kernels
    (300, 64, 1, 6),
    (100, 8, 2, 3),
    (77, 70, 3, 8),
    (50, 300, 4, 5),
    # degrees added for the paper's operator shapes; small batch with a split forward contraction
    (40, 12, 70, 15),
    (33, 6, 40, 24),
    (64, 300, 72, 2),
    (70, 20, 12, 7),
    # small batches whose input-gradient contraction is split over the outputs (both dx kernels)
    (33, 6, 130, 24),
    (64, 40, 200, 5),
    # very few inputs: both gradients from the one-tile kernel (full 64-row tile, ragged tile, several slices)
    (200, 8, 64, 6),
    (100, 5, 40, 8),
    (300, 16, 33, 3),
    # at most 32 and at most 64 rows at the degrees of the paper's operator shapes: waves side by side
    (30, 9, 200, 8),
    (50, 20, 130, 15),
]


@pytest.mark.parametrize("case", _select(CASES), ids=lambda c: "B%d_I%d_O%d_d%d" % c)
def test_mfma_family_on_cpu_emulation(emu_driver, case):
    B, I, O, d = case
    errs = _run(emu_driver, B, I, O, d, family=2)
    assert all(np.isfinite(e) and e <= 1e-5 for e in errs), errs


@pytest.mark.parametrize("case", [(129, 5, 257, 8), (40, 12, 70, 15), (60, 9, 72, 8), (50, 12, 72, 15)], ids=lambda c: "B%d_I%d_O%d_d%d" % c)
def test_single_slice_dC_written_by_the_slice_kernel(emu_driver, case):
    """One batch slice: the coefficient-gradient kernel turns its tile to [i][o][k] in LDS and writes dC
    itself (forced here at a small tile count; both output-tile widths, ragged tiles, the scalar and the
    16-byte copy-out)."""
    errs = _run(emu_driver, *case, family=2, tune=2 + 4)   # test hooks: direct dC at any tile count; at least 256 rows per slice
    assert all(np.isfinite(e) and e <= 1e-5 for e in errs), errs


@pytest.mark.parametrize("case", [(140, 65, 40, 5), (130, 73, 36, 6)], ids=lambda c: "B%d_I%d_O%d_d%d" % c)
def test_input_gradient_with_a_second_launch_for_the_last_features(emu_driver, case):
    """Feature counts just above a multiple of 32: feature-per-lane tiles plus a packed-column launch over
    the last 1 and 9 features (one and two column blocks), forced here at a small amount of work."""
    errs = _run(emu_driver, *case, family=2, tune=8)
    assert all(np.isfinite(e) and e <= 1e-5 for e in errs), errs


def test_generic_family_on_cpu_emulation(emu_driver):
    errs = _run(emu_driver, 37, 11, 9, 7, family=1)
    assert all(np.isfinite(e) and e <= 1e-5 for e in errs), errs


# (B, I, O, degree, table size): the table-interpolated form of each kernel family, a table too
# large for staging (any-degree kernels with the table in global memory) and the smallest table
LUT_CASES = [
    (130, 9, 64, 4, 65),
    (140, 40, 72, 6, 129),
    (129, 5, 257, 8, 33),
    (300, 64, 1, 6, 65),
    (100, 8, 2, 3, 17),
    (64, 300, 72, 2, 2),
    (40, 6, 20, 6, 4097),
]


@pytest.mark.parametrize("case", _select(LUT_CASES), ids=lambda c: "B%d_I%d_O%d_d%d_n%d" % c)
def test_table_variant_on_cpu_emulation(emu_driver, case):
    B, I, O, d, n = case
    errs = _run(emu_driver, B, I, O, d, family=2, lut_size=n)
    assert all(np.isfinite(e) and e <= 1e-5 for e in errs), errs


# the same with dx from the auxiliary derivative table (both tables staged in LDS): one case per kernel that
# evaluates a derivative - both matrix-core dx kernels, the streaming kernel, the few-inputs kernel
LUT2_CASES = [
    (140, 40, 72, 6, 129),
    (129, 5, 257, 8, 33),
    (300, 64, 1, 6, 65),
    (200, 8, 64, 6, 65),
]
QUICK |= {(140, 40, 72, 6, 129, "d"), (200, 8, 64, 6, 65, "d")}


@pytest.mark.parametrize("case", _select([c + ("d",) for c in LUT2_CASES]), ids=lambda c: "B%d_I%d_O%d_d%d_n%d_%s" % c)
def test_derivative_table_variant_on_cpu_emulation(emu_driver, case):
    B, I, O, d, n, _ = case
    errs = _run(emu_driver, B, I, O, d, family=2, lut_size=n, deriv_table=True)
    assert all(np.isfinite(e) and e <= 1e-5 for e in errs), errs


# (B, I, O, degree, basis): Legendre (1), Hermite (2), Fourier (3) on the matrix-core, streaming and any-degree kernels
BASIS_CASES = [
    (130, 9, 64, 4, 1),
    (140, 40, 72, 6, 2),
    (129, 5, 130, 8, 3),
    (300, 64, 1, 6, 3),
    (60, 11, 9, 7, 2),
]


@pytest.mark.parametrize("case", _select(BASIS_CASES), ids=lambda c: "B%d_I%d_O%d_d%d_basis%d" % c)
def test_other_bases_on_cpu_emulation(emu_driver, case):
    B, I, O, d, basis = case
    errs = _run(emu_driver, B, I, O, d, family=2, basis=basis)
    assert all(np.isfinite(e) and e <= 1e-5 for e in errs), errs


# (B, widths, degree): stack calls - forward of a narrow stack in one kernel (forced at these small batches),
# backward with every small slice sum in one launch: ragged
# last row tile, narrow and matrix-core last layers, a hidden width below 64
STACK_CASES = [
    (200, (8, 64, 64, 1), 6),
    (150, (9, 16, 48, 3), 4),
    (129, (5, 64, 12), 3),
]


@pytest.mark.parametrize("case", _select(STACK_CASES), ids=lambda c: "B%d_%s_d%d" % (c[0], "x".join(map(str, c[1])), c[2]))
def test_stack_calls_on_cpu_emulation(emu_driver, case):
    B, widths, d = case
    exe = os.path.join(os.path.dirname(emu_driver), "emu_stack_driver")
    x = wl.make_x(B, widths[0], 77)
    dy = wl.make_dy(B, widths[-1], 78)
    Cs = [wl.make_coeff(i, o, d, 80 + l) for l, (i, o) in enumerate(zip(widths[:-1], widths[1:]))]
    td = tempfile.mkdtemp(prefix="emu_")
    try:
        x.tofile(os.path.join(td, "x.bin"))
        dy.tofile(os.path.join(td, "dy.bin"))
        for l, c in enumerate(Cs):
            c.tofile(os.path.join(td, "C%d.bin" % l))
        env = dict(os.environ, CHEBYKAN_TEST_HOOKS="1")   # fuse the forward at this small batch
        r = subprocess.run([exe, td, str(B), str(d), str(len(Cs)), *map(str, widths)], capture_output=True, text=True,
                           timeout=600, env=env)
        assert r.returncode == 0, (r.stdout[-1000:], r.stderr[-4000:])
        ys = [np.fromfile(os.path.join(td, "y%d.bin" % l), dtype=np.float32).reshape(B, widths[l + 1])
              for l in range(len(Cs))]
        gs = [np.fromfile(os.path.join(td, "g%d.bin" % l), dtype=np.float32).reshape(B, widths[l])
              for l in range(len(Cs))] + [dy]
        dCs = [np.fromfile(os.path.join(td, "dC%d.bin" % l), dtype=np.float32).reshape(Cs[l].shape)
               for l in range(len(Cs))]
    finally:
        shutil.rmtree(td, ignore_errors=True)
    xin = x
    for l, c in enumerate(Cs):             # per layer, on the kernel's own fp32 layer input
        err = oracle.rel_err(ys[l], oracle.forward(xin, c))
        assert np.isfinite(err) and err <= 1e-5, (l, err)
        # backward of the layer on the kernels' own incoming gradient; the slice sums of all layers ran in one launch
        dx_ref, dC_ref = oracle.backward(xin, c, gs[l + 1])
        errs = (oracle.rel_err(gs[l], dx_ref), oracle.rel_err(dCs[l], dC_ref))
        assert all(np.isfinite(e) and e <= 1e-5 for e in errs), (l, errs)
        xin = ys[l]
