// C ABI of the library: argument validation, kernel choice, launches.
// See include/chebykan.h for the contract of every entry point.
#include <hip/hip_runtime.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "../../include/chebykan.h"
#include "dispatch.h"
#include "generic_kernels.h"
#include "launch.h"
#include "runtime.h"

namespace chebykan {

// Scratch of chebykan_backward_noalloc: one array per GPU that loads the library, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress - never a device
// address: everything below uses the per-device address that call returns.
static __device__ __align__(256) unsigned char scratch[CHEBYKAN_NOALLOC_SCRATCH_BYTES];

// Device address of `scratch` on the current device, looked up once per device.
static chebykan_status scratch_address(void** out)
{
    constexpr int MAX_DEVICES = 64;
    static std::atomic<void*> address[MAX_DEVICES];
    static std::mutex lookup_mutex;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        return CHEBYKAN_ERR_DEVICE;
    }
    void* p = address[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(lookup_mutex);
        p = address[dev].load();
        if (!p) {
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                (void)hipGetLastError();
                return CHEBYKAN_ERR_LAUNCH;
            }
            address[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return CHEBYKAN_OK;
}

static bool shape_ok(int64_t batch, int in, int out, int degree)
{
    if (batch < 0 || in <= 0 || out <= 0 || degree < 0 || degree > CHEBYKAN_MAX_DEGREE) return false;
    const int64_t lim = (int64_t)1 << 40;  // element counts stay far inside int64
    if (batch * in > lim || batch * out > lim) return false;
    if ((int64_t)in * out * (degree + 1) > ((int64_t)1 << 31) - 1) return false;
    if (batch > ((int64_t)1 << 31) - 1) return false;
    return true;
}

static chebykan_status launch_status()
{
    return hipGetLastError() == hipSuccess ? CHEBYKAN_OK : CHEBYKAN_ERR_LAUNCH;
}

static void generic_forward(const float* x, const float* C, float* y, int64_t B, int I, int O, int d,
                            hipStream_t s)
{
    const ScopedOps ops(OP_FWD);
    dim3 block(64, 4), grid((unsigned)((B + 3) / 4), (unsigned)((O + 63) / 64));
    launch<generic_forward_kernel>(grid, block, 0, s, x, C, y, B, I, O, d);
}

static void generic_dx(const float* x, const float* C, const float* dy, float* dx, int64_t B, int I, int O,
                       int d, hipStream_t s)
{
    const ScopedOps ops(OP_DX);
    dim3 block(64, 4), grid((unsigned)((B + 3) / 4), (unsigned)((I + 63) / 64));
    launch<generic_dx_kernel>(grid, block, 0, s, x, C, dy, dx, B, I, O, d);
}

static void generic_dC(const float* x, const float* dy, float* dC, int64_t B, int I, int O, int d,
                       hipStream_t s)
{
    const ScopedOps ops(OP_DC);
    const int64_t n = (int64_t)I * O * (d + 1);
    launch<generic_dC_kernel>(dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, x, dy, dC, B, I,
                       O, d);
}

static void generic_forward_table(const float* x, const float* C, const float* lut, int n, float* y, int64_t B,
                                  int I, int O, int d, hipStream_t s)
{
    const ScopedOps ops(OP_FWD);
    dim3 block(64, 4), grid((unsigned)((B + 3) / 4), (unsigned)((O + 63) / 64));
    launch<generic_forward_table_kernel>(grid, block, 0, s, x, C, lut, n, y, B, I, O, d);
}

static void generic_dx_table(const float* x, const float* C, const float* dy, const float* lut, int n, float* dx,
                             int64_t B, int I, int O, int d, hipStream_t s)
{
    const ScopedOps ops(OP_DX);
    dim3 block(64, 4), grid((unsigned)((B + 3) / 4), (unsigned)((I + 63) / 64));
    launch<generic_dx_table_kernel>(grid, block, 0, s, x, C, dy, lut, n, dx, B, I, O, d);
}

static void generic_dx_table2(const float* x, const float* C, const float* dy, const float* dlut, int n, float* dx,
                              int64_t B, int I, int O, int d, hipStream_t s)
{
    const ScopedOps ops(OP_DX);
    dim3 block(64, 4), grid((unsigned)((B + 3) / 4), (unsigned)((I + 63) / 64));
    launch<generic_dx_table2_kernel>(grid, block, 0, s, x, C, dy, dlut, n, dx, B, I, O, d);
}

static void generic_dC_table(const float* x, const float* dy, const float* lut, int n, float* dC, int64_t B, int I,
                             int O, int d, hipStream_t s)
{
    const ScopedOps ops(OP_DC);
    const int64_t cnt = (int64_t)I * O * (d + 1);
    launch<generic_dC_table_kernel>(dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, s, x, dy, lut, n,
                       dC, B, I, O, d);
}

}  // namespace chebykan

using namespace chebykan;

extern "C" {

int chebykan_version(void) { return 1000; }

chebykan_status chebykan_init(void)
{
    const chebykan_status st = prepare_device();
    if (st != CHEBYKAN_OK) return st;
    void* p = nullptr;
    return scratch_address(&p);   // so that chebykan_backward_noalloc has nothing left to look up
}

const char* chebykan_status_string(chebykan_status status)
{
    switch (status) {
        case CHEBYKAN_OK: return "ok";
        case CHEBYKAN_ERR_NULL: return "a required pointer is NULL";
        case CHEBYKAN_ERR_SHAPE: return "invalid shape or degree";
        case CHEBYKAN_ERR_WORKSPACE: return "workspace missing or too small";
        case CHEBYKAN_ERR_DEVICE: return "no gfx950 device is current";
        case CHEBYKAN_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

size_t chebykan_workspace_bytes(int64_t batch, int in, int out, int degree, int pass)
{
    if (!shape_ok(batch, in, out, degree)) return 0;
    if (pass == CHEBYKAN_PASS_FORWARD) return forward_workspace_bytes(batch, in, out, degree);
    if (pass == CHEBYKAN_PASS_BACKWARD) return backward_workspace_bytes(batch, in, out, degree);
    return 0;
}

chebykan_status chebykan_forward(const float* x, const float* C, float* y, int64_t batch, int in, int out,
                                 int degree, void* workspace, size_t workspace_bytes,
                                 chebykan_stream_t stream)
{
    if (!C || (batch != 0 && (!x || !y))) return CHEBYKAN_ERR_NULL;  // empty tensors may be NULL
    if (!shape_ok(batch, in, out, degree)) return CHEBYKAN_ERR_SHAPE;
    const size_t need = forward_workspace_bytes(batch, in, out, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    if (batch == 0) return CHEBYKAN_OK;
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (kernel_family() != 1 && fast_forward(x, C, y, batch, in, out, degree, workspace, s)) return launch_status();
    generic_forward(x, C, y, batch, in, out, degree, s);
    return launch_status();
}

chebykan_status chebykan_backward(const float* x, const float* C, const float* dy, float* dx, float* dC,
                                  int64_t batch, int in, int out, int degree, void* workspace,
                                  size_t workspace_bytes, chebykan_stream_t stream)
{
    if (!C || (batch != 0 && (!x || !dy))) return CHEBYKAN_ERR_NULL;  // empty tensors may be NULL
    if (!dx && !dC && batch != 0) return CHEBYKAN_ERR_NULL;
    if (!shape_ok(batch, in, out, degree)) return CHEBYKAN_ERR_SHAPE;
    const size_t need = backward_workspace_bytes(batch, in, out, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (kernel_family() != 1 && batch > 0 && fast_backward(x, C, dy, dx, dC, batch, in, out, degree, workspace, s))
        return launch_status();
    if (dx && batch > 0) generic_dx(x, C, dy, dx, batch, in, out, degree, s);
    // batch == 0 still defines dC (all zeros): the generic kernel's empty sum gives that.
    if (dC) generic_dC(x, dy, dC, batch, in, out, degree, s);
    return launch_status();
}

chebykan_status chebykan_backward_noalloc(const float* x, const float* C, const float* dy, float* dx, float* dC,
                                          int64_t batch, int in, int out, int degree, chebykan_stream_t stream)
{
    if (!C || (batch != 0 && (!x || !dy))) return CHEBYKAN_ERR_NULL;
    if (!dx && !dC && batch != 0) return CHEBYKAN_ERR_NULL;
    if (!shape_ok(batch, in, out, degree)) return CHEBYKAN_ERR_SHAPE;
    if (backward_workspace_bytes(batch, in, out, degree) > (size_t)CHEBYKAN_NOALLOC_SCRATCH_BYTES)
        return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    void* ws = nullptr;
    const chebykan_status st = scratch_address(&ws);
    if (st != CHEBYKAN_OK) return st;
    // The kernels write every scratch element they later read within this call, so what an earlier
    // call left there does not matter and nothing is cleared.
    return chebykan_backward(x, C, dy, dx, dC, batch, in, out, degree, ws, CHEBYKAN_NOALLOC_SCRATCH_BYTES, stream);
}

chebykan_status chebykan_lut_build(float* lut, int degree, int lut_size)
{
    if (!lut) return CHEBYKAN_ERR_NULL;
    if (degree < 0 || degree > CHEBYKAN_MAX_DEGREE || lut_size < 2 || lut_size > CHEBYKAN_MAX_LUT_SIZE)
        return CHEBYKAN_ERR_SHAPE;
    // Samples of T_0..T_degree on the uniform grid, recurrence in double, rounded once to fp32.
    const double step = 2.0 / (double)(lut_size - 1);
    for (int i = 0; i < lut_size; ++i) {
        const double xi = i == lut_size - 1 ? 1.0 : (double)i * step - 1.0;
        double below = 1.0, here = xi;   // T_{k-1}, T_k
        lut[i] = 1.0f;
        if (degree >= 1) lut[(size_t)lut_size + i] = (float)xi;
        for (int k = 2; k <= degree; ++k) {
            const double above = 2.0 * xi * here - below;
            lut[(size_t)k * lut_size + i] = (float)above;
            below = here;
            here = above;
        }
    }
    return CHEBYKAN_OK;
}

chebykan_status chebykan_lut_build_derivative(float* dlut, int degree, int lut_size)
{
    if (!dlut) return CHEBYKAN_ERR_NULL;
    if (degree < 0 || degree > CHEBYKAN_MAX_DEGREE || lut_size < 2 || lut_size > CHEBYKAN_MAX_LUT_SIZE)
        return CHEBYKAN_ERR_SHAPE;
    // Samples of T_k' = k U_{k-1} on the uniform grid: second-kind recurrence in double, rounded once to fp32.
    const double step = 2.0 / (double)(lut_size - 1);
    for (int i = 0; i < lut_size; ++i) {
        const double xi = i == lut_size - 1 ? 1.0 : (double)i * step - 1.0;
        double second_below = 0.0, second_here = 1.0;   // U_{k-2}, U_{k-1}
        dlut[i] = 0.0f;
        for (int k = 1; k <= degree; ++k) {
            dlut[(size_t)k * lut_size + i] = (float)((double)k * second_here);
            const double second_above = 2.0 * xi * second_here - second_below;
            second_below = second_here;
            second_here = second_above;
        }
    }
    return CHEBYKAN_OK;
}

chebykan_status chebykan_backward_lut2(const float* x, const float* C, const float* dy, const float* lut,
                                       const float* dlut, int lut_size, float* dx, float* dC, int64_t batch, int in,
                                       int out, int degree, void* workspace, size_t workspace_bytes,
                                       chebykan_stream_t stream)
{
    if (!C || !lut || !dlut || (batch != 0 && (!x || !dy))) return CHEBYKAN_ERR_NULL;
    if (!dx && !dC && batch != 0) return CHEBYKAN_ERR_NULL;
    if (!shape_ok(batch, in, out, degree) || lut_size < 2 || lut_size > CHEBYKAN_MAX_LUT_SIZE)
        return CHEBYKAN_ERR_SHAPE;
    const size_t need = backward_workspace_bytes(batch, in, out, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (kernel_family() != 1 && batch > 0 &&
        fast_backward_table2(x, C, dy, lut, dlut, lut_size, dx, dC, batch, in, out, degree, workspace, s))
        return launch_status();
    // two tables too large for LDS, or a degree without table kernels: each gradient on its own path
    if (dx && batch > 0) generic_dx_table2(x, C, dy, dlut, lut_size, dx, batch, in, out, degree, s);
    if (dC) {
        if (kernel_family() != 1 && batch > 0 &&
            fast_backward_table(x, C, dy, lut, lut_size, nullptr, dC, batch, in, out, degree, workspace, s))
            return launch_status();
        generic_dC_table(x, dy, lut, lut_size, dC, batch, in, out, degree, s);
    }
    return launch_status();
}

chebykan_status chebykan_forward_lut(const float* x, const float* C, const float* lut, int lut_size, float* y,
                                     int64_t batch, int in, int out, int degree, void* workspace,
                                     size_t workspace_bytes, chebykan_stream_t stream)
{
    if (!C || !lut || (batch != 0 && (!x || !y))) return CHEBYKAN_ERR_NULL;
    if (!shape_ok(batch, in, out, degree) || lut_size < 2 || lut_size > CHEBYKAN_MAX_LUT_SIZE)
        return CHEBYKAN_ERR_SHAPE;
    const size_t need = forward_workspace_bytes(batch, in, out, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    if (batch == 0) return CHEBYKAN_OK;
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (kernel_family() != 1 && fast_forward_table(x, C, lut, lut_size, y, batch, in, out, degree, workspace, s))
        return launch_status();
    generic_forward_table(x, C, lut, lut_size, y, batch, in, out, degree, s);
    return launch_status();
}

chebykan_status chebykan_backward_lut(const float* x, const float* C, const float* dy, const float* lut,
                                      int lut_size, float* dx, float* dC, int64_t batch, int in, int out,
                                      int degree, void* workspace, size_t workspace_bytes,
                                      chebykan_stream_t stream)
{
    if (!C || !lut || (batch != 0 && (!x || !dy))) return CHEBYKAN_ERR_NULL;
    if (!dx && !dC && batch != 0) return CHEBYKAN_ERR_NULL;
    if (!shape_ok(batch, in, out, degree) || lut_size < 2 || lut_size > CHEBYKAN_MAX_LUT_SIZE)
        return CHEBYKAN_ERR_SHAPE;
    const size_t need = backward_workspace_bytes(batch, in, out, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (kernel_family() != 1 && batch > 0 &&
        fast_backward_table(x, C, dy, lut, lut_size, dx, dC, batch, in, out, degree, workspace, s))
        return launch_status();
    if (dx && batch > 0) generic_dx_table(x, C, dy, lut, lut_size, dx, batch, in, out, degree, s);
    if (dC) generic_dC_table(x, dy, lut, lut_size, dC, batch, in, out, degree, s);
    return launch_status();
}

static bool stack_ok(int n_layers, const int* widths, int degree, int64_t batch)
{
    if (n_layers < 1 || n_layers > CHEBYKAN_MAX_LAYERS || !widths) return false;
    for (int l = 0; l < n_layers; ++l)
        if (!shape_ok(batch, widths[l], widths[l + 1], degree)) return false;
    return true;
}

size_t chebykan_stack_workspace_bytes(int64_t batch, int n_layers, const int* widths, int degree)
{
    if (!widths || n_layers < 1 || n_layers > CHEBYKAN_MAX_LAYERS) return 0;
    size_t need = 0;
    for (int l = 0; l < n_layers; ++l) {
        const size_t f = chebykan_workspace_bytes(batch, widths[l], widths[l + 1], degree, CHEBYKAN_PASS_FORWARD);
        const size_t b = chebykan_workspace_bytes(batch, widths[l], widths[l + 1], degree, CHEBYKAN_PASS_BACKWARD);
        if (f > need) need = f;
        if (b > need) need = b;
    }
    // the backward pass keeps every layer's partial sums until its single combine launch
    if (stack_ok(n_layers, widths, degree, batch)) {
        const size_t all = stack_backward_workspace_bytes(n_layers, widths, degree, batch);
        if (all > need) need = all;
    }
    return need;
}

chebykan_status chebykan_stack_forward(int n_layers, const int* widths, int degree, int64_t batch,
                                       const float* const* C, float* const* act, void* workspace,
                                       size_t workspace_bytes, chebykan_stream_t stream)
{
    if (!widths || !C || !act) return CHEBYKAN_ERR_NULL;
    if (n_layers < 1 || n_layers > CHEBYKAN_MAX_LAYERS) return CHEBYKAN_ERR_SHAPE;
    for (int l = 0; l < n_layers; ++l)
        if (!C[l] || (batch != 0 && (!act[l] || !act[l + 1]))) return CHEBYKAN_ERR_NULL;
    if (!stack_ok(n_layers, widths, degree, batch)) return CHEBYKAN_ERR_SHAPE;
    const size_t need = chebykan_stack_workspace_bytes(batch, n_layers, widths, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    if (batch == 0) return CHEBYKAN_OK;
    // narrow stacks run all layers in one kernel, each workgroup keeping its rows' activations in LDS
    (void)hipGetLastError();
    if (kernel_family() != 1 && fast_chain_forward(n_layers, widths, degree, batch, C, act, (hipStream_t)stream))
        return launch_status();
    // every argument is validated: the per-layer calls below can only fail at launch
    for (int l = 0; l < n_layers; ++l) {
        const ScopedLayer layer(l);
        const chebykan_status st = chebykan_forward(act[l], C[l], act[l + 1], batch, widths[l], widths[l + 1], degree,
                                                    workspace, workspace_bytes, stream);
        if (st != CHEBYKAN_OK) return st;
    }
    return CHEBYKAN_OK;
}

chebykan_status chebykan_stack_backward(int n_layers, const int* widths, int degree, int64_t batch,
                                        const float* const* C, const float* const* act, float* const* grad,
                                        float* const* dC, void* workspace, size_t workspace_bytes,
                                        chebykan_stream_t stream)
{
    if (!widths || !C || !act || !grad || !dC) return CHEBYKAN_ERR_NULL;
    if (n_layers < 1 || n_layers > CHEBYKAN_MAX_LAYERS) return CHEBYKAN_ERR_SHAPE;
    for (int l = 0; l < n_layers; ++l) {
        if (!C[l] || (batch != 0 && (!act[l] || !grad[l + 1]))) return CHEBYKAN_ERR_NULL;
        if (l == 0 && !grad[0] && !dC[0] && batch != 0) return CHEBYKAN_ERR_NULL;   // layer 0 would have nothing to do
    }
    if (!stack_ok(n_layers, widths, degree, batch)) return CHEBYKAN_ERR_SHAPE;
    const size_t need = chebykan_stack_workspace_bytes(batch, n_layers, widths, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    if (batch > 0 && kernel_family() != 1) {
        (void)hipGetLastError();
        if (fast_stack_backward(n_layers, widths, degree, batch, C, act, grad, dC, workspace, (hipStream_t)stream))
            return launch_status();
    }
    for (int l = n_layers - 1; l >= 0; --l) {
        const ScopedLayer layer(l);
        const chebykan_status st = chebykan_backward(act[l], C[l], grad[l + 1], grad[l], dC[l], batch, widths[l],
                                                     widths[l + 1], degree, workspace, workspace_bytes, stream);
        if (st != CHEBYKAN_OK) return st;
    }
    return CHEBYKAN_OK;
}

static bool basis_ok(int basis, int degree)
{
    if (basis < CHEBYKAN_BASIS_CHEBYSHEV || basis > CHEBYKAN_BASIS_FOURIER) return false;
    return basis != CHEBYKAN_BASIS_FOURIER || degree % 2 == 0;
}

chebykan_status chebykan_forward_basis(int basis, const float* x, const float* C, float* y, int64_t batch, int in,
                                       int out, int degree, void* workspace, size_t workspace_bytes,
                                       chebykan_stream_t stream)
{
    if (basis == CHEBYKAN_BASIS_CHEBYSHEV)
        return chebykan_forward(x, C, y, batch, in, out, degree, workspace, workspace_bytes, stream);
    if (!C || (batch != 0 && (!x || !y))) return CHEBYKAN_ERR_NULL;
    if (!shape_ok(batch, in, out, degree) || !basis_ok(basis, degree)) return CHEBYKAN_ERR_SHAPE;
    const size_t need = forward_workspace_bytes(batch, in, out, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    if (batch == 0) return CHEBYKAN_OK;
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (kernel_family() != 1 && fast_forward_family(basis, x, C, y, batch, in, out, degree, workspace, s))
        return launch_status();
    const ScopedOps ops(OP_FWD);
    dim3 block(64, 4), grid((unsigned)((batch + 3) / 4), (unsigned)((out + 63) / 64));
    launch<generic_forward_family_kernel>(grid, block, 0, s, basis, x, C, y, batch, in, out, degree);
    return launch_status();
}

chebykan_status chebykan_backward_basis(int basis, const float* x, const float* C, const float* dy, float* dx,
                                        float* dC, int64_t batch, int in, int out, int degree, void* workspace,
                                        size_t workspace_bytes, chebykan_stream_t stream)
{
    if (basis == CHEBYKAN_BASIS_CHEBYSHEV)
        return chebykan_backward(x, C, dy, dx, dC, batch, in, out, degree, workspace, workspace_bytes, stream);
    if (!C || (batch != 0 && (!x || !dy))) return CHEBYKAN_ERR_NULL;
    if (!dx && !dC && batch != 0) return CHEBYKAN_ERR_NULL;
    if (!shape_ok(batch, in, out, degree) || !basis_ok(basis, degree)) return CHEBYKAN_ERR_SHAPE;
    const size_t need = backward_workspace_bytes(batch, in, out, degree);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CHEBYKAN_ERR_WORKSPACE;
    const chebykan_status dev = prepare_device();
    if (dev != CHEBYKAN_OK) return dev;
    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (kernel_family() != 1 && batch > 0 &&
        fast_backward_family(basis, x, C, dy, dx, dC, batch, in, out, degree, workspace, s))
        return launch_status();
    if (dx && batch > 0) {
        const ScopedOps ops(OP_DX);
        dim3 block(64, 4), grid((unsigned)((batch + 3) / 4), (unsigned)((in + 63) / 64));
        launch<generic_dx_family_kernel>(grid, block, 0, s, basis, x, C, dy, dx, batch, in, out, degree);
    }
    if (dC) {
        const ScopedOps ops(OP_DC);
        const int64_t cnt = (int64_t)in * out * (degree + 1);
        launch<generic_dC_family_kernel>(dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, s, basis, x, dy,
                           dC, batch, in, out, degree);
    }
    return launch_status();
}

}  // extern "C"
