/*
 * chebykan.h - C ABI of the fused Chebyshev-KAN layer for AMD MI355X (gfx950).
 *
 * One layer maps x[batch,in] to y[batch,out] through per-edge Chebyshev
 * expansions of tanh(x) (paper Sec. 2.2: Eq. 2 for the basis, Eq. 3 and the
 * Fig. 3 caption for the contraction; Alg. 1 for forward, Alg. 2 for backward):
 *
 *   u[b,i]    = tanh(x[b,i])
 *   T_0 = 1, T_1 = u, T_{k+1} = 2 u T_k - T_{k-1}
 *   y[b,o]    = sum_i sum_{k=0..degree} C[i,o,k] * T_k(u[b,i])
 *   dC[i,o,k] = sum_b T_k(u[b,i]) * dy[b,o]
 *   dx[b,i]   = (1 - u^2) * sum_o dy[b,o] * sum_{k=1..degree} C[i,o,k] * T_k'(u)
 *
 * There is no bias term.  dx is the gradient with respect to the raw input, so
 * it carries the tanh derivative.  chebykan_forward / chebykan_backward evaluate
 * the basis and its derivative exactly (three-term recurrences); the *_lut entry
 * points further down are the paper's table-interpolated variant.
 *
 * Conventions common to every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller, fp32,
 *    row-major and contiguous, at least 4-byte aligned (16-byte alignment of
 *    the base pointers enables the vectorised paths):
 *        x  [batch, in]      C  [in, out, degree+1]   (the paper's original
 *        y  [batch, out]     dC [in, out, degree+1]    coefficient layout,
 *        dy [batch, out]     dx [batch, in]            Sec. 4.5.1)
 *  - Outputs are OVERWRITTEN (never accumulated into); inputs are not modified;
 *    outputs must not alias inputs.
 *  - `workspace` is device memory owned by the caller, at least
 *    chebykan_workspace_bytes(...) bytes, 256-byte aligned; it may be NULL when
 *    that size is 0.  Its contents are scratch: undefined before and after.
 *  - `stream` is a hipStream_t passed as an opaque pointer (NULL = the null
 *    stream).  All work is enqueued on it; the call returns without
 *    synchronising.  The library allocates nothing and frees nothing.
 *  - Entry points may be called from several host threads at once (on
 *    different streams or devices); the library keeps no per-call state.
 *  - Results are bitwise reproducible from run to run for fixed shapes: every
 *    reduction has a fixed order and no floating-point atomics are used.
 *  - batch == 0 is a successful no-op for forward and dx; dC is then zeroed.
 *    Pointers to tensors that have no elements (x, y, dy, dx at batch == 0)
 *    may be NULL.
 *  - Errors are reported by return code only.  On any error nothing has been
 *    enqueued.
 */
#ifndef CHEBYKAN_H
#define CHEBYKAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CHEBYKAN_MAX_DEGREE 32

typedef enum chebykan_status {
    CHEBYKAN_OK = 0,
    CHEBYKAN_ERR_NULL = -1,      /* a required pointer is NULL                         */
    CHEBYKAN_ERR_SHAPE = -2,     /* batch < 0, in/out <= 0, degree < 0 or > MAX_DEGREE,
                                    or a tensor would exceed 2^31-1 rows*cols limits   */
    CHEBYKAN_ERR_WORKSPACE = -3, /* workspace NULL or smaller than required            */
    CHEBYKAN_ERR_DEVICE = -4,    /* current device is not a gfx950 part                */
    CHEBYKAN_ERR_LAUNCH = -5     /* HIP reported an error when launching               */
} chebykan_status;

typedef void *chebykan_stream_t; /* a hipStream_t */

/* pass selector for chebykan_workspace_bytes */
#define CHEBYKAN_PASS_FORWARD 0
#define CHEBYKAN_PASS_BACKWARD 1

/*
 * Bytes of workspace the given call needs (0 is possible).  Host-only, no GPU
 * access.  Returns 0 for invalid shapes (the compute call will report them).
 * Backward needs room for the per-slice partial coefficient gradients of the
 * deterministic two-stage reduction (the idea of the paper's Sec. 4.4 applied
 * to the batch axis).
 */
size_t chebykan_workspace_bytes(int64_t batch, int in, int out, int degree, int pass);

/*
 * Forward pass (paper Alg. 1 as a function; Eq. 2-3): writes y[batch,out].
 */
chebykan_status chebykan_forward(const float *x, const float *C, float *y,
                                 int64_t batch, int in, int out, int degree,
                                 void *workspace, size_t workspace_bytes,
                                 chebykan_stream_t stream);

/*
 * Backward pass (paper Alg. 2 as a function): writes dx[batch,in] and
 * dC[in,out,degree+1].  Either output pointer may be NULL to skip it (not both
 * required).  Nothing is kept from the forward call: u, T_k and T_k' are
 * regenerated from x.
 */
chebykan_status chebykan_backward(const float *x, const float *C, const float *dy,
                                  float *dx, float *dC,
                                  int64_t batch, int in, int out, int degree,
                                  void *workspace, size_t workspace_bytes,
                                  chebykan_stream_t stream);

/*
 * chebykan_backward for callers that can neither allocate nor hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same
 * arguments (without the workspace) and same results, bit for bit, as chebykan_backward; the
 * partial coefficient gradients and split-contraction planes go to a scratch array of
 * CHEBYKAN_NOALLOC_SCRATCH_BYTES that is part of the library's device image (every GPU the
 * library runs on holds it until the process ends).  A shape whose
 * chebykan_workspace_bytes(..., CHEBYKAN_PASS_BACKWARD) exceeds that size is refused with
 * CHEBYKAN_ERR_WORKSPACE and nothing is enqueued.  The call allocates and frees nothing; its
 * only set-up is a symbol-address lookup on the first call per device, which chebykan_init does
 * ahead of time (call that before a stream capture).  All calls on one GPU share the one array:
 * two such calls that may run at the same time on that GPU (different streams, or graphs
 * replayed concurrently) race and give undefined results - keep them on one stream or order them.
 * The array keeps what the last call left in it; no call depends on its contents.
 */
#define CHEBYKAN_NOALLOC_SCRATCH_BYTES (32u << 20)
chebykan_status chebykan_backward_noalloc(const float *x, const float *C, const float *dy,
                                          float *dx, float *dC,
                                          int64_t batch, int in, int out, int degree,
                                          chebykan_stream_t stream);

/*
 * Table-interpolated variant (paper Sec. 4.2, "Polynomial Operators Acceleration
 * via LUT").  The basis is not evaluated by the recurrence but read from a table
 *
 *   LUT[k][i] = T_k(-1 + i*Delta),  Delta = 2/(lut_size-1),  k = 0..degree,
 *                                                             i = 0..lut_size-1   (Sec. 4.2.1)
 *
 * by linear interpolation (Sec. 4.2.2): with u = tanh(x), pos = (u+1)/2*(lut_size-1),
 * c = min(floor(pos), lut_size-2), f = pos - c,
 *
 *   T_k(u)  ~ LUT[k][c] + f*(LUT[k][c+1] - LUT[k][c])
 *   T_k'(u) ~ (LUT[k][c+1] - LUT[k][c]) / Delta        (difference of adjacent samples)
 *
 * and y, dC, dx are formed from these exactly as in the exact entry points (dx
 * again includes the factor 1 - u^2).  The result is an APPROXIMATION of the exact
 * layer: the value error is at most Delta^2/8 * k^2(k^2-1)/3 per basis function,
 * the derivative is only first-order accurate (error up to Delta * k^2(k^2-1)/3).
 *
 * chebykan_lut_build fills a HOST array of (degree+1)*lut_size floats, row k at
 * lut + k*lut_size, from the recurrence in double precision (the "offline
 * construction on the CPU" of Sec. 4.2.1); the caller copies it to the device.
 *
 * chebykan_forward_lut / chebykan_backward_lut take that table as a DEVICE
 * pointer `lut` in the same layout; every other argument, the workspace size
 * (chebykan_workspace_bytes of the same shape), ownership, overwrite semantics,
 * reproducibility and error behaviour are those of chebykan_forward /
 * chebykan_backward.  Tables of up to 80 KiB ((degree+1)*lut_size*4 bytes) at
 * degrees 2..8 are staged in on-chip memory by the matrix-core kernels; larger
 * tables and other degrees run on the any-degree kernels, which read the table
 * from global memory.  2 <= lut_size <= CHEBYKAN_MAX_LUT_SIZE, else
 * CHEBYKAN_ERR_SHAPE.
 */
#define CHEBYKAN_MAX_LUT_SIZE (1 << 20)
chebykan_status chebykan_lut_build(float *lut, int degree, int lut_size);
chebykan_status chebykan_forward_lut(const float *x, const float *C, const float *lut, int lut_size, float *y,
                                     int64_t batch, int in, int out, int degree,
                                     void *workspace, size_t workspace_bytes, chebykan_stream_t stream);
chebykan_status chebykan_backward_lut(const float *x, const float *C, const float *dy, const float *lut,
                                      int lut_size, float *dx, float *dC,
                                      int64_t batch, int in, int out, int degree,
                                      void *workspace, size_t workspace_bytes, chebykan_stream_t stream);

/*
 * Second-order derivative for the table variant.  Sec. 4.2.2 names two sources for the
 * derivative: the difference of neighbouring samples (chebykan_backward_lut above, first order
 * in Delta) or an auxiliary table.  Here the auxiliary table holds samples of the derivative,
 *
 *   dLUT[k][i] = T_k'(-1 + i*Delta) = k U_{k-1}(-1 + i*Delta),     same grid, same layout,
 *   T_k'(u) ~ dLUT[k][c] + f*(dLUT[k][c+1] - dLUT[k][c])            same cell c and fraction f,
 *
 * whose error is at most Delta^2/8 * k^2(k^2-1)(k^2-4)/15 and which is continuous across table
 * knots.  chebykan_lut_build_derivative fills a HOST array like chebykan_lut_build does;
 * chebykan_backward_lut2 is chebykan_backward_lut with `dlut` (DEVICE, same layout as `lut`)
 * supplying the derivative in dx; dC and every other convention are unchanged.  The forward
 * pass of this variant is chebykan_forward_lut.  Both tables are staged on chip together when
 * 2*(degree+1)*lut_size*4 bytes <= 80 KiB at degrees 2..8; otherwise the any-degree kernels run.
 */
chebykan_status chebykan_lut_build_derivative(float *dlut, int degree, int lut_size);
chebykan_status chebykan_backward_lut2(const float *x, const float *C, const float *dy, const float *lut,
                                       const float *dlut, int lut_size, float *dx, float *dC,
                                       int64_t batch, int in, int out, int degree,
                                       void *workspace, size_t workspace_bytes, chebykan_stream_t stream);

/*
 * Other KAN bases on the same layer skeleton (paper Sec. 2.3: every variant expands
 * each input into K = degree+1 basis functions by a short recurrence and contracts
 * them with C; Sec. 6.3 reports the method on Fourier, Legendre and Hermite KANs).
 * The paper prints no formulas for these bases; the textbook ones are used:
 *
 *   CHEBYKAN_BASIS_CHEBYSHEV  T_k(tanh x)                     (= chebykan_forward/backward)
 *   CHEBYKAN_BASIS_LEGENDRE   P_k(tanh x), (k+1)P_{k+1} = (2k+1)u P_k - k P_{k-1}
 *   CHEBYKAN_BASIS_HERMITE    H_k(tanh x), physicists': H_{k+1} = 2u H_k - 2k H_{k-1}
 *   CHEBYKAN_BASIS_FOURIER    B_0 = 1, B_{2m-1} = cos(m x), B_{2m} = sin(m x) of the raw
 *                             input, m = 1..degree/2; degree must be even
 *
 *   y[b,o] = sum_i sum_k C[i,o,k] B_k(x[b,i]),  dC[i,o,k] = sum_b B_k(x[b,i]) dy[b,o],
 *   dx[b,i] = sum_o dy[b,o] sum_k C[i,o,k] dB_k/dx(x[b,i])
 *
 * Tensors, layouts, workspace (chebykan_workspace_bytes of the same shape),
 * ownership, overwrite semantics, reproducibility and errors are those of
 * chebykan_forward / chebykan_backward; an unknown basis or an odd Fourier degree
 * gives CHEBYKAN_ERR_SHAPE.  Degrees 3, 4, 5, 6, 8 (Fourier: 4, 6, 8) run on the
 * matrix-core kernels, every other degree up to CHEBYKAN_MAX_DEGREE on the
 * any-degree kernels.
 */
#define CHEBYKAN_BASIS_CHEBYSHEV 0
#define CHEBYKAN_BASIS_LEGENDRE 1
#define CHEBYKAN_BASIS_HERMITE 2
#define CHEBYKAN_BASIS_FOURIER 3
chebykan_status chebykan_forward_basis(int basis, const float *x, const float *C, float *y,
                                       int64_t batch, int in, int out, int degree,
                                       void *workspace, size_t workspace_bytes, chebykan_stream_t stream);
chebykan_status chebykan_backward_basis(int basis, const float *x, const float *C, const float *dy,
                                        float *dx, float *dC,
                                        int64_t batch, int in, int out, int degree,
                                        void *workspace, size_t workspace_bytes, chebykan_stream_t stream);

/*
 * Whole stacks in one call (the paper evaluates three-layer Chebyshev-KAN stacks,
 * Sec. 6.1 Table 2): layer l maps widths[l] -> widths[l+1] inputs, all layers share
 * `degree`, and the layers are chained directly, act[l+1] = layer_l(act[l]).
 *
 * All array arguments are HOST arrays of DEVICE pointers (n_layers or n_layers+1
 * entries) that the call reads before it returns:
 *   C[l]    coefficients of layer l                 [widths[l], widths[l+1], degree+1]
 *   act[l]  activations: act[0] is the input x (read only), act[l+1] receives the
 *           output of layer l; chebykan_stack_backward reads act[0..n_layers-1]
 *   grad[l] gradient with respect to act[l]: grad[n_layers] is the incoming dy (read
 *           only), grad[l] for l < n_layers is written; grad[0] may be NULL when the
 *           gradient with respect to the stack's input is not wanted
 *   dC[l]   coefficient gradients, same shape as C[l]; an entry may be NULL (skipped)
 * The workspace must hold chebykan_stack_workspace_bytes(...) bytes (the largest
 * per-layer requirement; the layers run one after the other on `stream`).
 * 1 <= n_layers <= CHEBYKAN_MAX_LAYERS.  Everything else - overwrite semantics,
 * reproducibility, validation order and error codes - is as for the single-layer
 * calls; on any error nothing has been enqueued.
 */
#define CHEBYKAN_MAX_LAYERS 64
size_t chebykan_stack_workspace_bytes(int64_t batch, int n_layers, const int *widths, int degree);
chebykan_status chebykan_stack_forward(int n_layers, const int *widths, int degree, int64_t batch,
                                       const float *const *C, float *const *act,
                                       void *workspace, size_t workspace_bytes, chebykan_stream_t stream);
chebykan_status chebykan_stack_backward(int n_layers, const int *widths, int degree, int64_t batch,
                                        const float *const *C, const float *const *act,
                                        float *const *grad, float *const *dC,
                                        void *workspace, size_t workspace_bytes, chebykan_stream_t stream);

/*
 * Prepares the CURRENT device for the library: checks that it is a gfx950 part and raises the
 * dynamic-LDS limit of every kernel of the library on it.  Every entry point does this by itself
 * on its first call on a device, so calling chebykan_init is optional - except that function
 * attributes cannot be changed while a stream is being captured: a caller who captures the
 * library's launches into a HIP graph calls chebykan_init (or any entry point) once on that device
 * before the capture starts.  Idempotent and thread-safe; enqueues nothing.
 * CHEBYKAN_ERR_DEVICE when no gfx950 device is current, CHEBYKAN_ERR_LAUNCH if HIP refuses.
 */
chebykan_status chebykan_init(void);

/* Human-readable name of a status code (static storage, never NULL). */
const char *chebykan_status_string(chebykan_status status);

/* Library/ABI version: major*1000 + minor. */
int chebykan_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CHEBYKAN_H */
