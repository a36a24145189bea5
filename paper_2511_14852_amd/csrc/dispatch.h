// Internal interface between the C ABI and the specialised kernel families
// (matrix-core kernels for wide layers, streaming kernels for very narrow ones).
// Each fast_* function either enqueues the whole operation on `s` and returns
// true, or enqueues nothing and returns false (shape/degree not specialised:
// the caller then uses the any-degree kernels).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace chebykan {

size_t forward_workspace_bytes(int64_t B, int I, int O, int d);
size_t backward_workspace_bytes(int64_t B, int I, int O, int d);

bool fast_forward(const float* x, const float* C, float* y, int64_t B, int I, int O, int d, void* ws,
                  hipStream_t s);
// dx and/or dC may be null (skipped).
bool fast_backward(const float* x, const float* C, const float* dy, float* dx, float* dC, int64_t B, int I,
                   int O, int d, void* ws, hipStream_t s);

// Table-interpolated variant; lut is a device pointer to [d+1][n] samples.  False when the degree
// has no table kernels or the table does not fit beside the tiles in LDS.
bool fast_forward_table(const float* x, const float* C, const float* lut, int n, float* y, int64_t B, int I, int O,
                        int d, void* ws, hipStream_t s);
bool fast_backward_table(const float* x, const float* C, const float* dy, const float* lut, int n, float* dx,
                         float* dC, int64_t B, int I, int O, int d, void* ws, hipStream_t s);

// The same with the auxiliary derivative table dlut ([d+1][n], device): both tables must fit in LDS together.
bool fast_backward_table2(const float* x, const float* C, const float* dy, const float* lut, const float* dlut, int n,
                          float* dx, float* dC, int64_t B, int I, int O, int d, void* ws, hipStream_t s);

// Forward of a whole narrow stack in one launch (act[0] input, act[l+1] output of layer l).  False when
// the stack is not eligible (then nothing is enqueued and the caller runs the layers one by one).
bool fast_chain_forward(int n_layers, const int* widths, int d, int64_t B, const float* const* C, float* const* act,
                        hipStream_t s);

// Backward of a whole stack with every slice sum in one launch at the end; the workspace holds one region per
// layer (stack_backward_workspace_bytes).  False when a layer has no specialised kernels (nothing enqueued).
size_t stack_backward_workspace_bytes(int n_layers, const int* widths, int d, int64_t B);
bool fast_stack_backward(int n_layers, const int* widths, int d, int64_t B, const float* const* C,
                         const float* const* act, float* const* grad, float* const* dC, void* ws, hipStream_t s);

// Other bases (kind 1 Legendre, 2 Hermite, 3 Fourier).  False when the degree has no kernels for the family.
bool fast_forward_family(int kind, const float* x, const float* C, float* y, int64_t B, int I, int O, int d,
                         void* ws, hipStream_t s);
bool fast_backward_family(int kind, const float* x, const float* C, const float* dy, float* dx, float* dC,
                          int64_t B, int I, int O, int d, void* ws, hipStream_t s);

}  // namespace chebykan
