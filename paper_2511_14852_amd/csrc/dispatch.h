// Internal interface between the C ABI and the MFMA kernel family.
// Each mfma_* function either enqueues the whole operation on `s` and returns
// true, or enqueues nothing and returns false (shape/degree not specialised).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace chebykan {

size_t forward_workspace_bytes(int64_t B, int I, int O, int d);
size_t backward_workspace_bytes(int64_t B, int I, int O, int d);

bool mfma_forward(const float* x, const float* C, float* y, int64_t B, int I, int O, int d, void* ws,
                  hipStream_t s);
bool mfma_dx(const float* x, const float* C, const float* dy, float* dx, int64_t B, int I, int O, int d,
             void* ws, hipStream_t s);
bool mfma_dC(const float* x, const float* dy, float* dC, int64_t B, int I, int O, int d, void* ws,
             hipStream_t s);

}  // namespace chebykan
