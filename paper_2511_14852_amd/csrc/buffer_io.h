// Bounds-checked global loads through gfx950 buffer instructions.
//
// A BufferView describes a run of floats; loads whose byte range does not lie inside it
// return 0 in hardware (raw buffer addressing, stride 0).  Kernels use this instead of
// per-lane `if (in_range)` loads: no exec-mask branches are generated, so producer code
// stays in one basic block that the scheduler can interleave with MFMA issue, and ragged
// tile edges cost nothing.  Offsets are 32-bit byte offsets, so a view must be based
// close enough to the data it addresses (callers base views at their tile).
#ifndef CHEBYKAN_BUFFER_IO_H
#define CHEBYKAN_BUFFER_IO_H
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace chebykan {

typedef float bufx4 __attribute__((ext_vector_type(4)));

struct BufferView {
    __amdgpu_buffer_rsrc_t rsrc;
};

// n_floats < 0 is treated as empty.
__device__ __forceinline__ BufferView make_view(const float* base, int64_t n_floats)
{
    int64_t bytes = n_floats > 0 ? n_floats * 4 : 0;
    if (bytes > 0xfffffffcLL) bytes = 0xfffffffcLL;
    BufferView v;
    v.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)(uint32_t)bytes, 0x00020000);
    return v;
}

// element `index` (in floats) of the view, or 0 beyond its end
__device__ __forceinline__ float load1(const BufferView& v, uint32_t index)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(v.rsrc, (int)(index * 4u), 0, 0));
}

// four consecutive floats from any 4-byte aligned position; elements beyond the end read as zero
__device__ __forceinline__ bufx4 load4(const BufferView& v, uint32_t index)
{
    return __builtin_bit_cast(bufx4, __builtin_amdgcn_raw_buffer_load_b128(v.rsrc, (int)(index * 4u), 0, 0));
}

}  // namespace chebykan
#endif  // CHEBYKAN_BUFFER_IO_H
