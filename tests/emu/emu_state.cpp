// Definitions of the emulator's global state (see shim/hip/hip_runtime.h).
#include <hip/hip_runtime.h>
thread_local emu_uint3 threadIdx, blockIdx;
emu_uint3 blockDim, gridDim;
EmuBlockState* emu_block = nullptr;
thread_local int emu_tid = 0;
namespace chebykan {
float lds[EMU_LDS_FLOATS] __attribute__((aligned(16)));
}
