// CPU stand-in for <hip/hip_runtime.h>, used ONLY by the host-side kernel-logic
// tests: it lets the library's HIP sources compile with a host compiler and run
// each workgroup as a group of OS threads, so that indexing, tiling, barriers
// and bounds can be checked (under AddressSanitizer) without a GPU.
//
//  - a launch runs its workgroups one after another; the threads of a workgroup
//    run concurrently and meet at __syncthreads();
//  - dynamic LDS is one global array, NaN-filled before every workgroup and
//    poisoned past the launch's size, so reads of unwritten or out-of-range LDS
//    show up;
//  - the 32x32x2 fp32 MFMA is emulated per wave from its documented operand
//    layout (A[row=l%32][k=l/32], B[k=l/32][col=l%32], D reg r ->
//    row 8*(r/4)+4*(l/32)+r%4, col l%32).
// Nothing in the product path includes this file.
#pragma once
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <thread>
#include <vector>

#if defined(__has_feature)
#if __has_feature(address_sanitizer)
#include <sanitizer/asan_interface.h>
#define EMU_ASAN 1
#endif
#endif
#ifndef EMU_ASAN
#define ASAN_POISON_MEMORY_REGION(a, n) ((void)(a), (void)(n))
#define ASAN_UNPOISON_MEMORY_REGION(a, n) ((void)(a), (void)(n))
#endif

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __shared__
#define __align__(n) __attribute__((aligned(n)))
#define __launch_bounds__(...)
#define __restrict__ __restrict

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
struct emu_uint3 { unsigned x, y, z; };
extern thread_local emu_uint3 threadIdx, blockIdx;
extern emu_uint3 blockDim, gridDim;

typedef void* hipStream_t;
typedef int hipError_t;
constexpr hipError_t hipSuccess = 0;
struct hipDeviceProp_t { char gcnArchName[256]; };
constexpr int hipFuncAttributeMaxDynamicSharedMemorySize = 8;
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipGetDeviceProperties(hipDeviceProp_t* p, int) { strcpy(p->gcnArchName, "gfx950:emulated"); return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void*, int, int) { return hipSuccess; }
// a __device__ array is ordinary host memory here
#define HIP_SYMBOL(x) x
template <class T>
inline hipError_t hipGetSymbolAddress(void** p, T& symbol) { *p = (void*)&symbol; return hipSuccess; }
// events (the library's optional kernel timing): accepted, never timed
typedef void* hipEvent_t;
inline hipError_t hipEventCreate(hipEvent_t* e) { *e = nullptr; return hipSuccess; }
inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }

namespace chebykan {
constexpr int EMU_LDS_FLOATS = 160 * 1024 / 4;
extern float lds[EMU_LDS_FLOATS] __attribute__((aligned(16)));
}

struct EmuBlockState {
    pthread_barrier_t block_barrier;
    pthread_barrier_t wave_barrier[16];
    float exA[16][64], exB[16][64];
    int nthreads;
};
extern EmuBlockState* emu_block;
extern thread_local int emu_tid;

inline void __syncthreads() { pthread_barrier_wait(&emu_block->block_barrier); }

typedef float emu_floatx16 __attribute__((ext_vector_type(16)));
inline emu_floatx16 emu_mfma_f32_32x32x2f32(float a, float b, emu_floatx16 c, int, int, int)
{
    const int w = emu_tid / 64, lane = emu_tid % 64;
    emu_block->exA[w][lane] = a;
    emu_block->exB[w][lane] = b;
    pthread_barrier_wait(&emu_block->wave_barrier[w]);
    const int col = lane % 32, h = lane / 32;
    for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r / 4) + 4 * h + (r % 4);
        float acc = c[r];
        for (int k = 0; k < 2; ++k) acc = fmaf(emu_block->exA[w][k * 32 + row], emu_block->exB[w][k * 32 + col], acc);
        c[r] = acc;
    }
    pthread_barrier_wait(&emu_block->wave_barrier[w]);
    return c;
}
#define __builtin_amdgcn_mfma_f32_32x32x2f32 emu_mfma_f32_32x32x2f32

// stand-in for csrc/buffer_io.h (same include guard): bounds-checked loads, 0 beyond the end
#define CHEBYKAN_BUFFER_IO_H
namespace chebykan {
typedef float bufx4 __attribute__((ext_vector_type(4)));
struct BufferView { const float* base; int64_t n; };
inline BufferView make_view(const float* base, int64_t n_floats)
{
    int64_t n = n_floats > 0 ? n_floats : 0;
    if (n > 0x3fffffffLL) n = 0x3fffffffLL;
    return BufferView{base, n};
}
inline float load1(const BufferView& v, uint32_t index) { return (int64_t)index < v.n ? v.base[index] : 0.0f; }
inline bufx4 load4(const BufferView& v, uint32_t index)
{
    // any 4-byte aligned position; the range check is per element, as the hardware's is per dword
    bufx4 r = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int q = 0; q < 4; ++q)
        if ((int64_t)index + q < v.n) r[q] = v.base[index + q];
    return r;
}
}  // namespace chebykan

// data-parallel-primitive move as used for the row reductions: row_shr:n (0x110+n),
// row_bcast:15 (0x142), row_bcast:31 (0x143); every lane of the wave must take part.
inline int emu_update_dpp(int old, int src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl)
{
    (void)bank_mask;
    const int w = emu_tid / 64, lane = emu_tid % 64;
    int* ex = reinterpret_cast<int*>(emu_block->exA[w]);
    ex[lane] = src;
    pthread_barrier_wait(&emu_block->wave_barrier[w]);
    int result = old;
    const int row = lane / 16, pos = lane % 16;
    if ((row_mask >> row) & 1) {
        if (ctrl >= 0x111 && ctrl <= 0x11f) {
            const int n = ctrl - 0x110;
            if (pos - n >= 0) result = ex[lane - n];
            else if (bound_ctrl) result = 0;
        } else if (ctrl == 0x142) {
            if (row > 0) result = ex[row * 16 - 1];
            else if (bound_ctrl) result = 0;
        } else if (ctrl == 0x143) {
            if (row >= 2) result = ex[31];
            else if (bound_ctrl) result = 0;
        } else {
            fprintf(stderr, "emu_update_dpp: control %x not emulated\n", ctrl);
            abort();
        }
    }
    pthread_barrier_wait(&emu_block->wave_barrier[w]);
    return result;
}
#define __builtin_amdgcn_update_dpp emu_update_dpp

inline float emu_exp2f(float x) { return exp2f(x); }
inline float emu_rcpf(float x) { return 1.0f / x; }
#define __builtin_amdgcn_exp2f emu_exp2f
#define __builtin_amdgcn_sched_group_barrier(mask, size, id) ((void)0)
#define __builtin_amdgcn_sched_barrier(mask) ((void)0)
#define CHEBYKAN_OPAQUE(v) ((void)0)
#define CHEBYKAN_LDS_OPERAND(p) (*(p))
#define CHEBYKAN_LDS_STORE(p, v) (*(p) = (v))
#define __builtin_amdgcn_rcpf emu_rcpf

// wave-level exchange: every lane of the wave must take part
inline float __shfl_xor(float v, int mask, int width = 64)
{
    (void)width;
    const int w = emu_tid / 64, lane = emu_tid % 64;
    emu_block->exA[w][lane] = v;
    pthread_barrier_wait(&emu_block->wave_barrier[w]);
    const float r = emu_block->exA[w][lane ^ mask];
    pthread_barrier_wait(&emu_block->wave_barrier[w]);
    return r;
}

template <class Kernel, class... Args>
void emu_launch(Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, Args... args)
{
    const int nthreads = (int)(block.x * block.y * block.z);
    if (nthreads % 64 != 0 || nthreads > 1024 || lds_bytes > sizeof(chebykan::lds)) {
        fprintf(stderr, "emu_launch: bad launch shape\n");
        abort();
    }
    blockDim = {block.x, block.y, block.z};
    gridDim = {grid.x, grid.y, grid.z};
    EmuBlockState st;
    st.nthreads = nthreads;
    emu_block = &st;
    for (unsigned bz = 0; bz < grid.z; ++bz)
        for (unsigned by = 0; by < grid.y; ++by)
            for (unsigned bx = 0; bx < grid.x; ++bx) {
                ASAN_UNPOISON_MEMORY_REGION(chebykan::lds, sizeof(chebykan::lds));
                for (int i = 0; i < chebykan::EMU_LDS_FLOATS; ++i) chebykan::lds[i] = NAN;
                ASAN_POISON_MEMORY_REGION((char*)chebykan::lds + lds_bytes, sizeof(chebykan::lds) - lds_bytes);
                pthread_barrier_init(&st.block_barrier, nullptr, nthreads);
                for (int w = 0; w < nthreads / 64; ++w) pthread_barrier_init(&st.wave_barrier[w], nullptr, 64);
                std::vector<std::thread> th;
                th.reserve(nthreads);
                for (int t = 0; t < nthreads; ++t)
                    th.emplace_back([=]() {
                        emu_tid = t;
                        threadIdx = {t % block.x, (t / block.x) % block.y, t / (block.x * block.y)};
                        blockIdx = {bx, by, bz};
                        kernel(args...);
                    });
                for (auto& x : th) x.join();
                pthread_barrier_destroy(&st.block_barrier);
                for (int w = 0; w < nthreads / 64; ++w) pthread_barrier_destroy(&st.wave_barrier[w]);
            }
    ASAN_UNPOISON_MEMORY_REGION(chebykan::lds, sizeof(chebykan::lds));
}
#define hipLaunchKernelGGL(kernel, grid, block, ldsbytes, stream, ...) \
    emu_launch(kernel, grid, block, (size_t)(ldsbytes), __VA_ARGS__)
