// One place through which every kernel of the library is launched.
//
// launch<Kernel, MaxLds, Tags<...>>(grid, block, lds_bytes, stream, args...) does three things:
//  - it makes the kernel known to a process-wide registry when the library is loaded (a static
//    member that every use of launch<> instantiates), with the largest dynamic LDS size the
//    kernel may be launched with.  prepare_device() walks that registry once per device and raises
//    hipFuncAttributeMaxDynamicSharedMemorySize for every kernel, so that no launch ever has to
//    change a function attribute: the first real call may sit inside a stream capture, and two
//    host threads may launch the same kernel at once;
//  - it enqueues the kernel on the caller's stream;
//  - when the calling thread has switched kernel timing on (chebykan_trace_begin, a measurement
//    aid), it brackets the launch with two event records on that stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace chebykan {

struct KernelRecord {
    const void* fn;        // host-side handle of the kernel
    int max_lds_bytes;     // largest dynamic LDS size it is launched with (0: never above the 64 KiB default)
    const char* name;      // the launch<> instantiation's signature: the kernel's name and, in Tags<...>, its template arguments
    KernelRecord* next;
};

// Fills in a record and adds it to the registry (called from static initialisers at load time).
// The record itself is zero-initialised static storage, so it needs no initialiser of its own that
// could run after this one.
bool register_kernel(KernelRecord* rec, const void* fn, int max_lds_bytes, const char* name);
// First record of the registry.
KernelRecord* kernel_registry();

// What the calling thread's launches compute, for the timing report: the layer of a stack call
// they belong to (-1: every layer at once; 0 for single-layer calls) and which results
// (OP_* bits; OP_SUM marks a kernel that only adds partial results).  Set by the dispatch code
// through the two scoped helpers; read only while timing is on.
enum : int { OP_FWD = 1, OP_DX = 2, OP_DC = 4, OP_SUM = 8 };
struct LaunchContext {
    int layer;
    int ops;
    float share;   // part of that work this launch does (an output range tiled by two launches), 1 by default
    int layer2;    // a launch that holds two operations: the second one's layer and outputs (ops2 = 0: none)
    int ops2;
};
extern thread_local LaunchContext g_launch_context;
struct ScopedOps {
    int saved;
    explicit ScopedOps(int ops) : saved(g_launch_context.ops) { g_launch_context.ops = ops; }
    ~ScopedOps() { g_launch_context.ops = saved; }
};
struct ScopedShare {
    float saved;
    explicit ScopedShare(float share) : saved(g_launch_context.share) { g_launch_context.share = share; }
    ~ScopedShare() { g_launch_context.share = saved; }
};
struct ScopedSecond {
    int saved_layer, saved_ops;
    ScopedSecond(int layer, int ops) : saved_layer(g_launch_context.layer2), saved_ops(g_launch_context.ops2)
    {
        g_launch_context.layer2 = layer;
        g_launch_context.ops2 = ops;
    }
    ~ScopedSecond()
    {
        g_launch_context.layer2 = saved_layer;
        g_launch_context.ops2 = saved_ops;
    }
};
struct ScopedLayer {
    int saved;
    explicit ScopedLayer(int layer) : saved(g_launch_context.layer) { g_launch_context.layer = layer; }
    ~ScopedLayer() { g_launch_context.layer = saved; }
};

// Kernel timing of the calling thread: null when off.
struct TraceSink;
extern thread_local TraceSink* g_trace;
void trace_before(TraceSink* sink, const char* name, dim3 grid, dim3 block, hipStream_t s);
void trace_after(TraceSink* sink, hipStream_t s);

// The template arguments of a kernel, repeated as types for the timing report (a function's
// signature string spells out type arguments but not those of a function it points to).
template <class... T>
struct Tags {};
template <int N>
struct Int {};

template <auto Kernel, int MaxLds, class TagList>
struct KernelEntry {
    static const char* signature() { return __PRETTY_FUNCTION__; }
    static KernelRecord record;
    static bool registered;
};
template <auto Kernel, int MaxLds, class TagList>
KernelRecord KernelEntry<Kernel, MaxLds, TagList>::record;
template <auto Kernel, int MaxLds, class TagList>
bool KernelEntry<Kernel, MaxLds, TagList>::registered =
    register_kernel(&KernelEntry<Kernel, MaxLds, TagList>::record, reinterpret_cast<const void*>(Kernel), MaxLds,
                    KernelEntry<Kernel, MaxLds, TagList>::signature());

template <auto Kernel, int MaxLds = 0, class TagList = Tags<>, class... Args>
inline void launch(dim3 grid, dim3 block, size_t lds_bytes, hipStream_t s, Args... args)
{
    using Entry = KernelEntry<Kernel, MaxLds, TagList>;
    // naming the member keeps its initialiser (the registration, run when the library is loaded) in the library
    if (!Entry::registered)
        Entry::registered = register_kernel(&Entry::record, reinterpret_cast<const void*>(Kernel), MaxLds, Entry::signature());
    TraceSink* sink = g_trace;
    if (sink) trace_before(sink, Entry::record.name, grid, block, s);
    hipLaunchKernelGGL(Kernel, grid, block, lds_bytes, s, args...);
    if (sink) trace_after(sink, s);
}

}  // namespace chebykan
