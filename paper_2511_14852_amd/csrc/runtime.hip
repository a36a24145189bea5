// Process-wide state of the library: the kernel registry, per-device preparation, the
// kernel-family override and the optional kernel timing.  No kernels here.
#include <hip/hip_runtime.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/chebykan.h"
#include "../../include/chebykan_tools.h"
#include "launch.h"
#include "runtime.h"

namespace chebykan {

// ------------------------------------------------------------- kernel registry
// A singly linked list that static initialisers of every translation unit push onto while the
// library is loaded; guarded because a late registration (see below) may come from any thread.
static std::mutex& registry_mutex()
{
    static std::mutex m;
    return m;
}
static std::atomic<KernelRecord*>& registry_head()
{
    static std::atomic<KernelRecord*> head{nullptr};
    return head;
}

constexpr int MAX_DEVICES = 64;
// per device ordinal: 0 not prepared, 1 ready, -1 not a gfx950 part
static std::atomic<int> g_device_state[MAX_DEVICES];
static std::atomic<bool> g_any_prepared{false};

// Dynamic LDS up to this size needs no function attribute.
constexpr int DEFAULT_LDS_LIMIT = 48 * 1024;

static bool allow_lds(const KernelRecord* rec)
{
    if (rec->max_lds_bytes <= DEFAULT_LDS_LIMIT) return true;
    if (hipFuncSetAttribute(rec->fn, hipFuncAttributeMaxDynamicSharedMemorySize, rec->max_lds_bytes) == hipSuccess)
        return true;
    (void)hipGetLastError();
    return false;
}

bool register_kernel(KernelRecord* rec, const void* fn, int max_lds_bytes, const char* name)
{
    std::lock_guard<std::mutex> lock(registry_mutex());
    for (KernelRecord* r = registry_head().load(); r; r = r->next)
        if (r == rec) return true;
    rec->fn = fn;
    rec->max_lds_bytes = max_lds_bytes;
    rec->name = name;
    rec->next = registry_head().load();
    registry_head().store(rec);
    // A kernel that becomes known only after a device was prepared (never the case when the
    // static initialisers ran at load time) gets its attribute on the current device now.
    // No HIP call is made while the library is being loaded.
    if (g_any_prepared.load()) {
        int dev = -1;
        if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < MAX_DEVICES && g_device_state[dev].load() == 1)
            (void)allow_lds(rec);
        else
            (void)hipGetLastError();
    }
    return true;
}

KernelRecord* kernel_registry() { return registry_head().load(); }

chebykan_status prepare_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        return CHEBYKAN_ERR_DEVICE;
    }
    const int state = g_device_state[dev].load(std::memory_order_acquire);
    if (state != 0) return state > 0 ? CHEBYKAN_OK : CHEBYKAN_ERR_DEVICE;

    static std::mutex prepare_mutex;
    std::lock_guard<std::mutex> lock(prepare_mutex);
    if (g_device_state[dev].load() != 0) return g_device_state[dev].load() > 0 ? CHEBYKAN_OK : CHEBYKAN_ERR_DEVICE;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return CHEBYKAN_ERR_DEVICE;
    }
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
        g_device_state[dev].store(-1, std::memory_order_release);
        return CHEBYKAN_ERR_DEVICE;
    }
    // every kernel of the library may use the LDS size it was registered with from now on
    for (const KernelRecord* r = kernel_registry(); r; r = r->next)
        if (!allow_lds(r)) return CHEBYKAN_ERR_LAUNCH;   // state stays 0: the next call tries again
    g_any_prepared.store(true);
    g_device_state[dev].store(1, std::memory_order_release);
    return CHEBYKAN_OK;
}

// ------------------------------------------------------------- kernel family
static std::atomic<int> g_family{0};   // 0 automatic, 1 any-degree kernels, 2 matrix-core kernels
int kernel_family() { return g_family.load(std::memory_order_relaxed); }

// ------------------------------------------------------------- kernel timing
struct TraceRecord {
    const char* signature;
    unsigned grid[3], block;
    LaunchContext context;
};
struct TraceSink {
    std::vector<hipEvent_t> events;     // two per kernel, created by chebykan_trace_begin
    std::vector<TraceRecord> records;
    int capacity = 0;
    int dropped = 0;                    // launches beyond the capacity (not timed)
    bool open = false;
    std::string name;                   // scratch for chebykan_trace_get
};
thread_local TraceSink* g_trace = nullptr;
thread_local LaunchContext g_launch_context = {0, 0, 1.0f, 0, 0};
static thread_local TraceSink* g_sink = nullptr;   // this thread's sink, collecting or not

void trace_before(TraceSink* sink, const char* signature, dim3 grid, dim3 block, hipStream_t s)
{
    if ((int)sink->records.size() >= sink->capacity) {
        ++sink->dropped;
        sink->open = false;
        return;
    }
    (void)hipEventRecord(sink->events[2 * sink->records.size()], s);
    sink->records.push_back(TraceRecord{signature, {grid.x, grid.y, grid.z}, block.x * block.y * block.z, g_launch_context});
    sink->open = true;
}

void trace_after(TraceSink* sink, hipStream_t s)
{
    if (!sink->open) return;
    (void)hipEventRecord(sink->events[2 * sink->records.size() - 1], s);
    sink->open = false;
}

static void free_sink()
{
    if (!g_sink) return;
    for (hipEvent_t e : g_sink->events) (void)hipEventDestroy(e);
    delete g_sink;
    g_sink = nullptr;
    g_trace = nullptr;
}

}  // namespace chebykan

using namespace chebykan;

extern "C" {

int chebykan_set_kernel_family(int family)
{
    const int prev = g_family.load();
    if (family >= 0 && family <= 2) g_family.store(family);
    return prev;
}

chebykan_status chebykan_trace_begin(int max_kernels)
{
    if (max_kernels <= 0 || max_kernels > (1 << 20)) return CHEBYKAN_ERR_SHAPE;
    free_sink();
    TraceSink* sink = new TraceSink;
    sink->capacity = max_kernels;
    sink->events.reserve(2 * (size_t)max_kernels);
    sink->records.reserve((size_t)max_kernels);
    for (int i = 0; i < 2 * max_kernels; ++i) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) {
            (void)hipGetLastError();
            g_sink = sink;
            free_sink();
            return CHEBYKAN_ERR_LAUNCH;
        }
        sink->events.push_back(e);
    }
    g_sink = sink;
    g_trace = sink;
    return CHEBYKAN_OK;
}

int chebykan_trace_end(int* dropped)
{
    g_trace = nullptr;
    if (dropped) *dropped = g_sink ? g_sink->dropped : 0;
    return g_sink ? (int)g_sink->records.size() : 0;
}

chebykan_status chebykan_trace_get(int index, const char** name, unsigned grid[3], unsigned* block, int* layer, int* ops,
                                   float* share, int* layer2, int* ops2, float* microseconds)
{
    TraceSink* sink = g_sink;
    if (!sink || g_trace) return CHEBYKAN_ERR_NULL;               // nothing collected, or still collecting
    if (index < 0 || index >= (int)sink->records.size()) return CHEBYKAN_ERR_SHAPE;
    const TraceRecord& r = sink->records[(size_t)index];
    if (name) {
        // the signature ends "[Kernel = &<kernel>, MaxLds = N, TagList = chebykan::Tags<<template arguments>>]"
        const std::string sig = r.signature;
        std::string s = sig;
        const size_t a = sig.find("Kernel = &");
        const size_t b = sig.find(", MaxLds", a == std::string::npos ? 0 : a);
        const size_t c = sig.find("Tags<", b == std::string::npos ? 0 : b);
        const size_t e = sig.rfind(">]");
        if (a != std::string::npos && b != std::string::npos && c != std::string::npos && e != std::string::npos && e >= c + 5) {
            s = sig.substr(a + 10, b - a - 10);
            const std::string tags = sig.substr(c + 5, e - c - 5);
            if (!tags.empty()) s += "<" + tags + ">";
        }
        for (size_t p; (p = s.find("chebykan::")) != std::string::npos;) s.erase(p, 10);
        for (size_t p; (p = s.find("(anonymous namespace)::")) != std::string::npos;) s.erase(p, 23);
        for (size_t p; (p = s.find("Int<")) != std::string::npos;) {   // Int<N> stands for the integer argument N
            const size_t q = s.find('>', p);
            if (q == std::string::npos) break;
            s.erase(q, 1);
            s.erase(p, 4);
        }
        sink->name = s;
        *name = sink->name.c_str();
    }
    if (grid) { grid[0] = r.grid[0]; grid[1] = r.grid[1]; grid[2] = r.grid[2]; }
    if (block) *block = r.block;
    if (layer) *layer = r.context.layer;
    if (ops) *ops = r.context.ops;
    if (share) *share = r.context.share;
    if (layer2) *layer2 = r.context.layer2;
    if (ops2) *ops2 = r.context.ops2;
    if (microseconds) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, sink->events[2 * (size_t)index], sink->events[2 * (size_t)index + 1]) != hipSuccess) {
            (void)hipGetLastError();
            return CHEBYKAN_ERR_LAUNCH;                            // the stream has not reached the second event yet
        }
        *microseconds = ms * 1000.0f;
    }
    return CHEBYKAN_OK;
}

void chebykan_trace_free(void) { free_sink(); }

}  // extern "C"
