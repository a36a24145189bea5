/*
 * chebykan_tools.h - test and measurement aids of libchebykan.  Nothing here is part of the
 * paper's method or needed to use the layer (that interface is chebykan.h): a kernel-family
 * override for tests, two roofline calibration kernels, and per-kernel timing for benchmarks.
 */
#ifndef CHEBYKAN_TOOLS_H
#define CHEBYKAN_TOOLS_H

#include "chebykan.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Kernel-family override: 0 = automatic choice (default), 1 = force the any-degree kernels,
 * 2 = force the matrix-core kernels where the shape supports them.  Process-wide (an atomic);
 * returns the previous value.  Other values are ignored.
 */
int chebykan_set_kernel_family(int family);

/*
 * Roofline calibration: what the GPU sustains on the two limits the layer kernels are priced
 * against.
 *
 * chebykan_calibrate_mfma enqueues `workgroups` workgroups of 4 waves, each wave issuing
 * iterations*32 register-only v_mfma_f32_32x32x2_f32 (no memory traffic in the loop).  `sink` is
 * device memory of at least workgroups*256 floats that the kernel overwrites; *flops (host
 * pointer, may be NULL) receives the number of floating-point operations of the launch.  The
 * caller times the launch.
 *
 * chebykan_calibrate_copy enqueues dst[0..n) = src[0..n) as a plain streaming copy (16 bytes per
 * thread): n*4 bytes read and n*4 bytes written.  dst and src are device pointers, 16-byte
 * aligned, non-overlapping; n is a multiple of 4.
 *
 * Both return CHEBYKAN_ERR_NULL / CHEBYKAN_ERR_SHAPE for bad arguments and CHEBYKAN_ERR_LAUNCH if
 * HIP refuses the launch; nothing is allocated.
 */
chebykan_status chebykan_calibrate_mfma(float *sink, int workgroups, int iterations, double *flops,
                                        chebykan_stream_t stream);
chebykan_status chebykan_calibrate_copy(float *dst, const float *src, int64_t n, chebykan_stream_t stream);

/*
 * Per-kernel timing.  Between chebykan_trace_begin and chebykan_trace_end every kernel that the
 * library launches FROM THE CALLING THREAD is bracketed by two hipEventRecord calls on the stream
 * it is launched on; afterwards chebykan_trace_get returns, for the index-th launch in launch
 * order, the kernel's name with its template arguments (storage valid until the next call on this
 * thread), its grid and block size, what it computes - `layer`: the layer of a stack call it
 * belongs to (0 for single-layer calls, -1 for a kernel that covers every layer of the stack),
 * `ops`: CHEBYKAN_OP_* bits, `share`: the part of that work this launch does (below 1 when two
 * launches tile one output range), `layer2` / `ops2`: the same for a second operation when the
 * launch holds two (ops2 = 0 otherwise) - and the time between its two events in microseconds.
 *
 * chebykan_trace_begin creates 2*max_kernels events (the only calls here that allocate); launches
 * beyond max_kernels are not timed and are counted in *dropped by chebykan_trace_end, which
 * returns the number of timed launches.  The caller must have synchronised the stream(s) before
 * chebykan_trace_get (else CHEBYKAN_ERR_LAUNCH); CHEBYKAN_ERR_NULL when nothing was collected or
 * collection is still on, CHEBYKAN_ERR_SHAPE for a bad index.  Any output pointer may be NULL.  chebykan_trace_free destroys the events.  Event records cannot be
 * captured into a graph by a thread that is timing; the layer entry points behave as always
 * otherwise (an event record costs about a microsecond on the stream).
 */
#define CHEBYKAN_OP_FORWARD 1   /* the kernel computes y                                  */
#define CHEBYKAN_OP_DX 2        /* ... dx                                                */
#define CHEBYKAN_OP_DC 4        /* ... dC (or its per-slice partial sums)                */
#define CHEBYKAN_OP_SUM 8       /* ... only adds partial results of the marked output(s) */
chebykan_status chebykan_trace_begin(int max_kernels);
int chebykan_trace_end(int *dropped);
chebykan_status chebykan_trace_get(int index, const char **name, unsigned grid[3], unsigned *block,
                                   int *layer, int *ops, float *share, int *layer2, int *ops2,
                                   float *microseconds);
void chebykan_trace_free(void);

#ifdef __cplusplus
}
#endif
#endif /* CHEBYKAN_TOOLS_H */
