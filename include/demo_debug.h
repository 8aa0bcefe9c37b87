/*
 * demo_debug.h -- measurement and test hooks of libdemo.so.  Nothing here is part of the method: these
 * calls time kernels, select kernel families for cross-checks, and probe the memory system.  They follow
 * the conventions of demo.h (device pointers owned by the caller, status codes, asynchronous launches on
 * `hip_stream`).
 */
#ifndef DEMO_DEBUG_H_
#define DEMO_DEBUG_H_

#include "demo.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel timing with HIP events recorded on the call's own stream around each
 * kernel launch.  demo_set_timing(ctx, 1) opens a measurement window (and clears
 * the previous one); every encode / decode / step call then records one event
 * pair per kernel it launches, without synchronising.  demo_last_kernel_ms blocks
 * until the recorded events have completed and returns the average duration in
 * milliseconds over the launches of the window (the 256 most recent at most).
 * which: 0 = encode order-2 kernel, 1 = encode order-1, 2 = decode order-2,
 * 3 = decode order-1.  DEMO_ERR_ARG if nothing was recorded for `which`.  */
int demo_set_timing(demo_ctx* ctx, int enabled);
int demo_last_kernel_ms(demo_ctx* ctx, int which, float* ms);

/* Bandwidth probe: one plain streaming copy kernel of nbytes (a multiple of 16, both pointers
 * 16-byte aligned, device memory) from src to dst.  It is what the HBM traffic counters are
 * calibrated with (a copy of known size) and gives the copy bandwidth this GPU reaches; while
 * timing is enabled its duration is recorded in slot 1 of demo_last_kernel_ms.  Not part of the
 * method.  */
int demo_copy_probe(demo_ctx* ctx, void* dst, const void* src, int64_t nbytes, void* hip_stream);

/* Kernel family used by later calls: 1 (default) = the fastest kernels available
 * for the chunk size, 0 = the generic LDS-staged kernels only (kept selectable so
 * that the two families can be checked against each other), 2 = as 1, but the s = 64
 * decode of the DCT stays on its mirror-folded float32 instances where the full-product
 * instance on the float16 matrix pipe would take over (64 < W k <= 2048, sum or mean),
 * so that the two can be timed and checked against each other.  */
int demo_set_variant(demo_ctx* ctx, int variant);

/* Memory-system probe with the launch shape of the wavefront kernels (one workgroup of eight wavefronts
 * per compute unit, 16 bytes per lane and access, eight accesses in flight per lane), over nbytes (a multiple
 * of 16, pointers 16-byte aligned, device memory):
 *   mode 0  copy src -> dst with the default cache policy (what demo_copy_probe does, in this launch shape);
 *   mode 1  copy src -> dst with non-temporal loads and stores, the policy of the kernels' tensor accesses;
 *   mode 2  read src only, non-temporal (dst receives 16 bytes per wavefront so that the reads cannot be
 *           dropped; it must hold at least 64 KiB);
 *   mode 3  write dst only, non-temporal (src is not read);   mode 4  write dst only, default cache policy.
 * Timed like demo_copy_probe (slot 1 of demo_last_kernel_ms).  DEMO_ERR_ARG for an unknown mode.  */
int demo_stream_probe(demo_ctx* ctx, void* dst, const void* src, int64_t nbytes, int mode, void* hip_stream);

/* Time attribution for the s = 64 encode kernel (bfloat16 gradients, DCT): later demo_encode calls run a
 * cut-down copy of the kernel that does NOT encode.  stage 1 = the memory stream only (loads of g and m with
 * the cross-chunk prefetch, momentum update, store of m, k payload pairs per chunk): the time the kernel's own
 * access pattern takes with no transform at all; 2 = stage 1 plus the two DCT products; 3 = stage 2 plus
 * top-k and the payload (everything but the reconstruction); 0 = the real kernel (default).  The differences
 * between consecutive stages are the costs of the phases.  Momentum and payload contents after a stage 1..3
 * call are meaningless.  DEMO_ERR_ARG outside 0..3; a call with float32 gradients, another chunk size or
 * another projection matrix while a stage is set returns DEMO_ERR_UNSUPPORTED.  */
int demo_debug_set_encode_stage(demo_ctx* ctx, int stage);

/* The same for the s = 64 decode kernel (64 < W * k <= 2048, sum or mean): stage 1 = the memory stream only
 * (payload and parameter loads with the cross-chunk prefetch, update of the parameters with whatever the tile
 * holds, stores); 2 = stage 1 plus the scatter-add into the tile; 0 = the real kernel.  Parameters after a
 * stage 1 or 2 call are meaningless.  DEMO_ERR_ARG outside 0..2; calls the stages do not cover return
 * DEMO_ERR_UNSUPPORTED while one is set.  */
int demo_debug_set_decode_stage(demo_ctx* ctx, int stage);

#ifdef __cplusplus
}
#endif
#endif /* DEMO_DEBUG_H_ */
