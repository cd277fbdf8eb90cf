// Developer aids of libequarx (declared in include/equarx_devtools.h): the
// calibration kernels the benchmark sets beside the real ones, the self-tests
// of the kernels' arithmetic shortcuts, and the hooks that attach HIP events
// to the launches of the next entry-point call.  None of them is part of the
// method; the product's entry points live in equarx_api.hip.
#include "equarx_devtools.h"

#include "equarx_devtools_kernels.hpp"
#include "equarx_launch.hpp"
#include "equarx_passes.hpp"

using namespace equarx;
using namespace equarx::host;

extern "C" {

int equarx_calib_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    LaunchCtx ctx(stream);
    if (bytes == 0) return EQUARX_OK;
    if (!src || !dst) return EQUARX_NULL_POINTER;
    if (bytes % 16 != 0) return EQUARX_BAD_SHAPE;
    if (misaligned(src, kAlign) || misaligned(dst, kAlign)) return EQUARX_MISALIGNED;
    Aliasing mem;
    mem.reads(src, bytes);
    mem.writes(dst, bytes);
    if (int st = mem.check()) return st;
    const int64_t nvec = (int64_t)(bytes / 16);
    const int64_t per_wg = kThreads * 4;
    ctx.launch(copy_kernel, (unsigned)((nvec + per_wg - 1) / per_wg), kThreads, static_cast<const u32x4 *>(src),
               static_cast<u32x4 *>(dst), nvec);
    return ctx.status();
}

int equarx_calib_empty_launches(int32_t count, int32_t workgroups, void *stream)
{
    LaunchCtx ctx(stream);
    if (count < 0 || count > 4096 || workgroups < 1 || workgroups > (1 << 20)) return EQUARX_BAD_SHAPE;
    for (int32_t i = 0; i < count; ++i) ctx.launch(empty_kernel, (unsigned)workgroups, kThreads, 0);
    return ctx.status();
}

int equarx_calib_hop_traffic(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, int8_t *codes0,
                             float *scales0, int8_t *codes1, float *scales1, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (n % block != 0) return EQUARX_BAD_SHAPE;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!codes0 || !scales0 || !codes1 || !scales1) return EQUARX_NULL_POINTER;
    if (misaligned(codes0, kAlign) || misaligned(scales0, kAlign) || misaligned(codes1, kAlign) ||
        misaligned(scales1, kAlign))
        return EQUARX_MISALIGNED;
    const size_t scale_bytes = (size_t)(n / block) * sizeof(float);
    Aliasing mem;
    for (int32_t i = 0; i < P; ++i) {
        if (!partials_bf16[i]) return EQUARX_NULL_POINTER;
        if (misaligned(partials_bf16[i], kAlign)) return EQUARX_MISALIGNED;
        mem.reads(partials_bf16[i], (size_t)n * 2);
    }
    mem.writes(codes0, (size_t)n);
    mem.writes(scales0, scale_bytes);
    mem.writes(codes1, (size_t)n);
    mem.writes(scales1, scale_bytes);
    if (int st = mem.check()) return st;
    const int64_t lanes = n / kLaneElems;
    u32x2 *c[2] = {reinterpret_cast<u32x2 *>(codes0), reinterpret_cast<u32x2 *>(codes1)};
    float *s[2] = {scales0, scales1};
#define CALL(BB)                                                                                                   \
    case BB:                                                                                                       \
        for (int32_t i = 1; i < P; ++i) {                                                                          \
            ctx.launch(hop_traffic_kernel<BB, kTilesHop>, grid_for(n, kTilesHop), kThreads,                        \
                       reinterpret_cast<const u32x4 *>(partials_bf16[i]), c[(i - 1) & 1], s[(i - 1) & 1], lanes,   \
                       c[i & 1], s[i & 1]);                                                                        \
        }                                                                                                          \
        break;
    switch (block) {
        CALL(32) CALL(64) CALL(128) CALL(256) CALL(512)
        default: break;
    }
#undef CALL
    return ctx.status();
}

int equarx_calib_interleaved_chains(const void *const *partials_bf16, int32_t M, int32_t P, int64_t n, int32_t block,
                                    void *const *out_bf16, void *const *workspaces, size_t workspace_bytes,
                                    int32_t streaming, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS || M < 1 || M > EQUARX_CALIB_MAX_CHAINS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16 || !out_bf16 || !workspaces) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    const size_t need = equarx_workspace_bytes(P, n, block);
    if (workspace_bytes < need) return EQUARX_WORKSPACE_TOO_SMALL;
    const int64_t nb = blocks_of(n, block);
    const size_t codes = round_up((size_t)n, kWorkspaceAlign);
    const size_t scales = round_up((size_t)nb * sizeof(float), kWorkspaceAlign);
    for (int32_t m = 0; m < M; ++m) {
        if (!out_bf16[m] || !workspaces[m]) return EQUARX_NULL_POINTER;
        if (misaligned(out_bf16[m], kAlign) || misaligned(workspaces[m], kWorkspaceAlign)) return EQUARX_MISALIGNED;
        Aliasing mem;       // chain m's inputs against everything any chain writes
        for (int32_t i = 0; i < P; ++i) {
            const void *x = partials_bf16[(size_t)m * P + i];
            if (!x) return EQUARX_NULL_POINTER;
            if (misaligned(x, kAlign)) return EQUARX_MISALIGNED;
            mem.reads(x, (size_t)n * 2);
        }
        for (int32_t k = 0; k < M; ++k) {
            mem.writes(out_bf16[k], (size_t)n * 2);
            mem.writes(workspaces[k], need);
        }
        if (int st = mem.check()) return st;
    }
    const bool stream_wire = streaming != 0;
    // pass by pass over all chains: chain m's wire i is read M-1 launches after it was written
    for (int32_t pass = 0; pass <= P; ++pass) {
        for (int32_t m = 0; m < M; ++m) {
            char *w = static_cast<char *>(workspaces[m]);
            int8_t *c[2] = {reinterpret_cast<int8_t *>(w), reinterpret_cast<int8_t *>(w + codes + scales)};
            float *s[2] = {reinterpret_cast<float *>(w + codes), reinterpret_cast<float *>(w + 2 * codes + scales)};
            const void *x = partials_bf16[(size_t)m * P + (pass < P ? pass : 0)];
            if (pass == 0) {
                do_quantize(x, n, block, c[0], s[0], ctx, stream_wire);
            } else if (pass < P) {
                do_hop(c[(pass - 1) & 1], s[(pass - 1) & 1], x, n, block, c[pass & 1], s[pass & 1], ctx, stream_wire);
            } else {
                do_dequantize(c[(P - 1) & 1], s[(P - 1) & 1], n, block, out_bf16[m], ctx, stream_wire);
            }
        }
    }
    return ctx.status();
}

int equarx_selftest_quotients(uint32_t first_bits, uint64_t count, uint64_t *mismatches, void *stream)
{
    LaunchCtx ctx(stream);
    if (count == 0) return EQUARX_OK;
    if (!mismatches) return EQUARX_NULL_POINTER;
    if (misaligned(mismatches, 8)) return EQUARX_MISALIGNED;
    if ((uint64_t)first_bits + count > 0x7F800000ull) return EQUARX_BAD_SHAPE;     // positive finite patterns only
    const uint64_t wgs = (count + kThreads - 1) / kThreads;
    ctx.launch(selftest_quotients_kernel, (unsigned)(wgs < 16384 ? wgs : 16384), kThreads, first_bits, count,
               reinterpret_cast<unsigned long long *>(mismatches));
    return ctx.status();
}

int equarx_selftest_rounding(uint32_t first_bits, uint64_t count, uint64_t *mismatches, void *stream)
{
    LaunchCtx ctx(stream);
    if (count == 0) return EQUARX_OK;
    if (!mismatches) return EQUARX_NULL_POINTER;
    if (misaligned(mismatches, 8)) return EQUARX_MISALIGNED;
    if ((uint64_t)first_bits + count > 0x43000000ull) return EQUARX_BAD_SHAPE;     // |p| < 128 only
    const uint64_t wgs = (count + kThreads - 1) / kThreads;
    ctx.launch(selftest_rounding_kernel, (unsigned)(wgs < 16384 ? wgs : 16384), kThreads, first_bits, count,
               reinterpret_cast<unsigned long long *>(mismatches));
    return ctx.status();
}

int equarx_eval_quotients(const float *absmax, int64_t n, float *scale, float *inv, void *stream)
{
    LaunchCtx ctx(stream);
    if (n < 0 || n > ((int64_t)1 << 31)) return EQUARX_BAD_SHAPE;
    if (n == 0) return EQUARX_OK;
    if (!absmax || !scale || !inv) return EQUARX_NULL_POINTER;
    if (misaligned(absmax, 4) || misaligned(scale, 4) || misaligned(inv, 4)) return EQUARX_MISALIGNED;
    ctx.launch(eval_quotients_kernel, (unsigned)((n + kThreads - 1) / kThreads), kThreads, absmax, n, scale, inv);
    return ctx.status();
}

void equarx_time_next_launch(void *start_event, void *stop_event)
{
    t_pending_hooks.launch_start = static_cast<hipEvent_t>(start_event);
    t_pending_hooks.launch_stop = static_cast<hipEvent_t>(stop_event);
}

void equarx_time_launch_span(int32_t first, int32_t last, void *start_event, void *stop_event)
{
    t_pending_hooks.span_start = nullptr;
    t_pending_hooks.span_stop = nullptr;
    if (first < 0 || last < first || !start_event || !stop_event) return;
    t_pending_hooks.span_first = first;
    t_pending_hooks.span_last = last;
    t_pending_hooks.span_start = static_cast<hipEvent_t>(start_event);
    t_pending_hooks.span_stop = static_cast<hipEvent_t>(stop_event);
}

void equarx_time_cancel(void) { t_pending_hooks = TimingHooks{}; }

}  // extern "C"
