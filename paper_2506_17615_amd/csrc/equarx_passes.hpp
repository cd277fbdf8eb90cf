// The three per-pass launches of the hop-by-hop chain -- quantize, hop, dequantize -- chosen by block size.
// Shared by the translation units of libequarx that launch them (the entry points and the calibration aids).
#pragma once

#include "equarx_device.hpp"
#include "equarx_launch.hpp"

namespace equarx {
namespace host {

// `streaming`: the wire these passes write or read is not read back soon through this device's caches (a ring
// step between devices, as opposed to the single-device chain, whose next launch reads what this one wrote).
template <int B>
void launch_quantize(const uint16_t *x, int64_t n, int8_t *codes, float *scales, LaunchCtx &ctx, bool streaming = false)
{
    const unsigned grid = grid_for(n, kTilesQuantize);
    if (streaming) {
        ctx.launch(quantize_kernel<B, kTilesQuantize, true>, grid, kThreads, x, n, codes, scales, blocks_of(n, B));
    } else {
        ctx.launch(quantize_kernel<B, kTilesQuantize, false>, grid, kThreads, x, n, codes, scales, blocks_of(n, B));
    }
}

template <int B>
void launch_hop(const int8_t *cin, const float *sin, const uint16_t *x, int64_t n, int8_t *cout, float *sout,
                LaunchCtx &ctx, bool streaming = false)
{
    const unsigned grid = grid_for(n, kTilesHop);
    if (streaming) {
        ctx.launch(hop_kernel<B, kTilesHop, true>, grid, kThreads, cin, sin, x, n, cout, sout, blocks_of(n, B));
    } else {
        ctx.launch(hop_kernel<B, kTilesHop, false>, grid, kThreads, cin, sin, x, n, cout, sout, blocks_of(n, B));
    }
}

template <int B>
void launch_dequantize(const int8_t *codes, const float *scales, int64_t n, uint16_t *out, LaunchCtx &ctx,
                       bool streaming = false)
{
    const unsigned grid = grid_for(n, kTilesDequantize);
    if (streaming) {
        ctx.launch(dequantize_kernel<B, kTilesDequantize, true>, grid, kThreads, codes, scales, n, out, blocks_of(n, B));
    } else {
        ctx.launch(dequantize_kernel<B, kTilesDequantize, false>, grid, kThreads, codes, scales, n, out, blocks_of(n, B));
    }
}

#define EQUARX_DISPATCH_BLOCK(block, CALL)      \
    switch (block) {                            \
        case 32: CALL(32); break;               \
        case 64: CALL(64); break;               \
        case 128: CALL(128); break;             \
        case 256: CALL(256); break;             \
        case 512: CALL(512); break;             \
        default: break;                         \
    }

inline void do_quantize(const void *x, int64_t n, int32_t block, int8_t *codes, float *scales, LaunchCtx &ctx,
                        bool streaming = false)
{
#define CALL(BB) launch_quantize<BB>(static_cast<const uint16_t *>(x), n, codes, scales, ctx, streaming)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
}

inline void do_hop(const int8_t *cin, const float *sin, const void *x, int64_t n, int32_t block, int8_t *cout,
                   float *sout, LaunchCtx &ctx, bool streaming = false)
{
#define CALL(BB) launch_hop<BB>(cin, sin, static_cast<const uint16_t *>(x), n, cout, sout, ctx, streaming)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
}

inline void do_dequantize(const int8_t *codes, const float *scales, int64_t n, int32_t block, void *out,
                          LaunchCtx &ctx, bool streaming = false)
{
#define CALL(BB) launch_dequantize<BB>(codes, scales, n, static_cast<uint16_t *>(out), ctx, streaming)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
}

}  // namespace host
}  // namespace equarx
