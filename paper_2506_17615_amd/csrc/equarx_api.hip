// Host side of libequarx: argument validation, kernel selection and launch.
// The C ABI is declared and documented in include/equarx.h.
#include "equarx.h"

#include <atomic>

#include "equarx_device.hpp"
#include "equarx_launch.hpp"
#include "equarx_passes.hpp"
#include "equarx_strided.hpp"

// Wire buffers of equarx_reduce_quantized_static, for callers that cannot allocate: one array per GPU, created
// when the library's code object is loaded on that GPU and held until the process ends.  In host code this name
// is only a handle for hipGetSymbolAddress -- never a device address.
static __device__ __align__(256) unsigned char scratch[EQUARX_STATIC_WORKSPACE_BYTES];

namespace {

using namespace equarx;
using namespace equarx::host;

// The device address of `scratch` on each GPU, resolved on the first call made with that GPU current.
constexpr int kMaxDevices = 64;
std::atomic<unsigned char *> g_scratch_on_device[kMaxDevices];

// EQUARX_OK and the current device's copy of `scratch`, or EQUARX_DEVICE_ERROR.
int static_scratch(unsigned char **ptr)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return EQUARX_DEVICE_ERROR;
    unsigned char *p = g_scratch_on_device[device].load(std::memory_order_acquire);
    if (!p) {
        void *resolved = nullptr;
        if (hipGetSymbolAddress(&resolved, HIP_SYMBOL(scratch)) != hipSuccess || !resolved) {
            (void)hipGetLastError();
            return EQUARX_DEVICE_ERROR;
        }
        p = static_cast<unsigned char *>(resolved);     // two threads racing here resolve the same address
        g_scratch_on_device[device].store(p, std::memory_order_release);
    }
    *ptr = p;
    return EQUARX_OK;
}

template <int B>
void launch_head(const uint16_t *x0, const uint16_t *x1, int64_t n, int8_t *cout, float *sout, LaunchCtx &ctx)
{
    ctx.launch(head_kernel<B, kTilesHead>, grid_for(n, kTilesHead), kThreads, x0, x1, n, cout, sout, blocks_of(n, B));
}

template <int B>
void launch_tail(const int8_t *cin, const float *sin, const uint16_t *x, int64_t n, uint16_t *out, LaunchCtx &ctx,
                 bool ag = true)
{
    if (ag) {
        ctx.launch(tail_kernel<B, kTilesTail, true>, grid_for(n, kTilesTail), kThreads, cin, sin, x, n, out, blocks_of(n, B));
    } else {
        ctx.launch(tail_kernel<B, kTilesTail, false>, grid_for(n, kTilesTail), kThreads, cin, sin, x, n, out, blocks_of(n, B));
    }
}

// P >= 3: [Q_B(x_0) + hop 1], hops 2 .. P-2, [hop P-1 + quantize/dequantize pair]; c_i lives in wire buffer i & 1.
template <int B>
void launch_fused_ends(const PartialTable &tab, int P, int64_t n, int8_t *const (&c)[2], float *const (&s)[2],
                       uint16_t *out, LaunchCtx &ctx)
{
    launch_head<B>(tab.x[0], tab.x[1], n, c[1], s[1], ctx);
    for (int i = 2; i + 1 < P; ++i) launch_hop<B>(c[(i - 1) & 1], s[(i - 1) & 1], tab.x[i], n, c[i & 1], s[i & 1], ctx);
    launch_tail<B>(c[(P - 2) & 1], s[(P - 2) & 1], tab.x[P - 1], n, out, ctx);
}

// Full loop in ring order, hop by hop: P launches, each over all P shards (one grid row per shard).
template <int B>
void launch_ring_hops(const PartialTable &tab, int P, int64_t n, bool ag, int8_t *const (&c)[3], float *const (&s)[3],
                      uint16_t *out, LaunchCtx &ctx)
{
    const int64_t nb = blocks_of(n, B);
    const int64_t shard_elems = (nb + P - 1) / P * B;       // ceil(nb / P) blocks per shard, as the single launch
    const unsigned gx = grid_for(shard_elems, kTilesHop), gy = (unsigned)P;
    ctx.launch2d(quantize_ring_kernel<B, kTilesHop>, gx, gy, kThreads, tab, P, n, shard_elems, c[0], s[0]);
    for (int i = 1; i + 1 < P; ++i) {
        ctx.launch2d(hop_ring_kernel<B, kTilesHop>, gx, gy, kThreads, c[(i - 1) & 1], s[(i - 1) & 1], tab, P, i, n, shard_elems,
                 c[i & 1], s[i & 1]);
    }
    if (ag) {
        ctx.launch2d(tail_ring_kernel<B, kTilesHop, true>, gx, gy, kThreads, c[(P - 2) & 1], s[(P - 2) & 1], tab, P, P - 1, n,
                 shard_elems, out);
    } else {
        ctx.launch2d(tail_ring_kernel<B, kTilesHop, false>, gx, gy, kThreads, c[(P - 2) & 1], s[(P - 2) & 1], tab, P, P - 1, n,
                 shard_elems, out);
    }
}

// Single-launch chain, measured on MI355X (27B-shaped size): 4 tiles per thread is fastest (63 us; 1, 2, 6, 8
// tiles and 512- or 1024-thread groups are 1-8 % slower).
#ifndef EQUARX_TILES_CHAIN
#define EQUARX_TILES_CHAIN 4
#endif
constexpr int kTilesChain = EQUARX_TILES_CHAIN;
static_assert(kMaxPartials == EQUARX_MAX_PARTIALS && kMaxBatch == EQUARX_MAX_PARTIALS, "header and device limits differ");

// Shape of a chain launch: the whole tensor in array order, or (ring layout) one grid row per shard.
struct ChainGrid {
    unsigned x, y;
    int64_t shard_elems;
};

inline ChainGrid chain_grid(int64_t n, int32_t block, int32_t P, bool ring, int tiles)
{
    ChainGrid g;
    if (ring) {
        const int64_t nb = blocks_of(n, block);
        g.shard_elems = (nb + P - 1) / P * block;           // ceil(nb / P) blocks per shard
        g.x = grid_for(g.shard_elems, tiles);
        g.y = (unsigned)P;
    } else {
        g.shard_elems = 0;
        g.x = grid_for(n, tiles);
        g.y = 1;
    }
    return g;
}

// Which chain kernel a message gets, by its size in 2048-element tiles (measured on MI355X, P = 8 and 16):
//   up to kChainSmallTiles     the latency-shaped kernel (one tile per workgroup, batched loads): 4.8 us vs 7.6 us
//                              at 344 k elements;
//   up to kChainMediumTiles    the bandwidth kernel with one tile per thread, so that every compute unit gets
//                              work: 8.4 us vs 9.8 us at 2 M elements;
//   above                      kTilesChain tiles per thread.
#ifndef EQUARX_CHAIN_SMALL_MAX_TILES
#define EQUARX_CHAIN_SMALL_MAX_TILES 512
#endif
#ifndef EQUARX_CHAIN_MEDIUM_MAX_TILES
#define EQUARX_CHAIN_MEDIUM_MAX_TILES 2048
#endif
constexpr int64_t kChainSmallTiles = EQUARX_CHAIN_SMALL_MAX_TILES;
constexpr int64_t kChainMediumTiles = EQUARX_CHAIN_MEDIUM_MAX_TILES;

template <int B, int K>
void launch_chain_k(const PartialTable &tab, int P, int64_t n, bool rs, bool ag, bool ring, uint16_t *out,
                    int8_t *wire_codes, float *wire_scales, int64_t c_step, int64_t s_step, LaunchCtx &ctx)
{
    const ChainGrid g = chain_grid(n, B, P, ring, K);
#define EQUARX_CHAIN(RS, AG, WIRE)                                                                        \
    ctx.launch2d(chain_kernel<B, K, RS, AG, WIRE>, g.x, g.y, kThreads, tab, P, n, g.shard_elems, out, wire_codes,   \
             wire_scales, c_step, s_step)
    if (rs && ag) {
        if (wire_codes) {
            EQUARX_CHAIN(true, true, true);
        } else {
            EQUARX_CHAIN(true, true, false);
        }
    } else if (rs) {
        EQUARX_CHAIN(true, false, false);
    } else {
        EQUARX_CHAIN(false, true, false);
    }
#undef EQUARX_CHAIN
}

template <int B>
void launch_chain(const PartialTable &tab, int P, int64_t n, bool rs, bool ag, bool ring, uint16_t *out,
                  int8_t *wire_codes, float *wire_scales, int64_t c_step, int64_t s_step, LaunchCtx &ctx)
{
    const int64_t tiles = (n + kTileElems - 1) / kTileElems;
    if (rs && ag && !ring && tiles <= kChainSmallTiles) {
        const unsigned grid = grid_for(n, 1);
        if (wire_codes) {
            ctx.launch(chain_small_kernel<B, true>, grid, kThreads, tab, P, n, out, wire_codes, wire_scales, c_step, s_step);
        } else {
            ctx.launch(chain_small_kernel<B, false>, grid, kThreads, tab, P, n, out, wire_codes, wire_scales, c_step, s_step);
        }
    } else if (tiles <= kChainMediumTiles) {
        launch_chain_k<B, 1>(tab, P, n, rs, ag, ring, out, wire_codes, wire_scales, c_step, s_step, ctx);
    } else {
        launch_chain_k<B, kTilesChain>(tab, P, n, rs, ag, ring, out, wire_codes, wire_scales, c_step, s_step, ctx);
    }
}

#ifndef EQUARX_TILES_SEMI
#define EQUARX_TILES_SEMI 2       // measured at the 27B shape: 66 us against 67.5 us with 4 (two running sums per tile)
#endif
constexpr int kTilesSemi = EQUARX_TILES_SEMI;

template <int B>
void launch_semi(const PartialTable &tab, int P, int64_t n, bool ag, bool ring, uint16_t *out, LaunchCtx &ctx)
{
    const ChainGrid g = chain_grid(n, B, P, ring, kTilesSemi);
    if (ag) {
        ctx.launch2d(semi_kernel<B, kTilesSemi, true>, g.x, g.y, kThreads, tab, P, n, g.shard_elems, out);
    } else {
        ctx.launch2d(semi_kernel<B, kTilesSemi, false>, g.x, g.y, kThreads, tab, P, n, g.shard_elems, out);
    }
}

#ifndef EQUARX_TILES_FLAT
#define EQUARX_TILES_FLAT 4
#endif
constexpr int kTilesFlat = EQUARX_TILES_FLAT;

template <int B, bool kStream>
void launch_flat_as(const uint16_t *local, const WireTable &tab, int R, int64_t n, uint16_t *out, int8_t *codes_out,
                    float *scales_out, LaunchCtx &ctx, bool ag)
{
    const unsigned grid = grid_for(n, kTilesFlat);
    const int64_t nb = blocks_of(n, B);
    if (!ag) {      // bf16 output of the unquantized sum; callers pass out and no wire
        ctx.launch(flat_kernel<B, kTilesFlat, true, false, false, kStream>, grid, kThreads, local, tab, R, n, out, codes_out, scales_out, nb);
    } else if (out && codes_out) {
        ctx.launch(flat_kernel<B, kTilesFlat, true, true, true, kStream>, grid, kThreads, local, tab, R, n, out, codes_out, scales_out, nb);
    } else if (out) {
        ctx.launch(flat_kernel<B, kTilesFlat, true, false, true, kStream>, grid, kThreads, local, tab, R, n, out, codes_out, scales_out, nb);
    } else {
        ctx.launch(flat_kernel<B, kTilesFlat, false, true, true, kStream>, grid, kThreads, local, tab, R, n, out, codes_out, scales_out, nb);
    }
}

// streaming: the received wires are read, and the outgoing wire is written, with non-temporal hints.
template <int B>
void launch_flat(const uint16_t *local, const WireTable &tab, int R, int64_t n, uint16_t *out, int8_t *codes_out,
                 float *scales_out, LaunchCtx &ctx, bool ag = true, bool streaming = false)
{
    if (streaming) {
        launch_flat_as<B, true>(local, tab, R, n, out, codes_out, scales_out, ctx, ag);
    } else {
        launch_flat_as<B, false>(local, tab, R, n, out, codes_out, scales_out, ctx, ag);
    }
}

// The per-step entry points are what a device calls once per step of a collective: equarx_quantize,
// equarx_reduce_stage and equarx_dequantize in a ring, equarx_quantize_batch and equarx_reduce_flat around an
// all-to-all.  The wire they read came from another device and the wire they write goes to one, so they access it
// with non-temporal hints.  The chain entry points, which run every step on this device, know that the next launch
// reads what this one wrote and keep the wire cacheable.
constexpr bool kWireLeavesTheDevice = true;

// The output of a chain may BE one of the partials (in-place reduction: every
// kernel reads an element of every partial before the thread that owns the
// element writes it, and in the hop-by-hop schedules the output is written by
// the last launch only): partials and output carry this tag, so the output may
// coincide with a partial exactly and may not overlap one in any other way.
constexpr int kInPlace = 1;

// Validates the P device pointers of a chain call and lists them as read.
inline int check_partials(const void *const *partials_bf16, int32_t P, int64_t n, Aliasing &mem)
{
    for (int32_t i = 0; i < P; ++i) {
        if (!partials_bf16[i]) return EQUARX_NULL_POINTER;
        if (misaligned(partials_bf16[i], kAlign)) return EQUARX_MISALIGNED;
        mem.reads(partials_bf16[i], (size_t)n * sizeof(uint16_t), kInPlace);
    }
    return EQUARX_OK;
}

// ... and copies them into the kernel's table.
inline int fill_table(const void *const *partials_bf16, int32_t P, int64_t n, Aliasing &mem, PartialTable &tab)
{
    for (int32_t i = 0; i < kMaxPartials; ++i) tab.x[i] = nullptr;
    if (int st = check_partials(partials_bf16, P, n, mem)) return st;
    for (int32_t i = 0; i < P; ++i) tab.x[i] = static_cast<const uint16_t *>(partials_bf16[i]);
    return EQUARX_OK;
}

// The two (semi-loop: three, semi-loop in ring order: four) wire buffers inside a workspace: codes, then scales, each part rounded up to
// the workspace alignment.
struct WireBuffers {
    int8_t *c[4];
    float *s[4];
};

inline WireBuffers carve_workspace(void *workspace, int64_t n, int64_t scales_count)
{
    const size_t codes = round_up((size_t)n, kWorkspaceAlign);
    const size_t scales = round_up((size_t)scales_count * sizeof(float), kWorkspaceAlign);
    char *w = static_cast<char *>(workspace);
    WireBuffers b;
    for (int i = 0; i < 4; ++i) {       // pairs beyond the second exist only in the semi-loop's larger workspaces
        b.c[i] = reinterpret_cast<int8_t *>(w + (size_t)i * (codes + scales));
        b.s[i] = reinterpret_cast<float *>(w + (size_t)i * (codes + scales) + codes);
    }
    return b;
}

// Semi-loop in ring order, hop by hop: h = P/2 launches in which both chains of every shard advance one device
// (grid row = shard, grid layer = direction), then the owners' launch.  Wire buffers: direction d ping-pongs between
// buffers 2d and 2d + 1.
template <int B>
void launch_semi_ring_hops(const PartialTable &tab, int P, int64_t n, bool ag, const WireBuffers &w, uint16_t *out,
                           LaunchCtx &ctx)
{
    const int64_t nb = blocks_of(n, B);
    const int64_t shard_elems = (nb + P - 1) / P * B;       // ceil(nb / P) blocks per shard, as the single launch
    const unsigned gx = grid_for(shard_elems, kTilesHop), gy = (unsigned)P;
    const int h = P / 2, count[2] = {P - 1 - h, h};
    for (int t = 0; t < h; ++t) {
        WirePair in, to;
        for (int d = 0; d < 2; ++d) {
            in.codes[d] = w.c[2 * d + ((t + 1) & 1)];
            in.scales[d] = w.s[2 * d + ((t + 1) & 1)];
            to.codes[d] = w.c[2 * d + (t & 1)];
            to.scales[d] = w.s[2 * d + (t & 1)];
        }
        ctx.launch3d(semi_ring_step_kernel<B, kTilesHop>, gx, gy, 2u, kThreads, tab, P, t, n, shard_elems, in, to);
    }
    WireTable wires;
    for (int r = 0; r < kMaxPartials; ++r) {
        wires.codes[r] = nullptr;
        wires.scales[r] = nullptr;
    }
    int received = 0;
    for (int d = 0; d < 2; ++d) {       // counter-clockwise first, as the single launch adds them
        if (count[d] == 0) continue;
        wires.codes[received] = w.c[2 * d + ((count[d] - 1) & 1)];
        wires.scales[received] = w.s[2 * d + ((count[d] - 1) & 1)];
        ++received;
    }
    if (ag) {
        ctx.launch2d(semi_ring_owner_kernel<B, kTilesFlat, true>, grid_for(shard_elems, kTilesFlat), gy, kThreads, tab, P, n, shard_elems,
                     wires, received, out);
    } else {
        ctx.launch2d(semi_ring_owner_kernel<B, kTilesFlat, false>, grid_for(shard_elems, kTilesFlat), gy, kThreads, tab, P, n,
                     shard_elems, wires, received, out);
    }
}


// ---- strided (Sec. 3.2) geometry ----

inline int check_strided(int64_t n, int32_t chunks)
{
    if (chunks != 32 && chunks != 64 && chunks != 128) return EQUARX_BAD_BLOCK;
    if (n < 0 || too_long(n) || n % ((int64_t)kChunk * chunks) != 0) return EQUARX_BAD_SHAPE;
    return EQUARX_OK;
}

inline unsigned strided_grid(int64_t n, int32_t chunks)
{
    return (unsigned)(n / ((int64_t)kChunk * chunks) * kSlicesPerChunk);
}

#define EQUARX_DISPATCH_CHUNKS(chunks, CALL) \
    switch (chunks) {                        \
        case 32: CALL(32 / kChunkGroups); break;   \
        case 64: CALL(64 / kChunkGroups); break;   \
        case 128: CALL(128 / kChunkGroups); break; \
        default: break;                      \
    }

// One tensor as the source of a per-pass strided kernel.
inline StridedSource one_tensor(const void *x)
{
    StridedSource src;
    for (int i = 0; i < kMaxPartials; ++i) src.tab.x[i] = nullptr;
    src.tab.x[0] = static_cast<const uint16_t *>(x);
    src.P = 1;
    src.per_shard = 0;
    src.offset = 0;
    return src;
}

// Partial `offset` of a chain (per_shard == 0), or in the ring layout the partial of device (k + offset) mod P for
// every shard k at once (per_shard minishards per shard).
inline StridedSource chain_source(const PartialTable &tab, int P, int per_shard, int offset)
{
    StridedSource src;
    src.tab = tab;
    src.P = P;
    src.per_shard = per_shard;
    src.offset = offset;
    return src;
}

void do_quantize_strided(const StridedSource &src, int64_t n, int32_t chunks, int8_t *codes, float *scales, LaunchCtx &ctx)
{
#define CALL(RR) ctx.launch(quantize_strided_kernel<RR>, strided_grid(n, chunks), kThreads, src, codes, scales)
    EQUARX_DISPATCH_CHUNKS(chunks, CALL)
#undef CALL
}

void do_hop_strided(const int8_t *cin, const float *sin, const StridedSource &src, int64_t n, int32_t chunks, int8_t *cout,
                    float *sout, LaunchCtx &ctx)
{
#define CALL(RR) ctx.launch(hop_strided_kernel<RR>, strided_grid(n, chunks), kThreads, cin, sin, src, cout, sout)
    EQUARX_DISPATCH_CHUNKS(chunks, CALL)
#undef CALL
}

void do_owner_strided(const StridedSource &own, const StridedWires &wires, int received, int64_t n, int32_t chunks, bool ag,
                      uint16_t *out, LaunchCtx &ctx)
{
#define CALL(RR)                                                                                                           \
    do {                                                                                                                   \
        if (ag) ctx.launch(owner_strided_kernel<RR, true>, strided_grid(n, chunks), kThreads, own, wires, received, out);  \
        else ctx.launch(owner_strided_kernel<RR, false>, strided_grid(n, chunks), kThreads, own, wires, received, out);    \
    } while (0)
    EQUARX_DISPATCH_CHUNKS(chunks, CALL)
#undef CALL
}

// The single-launch chain and its flavours: chunks = 8 * W * R (see chain_strided_kernel), 4 * W workgroups per minishard.
template <int R, int W>
void launch_chain_strided_as(const PartialTable &tab, int P, unsigned grid, int per_shard, bool semi, bool rs, bool ag,
                             uint16_t *out, LaunchCtx &ctx)
{
    if (semi && ag) ctx.launch(chain_strided_kernel<R, W, true, true, true>, grid, kThreads, tab, P, per_shard, out);
    else if (semi) ctx.launch(chain_strided_kernel<R, W, true, true, false>, grid, kThreads, tab, P, per_shard, out);
    else if (rs && ag) ctx.launch(chain_strided_kernel<R, W, false, true, true>, grid, kThreads, tab, P, per_shard, out);
    else if (rs) ctx.launch(chain_strided_kernel<R, W, false, true, false>, grid, kThreads, tab, P, per_shard, out);
    else ctx.launch(chain_strided_kernel<R, W, false, false, true>, grid, kThreads, tab, P, per_shard, out);
}

// ring: shards of ceil(minishards / P) whole minishards, shard k in the order a ring gives it.
void launch_chain_strided(const PartialTable &tab, int P, int64_t n, int32_t chunks, bool semi, bool rs, bool ag,
                          bool ring, uint16_t *out, LaunchCtx &ctx)
{
    const int64_t minishards = n / ((int64_t)kChunk * chunks);
    const int per_shard = ring ? (int)((minishards + P - 1) / P) : 0;
    const unsigned ms = (unsigned)minishards;
    switch (chunks) {
        case 32: launch_chain_strided_as<4, 1>(tab, P, ms * 4, per_shard, semi, rs, ag, out, ctx); break;
        case 64: launch_chain_strided_as<8, 1>(tab, P, ms * 4, per_shard, semi, rs, ag, out, ctx); break;
        case 128: launch_chain_strided_as<8, 2>(tab, P, ms * 8, per_shard, semi, rs, ag, out, ctx); break;
        default: break;
    }
}

void do_dequantize_strided(const int8_t *codes, const float *scales, int64_t n, int32_t chunks, void *out,
                           LaunchCtx &ctx)
{
    ctx.launch(dequantize_strided_kernel<kTilesDequantize>, grid_for(n, kTilesDequantize), kThreads, codes, scales, n, (int)chunks,
           static_cast<uint16_t *>(out));
}

}  // namespace

extern "C" {

int64_t equarx_num_blocks(int64_t n, int32_t block)
{
    if (check_shape(n, block) != EQUARX_OK) return 0;
    return blocks_of(n, block);
}

int64_t equarx_wire_row_codes(int64_t n)
{
    return n < 0 ? 0 : (int64_t)round_up((size_t)n, kAlign);
}

int64_t equarx_wire_row_scales(int64_t n, int32_t block)
{
    if (check_shape(n, block) != EQUARX_OK) return 0;
    return (int64_t)round_up((size_t)blocks_of(n, block), kAlign / sizeof(float));
}

size_t equarx_workspace_bytes(int32_t P, int64_t n, int32_t block)
{
    if (P < 1 || P > EQUARX_MAX_PARTIALS || check_shape(n, block) != EQUARX_OK) return 0;
    const size_t codes = round_up((size_t)n, kWorkspaceAlign);
    const size_t scales = round_up((size_t)blocks_of(n, block) * sizeof(float), kWorkspaceAlign);
    return 2 * (codes + scales);
}

const char *equarx_status_string(int status)
{
    switch (status) {
        case EQUARX_OK: return "ok";
        case EQUARX_NULL_POINTER: return "a required pointer is NULL";
        case EQUARX_BAD_SHAPE: return "bad shape: n < 0, P out of range, or forbidden overlap of buffers";
        case EQUARX_BAD_BLOCK: return "block size must be 32, 64, 128, 256 or 512";
        case EQUARX_MISALIGNED: return "a data pointer is not 16-byte aligned";
        case EQUARX_WORKSPACE_TOO_SMALL:
            return "workspace (the caller's, or the static array of equarx_reduce_quantized_static) is smaller than the "
                   "call needs: see equarx_workspace_bytes() / equarx_variant_workspace_bytes()";
        case EQUARX_DEVICE_ERROR: return "the HIP runtime reported an error at kernel launch";
        default: return "unknown status";
    }
}

int equarx_quantize(const void *x_bf16, int64_t n, int32_t block, int8_t *codes, float *scales, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (n == 0) return EQUARX_OK;
    if (!x_bf16 || !codes || !scales) return EQUARX_NULL_POINTER;
    if (misaligned(x_bf16, kAlign) || misaligned(codes, kAlign) || misaligned(scales, kAlign)) return EQUARX_MISALIGNED;
    Aliasing mem;
    mem.reads(x_bf16, (size_t)n * 2);
    mem.writes(codes, (size_t)n);
    mem.writes(scales, (size_t)blocks_of(n, block) * sizeof(float));
    if (int st = mem.check()) return st;
    do_quantize(x_bf16, n, block, codes, scales, ctx, kWireLeavesTheDevice);
    return ctx.status();
}

int equarx_quantize_batch(const void *const *x_bf16, int8_t *const *codes, float *const *scales, int32_t count,
                          int64_t n, int32_t block, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (count < 0 || count > kMaxBatch) return EQUARX_BAD_SHAPE;
    if (count == 0 || n == 0) return EQUARX_OK;
    if (!x_bf16 || !codes || !scales) return EQUARX_NULL_POINTER;
    QuantizeBatch tab;
    for (int32_t i = 0; i < kMaxBatch; ++i) {
        tab.x[i] = nullptr;
        tab.codes[i] = nullptr;
        tab.scales[i] = nullptr;
    }
    Aliasing mem;
    const size_t scale_bytes = (size_t)blocks_of(n, block) * sizeof(float);
    for (int32_t i = 0; i < count; ++i) {
        if (!x_bf16[i] || !codes[i] || !scales[i]) return EQUARX_NULL_POINTER;
        if (misaligned(x_bf16[i], kAlign) || misaligned(codes[i], kAlign) || misaligned(scales[i], kAlign))
            return EQUARX_MISALIGNED;
        mem.reads(x_bf16[i], (size_t)n * 2);
        mem.writes(codes[i], (size_t)n);
        mem.writes(scales[i], scale_bytes);
        tab.x[i] = static_cast<const uint16_t *>(x_bf16[i]);
        tab.codes[i] = codes[i];
        tab.scales[i] = scales[i];
    }
    if (int st = mem.check()) return st;      // two tensors sharing an output, or an output inside an input
#define CALL(BB)                                                                                                  \
    ctx.launch2d(quantize_batch_kernel<BB, kTilesQuantize, kWireLeavesTheDevice>, grid_for(n, kTilesQuantize), (unsigned)count, \
                 kThreads, tab, n, blocks_of(n, BB))
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return ctx.status();
}

int equarx_dequantize(const int8_t *codes, const float *scales, int64_t n, int32_t block, void *out_bf16,
                      void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (n == 0) return EQUARX_OK;
    if (!codes || !scales || !out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(codes, kAlign) || misaligned(scales, kAlign) || misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    Aliasing mem;
    mem.reads(codes, (size_t)n);
    mem.reads(scales, (size_t)blocks_of(n, block) * sizeof(float));
    mem.writes(out_bf16, (size_t)n * 2);
    if (int st = mem.check()) return st;
    do_dequantize(codes, scales, n, block, out_bf16, ctx, kWireLeavesTheDevice);
    return ctx.status();
}

// What a hop reads and writes: the wire may be updated in place (codes over codes, scales over scales, each
// coinciding exactly); nothing else may share memory with what is written.
static int check_hop_memory(const int8_t *codes_in, const float *scales_in, const void *local_bf16, int64_t n,
                            int64_t scales_count, const int8_t *codes_out, const float *scales_out)
{
    Aliasing mem;
    mem.reads(codes_in, (size_t)n, 1);
    mem.reads(scales_in, (size_t)scales_count * sizeof(float), 2);
    mem.reads(local_bf16, (size_t)n * 2);
    mem.writes(codes_out, (size_t)n, 1);
    mem.writes(scales_out, (size_t)scales_count * sizeof(float), 2);
    return mem.check();
}

int equarx_reduce_stage(const int8_t *codes_in, const float *scales_in, const void *local_bf16, int64_t n,
                        int32_t block, int8_t *codes_out, float *scales_out, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (n == 0) return EQUARX_OK;
    if (!codes_in || !scales_in || !local_bf16 || !codes_out || !scales_out) return EQUARX_NULL_POINTER;
    if (misaligned(codes_in, kAlign) || misaligned(scales_in, kAlign) || misaligned(local_bf16, kAlign) ||
        misaligned(codes_out, kAlign) || misaligned(scales_out, kAlign))
        return EQUARX_MISALIGNED;
    if (int st = check_hop_memory(codes_in, scales_in, local_bf16, n, blocks_of(n, block), codes_out, scales_out)) return st;
    do_hop(codes_in, scales_in, local_bf16, n, block, codes_out, scales_out, ctx, kWireLeavesTheDevice);
    return ctx.status();
}

int equarx_reduce_quantized(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, void *out_bf16,
                            void *workspace, size_t workspace_bytes, int8_t *wire_codes, float *wire_scales,
                            void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if ((wire_codes == nullptr) != (wire_scales == nullptr)) return EQUARX_NULL_POINTER;
    const bool keep_wire = wire_codes != nullptr;
    if (!keep_wire && !workspace) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    Aliasing mem;
    if (int st = check_partials(partials_bf16, P, n, mem)) return st;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    const int64_t nb = blocks_of(n, block);
    WireBuffers w{};
    int64_t c_step = 0, s_step = 0;     // distance between successive wire rows when they are kept
    if (keep_wire) {
        if (misaligned(wire_codes, kAlign) || misaligned(wire_scales, kAlign)) return EQUARX_MISALIGNED;
        c_step = equarx_wire_row_codes(n);
        s_step = equarx_wire_row_scales(n, block);
        mem.writes(wire_codes, (size_t)P * c_step);
        mem.writes(wire_scales, (size_t)P * s_step * sizeof(float));
    } else {
        if (misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
        const size_t need = equarx_workspace_bytes(P, n, block);
        if (workspace_bytes < need) return EQUARX_WORKSPACE_TOO_SMALL;
        mem.writes(workspace, need);
        w = carve_workspace(workspace, n, nb);
    }
    if (int st = mem.check()) return st;

    int8_t *c_prev = keep_wire ? wire_codes : w.c[0];
    float *s_prev = keep_wire ? wire_scales : w.s[0];
    do_quantize(partials_bf16[0], n, block, c_prev, s_prev, ctx);
    for (int32_t i = 1; i < P; ++i) {
        int8_t *c_next = keep_wire ? wire_codes + i * c_step : w.c[i & 1];
        float *s_next = keep_wire ? wire_scales + i * s_step : w.s[i & 1];
        do_hop(c_prev, s_prev, partials_bf16[i], n, block, c_next, s_next, ctx);
        c_prev = c_next;
        s_prev = s_next;
    }
    do_dequantize(c_prev, s_prev, n, block, out_bf16, ctx);
    return ctx.status();
}

int equarx_reduce_quantized_static(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                                   void *out_bf16, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    if (equarx_workspace_bytes(P, n, block) > (size_t)EQUARX_STATIC_WORKSPACE_BYTES) return EQUARX_WORKSPACE_TOO_SMALL;
    Aliasing mem;
    if (int st = check_partials(partials_bf16, P, n, mem)) return st;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    if (int st = mem.check()) return st;
    unsigned char *wire = nullptr;
    if (int st = static_scratch(&wire)) return st;
    // Nothing in the array has to start at zero: pass 0 writes wire buffer 0 completely before hop 1 reads it,
    // and every later hop reads only what the launch before it wrote.
    const WireBuffers w = carve_workspace(wire, n, blocks_of(n, block));
    do_quantize(partials_bf16[0], n, block, w.c[0], w.s[0], ctx);
    for (int32_t i = 1; i < P; ++i) {
        do_hop(w.c[(i - 1) & 1], w.s[(i - 1) & 1], partials_bf16[i], n, block, w.c[i & 1], w.s[i & 1], ctx);
    }
    do_dequantize(w.c[(P - 1) & 1], w.s[(P - 1) & 1], n, block, out_bf16, ctx);
    return ctx.status();
}

int equarx_reduce_quantized_fused_ends(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                                       void *out_bf16, void *workspace, size_t workspace_bytes, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    PartialTable tab;
    Aliasing mem;
    if (int st = fill_table(partials_bf16, P, n, mem, tab)) return st;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    uint16_t *out = static_cast<uint16_t *>(out_bf16);
    if (P <= 2) {       // both ends meet: the chain is one launch and needs no wire
        if (int st = mem.check()) return st;
#define CALL(BB) launch_chain<BB>(tab, P, n, true, true, false, out, nullptr, nullptr, 0, 0, ctx)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
        return ctx.status();
    }
    if (!workspace) return EQUARX_NULL_POINTER;
    if (misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
    const size_t need = equarx_workspace_bytes(P, n, block);
    if (workspace_bytes < need) return EQUARX_WORKSPACE_TOO_SMALL;
    mem.writes(workspace, need);
    if (int st = mem.check()) return st;
    const WireBuffers w = carve_workspace(workspace, n, blocks_of(n, block));
    int8_t *const c[2] = {w.c[0], w.c[1]};
    float *const s[2] = {w.s[0], w.s[1]};
#define CALL(BB) launch_fused_ends<BB>(tab, P, n, c, s, out, ctx)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return ctx.status();
}

int equarx_reduce_fused(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, void *out_bf16,
                        int8_t *wire_codes, float *wire_scales, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if ((wire_codes == nullptr) != (wire_scales == nullptr)) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    if (wire_codes && (misaligned(wire_codes, kAlign) || misaligned(wire_scales, kAlign))) return EQUARX_MISALIGNED;
    PartialTable tab;
    Aliasing mem;
    if (int st = fill_table(partials_bf16, P, n, mem, tab)) return st;
    const int64_t c_step = equarx_wire_row_codes(n);
    const int64_t s_step = equarx_wire_row_scales(n, block);
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    mem.writes(wire_codes, (size_t)P * c_step);
    mem.writes(wire_scales, (size_t)P * s_step * sizeof(float));
    if (int st = mem.check()) return st;
#define CALL(BB)                                                                                               \
    launch_chain<BB>(tab, P, n, true, true, false, static_cast<uint16_t *>(out_bf16), wire_codes, wire_scales, \
                     c_step, s_step, ctx)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return ctx.status();
}

int equarx_reduce_variant(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, uint32_t flags,
                          void *out_bf16, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    const uint32_t known = EQUARX_SEMI_LOOP | EQUARX_RS_UNQUANTIZED | EQUARX_AG_UNQUANTIZED | EQUARX_RING_ORDER;
    if (flags & ~known) return EQUARX_BAD_SHAPE;
    const bool semi = flags & EQUARX_SEMI_LOOP, rs = !(flags & EQUARX_RS_UNQUANTIZED);
    const bool ag = !(flags & EQUARX_AG_UNQUANTIZED), ring = flags & EQUARX_RING_ORDER;
    if (!rs && !ag) return EQUARX_BAD_SHAPE;        // nothing quantized: not this library's business
    if (semi && !rs) return EQUARX_BAD_SHAPE;       // the semi-loop is a reduce-scatter schedule
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    PartialTable tab;
    Aliasing mem;
    if (int st = fill_table(partials_bf16, P, n, mem, tab)) return st;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    if (int st = mem.check()) return st;
    uint16_t *out = static_cast<uint16_t *>(out_bf16);
    if (semi) {
#define CALL(BB) launch_semi<BB>(tab, P, n, ag, ring, out, ctx)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    } else {
#define CALL(BB) launch_chain<BB>(tab, P, n, rs, ag, ring, out, nullptr, nullptr, 0, 0, ctx)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    }
    return ctx.status();
}

size_t equarx_variant_workspace_bytes(uint32_t flags, int32_t P, int64_t n, int32_t block)
{
    const size_t two = equarx_workspace_bytes(P, n, block);
    if (!(flags & EQUARX_SEMI_LOOP)) return two;
    // the semi-loop keeps one chain's wire while the other runs (three buffers); in ring order both chains advance
    // in the same launch and each ping-pongs between two buffers of its own (four)
    return (flags & EQUARX_RING_ORDER) ? two * 2 : two / 2 * 3;
}

int equarx_reduce_variant_hops(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, uint32_t flags,
                               void *out_bf16, void *workspace, size_t workspace_bytes, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (flags & ~(uint32_t)(EQUARX_SEMI_LOOP | EQUARX_AG_UNQUANTIZED | EQUARX_RING_ORDER)) return EQUARX_BAD_SHAPE;
    const bool semi = flags & EQUARX_SEMI_LOOP, ag = !(flags & EQUARX_AG_UNQUANTIZED);
    const bool ring = flags & EQUARX_RING_ORDER;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16 || !workspace) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign) || misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
    const size_t need = equarx_variant_workspace_bytes(flags, P, n, block);
    if (workspace_bytes < need) return EQUARX_WORKSPACE_TOO_SMALL;
    PartialTable tab;
    Aliasing mem;
    if (int st = fill_table(partials_bf16, P, n, mem, tab)) return st;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    mem.writes(workspace, need);
    if (int st = mem.check()) return st;

    const WireBuffers w = carve_workspace(workspace, n, blocks_of(n, block));
    int8_t *const c[3] = {w.c[0], w.c[1], w.c[2]};
    float *const s[3] = {w.s[0], w.s[1], w.s[2]};
    uint16_t *out = static_cast<uint16_t *>(out_bf16);

    if (semi && ring) {     // every launch is one semi-loop iteration of the ring on all P shards, both directions
#define CALL(BB) launch_semi_ring_hops<BB>(tab, P, n, ag, w, out, ctx)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
        return ctx.status();
    }
    if (!semi) {
        if (P == 1) {       // no hop: one launch quantizes/dequantizes (or copies) partial 0
#define CALL(BB) launch_chain<BB>(tab, P, n, true, ag, ring, out, nullptr, nullptr, 0, 0, ctx)
            EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
            return ctx.status();
        }
        if (ring) {         // every launch is one ring step on all P shards: grid row k takes device k+1+step's partial
#define CALL(BB) launch_ring_hops<BB>(tab, P, n, ag, c, s, out, ctx)
            EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
            return ctx.status();
        }
        // Q_B(x_0), hops 1 .. P-2, then the last hop with or without the all-gather's quantize/dequantize pair
        do_quantize(tab.x[0], n, block, c[0], s[0], ctx);
        for (int32_t i = 1; i + 1 < P; ++i) do_hop(c[(i - 1) & 1], s[(i - 1) & 1], tab.x[i], n, block, c[i & 1], s[i & 1], ctx);
#define CALL(BB) launch_tail<BB>(c[(P - 2) & 1], s[(P - 2) & 1], tab.x[P - 1], n, out, ctx, ag)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
        return ctx.status();
    }

    // Semi-loop (Sec. 3.3): partial 0 owns the result; the counter-clockwise chain h+1, ..., P-1 and the clockwise
    // chain h, h-1, ..., 1 each run hop by hop and end in a wire the owner receives; the owner adds them to its
    // own shard, counter-clockwise first.
    const int32_t h = P / 2, na = P - 1 - h, nbk = h;
    WireTable wires;
    for (int32_t r = 0; r < kMaxPartials; ++r) {
        wires.codes[r] = nullptr;
        wires.scales[r] = nullptr;
    }
    int32_t received = 0;
    int last_a = -1;
    if (na > 0) {
        do_quantize(tab.x[h + 1], n, block, c[0], s[0], ctx);
        for (int32_t k = 1; k < na; ++k) do_hop(c[(k - 1) & 1], s[(k - 1) & 1], tab.x[h + 1 + k], n, block, c[k & 1], s[k & 1], ctx);
        last_a = (na - 1) & 1;
        wires.codes[received] = c[last_a];
        wires.scales[received] = s[last_a];
        ++received;
    }
    if (nbk > 0) {
        const int u[2] = {last_a == 0 ? 1 : 0, 2};      // two buffers that do not hold the first chain's wire
        do_quantize(tab.x[h], n, block, c[u[0]], s[u[0]], ctx);
        for (int32_t k = 1; k < nbk; ++k) {
            do_hop(c[u[(k - 1) & 1]], s[u[(k - 1) & 1]], tab.x[h - k], n, block, c[u[k & 1]], s[u[k & 1]], ctx);
        }
        wires.codes[received] = c[u[(nbk - 1) & 1]];
        wires.scales[received] = s[u[(nbk - 1) & 1]];
        ++received;
    }
#define CALL(BB) launch_flat<BB>(tab.x[0], wires, received, n, out, nullptr, nullptr, ctx, ag)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return ctx.status();
}

int equarx_reduce_flat(const void *local_bf16, const int8_t *const *codes, const float *const *scales, int32_t R,
                       int64_t n, int32_t block, void *out_bf16, int8_t *codes_out, float *scales_out, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_shape(n, block)) return st;
    if (R < 0 || R >= EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (R > 0 && (!codes || !scales)) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!local_bf16) return EQUARX_NULL_POINTER;
    if ((codes_out == nullptr) != (scales_out == nullptr)) return EQUARX_NULL_POINTER;
    if (!out_bf16 && !codes_out) return EQUARX_NULL_POINTER;                    // nothing to write
    if (misaligned(local_bf16, kAlign) || (out_bf16 && misaligned(out_bf16, kAlign))) return EQUARX_MISALIGNED;
    if (codes_out && (misaligned(codes_out, kAlign) || misaligned(scales_out, kAlign))) return EQUARX_MISALIGNED;
    const size_t scale_bytes = (size_t)blocks_of(n, block) * sizeof(float);
    Aliasing mem;
    mem.reads(local_bf16, (size_t)n * 2);
    mem.writes(out_bf16, (size_t)n * 2);
    mem.writes(codes_out, (size_t)n);
    mem.writes(scales_out, scale_bytes);
    WireTable tab;
    for (int32_t r = 0; r < kMaxPartials; ++r) {
        tab.codes[r] = nullptr;
        tab.scales[r] = nullptr;
    }
    for (int32_t r = 0; r < R; ++r) {
        if (!codes[r] || !scales[r]) return EQUARX_NULL_POINTER;
        if (misaligned(codes[r], kAlign) || misaligned(scales[r], kAlign)) return EQUARX_MISALIGNED;
        mem.reads(codes[r], (size_t)n);
        mem.reads(scales[r], scale_bytes);
        tab.codes[r] = codes[r];
        tab.scales[r] = scales[r];
    }
    if (int st = mem.check()) return st;          // outputs must not share memory with inputs or one another
#define CALL(BB)                                                                                                  \
    launch_flat<BB>(static_cast<const uint16_t *>(local_bf16), tab, R, n, static_cast<uint16_t *>(out_bf16), codes_out, \
                    scales_out, ctx, true, kWireLeavesTheDevice)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return ctx.status();
}

int equarx_quantize_strided(const void *x_bf16, int64_t n, int32_t chunks, int8_t *codes, float *scales, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_strided(n, chunks)) return st;
    if (n == 0) return EQUARX_OK;
    if (!x_bf16 || !codes || !scales) return EQUARX_NULL_POINTER;
    if (misaligned(x_bf16, kAlign) || misaligned(codes, kAlign) || misaligned(scales, kAlign)) return EQUARX_MISALIGNED;
    Aliasing mem;
    mem.reads(x_bf16, (size_t)n * 2);
    mem.writes(codes, (size_t)n);
    mem.writes(scales, (size_t)(n / chunks) * sizeof(float));
    if (int st = mem.check()) return st;
    do_quantize_strided(one_tensor(x_bf16), n, chunks, codes, scales, ctx);
    return ctx.status();
}

int equarx_dequantize_strided(const int8_t *codes, const float *scales, int64_t n, int32_t chunks, void *out_bf16,
                              void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_strided(n, chunks)) return st;
    if (n == 0) return EQUARX_OK;
    if (!codes || !scales || !out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(codes, kAlign) || misaligned(scales, kAlign) || misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    Aliasing mem;
    mem.reads(codes, (size_t)n);
    mem.reads(scales, (size_t)(n / chunks) * sizeof(float));
    mem.writes(out_bf16, (size_t)n * 2);
    if (int st = mem.check()) return st;
    do_dequantize_strided(codes, scales, n, chunks, out_bf16, ctx);
    return ctx.status();
}

int equarx_reduce_stage_strided(const int8_t *codes_in, const float *scales_in, const void *local_bf16, int64_t n,
                                int32_t chunks, int8_t *codes_out, float *scales_out, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_strided(n, chunks)) return st;
    if (n == 0) return EQUARX_OK;
    if (!codes_in || !scales_in || !local_bf16 || !codes_out || !scales_out) return EQUARX_NULL_POINTER;
    if (misaligned(codes_in, kAlign) || misaligned(scales_in, kAlign) || misaligned(local_bf16, kAlign) ||
        misaligned(codes_out, kAlign) || misaligned(scales_out, kAlign))
        return EQUARX_MISALIGNED;
    if (int st = check_hop_memory(codes_in, scales_in, local_bf16, n, n / chunks, codes_out, scales_out)) return st;
    do_hop_strided(codes_in, scales_in, one_tensor(local_bf16), n, chunks, codes_out, scales_out, ctx);
    return ctx.status();
}

int equarx_reduce_quantized_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks,
                                    void *out_bf16, void *workspace, size_t workspace_bytes, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_strided(n, chunks)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16 || !workspace) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign) || misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
    Aliasing mem;
    if (int st = check_partials(partials_bf16, P, n, mem)) return st;
    // one scale per `chunks` elements: the same workspace as the contiguous chain with block = chunks
    const size_t need = equarx_workspace_bytes(P, n, chunks);
    if (workspace_bytes < need) return EQUARX_WORKSPACE_TOO_SMALL;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    mem.writes(workspace, need);
    if (int st = mem.check()) return st;
    const WireBuffers w = carve_workspace(workspace, n, n / chunks);
    do_quantize_strided(one_tensor(partials_bf16[0]), n, chunks, w.c[0], w.s[0], ctx);
    for (int32_t i = 1; i < P; ++i) {
        do_hop_strided(w.c[(i - 1) & 1], w.s[(i - 1) & 1], one_tensor(partials_bf16[i]), n, chunks, w.c[i & 1], w.s[i & 1], ctx);
    }
    do_dequantize_strided(w.c[(P - 1) & 1], w.s[(P - 1) & 1], n, chunks, out_bf16, ctx);
    return ctx.status();
}

int equarx_reduce_fused_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks, void *out_bf16,
                                void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_strided(n, chunks)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    PartialTable tab;
    Aliasing mem;
    if (int st = fill_table(partials_bf16, P, n, mem, tab)) return st;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    if (int st = mem.check()) return st;
    launch_chain_strided(tab, P, n, chunks, false, true, true, false, static_cast<uint16_t *>(out_bf16), ctx);
    return ctx.status();
}

int equarx_reduce_variant_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks,
                                  uint32_t flags, void *out_bf16, void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_strided(n, chunks)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (flags & ~(uint32_t)(EQUARX_SEMI_LOOP | EQUARX_RS_UNQUANTIZED | EQUARX_AG_UNQUANTIZED | EQUARX_RING_ORDER))
        return EQUARX_BAD_SHAPE;
    const bool semi = flags & EQUARX_SEMI_LOOP, rs = !(flags & EQUARX_RS_UNQUANTIZED);
    const bool ag = !(flags & EQUARX_AG_UNQUANTIZED), ring = flags & EQUARX_RING_ORDER;
    if (!rs && !ag) return EQUARX_BAD_SHAPE;        // nothing quantized
    if (semi && !rs) return EQUARX_BAD_SHAPE;       // the semi-loop is a reduce-scatter schedule
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    PartialTable tab;
    Aliasing mem;
    if (int st = fill_table(partials_bf16, P, n, mem, tab)) return st;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    if (int st = mem.check()) return st;
    launch_chain_strided(tab, P, n, chunks, semi, rs, ag, ring, static_cast<uint16_t *>(out_bf16), ctx);
    return ctx.status();
}

int equarx_reduce_variant_hops_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks,
                                       uint32_t flags, void *out_bf16, void *workspace, size_t workspace_bytes,
                                       void *stream)
{
    LaunchCtx ctx(stream);
    if (int st = check_strided(n, chunks)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (flags & ~(uint32_t)(EQUARX_SEMI_LOOP | EQUARX_AG_UNQUANTIZED | EQUARX_RING_ORDER)) return EQUARX_BAD_SHAPE;
    const bool semi = flags & EQUARX_SEMI_LOOP, ag = !(flags & EQUARX_AG_UNQUANTIZED), ring = flags & EQUARX_RING_ORDER;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16 || !workspace) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign) || misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
    // one scale per `chunks` elements: the contiguous variants' workspace with block = chunks
    const size_t need = equarx_variant_workspace_bytes(flags & ~(uint32_t)EQUARX_RING_ORDER, P, n, chunks);
    if (workspace_bytes < need) return EQUARX_WORKSPACE_TOO_SMALL;
    PartialTable tab;
    Aliasing mem;
    if (int st = fill_table(partials_bf16, P, n, mem, tab)) return st;
    mem.writes(out_bf16, (size_t)n * 2, kInPlace);
    mem.writes(workspace, need);
    if (int st = mem.check()) return st;

    const WireBuffers w = carve_workspace(workspace, n, n / chunks);
    int8_t *const c[3] = {w.c[0], w.c[1], w.c[2]};
    float *const s[3] = {w.s[0], w.s[1], w.s[2]};
    uint16_t *out = static_cast<uint16_t *>(out_bf16);
    StridedWires wires = {{nullptr, nullptr}, {nullptr, nullptr}};
    // Ring layout: shards of ceil(M / P) whole minishards; every launch is one ring step on all P shards at once,
    // the workgroups of shard k reading the partial of device (k + offset) mod P.  Array order: offset = partial.
    const int64_t minishards = n / ((int64_t)kChunk * chunks);
    const int per_shard = ring ? (int)((minishards + P - 1) / P) : 0;
    // position i of the full loop: a ring starts shard k's chain at device k+1 and ends it on device k
    const auto at = [&](int i) { return chain_source(tab, P, per_shard, ring ? (i + 1) % P : i); };
    // position i of the semi-loop counts from its owner: device k in a ring, partial 0 otherwise
    const auto around = [&](int i) { return chain_source(tab, P, per_shard, i); };

    if (!semi) {
        // Q_B(x_0), hops 1 .. P-2, then the device holding x_(P-1) adds the last wire and feeds the all-gather
        int received = 0;
        if (P > 1) {
            do_quantize_strided(at(0), n, chunks, c[0], s[0], ctx);
            for (int32_t i = 1; i + 1 < P; ++i) {
                do_hop_strided(c[(i - 1) & 1], s[(i - 1) & 1], at(i), n, chunks, c[i & 1], s[i & 1], ctx);
            }
            wires.codes[0] = c[(P - 2) & 1];
            wires.scales[0] = s[(P - 2) & 1];
            received = 1;
        }
        do_owner_strided(at(P - 1), wires, received, n, chunks, ag, out, ctx);
        return ctx.status();
    }

    // Semi-loop (Sec. 3.3): the owner is position 0; the chain h+1, h+2, ..., P-1 (na sends) and the chain h, h-1,
    // ..., 1 (nb >= na sends) each advance one device per launch, both in the same launch while both are under way
    // (grid row = chain), each on a wire buffer of its own that its hops rewrite in place; the owner receives the
    // shorter chain's wire first.
    const int32_t h = P / 2, na = P - 1 - h, nb = h;
    for (int32_t t = 0; t < nb; ++t) {
        StridedDirections dirs;
        dirs.d[0] = {h + 1 + t, t ? c[0] : nullptr, t ? s[0] : nullptr, c[0], s[0]};
        dirs.d[1] = {h - t, t ? c[1] : nullptr, t ? s[1] : nullptr, c[1], s[1]};
        if (t < na) {
#define CALL(RR) ctx.launch2d(semi_step_strided_kernel<RR>, strided_grid(n, chunks), 2u, kThreads, tab, (int)P, per_shard, dirs)
            EQUARX_DISPATCH_CHUNKS(chunks, CALL)
#undef CALL
        } else if (t == 0) {
            do_quantize_strided(around(h), n, chunks, c[1], s[1], ctx);
        } else {
            do_hop_strided(c[1], s[1], around(h - t), n, chunks, c[1], s[1], ctx);
        }
    }
    int received = 0;
    if (na > 0) {
        wires.codes[received] = c[0];
        wires.scales[received] = s[0];
        ++received;
    }
    if (nb > 0) {
        wires.codes[received] = c[1];
        wires.scales[received] = s[1];
        ++received;
    }
    do_owner_strided(around(0), wires, received, n, chunks, ag, out, ctx);
    return ctx.status();
}

}  // extern "C"
