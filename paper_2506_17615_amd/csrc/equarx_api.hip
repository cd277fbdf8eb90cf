// Host side of libequarx: argument validation, kernel selection and launch.
// The C ABI is declared and documented in include/equarx.h.
#include "equarx.h"

#include <hip/hip_ext.h>

#include "equarx_device.hpp"
#include "equarx_strided.hpp"

namespace {

using namespace equarx;

constexpr size_t kAlign = 16;          // every data pointer
constexpr size_t kWorkspaceAlign = 256;

// Tiles a thread keeps in flight (K): 2048*K elements per workgroup.
// Measured on MI355X at the 27B-shaped size: 3 beats 1, 2 and 4 by 2-5 %.
#ifndef EQUARX_TILES_QUANTIZE
#define EQUARX_TILES_QUANTIZE 3
#endif
#ifndef EQUARX_TILES_HOP
#define EQUARX_TILES_HOP 3
#endif
#ifndef EQUARX_TILES_DEQUANTIZE
#define EQUARX_TILES_DEQUANTIZE 3
#endif
// First and last launch of the ends-fused schedule: 2, 3 and 4 tiles are within 1 % of each other, 1 is 7 % slower.
#ifndef EQUARX_TILES_HEAD
#define EQUARX_TILES_HEAD 3
#endif
#ifndef EQUARX_TILES_TAIL
#define EQUARX_TILES_TAIL 3
#endif
constexpr int kTilesHead = EQUARX_TILES_HEAD;
constexpr int kTilesTail = EQUARX_TILES_TAIL;
constexpr int kTilesQuantize = EQUARX_TILES_QUANTIZE;
constexpr int kTilesHop = EQUARX_TILES_HOP;
constexpr int kTilesDequantize = EQUARX_TILES_DEQUANTIZE;

inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

inline bool block_ok(int32_t block)
{
    return block == 32 || block == 64 || block == 128 || block == 256 || block == 512;
}

inline int64_t blocks_of(int64_t n, int32_t block) { return (n + block - 1) / block; }

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline unsigned grid_for(int64_t n, int tiles)
{
    const int64_t per_wg = (int64_t)kTileElems * tiles;
    return (unsigned)((n + per_wg - 1) / per_wg);
}

// The grid is a 32-bit count of workgroups; 2048*K elements each.
inline bool too_long(int64_t n) { return n > ((int64_t)1 << 40); }

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? EQUARX_OK : EQUARX_DEVICE_ERROR;
}

// Profiling aid (equarx_time_next_launch): events the calling thread's next
// kernel launch carries, so that they record that kernel's own begin and end.
thread_local hipEvent_t t_start_event = nullptr;
thread_local hipEvent_t t_stop_event = nullptr;

// Profiling aid (equarx_time_launch_span): plain events recorded on the stream
// around a run of the calling thread's coming launches.
thread_local hipEvent_t t_span_start = nullptr;
thread_local hipEvent_t t_span_stop = nullptr;
thread_local int t_span_first = 0;      // launches still to pass before the start event is recorded
thread_local int t_span_last = 0;       // launches still to pass before the one the stop event follows

template <typename... KArgs, typename... Args>
inline void launch2d(void (*kernel)(KArgs...), unsigned grid_x, unsigned grid_y, hipStream_t s, Args... args)
{
    hipEvent_t e0 = t_start_event, e1 = t_stop_event;
    t_start_event = nullptr;
    t_stop_event = nullptr;
    if (t_span_start) {
        if (t_span_first == 0) {
            (void)hipEventRecord(t_span_start, s);
            t_span_start = nullptr;
        } else {
            --t_span_first;
        }
    }
    hipExtLaunchKernelGGL(kernel, dim3(grid_x, grid_y), dim3(kThreads), 0, s, e0, e1, 0, static_cast<KArgs>(args)...);
    if (t_span_stop) {
        if (t_span_last == 0) {
            (void)hipEventRecord(t_span_stop, s);
            t_span_stop = nullptr;
        } else {
            --t_span_last;
        }
    }
}

template <typename... KArgs, typename... Args>
inline void launch(void (*kernel)(KArgs...), unsigned grid, hipStream_t s, Args... args)
{
    launch2d(kernel, grid, 1u, s, args...);
}

template <int B>
void launch_quantize(const uint16_t *x, int64_t n, int8_t *codes, float *scales, hipStream_t s)
{
    launch(quantize_kernel<B, kTilesQuantize>, grid_for(n, kTilesQuantize), s, x, n, codes, scales, blocks_of(n, B));
}

template <int B>
void launch_hop(const int8_t *cin, const float *sin, const uint16_t *x, int64_t n, int8_t *cout, float *sout,
                hipStream_t s)
{
    launch(hop_kernel<B, kTilesHop>, grid_for(n, kTilesHop), s, cin, sin, x, n, cout, sout, blocks_of(n, B));
}

template <int B>
void launch_dequantize(const int8_t *codes, const float *scales, int64_t n, uint16_t *out, hipStream_t s)
{
    launch(dequantize_kernel<B, kTilesDequantize>, grid_for(n, kTilesDequantize), s, codes, scales, n, out,
           blocks_of(n, B));
}

template <int B>
void launch_head(const uint16_t *x0, const uint16_t *x1, int64_t n, int8_t *cout, float *sout, hipStream_t s)
{
    launch(head_kernel<B, kTilesHead>, grid_for(n, kTilesHead), s, x0, x1, n, cout, sout, blocks_of(n, B));
}

template <int B>
void launch_tail(const int8_t *cin, const float *sin, const uint16_t *x, int64_t n, uint16_t *out, hipStream_t s,
                 bool ag = true)
{
    if (ag) {
        launch(tail_kernel<B, kTilesTail, true>, grid_for(n, kTilesTail), s, cin, sin, x, n, out, blocks_of(n, B));
    } else {
        launch(tail_kernel<B, kTilesTail, false>, grid_for(n, kTilesTail), s, cin, sin, x, n, out, blocks_of(n, B));
    }
}

// P >= 3: [Q_B(x_0) + hop 1], hops 2 .. P-2, [hop P-1 + quantize/dequantize pair]; c_i lives in wire buffer i & 1.
template <int B>
void launch_fused_ends(const PartialTable &tab, int P, int64_t n, int8_t *const (&c)[2], float *const (&s)[2],
                       uint16_t *out, hipStream_t hs)
{
    launch_head<B>(tab.x[0], tab.x[1], n, c[1], s[1], hs);
    for (int i = 2; i + 1 < P; ++i) launch_hop<B>(c[(i - 1) & 1], s[(i - 1) & 1], tab.x[i], n, c[i & 1], s[i & 1], hs);
    launch_tail<B>(c[(P - 2) & 1], s[(P - 2) & 1], tab.x[P - 1], n, out, hs);
}

// Full loop in ring order, hop by hop: P launches, each over all P shards (one grid row per shard).
template <int B>
void launch_ring_hops(const PartialTable &tab, int P, int64_t n, bool ag, int8_t *const (&c)[3], float *const (&s)[3],
                      uint16_t *out, hipStream_t hs)
{
    const int64_t nb = blocks_of(n, B);
    const int64_t shard_elems = (nb + P - 1) / P * B;       // ceil(nb / P) blocks per shard, as the single launch
    const unsigned gx = grid_for(shard_elems, kTilesHop), gy = (unsigned)P;
    launch2d(quantize_ring_kernel<B, kTilesHop>, gx, gy, hs, tab, P, n, shard_elems, c[0], s[0]);
    for (int i = 1; i + 1 < P; ++i) {
        launch2d(hop_ring_kernel<B, kTilesHop>, gx, gy, hs, c[(i - 1) & 1], s[(i - 1) & 1], tab, P, i, n, shard_elems,
                 c[i & 1], s[i & 1]);
    }
    if (ag) {
        launch2d(tail_ring_kernel<B, kTilesHop, true>, gx, gy, hs, c[(P - 2) & 1], s[(P - 2) & 1], tab, P, P - 1, n,
                 shard_elems, out);
    } else {
        launch2d(tail_ring_kernel<B, kTilesHop, false>, gx, gy, hs, c[(P - 2) & 1], s[(P - 2) & 1], tab, P, P - 1, n,
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
                    int8_t *wire_codes, float *wire_scales, int64_t c_step, int64_t s_step, hipStream_t s)
{
    const ChainGrid g = chain_grid(n, B, P, ring, K);
#define EQUARX_CHAIN(RS, AG, WIRE)                                                                        \
    launch2d(chain_kernel<B, K, RS, AG, WIRE>, g.x, g.y, s, tab, P, n, g.shard_elems, out, wire_codes,   \
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
                  int8_t *wire_codes, float *wire_scales, int64_t c_step, int64_t s_step, hipStream_t s)
{
    const int64_t tiles = (n + kTileElems - 1) / kTileElems;
    if (rs && ag && !ring && tiles <= kChainSmallTiles) {
        const unsigned grid = grid_for(n, 1);
        if (wire_codes) {
            launch(chain_small_kernel<B, true>, grid, s, tab, P, n, out, wire_codes, wire_scales, c_step, s_step);
        } else {
            launch(chain_small_kernel<B, false>, grid, s, tab, P, n, out, wire_codes, wire_scales, c_step, s_step);
        }
    } else if (tiles <= kChainMediumTiles) {
        launch_chain_k<B, 1>(tab, P, n, rs, ag, ring, out, wire_codes, wire_scales, c_step, s_step, s);
    } else {
        launch_chain_k<B, kTilesChain>(tab, P, n, rs, ag, ring, out, wire_codes, wire_scales, c_step, s_step, s);
    }
}

#ifndef EQUARX_TILES_SEMI
#define EQUARX_TILES_SEMI 2       // measured at the 27B shape: 66 us against 67.5 us with 4 (two running sums per tile)
#endif
constexpr int kTilesSemi = EQUARX_TILES_SEMI;

template <int B>
void launch_semi(const PartialTable &tab, int P, int64_t n, bool ag, bool ring, uint16_t *out, hipStream_t s)
{
    const ChainGrid g = chain_grid(n, B, P, ring, kTilesSemi);
    if (ag) {
        launch2d(semi_kernel<B, kTilesSemi, true>, g.x, g.y, s, tab, P, n, g.shard_elems, out);
    } else {
        launch2d(semi_kernel<B, kTilesSemi, false>, g.x, g.y, s, tab, P, n, g.shard_elems, out);
    }
}

#ifndef EQUARX_TILES_FLAT
#define EQUARX_TILES_FLAT 4
#endif
constexpr int kTilesFlat = EQUARX_TILES_FLAT;

template <int B>
void launch_flat(const uint16_t *local, const WireTable &tab, int R, int64_t n, uint16_t *out, int8_t *codes_out,
                 float *scales_out, hipStream_t s, bool ag = true)
{
    const unsigned grid = grid_for(n, kTilesFlat);
    const int64_t nb = blocks_of(n, B);
    if (!ag) {      // bf16 output of the unquantized sum; callers pass out and no wire
        launch(flat_kernel<B, kTilesFlat, true, false, false>, grid, s, local, tab, R, n, out, codes_out, scales_out, nb);
    } else if (out && codes_out) {
        launch(flat_kernel<B, kTilesFlat, true, true>, grid, s, local, tab, R, n, out, codes_out, scales_out, nb);
    } else if (out) {
        launch(flat_kernel<B, kTilesFlat, true, false>, grid, s, local, tab, R, n, out, codes_out, scales_out, nb);
    } else {
        launch(flat_kernel<B, kTilesFlat, false, true>, grid, s, local, tab, R, n, out, codes_out, scales_out, nb);
    }
}

// The output of a chain may BE one of the partials (in-place reduction: every
// kernel reads an element of every partial before the thread that owns the
// element writes it, and in the hop-by-hop schedules the output is written by
// the last launch only).  An output that overlaps a partial without coinciding
// with it would be read after it was overwritten.
inline bool overlaps_without_coinciding(const void *partial, const void *out, int64_t n)
{
    if (!out || partial == out) return false;
    const uintptr_t a = reinterpret_cast<uintptr_t>(partial), b = reinterpret_cast<uintptr_t>(out);
    const uintptr_t bytes = (uintptr_t)n * sizeof(uint16_t);
    return a < b + bytes && b < a + bytes;
}

// Validates the P device pointers of a chain call.
inline int check_partials(const void *const *partials_bf16, int32_t P, int64_t n, const void *out_bf16)
{
    for (int32_t i = 0; i < P; ++i) {
        if (!partials_bf16[i]) return EQUARX_NULL_POINTER;
        if (misaligned(partials_bf16[i], kAlign)) return EQUARX_MISALIGNED;
        if (overlaps_without_coinciding(partials_bf16[i], out_bf16, n)) return EQUARX_BAD_SHAPE;
    }
    return EQUARX_OK;
}

// ... and copies them into the kernel's table.
inline int fill_table(const void *const *partials_bf16, int32_t P, int64_t n, const void *out_bf16, PartialTable &tab)
{
    for (int32_t i = 0; i < kMaxPartials; ++i) tab.x[i] = nullptr;
    if (int st = check_partials(partials_bf16, P, n, out_bf16)) return st;
    for (int32_t i = 0; i < P; ++i) tab.x[i] = static_cast<const uint16_t *>(partials_bf16[i]);
    return EQUARX_OK;
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

void do_quantize(const void *x, int64_t n, int32_t block, int8_t *codes, float *scales, hipStream_t s)
{
#define CALL(BB) launch_quantize<BB>(static_cast<const uint16_t *>(x), n, codes, scales, s)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
}

void do_hop(const int8_t *cin, const float *sin, const void *x, int64_t n, int32_t block, int8_t *cout, float *sout,
            hipStream_t s)
{
#define CALL(BB) launch_hop<BB>(cin, sin, static_cast<const uint16_t *>(x), n, cout, sout, s)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
}

void do_dequantize(const int8_t *codes, const float *scales, int64_t n, int32_t block, void *out, hipStream_t s)
{
#define CALL(BB) launch_dequantize<BB>(codes, scales, n, static_cast<uint16_t *>(out), s)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
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

void do_quantize_strided(const void *x, int64_t n, int32_t chunks, int8_t *codes, float *scales, hipStream_t s)
{
#define CALL(RR) \
    launch(quantize_strided_kernel<RR>, strided_grid(n, chunks), s, static_cast<const uint16_t *>(x), codes, scales)
    EQUARX_DISPATCH_CHUNKS(chunks, CALL)
#undef CALL
}

void do_hop_strided(const int8_t *cin, const float *sin, const void *x, int64_t n, int32_t chunks, int8_t *cout,
                    float *sout, hipStream_t s)
{
#define CALL(RR) \
    launch(hop_strided_kernel<RR>, strided_grid(n, chunks), s, cin, sin, static_cast<const uint16_t *>(x), cout, sout)
    EQUARX_DISPATCH_CHUNKS(chunks, CALL)
#undef CALL
}

void do_dequantize_strided(const int8_t *codes, const float *scales, int64_t n, int32_t chunks, void *out,
                           hipStream_t s)
{
    launch(dequantize_strided_kernel<kTilesDequantize>, grid_for(n, kTilesDequantize), s, codes, scales, n, (int)chunks,
           static_cast<uint16_t *>(out));
}

inline int check_shape(int64_t n, int32_t block)
{
    if (!block_ok(block)) return EQUARX_BAD_BLOCK;
    if (n < 0 || too_long(n)) return EQUARX_BAD_SHAPE;
    return EQUARX_OK;
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
        case EQUARX_WORKSPACE_TOO_SMALL: return "workspace is smaller than equarx_workspace_bytes()";
        case EQUARX_DEVICE_ERROR: return "the HIP runtime reported an error at kernel launch";
        default: return "unknown status";
    }
}

int equarx_quantize(const void *x_bf16, int64_t n, int32_t block, int8_t *codes, float *scales, void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (n == 0) return EQUARX_OK;
    if (!x_bf16 || !codes || !scales) return EQUARX_NULL_POINTER;
    if (misaligned(x_bf16, kAlign) || misaligned(codes, kAlign) || misaligned(scales, kAlign)) return EQUARX_MISALIGNED;
    do_quantize(x_bf16, n, block, codes, scales, static_cast<hipStream_t>(stream));
    return launch_status();
}

int equarx_quantize_batch(const void *const *x_bf16, int8_t *const *codes, float *const *scales, int32_t count,
                          int64_t n, int32_t block, void *stream)
{
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
    for (int32_t i = 0; i < count; ++i) {
        if (!x_bf16[i] || !codes[i] || !scales[i]) return EQUARX_NULL_POINTER;
        if (misaligned(x_bf16[i], kAlign) || misaligned(codes[i], kAlign) || misaligned(scales[i], kAlign))
            return EQUARX_MISALIGNED;
        for (int32_t j = 0; j < i; ++j) {
            if (codes[i] == codes[j] || scales[i] == scales[j]) return EQUARX_BAD_SHAPE;      // two tensors, one output
        }
        tab.x[i] = static_cast<const uint16_t *>(x_bf16[i]);
        tab.codes[i] = codes[i];
        tab.scales[i] = scales[i];
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
#define CALL(BB)                                                                                                     \
    launch2d(quantize_batch_kernel<BB, kTilesQuantize>, grid_for(n, kTilesQuantize), (unsigned)count, hs, tab, n, \
             blocks_of(n, BB))
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return launch_status();
}

int equarx_dequantize(const int8_t *codes, const float *scales, int64_t n, int32_t block, void *out_bf16,
                      void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (n == 0) return EQUARX_OK;
    if (!codes || !scales || !out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(codes, kAlign) || misaligned(scales, kAlign) || misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    do_dequantize(codes, scales, n, block, out_bf16, static_cast<hipStream_t>(stream));
    return launch_status();
}

int equarx_reduce_stage(const int8_t *codes_in, const float *scales_in, const void *local_bf16, int64_t n,
                        int32_t block, int8_t *codes_out, float *scales_out, void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (n == 0) return EQUARX_OK;
    if (!codes_in || !scales_in || !local_bf16 || !codes_out || !scales_out) return EQUARX_NULL_POINTER;
    if (misaligned(codes_in, kAlign) || misaligned(scales_in, kAlign) || misaligned(local_bf16, kAlign) ||
        misaligned(codes_out, kAlign) || misaligned(scales_out, kAlign))
        return EQUARX_MISALIGNED;
    do_hop(codes_in, scales_in, local_bf16, n, block, codes_out, scales_out, static_cast<hipStream_t>(stream));
    return launch_status();
}

int equarx_reduce_quantized(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, void *out_bf16,
                            void *workspace, size_t workspace_bytes, int8_t *wire_codes, float *wire_scales,
                            void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if ((wire_codes == nullptr) != (wire_scales == nullptr)) return EQUARX_NULL_POINTER;
    const bool keep_wire = wire_codes != nullptr;
    if (!keep_wire && !workspace) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    if (int st = check_partials(partials_bf16, P, n, out_bf16)) return st;
    const int64_t nb = blocks_of(n, block);
    int8_t *c[2];
    float *s[2];
    int64_t c_step = 0, s_step = 0;     // distance between successive wire rows when they are kept
    if (keep_wire) {
        if (misaligned(wire_codes, kAlign) || misaligned(wire_scales, kAlign)) return EQUARX_MISALIGNED;
        c_step = equarx_wire_row_codes(n);
        s_step = equarx_wire_row_scales(n, block);
        c[0] = wire_codes;
        s[0] = wire_scales;
        c[1] = nullptr;
        s[1] = nullptr;
    } else {
        if (misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
        if (workspace_bytes < equarx_workspace_bytes(P, n, block)) return EQUARX_WORKSPACE_TOO_SMALL;
        const size_t codes = round_up((size_t)n, kWorkspaceAlign);
        const size_t scales = round_up((size_t)nb * sizeof(float), kWorkspaceAlign);
        char *w = static_cast<char *>(workspace);
        c[0] = reinterpret_cast<int8_t *>(w);
        s[0] = reinterpret_cast<float *>(w + codes);
        c[1] = reinterpret_cast<int8_t *>(w + codes + scales);
        s[1] = reinterpret_cast<float *>(w + 2 * codes + scales);
    }

    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int8_t *c_prev = c[0];
    const float *s_prev = s[0];
    do_quantize(partials_bf16[0], n, block, c[0], s[0], hs);
    for (int32_t i = 1; i < P; ++i) {
        int8_t *c_next = keep_wire ? wire_codes + i * c_step : c[i & 1];
        float *s_next = keep_wire ? wire_scales + i * s_step : s[i & 1];
        do_hop(c_prev, s_prev, partials_bf16[i], n, block, c_next, s_next, hs);
        c_prev = c_next;
        s_prev = s_next;
    }
    do_dequantize(c_prev, s_prev, n, block, out_bf16, hs);
    return launch_status();
}

int equarx_reduce_quantized_fused_ends(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                                       void *out_bf16, void *workspace, size_t workspace_bytes, void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    PartialTable tab;
    if (int st = fill_table(partials_bf16, P, n, out_bf16, tab)) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    uint16_t *out = static_cast<uint16_t *>(out_bf16);
    if (P <= 2) {       // both ends meet: the chain is one launch and needs no wire
#define CALL(BB) launch_chain<BB>(tab, P, n, true, true, false, out, nullptr, nullptr, 0, 0, hs)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
        return launch_status();
    }
    if (!workspace) return EQUARX_NULL_POINTER;
    if (misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
    if (workspace_bytes < equarx_workspace_bytes(P, n, block)) return EQUARX_WORKSPACE_TOO_SMALL;
    const int64_t nb = blocks_of(n, block);
    const size_t codes = round_up((size_t)n, kWorkspaceAlign);
    const size_t scales = round_up((size_t)nb * sizeof(float), kWorkspaceAlign);
    char *w = static_cast<char *>(workspace);
    int8_t *const c[2] = {reinterpret_cast<int8_t *>(w), reinterpret_cast<int8_t *>(w + codes + scales)};
    float *const s[2] = {reinterpret_cast<float *>(w + codes), reinterpret_cast<float *>(w + 2 * codes + scales)};
#define CALL(BB) launch_fused_ends<BB>(tab, P, n, c, s, out, hs)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return launch_status();
}

int equarx_reduce_fused(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, void *out_bf16,
                        int8_t *wire_codes, float *wire_scales, void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if ((wire_codes == nullptr) != (wire_scales == nullptr)) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    if (wire_codes && (misaligned(wire_codes, kAlign) || misaligned(wire_scales, kAlign))) return EQUARX_MISALIGNED;
    PartialTable tab;
    if (int st = fill_table(partials_bf16, P, n, out_bf16, tab)) return st;
    const int64_t c_step = equarx_wire_row_codes(n);
    const int64_t s_step = equarx_wire_row_scales(n, block);
    hipStream_t hs = static_cast<hipStream_t>(stream);
#define CALL(BB)                                                                                               \
    launch_chain<BB>(tab, P, n, true, true, false, static_cast<uint16_t *>(out_bf16), wire_codes, wire_scales, \
                     c_step, s_step, hs)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return launch_status();
}

int equarx_reduce_variant(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, uint32_t flags,
                          void *out_bf16, void *stream)
{
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
    if (int st = fill_table(partials_bf16, P, n, out_bf16, tab)) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    uint16_t *out = static_cast<uint16_t *>(out_bf16);
    if (semi) {
#define CALL(BB) launch_semi<BB>(tab, P, n, ag, ring, out, hs)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    } else {
#define CALL(BB) launch_chain<BB>(tab, P, n, rs, ag, ring, out, nullptr, nullptr, 0, 0, hs)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    }
    return launch_status();
}

size_t equarx_variant_workspace_bytes(uint32_t flags, int32_t P, int64_t n, int32_t block)
{
    const size_t two = equarx_workspace_bytes(P, n, block);
    return (flags & EQUARX_SEMI_LOOP) ? two / 2 * 3 : two;      // the semi-loop keeps one chain's wire while the other runs
}

int equarx_reduce_variant_hops(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, uint32_t flags,
                               void *out_bf16, void *workspace, size_t workspace_bytes, void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (flags & ~(uint32_t)(EQUARX_SEMI_LOOP | EQUARX_AG_UNQUANTIZED | EQUARX_RING_ORDER)) return EQUARX_BAD_SHAPE;
    const bool semi = flags & EQUARX_SEMI_LOOP, ag = !(flags & EQUARX_AG_UNQUANTIZED);
    const bool ring = flags & EQUARX_RING_ORDER;
    if (semi && ring) return EQUARX_BAD_SHAPE;      // the per-shard semi-loop exists as a single launch only
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16 || !workspace) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign) || misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
    if (workspace_bytes < equarx_variant_workspace_bytes(flags, P, n, block)) return EQUARX_WORKSPACE_TOO_SMALL;
    PartialTable tab;
    if (int st = fill_table(partials_bf16, P, n, out_bf16, tab)) return st;

    const int64_t nb = blocks_of(n, block);
    const size_t codes = round_up((size_t)n, kWorkspaceAlign);
    const size_t scales = round_up((size_t)nb * sizeof(float), kWorkspaceAlign);
    char *w = static_cast<char *>(workspace);
    int8_t *c[3];
    float *s[3];
    for (int i = 0; i < 3; ++i) {       // the third pair exists only in the semi-loop's larger workspace
        c[i] = reinterpret_cast<int8_t *>(w + (size_t)i * (codes + scales));
        s[i] = reinterpret_cast<float *>(w + (size_t)i * (codes + scales) + codes);
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    uint16_t *out = static_cast<uint16_t *>(out_bf16);

    if (!semi) {
        if (P == 1) {       // no hop: one launch quantizes/dequantizes (or copies) partial 0
#define CALL(BB) launch_chain<BB>(tab, P, n, true, ag, ring, out, nullptr, nullptr, 0, 0, hs)
            EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
            return launch_status();
        }
        if (ring) {         // every launch is one ring step on all P shards: grid row k takes device k+1+step's partial
#define CALL(BB) launch_ring_hops<BB>(tab, P, n, ag, c, s, out, hs)
            EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
            return launch_status();
        }
        // Q_B(x_0), hops 1 .. P-2, then the last hop with or without the all-gather's quantize/dequantize pair
        do_quantize(tab.x[0], n, block, c[0], s[0], hs);
        for (int32_t i = 1; i + 1 < P; ++i) do_hop(c[(i - 1) & 1], s[(i - 1) & 1], tab.x[i], n, block, c[i & 1], s[i & 1], hs);
#define CALL(BB) launch_tail<BB>(c[(P - 2) & 1], s[(P - 2) & 1], tab.x[P - 1], n, out, hs, ag)
        EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
        return launch_status();
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
        do_quantize(tab.x[h + 1], n, block, c[0], s[0], hs);
        for (int32_t k = 1; k < na; ++k) do_hop(c[(k - 1) & 1], s[(k - 1) & 1], tab.x[h + 1 + k], n, block, c[k & 1], s[k & 1], hs);
        last_a = (na - 1) & 1;
        wires.codes[received] = c[last_a];
        wires.scales[received] = s[last_a];
        ++received;
    }
    if (nbk > 0) {
        const int u[2] = {last_a == 0 ? 1 : 0, 2};      // two buffers that do not hold the first chain's wire
        do_quantize(tab.x[h], n, block, c[u[0]], s[u[0]], hs);
        for (int32_t k = 1; k < nbk; ++k) {
            do_hop(c[u[(k - 1) & 1]], s[u[(k - 1) & 1]], tab.x[h - k], n, block, c[u[k & 1]], s[u[k & 1]], hs);
        }
        wires.codes[received] = c[u[(nbk - 1) & 1]];
        wires.scales[received] = s[u[(nbk - 1) & 1]];
        ++received;
    }
#define CALL(BB) launch_flat<BB>(tab.x[0], wires, received, n, out, nullptr, nullptr, hs, ag)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return launch_status();
}

int equarx_reduce_flat(const void *local_bf16, const int8_t *const *codes, const float *const *scales, int32_t R,
                       int64_t n, int32_t block, void *out_bf16, int8_t *codes_out, float *scales_out, void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (R < 0 || R >= EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (R > 0 && (!codes || !scales)) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!local_bf16) return EQUARX_NULL_POINTER;
    if ((codes_out == nullptr) != (scales_out == nullptr)) return EQUARX_NULL_POINTER;
    if (!out_bf16 && !codes_out) return EQUARX_NULL_POINTER;                    // nothing to write
    if (misaligned(local_bf16, kAlign) || (out_bf16 && misaligned(out_bf16, kAlign))) return EQUARX_MISALIGNED;
    if (codes_out && (misaligned(codes_out, kAlign) || misaligned(scales_out, kAlign))) return EQUARX_MISALIGNED;
    if (out_bf16 == local_bf16) return EQUARX_BAD_SHAPE;
    WireTable tab;
    for (int32_t r = 0; r < kMaxPartials; ++r) {
        tab.codes[r] = nullptr;
        tab.scales[r] = nullptr;
    }
    for (int32_t r = 0; r < R; ++r) {
        if (!codes[r] || !scales[r]) return EQUARX_NULL_POINTER;
        if (misaligned(codes[r], kAlign) || misaligned(scales[r], kAlign)) return EQUARX_MISALIGNED;
        if (codes[r] == codes_out || scales[r] == scales_out) return EQUARX_BAD_SHAPE;
        tab.codes[r] = codes[r];
        tab.scales[r] = scales[r];
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
#define CALL(BB)                                                                                                  \
    launch_flat<BB>(static_cast<const uint16_t *>(local_bf16), tab, R, n, static_cast<uint16_t *>(out_bf16), codes_out, \
                    scales_out, hs)
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return launch_status();
}

int equarx_quantize_strided(const void *x_bf16, int64_t n, int32_t chunks, int8_t *codes, float *scales, void *stream)
{
    if (int st = check_strided(n, chunks)) return st;
    if (n == 0) return EQUARX_OK;
    if (!x_bf16 || !codes || !scales) return EQUARX_NULL_POINTER;
    if (misaligned(x_bf16, kAlign) || misaligned(codes, kAlign) || misaligned(scales, kAlign)) return EQUARX_MISALIGNED;
    do_quantize_strided(x_bf16, n, chunks, codes, scales, static_cast<hipStream_t>(stream));
    return launch_status();
}

int equarx_dequantize_strided(const int8_t *codes, const float *scales, int64_t n, int32_t chunks, void *out_bf16,
                              void *stream)
{
    if (int st = check_strided(n, chunks)) return st;
    if (n == 0) return EQUARX_OK;
    if (!codes || !scales || !out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(codes, kAlign) || misaligned(scales, kAlign) || misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    do_dequantize_strided(codes, scales, n, chunks, out_bf16, static_cast<hipStream_t>(stream));
    return launch_status();
}

int equarx_reduce_stage_strided(const int8_t *codes_in, const float *scales_in, const void *local_bf16, int64_t n,
                                int32_t chunks, int8_t *codes_out, float *scales_out, void *stream)
{
    if (int st = check_strided(n, chunks)) return st;
    if (n == 0) return EQUARX_OK;
    if (!codes_in || !scales_in || !local_bf16 || !codes_out || !scales_out) return EQUARX_NULL_POINTER;
    if (misaligned(codes_in, kAlign) || misaligned(scales_in, kAlign) || misaligned(local_bf16, kAlign) ||
        misaligned(codes_out, kAlign) || misaligned(scales_out, kAlign))
        return EQUARX_MISALIGNED;
    do_hop_strided(codes_in, scales_in, local_bf16, n, chunks, codes_out, scales_out, static_cast<hipStream_t>(stream));
    return launch_status();
}

int equarx_reduce_quantized_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks,
                                    void *out_bf16, void *workspace, size_t workspace_bytes, void *stream)
{
    if (int st = check_strided(n, chunks)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16 || !workspace) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign) || misaligned(workspace, kWorkspaceAlign)) return EQUARX_MISALIGNED;
    if (int st = check_partials(partials_bf16, P, n, out_bf16)) return st;
    // one scale per `chunks` elements: the same workspace as the contiguous chain with block = chunks
    if (workspace_bytes < equarx_workspace_bytes(P, n, chunks)) return EQUARX_WORKSPACE_TOO_SMALL;
    const size_t codes = round_up((size_t)n, kWorkspaceAlign);
    const size_t scales = round_up((size_t)(n / chunks) * sizeof(float), kWorkspaceAlign);
    char *w = static_cast<char *>(workspace);
    int8_t *const c[2] = {reinterpret_cast<int8_t *>(w), reinterpret_cast<int8_t *>(w + codes + scales)};
    float *const s[2] = {reinterpret_cast<float *>(w + codes), reinterpret_cast<float *>(w + 2 * codes + scales)};
    hipStream_t hs = static_cast<hipStream_t>(stream);
    do_quantize_strided(partials_bf16[0], n, chunks, c[0], s[0], hs);
    for (int32_t i = 1; i < P; ++i) {
        do_hop_strided(c[(i - 1) & 1], s[(i - 1) & 1], partials_bf16[i], n, chunks, c[i & 1], s[i & 1], hs);
    }
    do_dequantize_strided(c[(P - 1) & 1], s[(P - 1) & 1], n, chunks, out_bf16, hs);
    return launch_status();
}

int equarx_reduce_fused_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks, void *out_bf16,
                                void *stream)
{
    if (int st = check_strided(n, chunks)) return st;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!out_bf16) return EQUARX_NULL_POINTER;
    if (misaligned(out_bf16, kAlign)) return EQUARX_MISALIGNED;
    PartialTable tab;
    if (int st = fill_table(partials_bf16, P, n, out_bf16, tab)) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
#define CALL(RR) launch(chain_strided_kernel<RR>, strided_grid(n, chunks), hs, tab, P, static_cast<uint16_t *>(out_bf16))
    EQUARX_DISPATCH_CHUNKS(chunks, CALL)
#undef CALL
    return launch_status();
}

int equarx_calib_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (bytes == 0) return EQUARX_OK;
    if (!src || !dst) return EQUARX_NULL_POINTER;
    if (bytes % 16 != 0) return EQUARX_BAD_SHAPE;
    if (misaligned(src, kAlign) || misaligned(dst, kAlign)) return EQUARX_MISALIGNED;
    const int64_t nvec = (int64_t)(bytes / 16);
    const int64_t per_wg = kThreads * 4;
    launch(copy_kernel, (unsigned)((nvec + per_wg - 1) / per_wg), static_cast<hipStream_t>(stream),
           static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), nvec);
    return launch_status();
}

int equarx_calib_hop_traffic(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, int8_t *codes0,
                             float *scales0, int8_t *codes1, float *scales1, void *stream)
{
    if (int st = check_shape(n, block)) return st;
    if (n % block != 0) return EQUARX_BAD_SHAPE;
    if (P < 1 || P > EQUARX_MAX_PARTIALS) return EQUARX_BAD_SHAPE;
    if (!partials_bf16) return EQUARX_NULL_POINTER;
    if (n == 0) return EQUARX_OK;
    if (!codes0 || !scales0 || !codes1 || !scales1) return EQUARX_NULL_POINTER;
    if (misaligned(codes0, kAlign) || misaligned(scales0, kAlign) || misaligned(codes1, kAlign) ||
        misaligned(scales1, kAlign))
        return EQUARX_MISALIGNED;
    if (codes0 == codes1 || scales0 == scales1) return EQUARX_BAD_SHAPE;
    PartialTable tab;
    if (int st = fill_table(partials_bf16, P, n, nullptr, tab)) return st;
    const int64_t lanes = n / kLaneElems;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    u32x2 *c[2] = {reinterpret_cast<u32x2 *>(codes0), reinterpret_cast<u32x2 *>(codes1)};
    float *s[2] = {scales0, scales1};
#define CALL(BB)                                                                                      \
    for (int32_t i = 1; i < P; ++i) {                                                                 \
        launch(hop_traffic_kernel<BB, kTilesHop>, grid_for(n, kTilesHop), hs,                         \
               reinterpret_cast<const u32x4 *>(tab.x[i]), c[(i - 1) & 1], s[(i - 1) & 1], lanes, c[i & 1], s[i & 1]); \
    }
    EQUARX_DISPATCH_BLOCK(block, CALL)
#undef CALL
    return launch_status();
}

int equarx_selftest_quotients(uint32_t first_bits, uint64_t count, uint64_t *mismatches, void *stream)
{
    if (count == 0) return EQUARX_OK;
    if (!mismatches) return EQUARX_NULL_POINTER;
    if (misaligned(mismatches, 8)) return EQUARX_MISALIGNED;
    if ((uint64_t)first_bits + count > 0x7F800000ull) return EQUARX_BAD_SHAPE;     // positive finite patterns only
    const uint64_t wgs = (count + kThreads - 1) / kThreads;
    launch(selftest_quotients_kernel, (unsigned)(wgs < 16384 ? wgs : 16384), static_cast<hipStream_t>(stream),
           first_bits, count, reinterpret_cast<unsigned long long *>(mismatches));
    return launch_status();
}

int equarx_selftest_rounding(uint32_t first_bits, uint64_t count, uint64_t *mismatches, void *stream)
{
    if (count == 0) return EQUARX_OK;
    if (!mismatches) return EQUARX_NULL_POINTER;
    if (misaligned(mismatches, 8)) return EQUARX_MISALIGNED;
    if ((uint64_t)first_bits + count > 0x43000000ull) return EQUARX_BAD_SHAPE;     // |p| < 128 only
    const uint64_t wgs = (count + kThreads - 1) / kThreads;
    launch(selftest_rounding_kernel, (unsigned)(wgs < 16384 ? wgs : 16384), static_cast<hipStream_t>(stream),
           first_bits, count, reinterpret_cast<unsigned long long *>(mismatches));
    return launch_status();
}

int equarx_eval_quotients(const float *absmax, int64_t n, float *scale, float *inv, void *stream)
{
    if (n < 0 || n > ((int64_t)1 << 31)) return EQUARX_BAD_SHAPE;
    if (n == 0) return EQUARX_OK;
    if (!absmax || !scale || !inv) return EQUARX_NULL_POINTER;
    if (misaligned(absmax, 4) || misaligned(scale, 4) || misaligned(inv, 4)) return EQUARX_MISALIGNED;
    launch(eval_quotients_kernel, (unsigned)((n + kThreads - 1) / kThreads), static_cast<hipStream_t>(stream), absmax, n,
           scale, inv);
    return launch_status();
}

void equarx_time_next_launch(void *start_event, void *stop_event)
{
    t_start_event = static_cast<hipEvent_t>(start_event);
    t_stop_event = static_cast<hipEvent_t>(stop_event);
}

void equarx_time_launch_span(int32_t first, int32_t last, void *start_event, void *stop_event)
{
    if (first < 0 || last < first || !start_event || !stop_event) {
        t_span_start = nullptr;
        t_span_stop = nullptr;
        return;
    }
    t_span_first = first;
    t_span_last = last;
    t_span_start = static_cast<hipEvent_t>(start_event);
    t_span_stop = static_cast<hipEvent_t>(stop_event);
}

}  // extern "C"
