// Device code of libequarx: gfx950 (CDNA4, wave64) kernels for the block-wise
// int8 quantized reduction of EQuARX (arXiv 2506.17615, Sec. 3.1-3.4).
//
// Work decomposition shared by all kernels
//   lane   : owns 8 consecutive elements of a tile (one 16-byte bf16 load, one
//            8-byte code load/store), so it sees the same elements in both
//            streams;
//   group  : the G = B/8 consecutive lanes that cover one quantization block
//            (G = 4 .. 64, always inside one wavefront), reduced with DPP row
//            operations and the gfx950 row-swap permutes;
//   wave   : 512 consecutive elements per tile;
//   block of 256 threads : 2048 consecutive elements per tile, K tiles per
//            thread in flight, tile k of a workgroup starting 2048*k further.
// Every load instruction of a workgroup therefore reads one contiguous 4 KiB
// (bf16) or 2 KiB (codes) span.  Elements past n read as zero -- a zero never
// changes a block's max-abs, so a ragged last block needs no special
// arithmetic -- and are not stored.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace equarx {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte access
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));   // one 8-byte access

// Build-time tuning knobs (defaults are what the library ships with).
#ifndef EQUARX_THREADS
#define EQUARX_THREADS 256          // threads per workgroup
#endif
#ifndef EQUARX_NT_LOAD_BF16
#define EQUARX_NT_LOAD_BF16 1       // bf16 inputs are read once: non-temporal loads
#endif
#ifndef EQUARX_NT_STORE_BF16
#define EQUARX_NT_STORE_BF16 1      // the bf16 output is not read again by this library
#endif
#ifndef EQUARX_CHAIN_PAIRED
#define EQUARX_CHAIN_PAIRED 1       // single-launch chain, blocks >= 128: two pieces of one block per lane
#endif
#ifndef EQUARX_SCHED_BARRIER
#define EQUARX_SCHED_BARRIER 1      // keep every load of a thread ahead of its arithmetic
#endif
constexpr int kLaneElems = 8;
constexpr int kThreads = EQUARX_THREADS;
constexpr int kTileElems = kThreads * kLaneElems;   // 2048 elements per workgroup tile

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

// Workgroups of a launch whose workgroups take `tiles` tiles each.
inline unsigned grid_for(int64_t n, int tiles)
{
    const int64_t per_wg = (int64_t)kTileElems * tiles;
    return (unsigned)((n + per_wg - 1) / per_wg);
}


// Smallest max-abs that still gets a non-zero scale: 127 * 2^-126, so that
// scale = absmax/127 stays a normal number and 127/absmax stays finite.
constexpr float kTinyAbsmax = 127.0f * 1.17549435e-38f;

// ---------------------------------------------------------------- lane exchange

template <int kCtrl>
__device__ __forceinline__ uint32_t dpp_read(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kCtrl, 0xf, 0xf, false);
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// Max over the G lanes of a group, result in every lane of the group.  The
// operand is the bit pattern of a non-negative float, for which unsigned
// integer order equals float order.  All 64 lanes of the wave must be active.
template <int G>
__device__ __forceinline__ uint32_t group_max_bits(uint32_t m)
{
    static_assert(G == 4 || G == 8 || G == 16 || G == 32 || G == 64, "group width");
    m = umax(m, dpp_read<0xB1>(m));                 // quad_perm:[1,0,3,2]  lane ^ 1
    m = umax(m, dpp_read<0x4E>(m));                 // quad_perm:[2,3,0,1]  lane ^ 2
    if (G >= 8) m = umax(m, dpp_read<0x141>(m));    // row_half_mirror      the other quad of 8
    if (G >= 16) m = umax(m, dpp_read<0x140>(m));   // row_mirror           the other half of 16
    if (G >= 32) {                                  // rows 0<->1 and 2<->3 trade places
        auto r = __builtin_amdgcn_permlane16_swap(m, m, false, false);
        m = umax(r[0], r[1]);
    }
    if (G >= 64) {                                  // lower and upper 32 lanes trade places
        auto r = __builtin_amdgcn_permlane32_swap(m, m, false, false);
        m = umax(r[0], r[1]);
    }
    return m;
}

// ---------------------------------------------------------------- element codecs

__device__ __forceinline__ void widen_bf16x8(const u32x4 &w, float (&f)[8])
{
    const uint32_t d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(d[i] << 16);
        f[2 * i + 1] = __uint_as_float(d[i] & 0xFFFF0000u);
    }
}

__device__ __forceinline__ void widen_i8x8(const u32x2 &w, float (&f)[8])
{
    const uint32_t d[2] = {w.x, w.y};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            f[4 * i + b] = (float)(int)(int8_t)(d[i] >> (8 * b));
        }
    }
}

__device__ __forceinline__ uint32_t narrow_bf16x2(float lo, float hi)
{
    // gfx950 converts in hardware (round to nearest, ties to even)
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    floatx2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

// ---------------------------------------------------------------- guarded tile I/O
// `full` is a compile-time constant at every call: the whole tile lies inside [0, n).

__device__ __forceinline__ u32x4 load_bf16x8(const uint16_t *p, int64_t at, int64_t n, bool full)
{
    if (full || at + kLaneElems <= n) {
        const u32x4 *v = reinterpret_cast<const u32x4 *>(p + at);
        return EQUARX_NT_LOAD_BF16 ? __builtin_nontemporal_load(v) : *v;
    }
    uint16_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = (at + i < n) ? p[at + i] : (uint16_t)0;
    u32x4 w;
    w.x = e[0] | ((uint32_t)e[1] << 16);
    w.y = e[2] | ((uint32_t)e[3] << 16);
    w.z = e[4] | ((uint32_t)e[5] << 16);
    w.w = e[6] | ((uint32_t)e[7] << 16);
    return w;
}

// Wire accesses come in two flavours.  kStream = false: ordinary cached accesses, for a wire that the next launch
// on this device reads back (the single-device chain: the 256 MB Infinity Cache still holds it).  kStream = true:
// non-temporal accesses, for a wire that arrives from and leaves for somewhere else, as in a ring step between
// devices: it is read once and what is written is not read here again.  Measured on MI355X at the 27B shape: with
// every wire cold, streaming accesses make a hop 15.8 us instead of 17.3 us; with a warm wire they make it 16.0 us
// instead of 14.7 us, because the next launch then misses the cache.
template <bool kStream = false>
__device__ __forceinline__ u32x2 load_i8x8(const int8_t *p, int64_t at, int64_t n, bool full)
{
    if (full || at + kLaneElems <= n) {
        const u32x2 *v = reinterpret_cast<const u32x2 *>(p + at);
        return kStream ? __builtin_nontemporal_load(v) : *v;
    }
    uint32_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = (at + i < n) ? (uint32_t)(uint8_t)p[at + i] : 0u;
    u32x2 w;
    w.x = e[0] | (e[1] << 8) | (e[2] << 16) | (e[3] << 24);
    w.y = e[4] | (e[5] << 8) | (e[6] << 16) | (e[7] << 24);
    return w;
}

template <bool kStream = false>
__device__ __forceinline__ void store_i8x8(int8_t *p, int64_t at, int64_t n, bool full, const u32x2 &w)
{
    if (full || at + kLaneElems <= n) {
        u32x2 *v = reinterpret_cast<u32x2 *>(p + at);
        if (kStream) {
            __builtin_nontemporal_store(w, v);
        } else {
            *v = w;
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (at + i < n) p[at + i] = (int8_t)(((i < 4 ? w.x : w.y) >> (8 * (i & 3))) & 0xFF);
    }
}

__device__ __forceinline__ void store_bf16x8(uint16_t *p, int64_t at, int64_t n, bool full, const u32x4 &w)
{
    if (full || at + kLaneElems <= n) {
        u32x4 *v = reinterpret_cast<u32x4 *>(p + at);
        if (EQUARX_NT_STORE_BF16) {
            __builtin_nontemporal_store(w, v);
        } else {
            *v = w;
        }
        return;
    }
    const uint32_t d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (at + i < n) p[at + i] = (uint16_t)(d[i >> 1] >> (16 * (i & 1)));
    }
}

// With all K tiles of a thread in one basic block the instruction scheduler
// would sink some loads between the arithmetic of earlier tiles to save
// registers; the kernels want every request in flight before the first wait.
__device__ __forceinline__ void loads_first()
{
#if EQUARX_SCHED_BARRIER
    __builtin_amdgcn_sched_barrier(0);
#endif
}

// ---------------------------------------------------------------- the two quotients of a block

// 127 / a is taken through the hardware reciprocal of a below this bound; from
// 2^126 on, 1/a is subnormal and the reciprocal is no longer accurate enough,
// so a/16 is used there.
constexpr float kRcpSafeBelow = 8.507059173e37f;    // 2^126

// scale = fl32(a / 127) and inv = fl32(127 / a), both CORRECTLY ROUNDED, for a
// block whose max-abs is a (scale = inv = 0 below the tiny threshold).
//
// The compiler's IEEE division costs about 11 instructions per quotient and
// every lane of a group computes both, which is a third of the hop's ALU work.
// These shorter sequences give the same bits:
//   a / 127 : q0 = a*c with c = fl32(1/127), then one exact-remainder
//             correction (the divisor is a constant whose reciprocal is known
//             to half an ulp);
//   127 / a : q0 = 127*rcp(a), then the same correction with the 1-ulp
//             hardware reciprocal.
// That they equal the IEEE quotient is not argued but CHECKED, exhaustively,
// over every finite fp32 a >= 127*2^-126 -- selftest_quotients_kernel below,
// run by the GPU tests.
__device__ __forceinline__ void block_quotients(float a, float &scale, float &inv)
{
    // Straight-line code (selects, no branches): the K tiles of a thread then
    // form one basic block and the compiler interleaves their dependent chains.
    const float c = 1.0f / 127.0f;                      // folded at compile time: fl32(1/127)
    const float q0 = a * c;
    const float e = __builtin_fmaf(-127.0f, q0, a);     // exact remainder a - 127*q0
    const float s = __builtin_fmaf(e, c, q0);
    // From 2^126 on, 1/a is subnormal: divide a/16 instead and scale the
    // quotient by 1/16, both exact (127/a >= 127*2^-128 is still normal).
    const float f = a < kRcpSafeBelow ? 1.0f : 0.0625f;
    const float af = a * f;
    const float y = __builtin_amdgcn_rcpf(af);
    const float p0 = 127.0f * y;
    const float r = __builtin_fmaf(-af, p0, 127.0f);    // exact remainder 127 - af*p0
    const float v = __builtin_fmaf(r, y, p0) * f;
    const bool tiny = a < kTinyAbsmax;                  // what the lanes computed above (inf, NaN) is dropped
    scale = tiny ? 0.0f : s;
    inv = tiny ? 0.0f : v;
}

// Reference form of the same two quotients: the compiler's IEEE division.
__device__ __forceinline__ void block_quotients_ieee(float a, float &scale, float &inv)
{
    if (a < kTinyAbsmax) {
        scale = 0.0f;
        inv = 0.0f;
    } else {
        scale = a / 127.0f;
        inv = 127.0f / a;
    }
}

// ---------------------------------------------------------------- Q_B on registers

// Quantize the 8 values a lane holds, given that the G lanes of its group hold
// one block.  r[i] receives the code of t[i] as a float (an integer in
// [-127, 127]); `scale` is the block's scale (the same in every lane of the group).
//
// kPositiveZero: a code that rounds to zero from below is -0.0 as a float,
// where the int8 code converted back would be +0.0.  Kernels that keep the
// codes as floats and multiply them again set this flag, which adds +0.0
// (turning -0.0 into +0.0 and changing nothing else); the sign of a zero
// product would otherwise leak into a sum whose other term is -0.0.
template <int G, bool kPositiveZero = false>
__device__ __forceinline__ void quantize_lane_f(const float (&t)[8], float (&r)[8], float &scale)
{
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) m = __builtin_fmaxf(m, __builtin_fabsf(t[i]));
    const float a = __uint_as_float(group_max_bits<G>(__float_as_uint(m)));

    float inv;
    block_quotients(a, scale, inv);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // |t*inv| <= 127*(1+2^-23): rounds to at most 127, no clamp needed
        r[i] = __builtin_rintf(t[i] * inv);
        if (kPositiveZero) r[i] += 0.0f;
    }
}

// Adding 1.5 * 2^23 to a float p, |p| < 2^22, rounds p to the nearest integer
// (ties to even, the sum's ulp being 1 and the constant even) and leaves that
// integer, in two's complement, in the low mantissa bits of the sum: the int8
// code of p is the sum's low byte.  Two instructions (multiply, add) where
// round + convert + mask would be four.
constexpr float kRoundMagic = 12582912.0f;

// Byte 0 of each of four words, gathered into one word.
__device__ __forceinline__ uint32_t gather_low_bytes(uint32_t b0, uint32_t b1, uint32_t b2, uint32_t b3)
{
    // v_perm_b32: selector 0..3 = byte of the second operand, 4..7 = byte of the first, 0x0c = zero
    const uint32_t lo = __builtin_amdgcn_perm(b1, b0, 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(b3, b2, 0x04000c0cu);
    return lo | hi;
}

// The 8 float-valued codes of a lane (integers in [-127, 127]) as packed int8.
__device__ __forceinline__ u32x2 pack_codes(const float (&r)[8])
{
    uint32_t b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) b[i] = __float_as_uint(r[i] + kRoundMagic);     // exact: r[i] is an integer
    u32x2 w;
    w.x = gather_low_bytes(b[0], b[1], b[2], b[3]);
    w.y = gather_low_bytes(b[4], b[5], b[6], b[7]);
    return w;
}

// Q_B of the 8 values of a lane, as packed int8 codes (same codes as
// quantize_lane_f followed by pack_codes).
template <int G>
__device__ __forceinline__ u32x2 quantize_lane(const float (&t)[8], float &scale)
{
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) m = __builtin_fmaxf(m, __builtin_fabsf(t[i]));
    const float a = __uint_as_float(group_max_bits<G>(__float_as_uint(m)));
    float inv;
    block_quotients(a, scale, inv);
    uint32_t b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) b[i] = __float_as_uint(t[i] * inv + kRoundMagic);   // two roundings: product, then sum
    u32x2 w;
    w.x = gather_low_bytes(b[0], b[1], b[2], b[3]);
    w.y = gather_low_bytes(b[4], b[5], b[6], b[7]);
    return w;
}

// ---------------------------------------------------------------- kernels
// Each kernel body exists twice: kFull = true for workgroups whose K tiles lie
// entirely inside [0, n) (straight-line vector code), kFull = false for the one
// workgroup that holds the ragged end (every access guarded).

// The K scales a group leader holds, stored after all K tiles are computed: one
// conditional region at the end instead of one per tile, so the tiles'
// arithmetic stays in a single basic block.
template <int B, int K, bool kFull>
__device__ __forceinline__ void store_group_scales(float *scales, const float (&scale)[K], int64_t wg_at, int64_t nb)
{
    constexpr int G = B / kLaneElems;
    if ((threadIdx.x % G) == 0) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int64_t blk = (wg_at + k * kTileElems + threadIdx.x * kLaneElems) / B;
            if (kFull || blk < nb) scales[blk] = scale[k];
        }
    }
}

template <int B, int K, bool kFull, bool kStream = false>
__device__ __forceinline__ void quantize_body(const uint16_t *__restrict__ x, int64_t n, int8_t *__restrict__ codes,
                                              float *__restrict__ scales, int64_t nb, int64_t wg_at)
{
    constexpr int G = B / kLaneElems;
    const int lane_at = threadIdx.x * kLaneElems;

    u32x4 xv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) xv[k] = load_bf16x8(x, wg_at + k * kTileElems + lane_at, n, kFull);
    loads_first();

    float scale[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        float t[8];
        widen_bf16x8(xv[k], t);
        const u32x2 w = quantize_lane<G>(t, scale[k]);
        store_i8x8<kStream>(codes, at, n, kFull, w);
    }
    store_group_scales<B, K, kFull>(scales, scale, wg_at, nb);
}

// Pass 0 of the chain: quantize a bf16 tensor.
template <int B, int K, bool kStream = false>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const uint16_t *__restrict__ x, int64_t n,
                                                            int8_t *__restrict__ codes, float *__restrict__ scales,
                                                            int64_t nb)
{
    const int64_t wg_at = (int64_t)blockIdx.x * (kTileElems * K);
    if (wg_at + kTileElems * K <= n) {
        quantize_body<B, K, true, kStream>(x, n, codes, scales, nb, wg_at);
    } else {
        quantize_body<B, K, false, kStream>(x, n, codes, scales, nb, wg_at);
    }
}

// Several tensors of the same length in one launch (blockIdx.y picks the
// tensor): what a device does before an all-to-all, when it quantizes one shard
// per peer.  One launch instead of one per shard spares the per-launch ramp.
constexpr int kMaxBatch = 64;

struct QuantizeBatch {
    const uint16_t *x[kMaxBatch];
    int8_t *codes[kMaxBatch];
    float *scales[kMaxBatch];
};

template <int B, int K, bool kStream = false>
__global__ __launch_bounds__(kThreads) void quantize_batch_kernel(const QuantizeBatch tab, int64_t n, int64_t nb)
{
    const uint16_t *x = tab.x[blockIdx.y];
    int8_t *codes = tab.codes[blockIdx.y];
    float *scales = tab.scales[blockIdx.y];
    const int64_t wg_at = (int64_t)blockIdx.x * (kTileElems * K);
    if (wg_at + kTileElems * K <= n) {
        quantize_body<B, K, true, kStream>(x, n, codes, scales, nb, wg_at);
    } else {
        quantize_body<B, K, false, kStream>(x, n, codes, scales, nb, wg_at);
    }
}

template <int B, int K, bool kFull, bool kStream = false>
__device__ __forceinline__ void hop_body(const int8_t *cin, const float *sin, const uint16_t *__restrict__ x,
                                         int64_t n, int8_t *cout, float *sout, int64_t nb, int64_t wg_at)
{
    constexpr int G = B / kLaneElems;
    const int lane_at = threadIdx.x * kLaneElems;

    u32x4 xv[K];
    u32x2 cv[K];
    float sv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        xv[k] = load_bf16x8(x, at, n, kFull);
        cv[k] = load_i8x8<kStream>(cin, at, n, kFull);
        const int64_t blk = at / B;
        sv[k] = (kFull || blk < nb) ? sin[blk] : 0.0f;
    }
    loads_first();

    float scale[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        float xf[8], qf[8], t[8];
        widen_bf16x8(xv[k], xf);
        widen_i8x8(cv[k], qf);
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = __builtin_fmaf(qf[i], sv[k], xf[i]);
        const u32x2 w = quantize_lane<G>(t, scale[k]);
        store_i8x8<kStream>(cout, at, n, kFull, w);
    }
    store_group_scales<B, K, kFull>(sout, scale, wg_at, nb);
}

// One hop: dequantize the incoming wire, add the local bf16 shard in fp32
// (one fused multiply-add per element), quantize the partial sum.  The output
// wire may be the input wire: a thread reads its own elements, and a group its
// own scale, before either is written.
template <int B, int K, bool kStream = false>
__global__ __launch_bounds__(kThreads) void hop_kernel(const int8_t *cin, const float *sin,
                                                       const uint16_t *__restrict__ x, int64_t n,
                                                       int8_t *cout, float *sout, int64_t nb)
{
    const int64_t wg_at = (int64_t)blockIdx.x * (kTileElems * K);
    if (wg_at + kTileElems * K <= n) {
        hop_body<B, K, true, kStream>(cin, sin, x, n, cout, sout, nb, wg_at);
    } else {
        hop_body<B, K, false, kStream>(cin, sin, x, n, cout, sout, nb, wg_at);
    }
}

template <int B, int K, bool kFull, bool kStream = false>
__device__ __forceinline__ void dequantize_body(const int8_t *__restrict__ codes, const float *__restrict__ scales,
                                                int64_t n, uint16_t *__restrict__ out, int64_t nb, int64_t wg_at)
{
    const int lane_at = threadIdx.x * kLaneElems;

    u32x2 cv[K];
    float sv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        cv[k] = load_i8x8<kStream>(codes, at, n, kFull);
        const int64_t blk = at / B;
        sv[k] = (kFull || blk < nb) ? scales[blk] : 0.0f;
    }

#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        float qf[8];
        widen_i8x8(cv[k], qf);
        u32x4 w;
        w.x = narrow_bf16x2(qf[0] * sv[k], qf[1] * sv[k]);
        w.y = narrow_bf16x2(qf[2] * sv[k], qf[3] * sv[k]);
        w.z = narrow_bf16x2(qf[4] * sv[k], qf[5] * sv[k]);
        w.w = narrow_bf16x2(qf[6] * sv[k], qf[7] * sv[k]);
        store_bf16x8(out, at, n, kFull, w);
    }
}

// Last pass: dequantize the wire to bf16.
template <int B, int K, bool kStream = false>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const int8_t *__restrict__ codes,
                                                              const float *__restrict__ scales, int64_t n,
                                                              uint16_t *__restrict__ out, int64_t nb)
{
    const int64_t wg_at = (int64_t)blockIdx.x * (kTileElems * K);
    if (wg_at + kTileElems * K <= n) {
        dequantize_body<B, K, true, kStream>(codes, scales, n, out, nb, wg_at);
    } else {
        dequantize_body<B, K, false, kStream>(codes, scales, n, out, nb, wg_at);
    }
}

// ---------------------------------------------------------------- the whole chain in one launch
// Blocks never interact, so a workgroup can run all hops on its own tiles with
// the running sum held in registers: the same operations in the same order as
// the hop-by-hop passes, hence the same bits.  The partials are read once each
// (the next one's loads are issued before the current hop's arithmetic); the
// wire is written only if the caller keeps it (kWire) and is never read back.
//
// Template knobs (the stage selection of Sec. 3.4):
//   kRS  what a device forwards during the reduce-scatter is quantized
//        (otherwise the running sum stays fp32 and is added with plain adds);
//   kAG  the finished sum is quantized once more for the all-gather and
//        dequantized (otherwise it is narrowed to bf16 directly).
// Ring layout: with shard_elems > 0 the tensor is cut into gridDim.y shards of
// shard_elems elements (a multiple of B) and shard k is reduced in the rotated
// order rot+0, rot+1, ... (mod P) with rot = k + rot_bias.

constexpr int kMaxPartials = 64;

struct PartialTable {
    const uint16_t *x[kMaxPartials];
};

template <int K, bool kFull>
__device__ __forceinline__ void load_tiles(const uint16_t *p, int64_t wg_at, int64_t n, u32x4 (&v)[K])
{
    const int lane_at = threadIdx.x * kLaneElems;
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] = load_bf16x8(p, wg_at + k * kTileElems + lane_at, n, kFull);
}

// Writes what the wire carries after a quantization of one tile (8 codes per
// lane starting at element `at`): row `row` of the kept wire.
template <int B, bool kFull>
__device__ __forceinline__ void store_wire_tile(int8_t *__restrict__ wire_codes, float *__restrict__ wire_scales,
                                                int64_t c_step, int64_t s_step, int row, int64_t at, int64_t n,
                                                const float (&r)[8], float s)
{
    constexpr int G = B / kLaneElems;
    store_i8x8(wire_codes + (int64_t)row * c_step, at, n, kFull, pack_codes(r));
    if ((threadIdx.x % G) == 0 && (kFull || at < n)) wire_scales[(int64_t)row * s_step + at / B] = s;
}

// out = bf16(v) for the 8 fp32 values of one lane.
template <bool kFull>
__device__ __forceinline__ void store_narrowed_tile(uint16_t *out, int64_t at, int64_t n,
                                                    const float (&v)[8])
{
    u32x4 w;
    w.x = narrow_bf16x2(v[0], v[1]);
    w.y = narrow_bf16x2(v[2], v[3]);
    w.z = narrow_bf16x2(v[4], v[5]);
    w.w = narrow_bf16x2(v[6], v[7]);
    store_bf16x8(out, at, n, kFull, w);
}

// The last step of a chain for one tile: quantize the finished fp32 sum once
// more and dequantize it (quantized all-gather, Sec. 3.4), or narrow it directly.
template <int B, bool kAG, bool kWire, bool kFull>
__device__ __forceinline__ void finish_tile(const float (&t)[8], uint16_t *out,
                                            int8_t *__restrict__ wire_codes, float *__restrict__ wire_scales,
                                            int64_t c_step, int64_t s_step, int row, int64_t at, int64_t n)
{
    constexpr int G = B / kLaneElems;
    if (kAG) {
        float r[8], s;
        quantize_lane_f<G, true>(t, r, s);      // +0.0 codes: the product below shows the sign of a zero
        if (kWire) store_wire_tile<B, kFull>(wire_codes, wire_scales, c_step, s_step, row, at, n, r, s);
        float d[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) d[j] = r[j] * s;
        store_narrowed_tile<kFull>(out, at, n, d);
    } else {
        store_narrowed_tile<kFull>(out, at, n, t);
    }
}

// ---------------------------------------------------------------- first and last launch of the end-fused schedule
//
// The hop-by-hop chain spends its first two launches on Q_B(x_0) and on hop 1,
// and its last two on hop P-1 and on the dequantization.  On one device each
// pair can share a launch: c_0 and c_(P-1) then stay in registers and 2 of the
// P+1 passes (and 2 of the P wire round trips) disappear.  Same operations in
// the same order, so the same bits.

// (c_1, s_1) = Q_B( fma(codes_0, s_0, x_1) ),  (codes_0, s_0) = Q_B(x_0) kept in registers.
template <int B, int K, bool kFull>
__device__ __forceinline__ void head_body(const uint16_t *__restrict__ x0, const uint16_t *__restrict__ x1, int64_t n,
                                          int8_t *__restrict__ cout, float *__restrict__ sout, int64_t nb,
                                          int64_t wg_at)
{
    constexpr int G = B / kLaneElems;
    const int lane_at = threadIdx.x * kLaneElems;
    u32x4 av[K], bv[K];
    load_tiles<K, kFull>(x0, wg_at, n, av);
    load_tiles<K, kFull>(x1, wg_at, n, bv);
    loads_first();
    float scale[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        float t[8], r[8], xf[8], s0;
        widen_bf16x8(av[k], t);
        quantize_lane_f<G, false>(t, r, s0);        // a -0.0 code only flips the sign of a zero sum, which Q_B ignores
        widen_bf16x8(bv[k], xf);
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = __builtin_fmaf(r[j], s0, xf[j]);
        const u32x2 w = quantize_lane<G>(t, scale[k]);
        store_i8x8(cout, at, n, kFull, w);
    }
    store_group_scales<B, K, kFull>(sout, scale, wg_at, nb);
}

template <int B, int K>
__global__ __launch_bounds__(kThreads) void head_kernel(const uint16_t *__restrict__ x0,
                                                        const uint16_t *__restrict__ x1, int64_t n,
                                                        int8_t *__restrict__ cout, float *__restrict__ sout,
                                                        int64_t nb)
{
    const int64_t wg_at = (int64_t)blockIdx.x * (kTileElems * K);
    if (wg_at + kTileElems * K <= n) {
        head_body<B, K, true>(x0, x1, n, cout, sout, nb, wg_at);
    } else {
        head_body<B, K, false>(x0, x1, n, cout, sout, nb, wg_at);
    }
}

// out = bf16( DQ( Q_B( fma(codes_in, s_in, x) ) ) ): the last hop and the quantized all-gather's pair (Sec. 3.4);
// kAG = false: out = bf16( fma(codes_in, s_in, x) ), the all-gather left unquantized.
template <int B, int K, bool kAG, bool kFull>
__device__ __forceinline__ void tail_body(const int8_t *__restrict__ cin, const float *__restrict__ sin,
                                          const uint16_t *x, int64_t n, uint16_t *out,
                                          int64_t nb, int64_t wg_at)
{
    const int lane_at = threadIdx.x * kLaneElems;
    u32x4 xv[K];
    u32x2 cv[K];
    float sv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        xv[k] = load_bf16x8(x, at, n, kFull);
        cv[k] = load_i8x8(cin, at, n, kFull);
        const int64_t blk = at / B;
        sv[k] = (kFull || blk < nb) ? sin[blk] : 0.0f;
    }
    loads_first();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        float xf[8], qf[8], t[8];
        widen_bf16x8(xv[k], xf);
        widen_i8x8(cv[k], qf);
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = __builtin_fmaf(qf[j], sv[k], xf[j]);
        finish_tile<B, kAG, false, kFull>(t, out, nullptr, nullptr, 0, 0, 0, wg_at + k * kTileElems + lane_at, n);
    }
}

template <int B, int K, bool kAG>
__global__ __launch_bounds__(kThreads) void tail_kernel(const int8_t *__restrict__ cin, const float *__restrict__ sin,
                                                        const uint16_t *x, int64_t n,      // out may be x (in place)
                                                        uint16_t *out, int64_t nb)
{
    const int64_t wg_at = (int64_t)blockIdx.x * (kTileElems * K);
    if (wg_at + kTileElems * K <= n) {
        tail_body<B, K, kAG, true>(cin, sin, x, n, out, nb, wg_at);
    } else {
        tail_body<B, K, kAG, false>(cin, sin, x, n, out, nb, wg_at);
    }
}

// Position -> partial index on a ring of P devices, without a division: the
// callers only ever step by one.
__device__ __forceinline__ int ring_next(int j, int P) { return j + 1 == P ? 0 : j + 1; }
__device__ __forceinline__ int ring_prev(int j, int P) { return j == 0 ? P - 1 : j - 1; }

// One hop on the K tiles of a workgroup: (what the previous device sends) = Q_B(t),
// t = fma(codes, scale, x) -- or a plain fp32 add when the reduce-scatter is
// not quantized.  The quantization does not need x, so it runs while x arrives.
//
// kPositiveZero (see quantize_lane_f) is needed only where the sign of a zero
// sum can reach the output, i.e. when the all-gather is NOT quantized; with a
// quantized all-gather a -0.0 code can only flip the sign of zero sums along
// the chain, which no max-abs, scale or integer code sees, and the last
// quantization hands out +0.0 codes.
template <int B, int K, bool kRS, bool kWire, bool kPositiveZero, bool kFull>
__device__ __forceinline__ void hop_tiles(float (&t)[K][8], const u32x4 (&x)[K], int8_t *__restrict__ wire_codes,
                                          float *__restrict__ wire_scales, int64_t c_step, int64_t s_step, int row,
                                          int64_t wg_at, int64_t n)
{
    constexpr int G = B / kLaneElems;
    const int lane_at = threadIdx.x * kLaneElems;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        if (kRS) {
            float r[8], s;
            quantize_lane_f<G, kPositiveZero>(t[k], r, s);
            if (kWire) {
                store_wire_tile<B, kFull>(wire_codes, wire_scales, c_step, s_step, row,
                                          wg_at + k * kTileElems + lane_at, n, r, s);
            }
            float xf[8];
            widen_bf16x8(x[k], xf);
#pragma unroll
            for (int j = 0; j < 8; ++j) t[k][j] = __builtin_fmaf(r[j], s, xf[j]);
        } else {
            float xf[8];
            widen_bf16x8(x[k], xf);
#pragma unroll
            for (int j = 0; j < 8; ++j) t[k][j] = t[k][j] + xf[j];
        }
    }
}

// Full-loop adder chain over the partials in the order rot, rot+1, ... (mod P).
// Per tile the only state carried from hop to hop is the fp32 sum t.  Each hop
// loads its partial and then computes; the quantization of the running sum
// does not need the new data and runs while it arrives.  Starting the loads a
// hop (or several) ahead was measured and is SLOWER on MI355X (63 -> 67..72 us
// at the 27B-shaped size): with three waves per SIMD and four 16-byte loads
// per lane in flight the memory system is already saturated, and more
// outstanding requests only lengthen its queues.
template <int B, int K, bool kRS, bool kAG, bool kWire, bool kFull>
__device__ __forceinline__ void chain_body(const PartialTable &tab, int P, int rot, int64_t n,
                                           uint16_t *out, int8_t *__restrict__ wire_codes,
                                           float *__restrict__ wire_scales, int64_t c_step, int64_t s_step,
                                           int64_t wg_at)
{
    const int lane_at = threadIdx.x * kLaneElems;
    float t[K][8];      // running fp32 sum
    u32x4 x0[K], xv[K];     // separate registers: partial 1 may be requested before partial 0 has arrived

    int j = rot >= P ? rot - P : rot;               // rot < 2P
    load_tiles<K, kFull>(tab.x[j], wg_at, n, x0);
#pragma unroll
    for (int k = 0; k < K; ++k) widen_bf16x8(x0[k], t[k]);
    for (int i = 1; i < P; ++i) {
        j = ring_next(j, P);
        load_tiles<K, kFull>(tab.x[j], wg_at, n, xv);
        hop_tiles<B, K, kRS, kWire, !kAG, kFull>(t, xv, wire_codes, wire_scales, c_step, s_step, i - 1, wg_at, n);
    }

#pragma unroll
    for (int k = 0; k < K; ++k) {
        finish_tile<B, kAG, kWire, kFull>(t[k], out, wire_codes, wire_scales, c_step, s_step, P - 1,
                                          wg_at + k * kTileElems + lane_at, n);
    }
}

// The same chain with TWO pieces per lane taken from the same block (B >= 128):
// the B/16 lanes of a block each hold elements [8l, 8l+8) and [B/2 + 8l, B/2 +
// 8l + 8) of it, so the max-abs reduction crosses half as many lanes and the
// two quotients are computed once per 16 elements instead of once per 8 --
// a fifth less arithmetic per element-hop in the one kernel whose vector ALU
// is busy half the time (measured at the 27B shape: 4 % faster).  Every wave
// access still covers whole 128-byte lines: the lanes of a block read B/2
// consecutive elements, B bytes, per load.  Same operations per element in the
// same order: same bits.  Full tiles only; the kept-wire form stays on chain_body.
template <int B, int K2, bool kRS, bool kAG>
__device__ __forceinline__ void chain_body_paired(const PartialTable &tab, int P, int rot,
                                                  uint16_t *out, int64_t wg_at)
{
    constexpr int Gh = B / 16;                      // lanes per block
    constexpr int kPairElems = 2 * kTileElems;      // 4096 elements per pair of pieces
    const int64_t lane_at = wg_at + (int64_t)(threadIdx.x / Gh) * B + (threadIdx.x % Gh) * kLaneElems;
    float t[K2][2][8];
    u32x4 x0[K2][2], xv[K2][2];

    int j = rot >= P ? rot - P : rot;
    {
        const uint16_t *p = tab.x[j];
#pragma unroll
        for (int k = 0; k < K2; ++k) {
#pragma unroll
            for (int h = 0; h < 2; ++h) x0[k][h] = load_bf16x8(p, lane_at + k * kPairElems + h * (B / 2), 0, true);
        }
    }
#pragma unroll
    for (int k = 0; k < K2; ++k) {
#pragma unroll
        for (int h = 0; h < 2; ++h) widen_bf16x8(x0[k][h], t[k][h]);
    }
    for (int i = 1; i < P; ++i) {
        j = ring_next(j, P);
        const uint16_t *p = tab.x[j];
#pragma unroll
        for (int k = 0; k < K2; ++k) {
#pragma unroll
            for (int h = 0; h < 2; ++h) xv[k][h] = load_bf16x8(p, lane_at + k * kPairElems + h * (B / 2), 0, true);
        }
#pragma unroll
        for (int k = 0; k < K2; ++k) {
            float xf[2][8];
            if (kRS) {
                float m = 0.0f;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) m = __builtin_fmaxf(m, __builtin_fabsf(t[k][h][e]));
                }
                const float a = __uint_as_float(group_max_bits<Gh>(__float_as_uint(m)));
                float s, inv;
                block_quotients(a, s, inv);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    widen_bf16x8(xv[k][h], xf[h]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float r = __builtin_rintf(t[k][h][e] * inv);
                        if (!kAG) r += 0.0f;        // see hop_tiles: only an unquantized all-gather shows a zero's sign
                        t[k][h][e] = __builtin_fmaf(r, s, xf[h][e]);
                    }
                }
            } else {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    widen_bf16x8(xv[k][h], xf[h]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) t[k][h][e] = t[k][h][e] + xf[h][e];
                }
            }
        }
    }

#pragma unroll
    for (int k = 0; k < K2; ++k) {
        if (kAG) {
            float m = 0.0f;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int e = 0; e < 8; ++e) m = __builtin_fmaxf(m, __builtin_fabsf(t[k][h][e]));
            }
            const float a = __uint_as_float(group_max_bits<Gh>(__float_as_uint(m)));
            float s, inv;
            block_quotients(a, s, inv);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float d[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) d[e] = (__builtin_rintf(t[k][h][e] * inv) + 0.0f) * s;
                store_narrowed_tile<true>(out, lane_at + k * kPairElems + h * (B / 2), 0, d);
            }
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) store_narrowed_tile<true>(out, lane_at + k * kPairElems + h * (B / 2), 0, t[k][h]);
        }
    }
}

// Where a workgroup works: its shard [lo, hi) and rotation, its first element.
struct Span {
    int64_t wg_at, hi;
    int rot;
    bool any;
};

template <int K>
__device__ __forceinline__ Span workgroup_span(int64_t n, int64_t shard_elems, int rot_bias)
{
    Span sp;
    int64_t lo = 0;
    sp.hi = n;
    sp.rot = 0;
    if (shard_elems > 0) {
        lo = (int64_t)blockIdx.y * shard_elems;
        sp.hi = lo + shard_elems < n ? lo + shard_elems : n;
        sp.rot = (int)blockIdx.y + rot_bias;
    }
    sp.wg_at = lo + (int64_t)blockIdx.x * (kTileElems * K);
    sp.any = sp.wg_at < sp.hi;
    return sp;
}

template <int B, int K, bool kRS, bool kAG, bool kWire>
__global__ __launch_bounds__(kThreads) void chain_kernel(const PartialTable tab, int P, int64_t n, int64_t shard_elems,
                                                         uint16_t *out, int8_t *__restrict__ wire_codes,
                                                         float *__restrict__ wire_scales, int64_t c_step,
                                                         int64_t s_step)
{
    const Span sp = workgroup_span<K>(n, shard_elems, 1);     // shard k: devices k+1, k+2, ..., k
    if (!sp.any) return;                                      // uniform over the workgroup
    if (sp.wg_at + kTileElems * K <= sp.hi) {
        if (EQUARX_CHAIN_PAIRED && B >= 128 && K % 2 == 0 && !kWire) {
            chain_body_paired<(B >= 128 ? B : 128), (K >= 2 ? K / 2 : 1), kRS, kAG>(tab, P, sp.rot, out, sp.wg_at);
        } else {
            chain_body<B, K, kRS, kAG, kWire, true>(tab, P, sp.rot, sp.hi, out, wire_codes, wire_scales, c_step,
                                                    s_step, sp.wg_at);
        }
    } else {
        chain_body<B, K, kRS, kAG, kWire, false>(tab, P, sp.rot, sp.hi, out, wire_codes, wire_scales, c_step, s_step,
                                                 sp.wg_at);
    }
}

// ---------------------------------------------------------------- ring order, hop by hop
//
// What all devices of a ring do in one step, as one launch: grid row k works on
// shard k, whose chain visits devices k+1, k+2, ..., k (mod P), so in step i it
// adds device (k + 1 + i)'s partial.  Same bodies as the plain per-pass
// kernels; only the partial, and the end of the range, depend on the grid row.

template <int B, int K>
__global__ __launch_bounds__(kThreads) void quantize_ring_kernel(const PartialTable tab, int P, int64_t n,
                                                                 int64_t shard_elems, int8_t *__restrict__ codes,
                                                                 float *__restrict__ scales)
{
    const Span sp = workgroup_span<K>(n, shard_elems, 1);
    if (!sp.any) return;
    const uint16_t *x = tab.x[sp.rot >= P ? sp.rot - P : sp.rot];
    const int64_t nb = (sp.hi + B - 1) / B;
    if (sp.wg_at + kTileElems * K <= sp.hi) {
        quantize_body<B, K, true>(x, sp.hi, codes, scales, nb, sp.wg_at);
    } else {
        quantize_body<B, K, false>(x, sp.hi, codes, scales, nb, sp.wg_at);
    }
}

template <int B, int K>
__global__ __launch_bounds__(kThreads) void hop_ring_kernel(const int8_t *cin, const float *sin, const PartialTable tab,
                                                            int P, int step, int64_t n, int64_t shard_elems,
                                                            int8_t *cout, float *sout)
{
    const Span sp = workgroup_span<K>(n, shard_elems, 1 + step);    // row + 1 + step < 2P
    if (!sp.any) return;
    const uint16_t *x = tab.x[sp.rot >= P ? sp.rot - P : sp.rot];
    const int64_t nb = (sp.hi + B - 1) / B;
    if (sp.wg_at + kTileElems * K <= sp.hi) {
        hop_body<B, K, true>(cin, sin, x, sp.hi, cout, sout, nb, sp.wg_at);
    } else {
        hop_body<B, K, false>(cin, sin, x, sp.hi, cout, sout, nb, sp.wg_at);
    }
}

template <int B, int K, bool kAG>
__global__ __launch_bounds__(kThreads) void tail_ring_kernel(const int8_t *__restrict__ cin,
                                                             const float *__restrict__ sin, const PartialTable tab,
                                                             int P, int step, int64_t n, int64_t shard_elems,
                                                             uint16_t *out)
{
    const Span sp = workgroup_span<K>(n, shard_elems, 1 + step);
    if (!sp.any) return;
    const uint16_t *x = tab.x[sp.rot >= P ? sp.rot - P : sp.rot];
    const int64_t nb = (sp.hi + B - 1) / B;
    if (sp.wg_at + kTileElems * K <= sp.hi) {
        tail_body<B, K, kAG, true>(cin, sin, x, sp.hi, out, nb, sp.wg_at);
    } else {
        tail_body<B, K, kAG, false>(cin, sin, x, sp.hi, out, nb, sp.wg_at);
    }
}

// Small messages: the same chain, organised for latency instead of bandwidth.
// With few tiles the bandwidth-shaped kernel leaves most compute units idle
// and pays one memory round trip per hop.  Here a workgroup takes ONE tile and
// requests the tiles of kSmallBatch partials at a time, two batches in flight
// (one being consumed, one arriving), so a chain of P hops costs about P /
// kSmallBatch round trips.  Every load is unconditional -- positions past the
// last partial re-read the last partial and are ignored -- because a load
// behind a condition makes the compiler wait for all outstanding loads where
// the paths join.
constexpr int kSmallBatch = 8;

template <int B, bool kWire, bool kFull>
__device__ __forceinline__ void chain_small_body(const PartialTable &tab, int P, int64_t n,
                                                 uint16_t *out, int8_t *__restrict__ wire_codes,
                                                 float *__restrict__ wire_scales, int64_t c_step, int64_t s_step,
                                                 int64_t wg_at)
{
    constexpr int D = kSmallBatch;
    const int lane_at = threadIdx.x * kLaneElems;
    float t[1][8];
    u32x4 a[D][1], b[D][1];

#pragma unroll
    for (int d = 0; d < D; ++d) load_tiles<1, kFull>(tab.x[d < P ? d : P - 1], wg_at, n, a[d]);

    for (int base = 0; base < P; base += 2 * D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int i = base + D + d;
            load_tiles<1, kFull>(tab.x[i < P ? i : P - 1], wg_at, n, b[d]);
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int i = base + d;
            if (i == 0) {
                widen_bf16x8(a[0][0], t[0]);
            } else if (i < P) {
                hop_tiles<B, 1, true, kWire, false, kFull>(t, a[d], wire_codes, wire_scales, c_step, s_step, i - 1,
                                                           wg_at, n);
            }
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int i = base + 2 * D + d;
            load_tiles<1, kFull>(tab.x[i < P ? i : P - 1], wg_at, n, a[d]);
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int i = base + D + d;
            if (i < P) {
                hop_tiles<B, 1, true, kWire, false, kFull>(t, b[d], wire_codes, wire_scales, c_step, s_step, i - 1,
                                                           wg_at, n);
            }
        }
    }
    finish_tile<B, true, kWire, kFull>(t[0], out, wire_codes, wire_scales, c_step, s_step, P - 1, wg_at + lane_at, n);
}

template <int B, bool kWire>
__global__ __launch_bounds__(kThreads) void chain_small_kernel(const PartialTable tab, int P, int64_t n,
                                                               uint16_t *out,
                                                               int8_t *__restrict__ wire_codes,
                                                               float *__restrict__ wire_scales, int64_t c_step,
                                                               int64_t s_step)
{
    const int64_t wg_at = (int64_t)blockIdx.x * kTileElems;
    if (wg_at + kTileElems <= n) {
        chain_small_body<B, kWire, true>(tab, P, n, out, wire_codes, wire_scales, c_step, s_step, wg_at);
    } else {
        chain_small_body<B, kWire, false>(tab, P, n, out, wire_codes, wire_scales, c_step, s_step, wg_at);
    }
}

// Semi-loop adder tree (Sec. 3.3).  Position 0 (device rot) owns the shard; the
// other positions follow in ring order.  With h = P/2 the counter-clockwise
// chain h+1, h+2, ..., P-1 and the clockwise chain h, h-1, ..., 1 each end in a
// quantized send to the owner, which adds them to its own fp32 shard, the
// shorter counter-clockwise chain first.
template <int B, int K, bool kAG, bool kFull>
__device__ __forceinline__ void semi_body(const PartialTable &tab, int P, int rot, int64_t n,
                                          uint16_t *out, int64_t wg_at)
{
    const int lane_at = threadIdx.x * kLaneElems;
    const int h = P / 2;
    float own[K][8], t[K][8];
    u32x4 xv[K];

    const int owner = rot >= P ? rot - P : rot;     // rot < 2P
    load_tiles<K, kFull>(tab.x[owner], wg_at, n, xv);
#pragma unroll
    for (int k = 0; k < K; ++k) widen_bf16x8(xv[k], own[k]);

#pragma unroll 1
    for (int dir = 0; dir < 2; ++dir) {
        // dir 0: positions h+1 .. P-1 ascending; dir 1: positions h .. 1 descending
        const int count = dir == 0 ? P - 1 - h : h;
        if (count <= 0) continue;
        int j = owner + (dir == 0 ? h + 1 : h);     // < 2P
        if (j >= P) j -= P;
        load_tiles<K, kFull>(tab.x[j], wg_at, n, xv);
#pragma unroll
        for (int k = 0; k < K; ++k) widen_bf16x8(xv[k], t[k]);
        for (int c = 1; c < count; ++c) {
            j = dir == 0 ? ring_next(j, P) : ring_prev(j, P);
            load_tiles<K, kFull>(tab.x[j], wg_at, n, xv);
            hop_tiles<B, K, true, false, !kAG, kFull>(t, xv, nullptr, nullptr, 0, 0, 0, wg_at, n);
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            constexpr int G = B / kLaneElems;
            float r[8], s;
            quantize_lane_f<G, !kAG>(t[k], r, s);                      // the send that reaches the owner
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) own[k][jj] = __builtin_fmaf(r[jj], s, own[k][jj]);
        }
    }

#pragma unroll
    for (int k = 0; k < K; ++k) {
        finish_tile<B, kAG, false, kFull>(own[k], out, nullptr, nullptr, 0, 0, 0, wg_at + k * kTileElems + lane_at, n);
    }
}

template <int B, int K, bool kAG>
__global__ __launch_bounds__(kThreads) void semi_kernel(const PartialTable tab, int P, int64_t n, int64_t shard_elems,
                                                        uint16_t *out)
{
    const Span sp = workgroup_span<K>(n, shard_elems, 0);     // shard k: owner is device k
    if (!sp.any) return;
    if (sp.wg_at + kTileElems * K <= sp.hi) {
        semi_body<B, K, kAG, true>(tab, P, sp.rot, sp.hi, out, sp.wg_at);
    } else {
        semi_body<B, K, kAG, false>(tab, P, sp.rot, sp.hi, out, sp.wg_at);
    }
}

// ---------------------------------------------------------------- flat one-shot reduce
// The reduce-scatter as an all-to-all followed by a local reduction (the
// decomposition Sec. 2 describes for ZeRO++, and the shape a full xGMI mesh
// favours over a ring): the owner of a shard holds its own bf16 shard and R
// received (codes, scales) pairs, each quantized once by its sender.  It
// dequantizes and accumulates them in fp32 in array order -- one fused
// multiply-add each -- and quantizes the sum once for the all-gather.

struct WireTable {
    const int8_t *codes[kMaxPartials];
    const float *scales[kMaxPartials];
};

template <int B, int K, bool kOutBf16, bool kOutWire, bool kAG, bool kFull, bool kStream = false>
__device__ __forceinline__ void flat_body(const uint16_t *local, const WireTable &tab, int R, int64_t n,
                                          uint16_t *out, int8_t *__restrict__ codes_out,
                                          float *__restrict__ scales_out, int64_t nb, int64_t wg_at)
{
    constexpr int G = B / kLaneElems;
    const int lane_at = threadIdx.x * kLaneElems;
    float acc[K][8];
    u32x4 xv[K];
    load_tiles<K, kFull>(local, wg_at, n, xv);
#pragma unroll
    for (int k = 0; k < K; ++k) widen_bf16x8(xv[k], acc[k]);

    for (int r = 0; r < R; ++r) {
        const int8_t *c = tab.codes[r];
        const float *sc = tab.scales[r];
        u32x2 cv[K];
        float sv[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int64_t at = wg_at + k * kTileElems + lane_at;
            cv[k] = load_i8x8<kStream>(c, at, n, kFull);
            const int64_t blk = at / B;
            sv[k] = (kFull || blk < nb) ? sc[blk] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            float qf[8];
            widen_i8x8(cv[k], qf);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[k][j] = __builtin_fmaf(qf[j], sv[k], acc[k][j]);
        }
    }

#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        if (!kAG) {                 // all-gather left unquantized (the semi-loop's owner, Sec. 3.3/3.4): no wire out
            store_narrowed_tile<kFull>(out, at, n, acc[k]);
            continue;
        }
        float q[8], s;
        quantize_lane_f<G, true>(acc[k], q, s);
        if (kOutWire) {
            store_i8x8<kStream>(codes_out, at, n, kFull, pack_codes(q));
            if ((threadIdx.x % G) == 0 && (kFull || at < n)) scales_out[at / B] = s;
        }
        if (kOutBf16) {
            float d[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) d[j] = q[j] * s;
            store_narrowed_tile<kFull>(out, at, n, d);
        }
    }
}

template <int B, int K, bool kOutBf16, bool kOutWire, bool kAG = true, bool kStream = false>
__global__ __launch_bounds__(kThreads) void flat_kernel(const uint16_t *local, const WireTable tab, int R,
                                                        int64_t n, uint16_t *out,
                                                        int8_t *__restrict__ codes_out, float *__restrict__ scales_out,
                                                        int64_t nb)
{
    const int64_t wg_at = (int64_t)blockIdx.x * (kTileElems * K);
    if (wg_at + kTileElems * K <= n) {
        flat_body<B, K, kOutBf16, kOutWire, kAG, true, kStream>(local, tab, R, n, out, codes_out, scales_out, nb, wg_at);
    } else {
        flat_body<B, K, kOutBf16, kOutWire, kAG, false, kStream>(local, tab, R, n, out, codes_out, scales_out, nb, wg_at);
    }
}

// ---------------------------------------------------------------- semi-loop in ring order, hop by hop
//
// What all devices of a ring do in one iteration of the semi-loop reduce-scatter (Sec. 3.3), as one launch: grid
// row k works on shard k, which device k owns; the devices k+1, k+2, ... sit around it at positions 1, 2, ....
// With h = P/2 the counter-clockwise chain runs over positions h+1, h+2, ..., P-1 and the clockwise chain over
// positions h, h-1, ..., 1; in iteration t both advance one device (blockIdx.z picks the direction), so the whole
// reduce-scatter takes h iterations, as the paper's N/2.  Same bodies as the plain per-pass kernels.

struct WirePair {           // one wire buffer per direction
    int8_t *codes[2];
    float *scales[2];
};

template <int B, int K>
__global__ __launch_bounds__(kThreads) void semi_ring_step_kernel(const PartialTable tab, int P, int t, int64_t n,
                                                                  int64_t shard_elems, const WirePair in,
                                                                  const WirePair out)
{
    const Span sp = workgroup_span<K>(n, shard_elems, 0);       // rot = the owner's device number
    if (!sp.any) return;
    const int dir = blockIdx.z, h = P / 2;
    const int count = dir == 0 ? P - 1 - h : h;                 // devices in this direction's chain
    if (t >= count) return;                                     // the shorter chain has already arrived
    int dev = sp.rot + (dir == 0 ? h + 1 + t : h - t);          // < 2P
    if (dev >= P) dev -= P;
    const uint16_t *x = tab.x[dev];
    const int64_t nb = (sp.hi + B - 1) / B;
    const bool full = sp.wg_at + kTileElems * K <= sp.hi;
    if (t == 0) {
        if (full) {
            quantize_body<B, K, true>(x, sp.hi, out.codes[dir], out.scales[dir], nb, sp.wg_at);
        } else {
            quantize_body<B, K, false>(x, sp.hi, out.codes[dir], out.scales[dir], nb, sp.wg_at);
        }
    } else if (full) {
        hop_body<B, K, true>(in.codes[dir], in.scales[dir], x, sp.hi, out.codes[dir], out.scales[dir], nb, sp.wg_at);
    } else {
        hop_body<B, K, false>(in.codes[dir], in.scales[dir], x, sp.hi, out.codes[dir], out.scales[dir], nb, sp.wg_at);
    }
}

// The owner's last step: its own shard plus the wires that arrived (counter-clockwise first), then the all-gather's
// quantize/dequantize pair or the plain narrowing.
template <int B, int K, bool kAG>
__global__ __launch_bounds__(kThreads) void semi_ring_owner_kernel(const PartialTable tab, int P, int64_t n,
                                                                   int64_t shard_elems, const WireTable wires,
                                                                   int received, uint16_t *out)
{
    const Span sp = workgroup_span<K>(n, shard_elems, 0);
    if (!sp.any) return;
    const uint16_t *own = tab.x[sp.rot >= P ? sp.rot - P : sp.rot];
    const int64_t nb = (sp.hi + B - 1) / B;
    if (sp.wg_at + kTileElems * K <= sp.hi) {
        flat_body<B, K, true, false, kAG, true>(own, wires, received, sp.hi, out, nullptr, nullptr, nb, sp.wg_at);
    } else {
        flat_body<B, K, true, false, kAG, false>(own, wires, received, sp.hi, out, nullptr, nullptr, nb, sp.wg_at);
    }
}

}  // namespace equarx
