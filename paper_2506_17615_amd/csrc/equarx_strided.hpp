// The paper's own block geometry on gfx950 (EQuARX, arXiv 2506.17615, Sec. 3.2).
//
// There a shard is cut into chunks of 8 x 128 = 1024 elements (the TPU's vector
// register shape, contiguous in its tiled memory layout) and a minishard of
// `chunks` consecutive chunks gets 1024 scales: scale j comes from the max-abs
// over position j of every chunk, so a quantization block is `chunks` entries
// that lie 1024 elements apart.  On the TPU this avoids any reduction inside a
// vector register.  On a GPU it means the opposite of the contiguous layout:
// no reduction over neighbouring elements (a lane keeps its own 8 positions),
// but one ACROSS the chunks of a minishard.
//
// Decomposition of the per-pass kernels (quantize, hop: codes go to memory, and
// 8-byte code pieces want 16 lanes or more side by side to fill a 128-byte
// line; the single-launch chain further down writes no codes and uses a
// layout without LDS): a workgroup of 256 threads takes one slice of 256 positions of
// one minishard.  Thread (g, l), g = 0..7, l = 0..31, owns positions 8l..8l+7
// of the slice in chunks g, g+8, g+16, ...; it keeps the raw inputs of its
// chunks/8 chunks in registers, so global memory is read once.  The 8 partial
// maxima per position meet in LDS (8 KiB), every thread derives the scales of
// its 8 positions, recomputes its values from the registers, scales, rounds
// and stores.  Loads of a half-wave cover 512 contiguous bytes.
#pragma once

#include "equarx_device.hpp"

namespace equarx {

constexpr int kChunk = 1024;                               // elements per chunk (8 x 128)
// Measured at the 27B-shaped size: 32 lanes per slice is best overall (16: within 2 % for 64 and 128 chunks, 8 %
// slower for 32; 64: 3 % slower for 32, 30 % slower for 128).  Capping the waves per SIMD at 2 or 3, or dropping
// the first of the two barriers (a kernel takes the maximum once), changes nothing beyond 2 %; the 8 x 8 in-wave
// layout of the single-launch chain makes these kernels 5-8 % slower (64-byte code pieces); workgroups of 512 or 1024
// threads with 1 or 2 KiB runs per chunk are no faster for 64 chunks and 4-100 % slower otherwise.
#ifndef EQUARX_STRIDED_SLICE_LANES
#define EQUARX_STRIDED_SLICE_LANES 32
#endif
constexpr int kSliceLanes = EQUARX_STRIDED_SLICE_LANES;    // lanes across a slice of a chunk
constexpr int kSlicePos = kSliceLanes * kLaneElems;        // 256 positions per workgroup
constexpr int kChunkGroups = kThreads / kSliceLanes;       // 8 groups of lanes, each walking every 8th chunk
constexpr int kSlicesPerChunk = kChunk / kSlicePos;        // 4 workgroups per minishard
static_assert(kThreads == 256, "the strided kernels are laid out for 256-thread workgroups");

struct StridedSpot {
    int64_t minishard;  // which minishard the workgroup works on
    int64_t elem;       // first element of the lane in chunk `g` of its minishard
    int64_t scale;      // index of the lane's first scale
    int g;              // chunk group
};

__device__ __forceinline__ StridedSpot strided_spot(int chunks)
{
    StridedSpot sp;
    const int l = threadIdx.x % kSliceLanes;
    sp.g = threadIdx.x / kSliceLanes;
    const int64_t ms = blockIdx.x / kSlicesPerChunk;
    const int pos = (blockIdx.x % kSlicesPerChunk) * kSlicePos + l * kLaneElems;
    sp.minishard = ms;
    sp.elem = ms * ((int64_t)kChunk * chunks) + (int64_t)sp.g * kChunk + pos;
    sp.scale = ms * kChunk + pos;
    return sp;
}

// The bf16 tensor a per-pass kernel reads.  Array order (per_shard == 0): partial `offset` for every workgroup.
// Ring layout (Sec. 3; per_shard > 0): the tensor is cut into shards of per_shard minishards, shard k ends on device
// k, and a launch is one ring step on every shard at once -- the workgroups of shard k read the partial of device
// (k + offset) mod P.  0 <= offset < P.
struct StridedSource {
    PartialTable tab;
    int P;
    int per_shard;
    int offset;
};

__device__ __forceinline__ const uint16_t *strided_source(const StridedSource &src, int64_t minishard)
{
    const int j = (src.per_shard > 0 ? (int)(minishard / src.per_shard) : 0) + src.offset;     // < 2P
    return src.tab.x[j >= src.P ? j - src.P : j];
}

// Max over the 8 chunk groups for each of the lane's 8 positions, through LDS.
// m: bit patterns of non-negative floats.  Every thread of the workgroup calls this.
__device__ __forceinline__ void across_chunks_max(uint32_t (&m)[8], uint32_t (*red)[kSlicePos])
{
    const int l = threadIdx.x % kSliceLanes;
    const int g = threadIdx.x / kSliceLanes;
    __syncthreads();                                        // the previous round's readers are done
    u32x4 *row = reinterpret_cast<u32x4 *>(&red[g][l * kLaneElems]);
    row[0] = u32x4{m[0], m[1], m[2], m[3]};
    row[1] = u32x4{m[4], m[5], m[6], m[7]};
    __syncthreads();
#pragma unroll
    for (int h = 0; h < kChunkGroups; ++h) {
        const u32x4 *other = reinterpret_cast<const u32x4 *>(&red[h][l * kLaneElems]);
        const u32x4 a = other[0], b = other[1];
        m[0] = umax(m[0], a.x); m[1] = umax(m[1], a.y); m[2] = umax(m[2], a.z); m[3] = umax(m[3], a.w);
        m[4] = umax(m[4], b.x); m[5] = umax(m[5], b.y); m[6] = umax(m[6], b.z); m[7] = umax(m[7], b.w);
    }
}

__device__ __forceinline__ void note_absmax(const float (&t)[8], uint32_t (&m)[8])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) m[j] = umax(m[j], __float_as_uint(t[j]) & 0x7FFFFFFFu);
}

__device__ __forceinline__ u32x2 scale_and_pack(const float (&t)[8], const float (&inv)[8])
{
    uint32_t b[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) b[j] = __float_as_uint(t[j] * inv[j] + kRoundMagic);  // rounds to the integer code
    u32x2 w;
    w.x = gather_low_bytes(b[0], b[1], b[2], b[3]);
    w.y = gather_low_bytes(b[4], b[5], b[6], b[7]);
    return w;
}

// R = chunks / 8 chunks per thread.
template <int R>
__device__ __forceinline__ void quantize_strided_body(const uint16_t *__restrict__ x, int8_t *__restrict__ codes,
                                                      float *__restrict__ scales, const StridedSpot &sp,
                                                      uint32_t (*red)[kSlicePos])
{
    u32x4 xv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        xv[r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(x + sp.elem + (int64_t)r * kChunkGroups * kChunk));
    }
    uint32_t m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float t[8];
        widen_bf16x8(xv[r], t);
        note_absmax(t, m);
    }
    across_chunks_max(m, red);

    float scale[8], inv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) block_quotients(__uint_as_float(m[j]), scale[j], inv[j]);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float t[8];
        widen_bf16x8(xv[r], t);
        *reinterpret_cast<u32x2 *>(codes + sp.elem + (int64_t)r * kChunkGroups * kChunk) = scale_and_pack(t, inv);
    }
    if (sp.g == 0) {
        float *s = scales + sp.scale;
        *reinterpret_cast<u32x4 *>(s) = u32x4{__float_as_uint(scale[0]), __float_as_uint(scale[1]),
                                              __float_as_uint(scale[2]), __float_as_uint(scale[3])};
        *reinterpret_cast<u32x4 *>(s + 4) = u32x4{__float_as_uint(scale[4]), __float_as_uint(scale[5]),
                                                  __float_as_uint(scale[6]), __float_as_uint(scale[7])};
    }
}

template <int R>
__global__ __launch_bounds__(kThreads) void quantize_strided_kernel(const StridedSource src,
                                                                    int8_t *__restrict__ codes,
                                                                    float *__restrict__ scales)
{
    __shared__ __align__(16) uint32_t red[kChunkGroups][kSlicePos];
    const StridedSpot sp = strided_spot(R * kChunkGroups);
    quantize_strided_body<R>(strided_source(src, sp.minishard), codes, scales, sp, red);
}

// One hop in the strided geometry.  Output wire may be the input wire: a
// workgroup holds all its inputs in registers before it stores anything.
template <int R>
__device__ __forceinline__ void hop_strided_body(const int8_t *cin, const float *sin, const uint16_t *__restrict__ x,
                                                 int8_t *cout, float *sout, const StridedSpot &sp,
                                                 uint32_t (*red)[kSlicePos])
{
    u32x4 xv[R];
    u32x2 cv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t at = sp.elem + (int64_t)r * kChunkGroups * kChunk;
        xv[r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(x + at));
        cv[r] = *reinterpret_cast<const u32x2 *>(cin + at);
    }
    float s_in[8];
    {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(sin + sp.scale);
        const u32x4 b = *reinterpret_cast<const u32x4 *>(sin + sp.scale + 4);
        s_in[0] = __uint_as_float(a.x); s_in[1] = __uint_as_float(a.y);
        s_in[2] = __uint_as_float(a.z); s_in[3] = __uint_as_float(a.w);
        s_in[4] = __uint_as_float(b.x); s_in[5] = __uint_as_float(b.y);
        s_in[6] = __uint_as_float(b.z); s_in[7] = __uint_as_float(b.w);
    }

    uint32_t m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float xf[8], qf[8], t[8];
        widen_bf16x8(xv[r], xf);
        widen_i8x8(cv[r], qf);
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = __builtin_fmaf(qf[j], s_in[j], xf[j]);
        note_absmax(t, m);
    }
    across_chunks_max(m, red);

    float scale[8], inv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) block_quotients(__uint_as_float(m[j]), scale[j], inv[j]);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float xf[8], qf[8], t[8];
        widen_bf16x8(xv[r], xf);
        widen_i8x8(cv[r], qf);
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = __builtin_fmaf(qf[j], s_in[j], xf[j]);      // same operands, same bits
        *reinterpret_cast<u32x2 *>(cout + sp.elem + (int64_t)r * kChunkGroups * kChunk) = scale_and_pack(t, inv);
    }
    if (sp.g == 0) {
        float *s = sout + sp.scale;
        *reinterpret_cast<u32x4 *>(s) = u32x4{__float_as_uint(scale[0]), __float_as_uint(scale[1]),
                                              __float_as_uint(scale[2]), __float_as_uint(scale[3])};
        *reinterpret_cast<u32x4 *>(s + 4) = u32x4{__float_as_uint(scale[4]), __float_as_uint(scale[5]),
                                                  __float_as_uint(scale[6]), __float_as_uint(scale[7])};
    }
}

template <int R>
__global__ __launch_bounds__(kThreads) void hop_strided_kernel(const int8_t *cin, const float *sin,
                                                               const StridedSource src, int8_t *cout, float *sout)
{
    __shared__ __align__(16) uint32_t red[kChunkGroups][kSlicePos];
    const StridedSpot sp = strided_spot(R * kChunkGroups);
    hop_strided_body<R>(cin, sin, strided_source(src, sp.minishard), cout, sout, sp, red);
}

// One iteration of the semi-loop reduce-scatter (Sec. 3.3) on both of its chains at once: grid row 0 advances the
// chain that walks up from device h+1, row 1 the one that walks down from device h, each by one device -- the
// first iteration quantizes the chain's first shard (no incoming wire: cin == nullptr), the later ones are hops on
// the chain's own wire buffer in place.  The two rows share nothing.
struct StridedDirection {
    int offset;             // as StridedSource::offset
    const int8_t *cin;      // nullptr: this is the chain's first device, it only quantizes its shard
    const float *sin;
    int8_t *cout;
    float *sout;
};

struct StridedDirections {
    StridedDirection d[2];
};

template <int R>
__global__ __launch_bounds__(kThreads) void semi_step_strided_kernel(const PartialTable tab, int P, int per_shard,
                                                                     const StridedDirections dirs)
{
    __shared__ __align__(16) uint32_t red[kChunkGroups][kSlicePos];
    const StridedSpot sp = strided_spot(R * kChunkGroups);
    const StridedDirection d = blockIdx.y == 0 ? dirs.d[0] : dirs.d[1];
    const int j = (per_shard > 0 ? (int)(sp.minishard / per_shard) : 0) + d.offset;     // < 2P
    const uint16_t *x = tab.x[j >= P ? j - P : j];
    if (d.cin == nullptr) {             // uniform over the workgroup
        quantize_strided_body<R>(x, d.cout, d.sout, sp, red);
    } else {
        hop_strided_body<R>(d.cin, d.sin, x, d.cout, d.sout, sp, red);
    }
}

// The last launch of a hop-by-hop flavour in the strided geometry: the device that ends up with the sum adds what
// it received to its own bf16 shard -- one wire at the end of the full loop, one or two at the owner of the
// semi-loop (Sec. 3.3: the shorter chain's wire first), none when it is alone -- each with one fused multiply-add
// per element, and hands the sum to the all-gather: quantized once more and dequantized (kAG), or narrowed to
// bf16 as it is (Sec. 3.4).  out may be `own`: a thread reads its elements before it writes them.
struct StridedWires {
    const int8_t *codes[2];
    const float *scales[2];
};

template <int R, bool kAG>
__global__ __launch_bounds__(kThreads) void owner_strided_kernel(const StridedSource src, const StridedWires wires,
                                                                 int received, uint16_t *out)
{
    __shared__ __align__(16) uint32_t red[kChunkGroups][kSlicePos];
    constexpr int chunks = R * kChunkGroups;
    const StridedSpot sp = strided_spot(chunks);
    const uint16_t *own = strided_source(src, sp.minishard);

    float acc[R][8];
    {
        u32x4 xv[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            xv[r] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4 *>(own + sp.elem + (int64_t)r * kChunkGroups * kChunk));
        }
#pragma unroll
        for (int r = 0; r < R; ++r) widen_bf16x8(xv[r], acc[r]);
    }
    for (int k = 0; k < received; ++k) {
        const int8_t *codes = wires.codes[k];
        const float *scales = wires.scales[k];
        u32x2 cv[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            cv[r] = *reinterpret_cast<const u32x2 *>(codes + sp.elem + (int64_t)r * kChunkGroups * kChunk);
        }
        const u32x4 a = *reinterpret_cast<const u32x4 *>(scales + sp.scale);
        const u32x4 b = *reinterpret_cast<const u32x4 *>(scales + sp.scale + 4);
        const float s_in[8] = {__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(a.z), __uint_as_float(a.w),
                               __uint_as_float(b.x), __uint_as_float(b.y), __uint_as_float(b.z), __uint_as_float(b.w)};
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float qf[8];
            widen_i8x8(cv[r], qf);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[r][j] = __builtin_fmaf(qf[j], s_in[j], acc[r][j]);
        }
    }

    float scale[8], inv[8];
    if (kAG) {
        uint32_t m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < R; ++r) note_absmax(acc[r], m);
        across_chunks_max(m, red);
#pragma unroll
        for (int j = 0; j < 8; ++j) block_quotients(__uint_as_float(m[j]), scale[j], inv[j]);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float d[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            d[j] = kAG ? (__builtin_rintf(acc[r][j] * inv[j]) + 0.0f) * scale[j] : acc[r][j];     // +0.0: the code as an integer
        }
        u32x4 w;
        w.x = narrow_bf16x2(d[0], d[1]);
        w.y = narrow_bf16x2(d[2], d[3]);
        w.z = narrow_bf16x2(d[4], d[5]);
        w.w = narrow_bf16x2(d[6], d[7]);
        __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>(out + sp.elem + (int64_t)r * kChunkGroups * kChunk));
    }
}

// ---------------------------------------------------------------- the chain and its flavours in one launch
//
// The full-loop chain, the semi-loop reduce-scatter (Sec. 3.3) and the stage
// knob (Sec. 3.4) with the blocks of Sec. 3.2, one launch each.  The running
// fp32 sums of a thread's chunks stay in registers from the first partial to
// the output; every quantized send needs the max-abs across the chunks of a
// minishard and nothing else from other threads.
//
// Layout: lane = 8 * g + l inside a wave, so the 8 chunk groups of a position
// sit in ONE wave, 8 lanes apart, and their maximum is three lane exchanges
// per value -- no LDS, no barrier.  A wave covers 64 positions (a 128-byte
// piece of each of 8 chunks per load) and, with W = 1, the chunks g, g+8, ...
// of its group: R = chunks/8 rows of 8 running sums per thread.  For 128
// chunks that would be 16 rows (128 sums, 64 load registers: one wave per
// SIMD), so there W = 2 waves share a position piece, wave w taking the chunk
// groups 8w .. 8w+7 (R = 8), and the two maxima meet through 256 bytes of LDS
// and one barrier per send (the buffer alternates, so the barrier of the next
// send also separates this send's reads from the writes of the one after).
// Same operations in the same order as the hop-by-hop strided chain, hence
// the same bits.

struct WaveSpot {
    int64_t minishard;  // which minishard the workgroup works on
    int64_t elem;       // first element of the lane in the first of its chunks
    int64_t scale;      // index of the lane's first scale
    int64_t row_step;   // elements between two consecutive chunks of the lane
    bool first_group;   // the lane stores the scales of its 8 positions
};

// W waves per position piece; a 256-thread workgroup covers (4 / W) * 64 positions: 4 * W workgroups per minishard.
template <int W>
__device__ __forceinline__ WaveSpot wave_spot(int chunks)
{
    static_assert(W == 1 || W == 2, "waves per position piece");
    constexpr int kPieces = (kThreads / 64) / W;                // position pieces per workgroup
    constexpr int kPerChunk = kChunk / (kPieces * 64);          // workgroups per minishard
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int g = (wave % W) * 8 + lane / 8;                    // chunk group, 0 .. 8W-1
    const int64_t ms = blockIdx.x / kPerChunk;
    const int pos = (blockIdx.x % kPerChunk) * (kPieces * 64) + (wave / W) * 64 + (lane % 8) * kLaneElems;
    WaveSpot sp;
    sp.minishard = ms;
    sp.elem = ms * ((int64_t)kChunk * chunks) + (int64_t)g * kChunk + pos;
    sp.scale = ms * kChunk + pos;
    sp.row_step = (int64_t)8 * W * kChunk;
    sp.first_group = g == 0;
    return sp;
}

constexpr int strided_wave_share(int chunks) { return chunks > 64 ? 2 : 1; }       // W for a minishard of `chunks`

// Max over all chunk groups for each of the lane's 8 positions.  Every thread of the workgroup calls this; `red`
// and `parity` matter for W = 2 only.
template <int W>
__device__ __forceinline__ void across_chunks_max_wave(uint32_t (&m)[8], uint32_t (*red)[kThreads / 64][64], int &parity)
{
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t v = m[j];
        v = umax(v, dpp_read<0x128>(v));                                    // row_ror:8: lane ^ 8 within a row of 16
        auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);      // lane ^ 16
        v = umax(a[0], a[1]);
        auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);      // lane ^ 32
        m[j] = umax(b[0], b[1]);
    }
    if (W == 2) {
        const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
        const int at = (lane % 8) * kLaneElems;
        if (lane < 8) {
            u32x4 *row = reinterpret_cast<u32x4 *>(&red[parity][wave][at]);
            row[0] = u32x4{m[0], m[1], m[2], m[3]};
            row[1] = u32x4{m[4], m[5], m[6], m[7]};
        }
        __syncthreads();
        const u32x4 *other = reinterpret_cast<const u32x4 *>(&red[parity][wave ^ 1][at]);
        const u32x4 a = other[0], b = other[1];
        m[0] = umax(m[0], a.x); m[1] = umax(m[1], a.y); m[2] = umax(m[2], a.z); m[3] = umax(m[3], a.w);
        m[4] = umax(m[4], b.x); m[5] = umax(m[5], b.y); m[6] = umax(m[6], b.z); m[7] = umax(m[7], b.w);
        parity ^= 1;
    }
}

struct ChunkMaxState {
    uint32_t (*red)[kThreads / 64][64];
    int parity;
};

template <int R>
__device__ __forceinline__ void load_strided(const uint16_t *x, const WaveSpot &sp, u32x4 (&xv)[R])
{
#pragma unroll
    for (int r = 0; r < R; ++r) {
        xv[r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(x + sp.elem + r * sp.row_step));
    }
}

template <int R>
__device__ __forceinline__ void widen_strided(const u32x4 (&xv)[R], float (&t)[R][8])
{
#pragma unroll
    for (int r = 0; r < R; ++r) widen_bf16x8(xv[r], t[r]);
}

// scale and inverse scale of the lane's 8 blocks for the sums t.
template <int R, int W>
__device__ __forceinline__ void strided_quotients(const float (&t)[R][8], ChunkMaxState &st, float (&scale)[8],
                                                  float (&inv)[8])
{
    uint32_t m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < R; ++r) note_absmax(t[r], m);
    across_chunks_max_wave<W>(m, st.red, st.parity);
#pragma unroll
    for (int j = 0; j < 8; ++j) block_quotients(__uint_as_float(m[j]), scale[j], inv[j]);
}

// The code of v as a float.  kPositiveZero: a value that rounds to zero from below gives +0.0, as the integer
// code converted back would (needed only where the sign of a zero sum can reach the output, i.e. when the
// all-gather is not quantized).
template <bool kPositiveZero>
__device__ __forceinline__ float code_of(float v, float inv)
{
    const float q = __builtin_rintf(v * inv);
    return kPositiveZero ? q + 0.0f : q;
}

// One hop: t <- fma(code(t), scale, x), what the device holding x has after it received the quantized t.
template <int R, int W, bool kPositiveZero>
__device__ __forceinline__ void strided_hop(float (&t)[R][8], const u32x4 (&xv)[R], ChunkMaxState &st)
{
    float scale[8], inv[8];
    strided_quotients<R, W>(t, st, scale, inv);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float xf[8];
        widen_bf16x8(xv[r], xf);
#pragma unroll
        for (int j = 0; j < 8; ++j) t[r][j] = __builtin_fmaf(code_of<kPositiveZero>(t[r][j], inv[j]), scale[j], xf[j]);
    }
}

// The send that ends a half chain of the semi-loop: acc <- fma(code(t), scale, acc).
template <int R, int W, bool kPositiveZero>
__device__ __forceinline__ void strided_send_into(const float (&t)[R][8], float (&acc)[R][8], ChunkMaxState &st)
{
    float scale[8], inv[8];
    strided_quotients<R, W>(t, st, scale, inv);
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[r][j] = __builtin_fmaf(code_of<kPositiveZero>(t[r][j], inv[j]), scale[j], acc[r][j]);
    }
}

// Waves per SIMD the compiler may plan for.  The full loop with a quantized reduce-scatter runs 3-4 us faster (of
// 63-75 at the 27B-shaped size) held to two waves than at the four its ~120 registers would allow: the loads of one
// partial per wave already fill the memory queues, and more waves only lengthen them.  The semi-loop (two dependent
// half chains) and the unquantized reduce-scatter measured the other way round and keep the default.
constexpr int strided_chain_waves(bool semi, bool rs) { return (!semi && rs) ? 2 : 8; }

// chunks = 8 * W * R.  kSemi: the semi-loop with partials[0] as the owner (always a quantized reduce-scatter);
// otherwise the full loop in array order with the reduce-scatter quantized (kRS) or added in plain fp32.  kAG: the
// finished sum is quantized once more and dequantized; otherwise narrowed to bf16 directly.
// Ring layout (Sec. 3): with per_shard > 0 the tensor is cut into shards of per_shard minishards and shard k ends
// on device k: the full loop takes the partials in the order k+1, k+2, ..., k (mod P), the semi-loop has device k
// as its owner and the devices k+1, k+2, ... around it.  per_shard == 0: array order everywhere.
template <int R, int W, bool kSemi, bool kRS, bool kAG>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, strided_chain_waves(kSemi, kRS))))
void chain_strided_kernel(const PartialTable tab, int P, int per_shard, uint16_t *out)
{
    static_assert(kRS || !kSemi, "the semi-loop is a quantized reduce-scatter");
    __shared__ __align__(16) uint32_t red[W > 1 ? 2 : 1][kThreads / 64][64];
    ChunkMaxState st{red, 0};
    constexpr int chunks = 8 * W * R;
    const WaveSpot sp = wave_spot<W>(chunks);
    // position i of the chain -> partial; `first` <= P and i < P, so one conditional subtraction wraps
    const int first = per_shard > 0 ? (int)(sp.minishard / per_shard) + (kSemi ? 0 : 1) : 0;
    const auto part = [&](int i) {
        const int j = first + i;
        return tab.x[j >= P ? j - P : j];
    };

    float sum[R][8];
    u32x4 xv[R];
    load_strided<R>(part(0), sp, xv);
    widen_strided<R>(xv, sum);
    if (kSemi) {
        const int h = P / 2;
        float t[R][8];
        if (h + 1 <= P - 1) {                       // h+1 -> h+2 -> ... -> P-1 -> owner: the shorter chain arrives first
            load_strided<R>(part(h + 1), sp, xv);
            widen_strided<R>(xv, t);
            for (int i = h + 2; i <= P - 1; ++i) {
                load_strided<R>(part(i), sp, xv);
                strided_hop<R, W, !kAG>(t, xv, st);
            }
            strided_send_into<R, W, !kAG>(t, sum, st);
        }
        if (h >= 1) {                               // h -> h-1 -> ... -> 1 -> owner
            load_strided<R>(part(h), sp, xv);
            widen_strided<R>(xv, t);
            for (int i = h - 1; i >= 1; --i) {
                load_strided<R>(part(i), sp, xv);
                strided_hop<R, W, !kAG>(t, xv, st);
            }
            strided_send_into<R, W, !kAG>(t, sum, st);
        }
    } else {
        for (int i = 1; i < P; ++i) {
            load_strided<R>(part(i), sp, xv);
            if (kRS) {
                strided_hop<R, W, !kAG>(sum, xv, st);
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    float xf[8];
                    widen_bf16x8(xv[r], xf);
#pragma unroll
                    for (int j = 0; j < 8; ++j) sum[r][j] = sum[r][j] + xf[j];
                }
            }
        }
    }

    float scale[8], inv[8];
    if (kAG) strided_quotients<R, W>(sum, st, scale, inv);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float d[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) d[j] = kAG ? code_of<true>(sum[r][j], inv[j]) * scale[j] : sum[r][j];
        u32x4 w;
        w.x = narrow_bf16x2(d[0], d[1]);
        w.y = narrow_bf16x2(d[2], d[3]);
        w.z = narrow_bf16x2(d[4], d[5]);
        w.w = narrow_bf16x2(d[6], d[7]);
        __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>(out + sp.elem + r * sp.row_step));
    }
}

// Dequantize in the strided geometry: element e uses scale (e / (1024*chunks)) * 1024 + e % 1024, so the 8
// elements of a lane use 8 consecutive scales.  n is a multiple of 1024, hence of the 2048-element tile.
template <int K>
__global__ __launch_bounds__(kThreads) void dequantize_strided_kernel(const int8_t *__restrict__ codes,
                                                                      const float *__restrict__ scales, int64_t n,
                                                                      int chunks, uint16_t *__restrict__ out)
{
    const int64_t wg_at = (int64_t)blockIdx.x * (kTileElems * K);
    const int lane_at = threadIdx.x * kLaneElems;
    const int64_t minishard = (int64_t)kChunk * chunks;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t at = wg_at + k * kTileElems + lane_at;
        if (at >= n) continue;                       // n % 8 == 0: a lane is inside or outside as a whole
        const u32x2 cv = *reinterpret_cast<const u32x2 *>(codes + at);
        const float *s = scales + (at / minishard) * kChunk + at % kChunk;
        const u32x4 a = *reinterpret_cast<const u32x4 *>(s);
        const u32x4 b = *reinterpret_cast<const u32x4 *>(s + 4);
        float qf[8];
        widen_i8x8(cv, qf);
        u32x4 w;
        w.x = narrow_bf16x2(qf[0] * __uint_as_float(a.x), qf[1] * __uint_as_float(a.y));
        w.y = narrow_bf16x2(qf[2] * __uint_as_float(a.z), qf[3] * __uint_as_float(a.w));
        w.z = narrow_bf16x2(qf[4] * __uint_as_float(b.x), qf[5] * __uint_as_float(b.y));
        w.w = narrow_bf16x2(qf[6] * __uint_as_float(b.z), qf[7] * __uint_as_float(b.w));
        __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>(out + at));
    }
}

}  // namespace equarx
