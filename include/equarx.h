/*
 * libequarx -- block-wise int8 quantized P-way reduction on one MI355X (gfx950).
 *
 * The compute path of EQuARX (arXiv 2506.17615): what each device does to the
 * data of a quantized AllReduce, with the inter-chip transfers replaced by
 * reads of buffers that live in the same GPU's HBM.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HBM of the current device) unless
 *     a parameter says HOST.  The caller owns every buffer; the library never
 *     allocates, frees or keeps a pointer after the call returns.
 *   - bf16 tensors are raw 16-bit patterns (upper half of an IEEE binary32).
 *   - A tensor of n elements is flat and contiguous.  Block b covers elements
 *     [b*block, min(n, (b+1)*block)); nb = ceil(n / block) blocks.  For a
 *     [rows, hidden] activation with hidden % block == 0, blocks run along
 *     hidden and never straddle rows.
 *   - codes: int8 [n], values in [-127, 127].  scales: fp32 [nb].
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it; no entry point synchronises.
 *   - Return value: an equarx_status.  A call that fails validation launches
 *     nothing and touches no memory.  n == 0 is valid and does nothing;
 *     n above 2^40 is EQUARX_BAD_SHAPE.  EQUARX_DEVICE_ERROR reports what the
 *     call's own kernel launches returned (a chain stops launching at the
 *     first failure); an error some earlier HIP call left pending on the
 *     thread is neither reported nor cleared.
 *   - Sharing memory between the buffers of one call: a buffer the call
 *     WRITES (an output, the workspace, a kept wire) may not overlap any other
 *     buffer of the call, not even partly -- EQUARX_BAD_SHAPE -- except where
 *     an entry point says that an output may BE an input; the two must then
 *     coincide exactly.  Buffers that are only read may overlap freely.
 *   - The library keeps no state between calls (the one exception, the static
 *     array of equarx_reduce_quantized_static, is described there) and may be
 *     called from several threads at once (on different streams, or on one).
 *   - Pointers must be 16-byte aligned (8-byte for codes, 4 for scales is not
 *     enough: every data pointer is checked against 16).
 *   - Supported block sizes: 32, 64, 128, 256, 512.
 *   - equarx_quantize, equarx_reduce_stage and equarx_dequantize are the calls
 *     one device of a ring makes per step, equarx_quantize_batch and
 *     equarx_reduce_flat the calls around an all-to-all: the wire they read
 *     arrived from another device and the wire they write leaves for one, so
 *     they access it with non-temporal hints (read once; not read here again).  The chain
 *     entry points run every step on this device and keep the wire cacheable
 *     for the next launch.  Same results either way; a chain composed by hand
 *     from the per-step calls on one device is a few percent slower than
 *     equarx_reduce_quantized.
 *   - NaN or infinite inputs give unspecified codes/scales but never a fault.
 */
#ifndef EQUARX_H
#define EQUARX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum equarx_status {
    EQUARX_OK = 0,
    EQUARX_NULL_POINTER = 1,        /* a required pointer is NULL */
    EQUARX_BAD_SHAPE = 2,           /* n < 0, P < 1, P > EQUARX_MAX_PARTIALS, or overlap that is not allowed */
    EQUARX_BAD_BLOCK = 3,           /* block not in {32, 64, 128, 256, 512} */
    EQUARX_MISALIGNED = 4,          /* a data pointer is not 16-byte aligned */
    EQUARX_WORKSPACE_TOO_SMALL = 5, /* workspace_bytes (or the static array) < what the call needs */
    EQUARX_DEVICE_ERROR = 6         /* a kernel launch of this call returned a HIP error */
} equarx_status;

#define EQUARX_MAX_PARTIALS 64

/*
 * Quantize a bf16 tensor block-wise to int8 (Sec. 3.2: symmetric, scale-only
 * quantization whose scale comes from a max-abs reduction; Sec. 3.1: the
 * first step of the reduce-scatter quantizes the shard before sending it).
 *
 * Per block: absmax = max |x|; scale = absmax / 127; codes =
 * rne(x * (127 / absmax)) (round to nearest, ties to even), both quotients
 * correctly rounded fp32.  absmax < 127 * 2^-126 gives scale 0, codes 0.
 *
 *   x_bf16 [n] in, codes [n] out, scales [nb] out.
 */
int equarx_quantize(const void *x_bf16, int64_t n, int32_t block,
                    int8_t *codes, float *scales, void *stream);

/*
 * equarx_quantize on `count` tensors of the same length n in one launch: what a
 * device does before an all-to-all reduce-scatter, when it quantizes one shard
 * per peer (see equarx_reduce_flat).  Tensor i: x_bf16[i] -> codes[i], scales[i].
 *
 *   x_bf16, codes, scales   HOST arrays of `count` device pointers
 *                           (0 <= count <= EQUARX_MAX_PARTIALS), read before
 *                           the call returns; no output may overlap another
 *                           output or any input (EQUARX_BAD_SHAPE).
 */
int equarx_quantize_batch(const void *const *x_bf16, int8_t *const *codes, float *const *scales, int32_t count,
                          int64_t n, int32_t block, void *stream);

/*
 * Dequantize int8 codes to bf16 (Sec. 3.4: the dequantize that ends a
 * quantized all-gather).  out = bf16_rne(fp32(code) * scale[block of the
 * element]).
 *
 *   codes [n] in, scales [nb] in, out_bf16 [n] out.
 */
int equarx_dequantize(const int8_t *codes, const float *scales, int64_t n, int32_t block,
                      void *out_bf16, void *stream);

/*
 * One reduce-scatter step as the receiving device performs it (Sec. 3 and
 * 3.1): dequantize the received shard to fp32, add the local -- unquantized --
 * bf16 shard, quantize the partial sum for the next send.
 *
 *   t = fma(fp32(codes_in), scales_in[block], fp32(local))   (one rounding)
 *   (codes_out, scales_out) = quantize(t) as in equarx_quantize.
 *
 * codes_out may BE codes_in and scales_out may BE scales_in (each block is read
 * completely before it is written); any other overlap between what the call
 * writes and its other buffers is EQUARX_BAD_SHAPE.
 */
int equarx_reduce_stage(const int8_t *codes_in, const float *scales_in, const void *local_bf16,
                        int64_t n, int32_t block,
                        int8_t *codes_out, float *scales_out, void *stream);

/*
 * The whole adder chain of the full-loop variant with reduce-scatter and
 * all-gather both quantized (Sec. 3.3 full-loop, Sec. 3.4), hop by hop:
 *
 *   (c0, s0) = quantize(x_0)
 *   (ci, si) = reduce_stage(c(i-1), s(i-1), x_i)      i = 1 .. P-1
 *   out      = dequantize(c(P-1), s(P-1))
 *
 * One kernel per line, P+1 launches; every wire buffer (ci, si) is written
 * once and read once.  P == 1 gives out = dequantize(quantize(x_0)).
 *
 *   partials_bf16   HOST array of P device pointers, each to n bf16 values,
 *                   in chain order; read before the call returns.
 *   out_bf16 [n]    device.  May BE one of the partials (in-place reduction,
 *                   as an AllReduce is usually called): every element of
 *                   every partial is read before the output element is
 *                   written.  An output that overlaps a partial without
 *                   coinciding with it is rejected (EQUARX_BAD_SHAPE).  The
 *                   same holds for every chain entry point below.
 *   workspace       device, at least equarx_workspace_bytes(P, n, block)
 *                   bytes, 256-byte aligned; holds the two ping-pong wire
 *                   buffers.  Not needed (may be NULL) when both wire_* are given.
 *   wire_codes      NULL, or device int8 [P][equarx_wire_row_codes(n)]:
 *                   receives the codes on the wire after every quantization
 *                   (row i = c_i in its first n entries; rows are padded so
 *                   that each starts 16-byte aligned).
 *   wire_scales     NULL, or device fp32 [P][equarx_wire_row_scales(n, block)],
 *                   row i = s_i in its first nb entries; must be given
 *                   together with wire_codes.
 */
int equarx_reduce_quantized(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                            void *out_bf16, void *workspace, size_t workspace_bytes,
                            int8_t *wire_codes, float *wire_scales, void *stream);

/*
 * equarx_reduce_quantized for callers that cannot allocate device memory and
 * have no workspace to hand in: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same kernels, same P+1 launches,
 * same bits; the two ping-pong wire buffers live in a static device array of
 * EQUARX_STATIC_WORKSPACE_BYTES that each GPU the library runs on holds from
 * the moment the library is loaded there until the process ends.  The call
 * allocates and frees nothing, on the device or through any library.
 *
 *   - equarx_workspace_bytes(P, n, block) above EQUARX_STATIC_WORKSPACE_BYTES
 *     is EQUARX_WORKSPACE_TOO_SMALL (80 MiB covers a 64 MiB bf16 message,
 *     32 Mi elements, at block 32: 72 MiB; larger blocks need less).
 *   - The first call on a GPU looks the array's address up
 *     (hipGetSymbolAddress; EQUARX_DEVICE_ERROR if that fails); make it
 *     outside a graph capture.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels
 *     may run at the same time (different streams, different threads) RACE
 *     on it.  Calls on one stream, or ordered by events, are safe; nothing in
 *     the array needs clearing between calls, whatever their sizes.
 * Other arguments as for equarx_reduce_quantized, without the kept wire.
 */
#define EQUARX_STATIC_WORKSPACE_BYTES (80u << 20)
int equarx_reduce_quantized_static(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                                   void *out_bf16, void *stream);

/*
 * The same hop-by-hop chain with its two ends fused: the first launch
 * quantizes partial 0 in registers and performs hop 1, the last launch performs
 * hop P-1 and the quantize/dequantize pair of the quantized all-gather
 * (Sec. 3.1, 3.4), so c_0 and c_(P-1) never reach memory: P-1 launches instead
 * of P+1, P-2 wire buffers written and read instead of P.  Same operations in
 * the same order, hence the same bits as equarx_reduce_quantized.  P <= 2 is a
 * single launch and ignores the workspace (which may then be NULL).
 *
 * Arguments as for equarx_reduce_quantized, without the optional kept wire.
 */
int equarx_reduce_quantized_fused_ends(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                                       void *out_bf16, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same adder chain (Sec. 3.3 full-loop, Sec. 3.4) in ONE launch.  Blocks
 * do not interact, so every workgroup runs all hops on its own tiles with the
 * running codes and scale in registers: same operations, same order, same
 * bits as equarx_reduce_quantized.  Each partial is read once; nothing
 * intermediate is written unless the wire arrays are given, and the wire is
 * never read back.  Needs no workspace.  On a single device this removes the
 * P+1 launches and the 2(P-1) wire passes of the hop-by-hop schedule; it is
 * not what a multi-device ring can do (there every hop's wire really crosses
 * a link), which is why it is a separate entry point.
 *
 * Arguments as for equarx_reduce_quantized (wire_codes / wire_scales optional,
 * same padded row layout).
 */
int equarx_reduce_fused(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                        void *out_bf16, int8_t *wire_codes, float *wire_scales, void *stream);

/*
 * Variants of the chain, each in one launch (no wire kept).  `flags` is a
 * combination of:
 *
 *   EQUARX_SEMI_LOOP       the semi-loop reduce-scatter of Sec. 3.3 instead of
 *                          the full loop: partials[0] owns the result, the
 *                          other partials follow in ring order around it; with
 *                          h = P/2 the chains h+1 -> h+2 -> ... -> P-1 and
 *                          h -> h-1 -> ... -> 1 each end in a quantized send to
 *                          the owner, which adds them to its own fp32 shard
 *                          (the shorter chain first).  Fewer requantizations
 *                          of smaller partial sums: lower error.
 *   EQUARX_RS_UNQUANTIZED  the stage knob of Sec. 3.4: the reduce-scatter adds
 *                          in plain fp32 (array order), only the all-gather
 *                          is quantized.  Not combinable with SEMI_LOOP.
 *   EQUARX_AG_UNQUANTIZED  the all-gather is not quantized: the owner's fp32
 *                          sum (last received wire dequantized + own shard)
 *                          is narrowed to bf16 directly.  Setting both
 *                          *_UNQUANTIZED flags is EQUARX_BAD_SHAPE.
 *   EQUARX_RING_ORDER      lay the reduction out as a ring does (Sec. 3): the
 *                          tensor is cut into P shards of ceil(nb/P) blocks,
 *                          shard k ends on device k and is reduced in the
 *                          order k+1, k+2, ..., k (full loop) or with device k
 *                          as the semi-loop owner and k+1, k+2, ... around it.
 *                          Without the flag every element uses array order.
 *
 * flags == 0 is equarx_reduce_fused without kept wire.  Other arguments as for
 * equarx_reduce_fused.
 */
#define EQUARX_SEMI_LOOP 1u
#define EQUARX_RS_UNQUANTIZED 2u
#define EQUARX_AG_UNQUANTIZED 4u
#define EQUARX_RING_ORDER 8u
int equarx_reduce_variant(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block, uint32_t flags,
                          void *out_bf16, void *stream);

/*
 * Variants of the chain in the schedule a ring imposes: one launch per hop,
 * every hop's wire written to memory once and read once (the single-launch
 * forms above keep it in registers).  Same bits as equarx_reduce_variant with
 * the same flags.
 *
 *   flags   any of EQUARX_AG_UNQUANTIZED, EQUARX_SEMI_LOOP, EQUARX_RING_ORDER.
 *           EQUARX_RS_UNQUANTIZED is rejected (EQUARX_BAD_SHAPE): without a
 *           quantized reduce-scatter there is no wire to write.
 *           full loop: Q_B(x_0), hops 1 .. P-2, and a last launch that performs
 *           hop P-1 and either the all-gather's quantize/dequantize pair or
 *           (EQUARX_AG_UNQUANTIZED) the narrowing to bf16: P launches.
 *           full loop with EQUARX_RING_ORDER: the same P launches, each of them
 *           one step of the ring on all P shards at once -- in step i, shard k
 *           takes the partial of device (k + 1 + i) mod P.
 *           semi-loop (Sec. 3.3): the two half chains hop by hop, then one
 *           launch in which the owner (partials[0]) adds the two received wires
 *           to its own shard, counter-clockwise first: P launches.
 *           semi-loop with EQUARX_RING_ORDER: P/2 launches, each of them one
 *           iteration of the ring's semi-loop on all P shards -- both chains
 *           of every shard advance one device per launch, as both directions
 *           of a ring do -- then the owners' launch: P/2 + 1 launches.
 *   workspace  equarx_variant_workspace_bytes(flags, P, n, block) bytes, 256-byte
 *           aligned (the semi-loop keeps one chain's last wire while the other
 *           chain runs: three wire buffers instead of two; in ring order each
 *           direction ping-pongs between two of its own: four).
 * Other arguments as for equarx_reduce_quantized (out_bf16 may be a partial).
 */
int equarx_reduce_variant_hops(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                               uint32_t flags, void *out_bf16, void *workspace, size_t workspace_bytes,
                               void *stream);
size_t equarx_variant_workspace_bytes(uint32_t flags, int32_t P, int64_t n, int32_t block);

/*
 * Flat one-shot reduce: the reduce-scatter done as an all-to-all followed by
 * a local reduction (the decomposition Sec. 2 describes for ZeRO++; on a full
 * xGMI mesh, where a ring is bound by one link of seven, it is the natural
 * shape).  Every other device has quantized its shard ONCE with
 * equarx_quantize; the owner holds its own bf16 shard and the R received
 * (codes, scales) pairs and computes
 *
 *   acc = fp32(local);  acc = fma(fp32(codes[r]), scales[r][block], acc)  r = 0 .. R-1, in array order
 *   (codes_out, scales_out) = quantize(acc)         what the all-gather carries (Sec. 3.4)
 *   out = bf16(fp32(codes_out) * scales_out[block])
 *
 * Two quantizations per value instead of the ring's P.
 *
 *   local_bf16 [n]     device.
 *   codes, scales      HOST arrays of R device pointers (int8 [n] / fp32 [nb]
 *                      each); 0 <= R < EQUARX_MAX_PARTIALS; read before return.
 *   out_bf16 [n]       device or NULL.
 *   codes_out [n], scales_out [nb]   device or both NULL; at least one of
 *                      out_bf16 and the (codes_out, scales_out) pair must be given.
 * No output may overlap an input or another output (EQUARX_BAD_SHAPE).
 */
int equarx_reduce_flat(const void *local_bf16, const int8_t *const *codes, const float *const *scales, int32_t R,
                       int64_t n, int32_t block, void *out_bf16, int8_t *codes_out, float *scales_out,
                       void *stream);

/*
 * The paper's own block geometry (Sec. 3.2, "VPU-friendly" quantization).
 *
 * The tensor is a sequence of chunks of 1024 elements (8 x 128, the TPU vector
 * register, contiguous in its tiled layout); a minishard is `chunks`
 * consecutive chunks and gets 1024 scales: scale j of a minishard comes from
 * the max-abs over position j of each of its chunks, so a quantization block
 * is the `chunks` elements  m*1024*chunks + c*1024 + j,  c = 0 .. chunks-1,
 * and its scale is scales[m*1024 + j].  (The paper's example: a shard of 64
 * chunks, 1024 scales, block size 64; with m minishards per shard, 64/m.)
 * Arithmetic exactly as in the contiguous entry points of the same name; only
 * the element -> block map differs.
 *
 *   chunks   32, 64 or 128 (else EQUARX_BAD_BLOCK); n must be a multiple of
 *            1024 * chunks (else EQUARX_BAD_SHAPE).  scales has n / chunks entries.
 *   equarx_reduce_quantized_strided: the hop-by-hop chain (P+1 launches);
 *            workspace of equarx_workspace_bytes(P, n, chunks) bytes, 256-byte aligned.
 *   equarx_reduce_stage_strided: codes_out / scales_out may BE codes_in / scales_in.
 *   equarx_reduce_fused_strided: the same chain in one launch (running sums in
 *            registers, no wire traffic, no workspace); same bits.
 *   equarx_reduce_variant_strided: the flavours of Sec. 3.3 / 3.4 in this
 *            geometry, one launch each: flags as for equarx_reduce_variant
 *            (EQUARX_SEMI_LOOP with partials[0] as the owner,
 *            EQUARX_RS_UNQUANTIZED, EQUARX_AG_UNQUANTIZED, same forbidden
 *            combinations).  EQUARX_RING_ORDER cuts the tensor into P shards
 *            of ceil(M/P) whole minishards (M = n / (1024 * chunks); a
 *            device's shard is what the paper cuts into minishards), shard k
 *            ending on device k as in equarx_reduce_variant.  flags == 0 gives
 *            the bits of equarx_reduce_fused_strided.  out_bf16 may BE one of
 *            the partials.
 *   equarx_reduce_variant_hops_strided: the same flavours hop by hop, one launch
 *            per send as a ring imposes (the paper's own setting: ring
 *            schedule, strided blocks): flags EQUARX_SEMI_LOOP,
 *            EQUARX_AG_UNQUANTIZED, EQUARX_RING_ORDER (anything else
 *            EQUARX_BAD_SHAPE); P launches for the full loop (one when
 *            P == 1), P/2 + 1 for the semi-loop (its two chains advance in
 *            the same launch), each of them in ring order one ring step on
 *            all P shards at once; workspace of
 *            equarx_variant_workspace_bytes(flags without EQUARX_RING_ORDER,
 *            P, n, chunks) bytes, 256-byte aligned (two wire buffers, three
 *            for the semi-loop); same bits as the single launch.
 */
int equarx_quantize_strided(const void *x_bf16, int64_t n, int32_t chunks,
                            int8_t *codes, float *scales, void *stream);
int equarx_dequantize_strided(const int8_t *codes, const float *scales, int64_t n, int32_t chunks,
                              void *out_bf16, void *stream);
int equarx_reduce_stage_strided(const int8_t *codes_in, const float *scales_in, const void *local_bf16,
                                int64_t n, int32_t chunks,
                                int8_t *codes_out, float *scales_out, void *stream);
int equarx_reduce_quantized_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks,
                                    void *out_bf16, void *workspace, size_t workspace_bytes, void *stream);
int equarx_reduce_fused_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks,
                                void *out_bf16, void *stream);
int equarx_reduce_variant_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks,
                                  uint32_t flags, void *out_bf16, void *stream);
int equarx_reduce_variant_hops_strided(const void *const *partials_bf16, int32_t P, int64_t n, int32_t chunks,
                                       uint32_t flags, void *out_bf16, void *workspace, size_t workspace_bytes,
                                       void *stream);

/* Bytes of workspace equarx_reduce_quantized needs (0 for invalid arguments). */
size_t equarx_workspace_bytes(int32_t P, int64_t n, int32_t block);

/* Number of blocks, ceil(n / block) (0 for invalid arguments). */
int64_t equarx_num_blocks(int64_t n, int32_t block);

/* Row lengths (in elements) of the optional wire_codes / wire_scales arrays:
 * n and nb rounded up to a multiple of 16 bytes. */
int64_t equarx_wire_row_codes(int64_t n);
int64_t equarx_wire_row_scales(int64_t n, int32_t block);

/* Static, NUL-terminated description of a status code. */
const char *equarx_status_string(int status);

#ifdef __cplusplus
}
#endif

#endif /* EQUARX_H */
