/*
 * Developer aids of libequarx: calibration kernels, self-tests of the kernels'
 * arithmetic shortcuts, and profiling hooks.  Exported by the same shared
 * library as the method's entry points (equarx.h) and following the same
 * conventions (device pointers, stream as void*, equarx_status return values),
 * but not part of the method: a caller that reduces tensors needs none of them.
 * The benchmark and the test suite do.
 */
#ifndef EQUARX_DEVTOOLS_H
#define EQUARX_DEVTOOLS_H

#include "equarx.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Plain 16-byte-vector device copy of `bytes` bytes (a multiple of 16, both
 * pointers 16-byte aligned): the calibration kernel the benchmark uses to
 * find the HBM bandwidth a streaming kernel can reach on this device. */
int equarx_calib_copy(const void *src, void *dst, size_t bytes, void *stream);

/* `count` launches (0 .. 4096), back to back on `stream`, of a kernel of
 * `workgroups` 256-thread workgroups that does nothing: what a launch costs on
 * this device before it moves a byte (the benchmark reports the pitch of such
 * launches beside the kernels' durations). */
int equarx_calib_empty_launches(int32_t count, int32_t workgroups, void *stream);

/* The chain's hops as memory traffic only: P-1 launches of a kernel with
 * exactly the loads and stores of equarx_reduce_stage (same tiling, same
 * access widths, the same ping-pong between two wire buffers, partial i read by
 * launch i) whose only computation is an XOR -- the time the memory system
 * alone needs for a hop, which the benchmark sets beside the hop kernel's.
 * n must be a multiple of block.  (codes0, scales0) is the input of launch 1,
 * which writes (codes1, scales1); launch 2 reads those and writes buffer 0,
 * and so on.  Per launch and per 8 consecutive elements (the partial as four
 * little-endian 32-bit words X0..X3, the codes read as two words C0, C1):
 * codes written = (X0^X2^C0, X1^X3^C1); scales written = scales read. */
int equarx_calib_hop_traffic(const void *const *partials_bf16, int32_t P, int64_t n, int32_t block,
                             int8_t *codes0, float *scales0, int8_t *codes1, float *scales1, void *stream);

/*
 * M independent hop-by-hop reductions of the same shape, their launches
 * interleaved pass by pass: pass 0 of chains 0 .. M-1, then pass 1 of chains
 * 0 .. M-1, and so on (launch number pass * M + m).  Each chain is exactly
 * equarx_reduce_quantized on its own inputs, workspace and output -- same
 * kernels, same bits -- but every wire is read M-1 launches after it was
 * written, so that with M large enough it no longer sits in a cache when the
 * next hop reads it: the benchmark's stand-in for a wire that arrives from
 * another device instead of from the previous launch.
 *
 *   partials_bf16   HOST array of M*P device pointers; chain m's partial i
 *                   is entry m*P + i.
 *   out_bf16        HOST array of M device pointers, bf16 [n] each; not in place.
 *   workspaces      HOST array of M device pointers, each to workspace_bytes
 *                   >= equarx_workspace_bytes(P, n, block) bytes, 256-byte aligned.
 *   streaming       0: the wire is accessed as the chain entry points access
 *                   it (cacheable); non-zero: as the per-step entry points do
 *                   (non-temporal hints).
 *   1 <= M <= EQUARX_CALIB_MAX_CHAINS.  No output or workspace may overlap
 *   any other buffer of the call.
 */
#define EQUARX_CALIB_MAX_CHAINS 64
int equarx_calib_interleaved_chains(const void *const *partials_bf16, int32_t M, int32_t P, int64_t n, int32_t block,
                                    void *const *out_bf16, void *const *workspaces, size_t workspace_bytes,
                                    int32_t streaming, void *stream);

/*
 * Self-tests of the kernels' arithmetic (used by the test suite).
 *
 * The quantizer needs, per block, scale = fl32(absmax / 127) and
 * inv = fl32(127 / absmax), correctly rounded (Sec. 3.2 leaves the formula
 * open; these are the readings the library documents).  The kernels compute
 * them with short reciprocal-based sequences instead of a full IEEE division.
 *
 * equarx_selftest_quotients compares those sequences with the IEEE division on
 * the device for the `count` consecutive fp32 bit patterns starting at
 * first_bits (positive, finite: first_bits + count <= 0x7F800000) and ADDS the
 * number of differing scales to mismatches[0] and of differing reciprocals to
 * mismatches[1] (device pointer, two uint64, zeroed by the caller).
 *
 * equarx_eval_quotients evaluates them for n caller-given values (device
 * arrays absmax[n] -> scale[n], inv[n]) so that a host can compare them with
 * its own division.
 */
int equarx_selftest_quotients(uint32_t first_bits, uint64_t count, uint64_t *mismatches, void *stream);

/* The kernels take the int8 code of a scaled value p (|p| <= 127 up to
 * rounding) from the low byte of fl32(p + 1.5 * 2^23) instead of rounding,
 * converting and masking.  This compares the two, for +p and -p, over `count`
 * consecutive fp32 bit patterns of |p| from first_bits (first_bits + count <=
 * 0x43000000, i.e. |p| < 128) and adds the number of differences to
 * mismatches[0] (device pointer, one uint64, zeroed by the caller). */
int equarx_selftest_rounding(uint32_t first_bits, uint64_t count, uint64_t *mismatches, void *stream);
int equarx_eval_quotients(const float *absmax, int64_t n, float *scale, float *inv, void *stream);

/*
 * Profiling hooks.  Each arms the calling thread's NEXT call of an entry point
 * of this library (equarx.h or this header) and nothing after it: that call
 * takes the setting over when it starts and drops it when it returns, whether
 * it launched kernels, had nothing to do (n == 0) or failed validation.  The
 * library's entry points themselves stay stateless; a caller that never uses
 * these hooks is never affected by them.  Event handles are hipEvent_t passed
 * as void*, created by the caller with timing enabled.
 *
 * equarx_time_next_launch: the FIRST kernel that call launches carries the two
 * events: after the stream has been synchronised, hipEventElapsedTime(start,
 * stop) is that one kernel's execution time.  Either handle may be NULL.  Meant
 * for kernels that run alone (a launch that carries events is dispatched
 * differently from one that does not).
 *
 * equarx_time_launch_span: counting that call's launches from 0, `start_event`
 * is recorded on the stream (hipEventRecord) just before launch `first` and
 * `stop_event` just after launch `last` (last >= first >= 0): the elapsed time
 * is that of launches first..last back to back, with nothing attached to the
 * kernels themselves.  E.g. hops 1..P-1 of equarx_reduce_quantized are its
 * launches 1..P-1.  Invalid arguments cancel a pending span.
 *
 * equarx_time_cancel: drops whatever is pending on the calling thread.
 */
void equarx_time_next_launch(void *start_event, void *stop_event);
void equarx_time_launch_span(int32_t first, int32_t last, void *start_event, void *stop_event);
void equarx_time_cancel(void);

#ifdef __cplusplus
}
#endif

#endif /* EQUARX_DEVTOOLS_H */
