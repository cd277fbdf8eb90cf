/*
 * EQuARX reference oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar CPU statement of what the quantized P-way reduction
 * computes.  It exists so that the HIP library can be checked against it; it
 * is not a fallback.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.  It shares no code, header, table or helper
 * with the HIP path.
 *
 * What it follows (EQuARX, arXiv 2506.17615):
 *   - Sec. 3 (ring reduce-scatter): a device adds the shard it received to its
 *     own, unquantized, counterpart and forwards the partial sum.
 *   - Sec. 3.1: what crosses the wire is quantized (codes + scale metadata);
 *     the receiver dequantizes to FP32, adds, and the step repeats N-1 times.
 *   - Sec. 3.2: symmetric (scale-only) block-wise quantization, the scale
 *     coming from a max-abs reduction over the block.
 *   - Sec. 3.3, full-loop variant: the adder chain is linear.
 *   - Sec. 3.4: quantizing the all-gather appends one more quantize /
 *     dequantize pair to the chain.
 *
 * Readings the paper leaves open (fixed here, listed in the design notes):
 *   block = B consecutive elements (the last block may be shorter);
 *   int8 codes in [-127, 127]; round-to-nearest-even; one fp32 scale per
 *   block, scale = absmax / 127; code = rne(fl32(v * fl32(127 / absmax)));
 *   absmax < 127 * 2^-126 gives scale 0 and all codes 0; dequantize-and-add
 *   is one fused multiply-add (single rounding); accumulation in fp32;
 *   chain order = order of the partials array.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math [-fopenmp] -shared -fPIC
 * Every floating-point operation below is meant to round exactly once, in
 * IEEE binary32 round-to-nearest-even; -ffp-contract=off keeps the compiler
 * from fusing the multiplies and adds that are written separately.
 *
 * Parity pins: every exported function is pinned by tests that do not call it
 * to produce their expected values (closed forms, exact rational arithmetic
 * on small inputs, the error bound of the method, a library bf16 cast, and
 * the error figures of the paper's Fig. 7).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of host threads the block loops use (1 = serial). Blocks are
 * independent, so threading never changes a bit of the result. */
void equarx_oracle_set_threads(int threads)
{
    g_threads = threads < 1 ? 1 : threads;
}

int equarx_oracle_get_threads(void)
{
#ifdef _OPENMP
    return g_threads;
#else
    return 1;
#endif
}

int equarx_oracle_has_openmp(void)
{
#ifdef _OPENMP
    return 1;
#else
    return 0;
#endif
}

/* ---- bf16 <-> fp32 ------------------------------------------------------ */

/* bf16 is the upper half of a binary32 pattern: widening is exact. */
static float widen_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Narrow binary32 to bf16, round-to-nearest, ties to even.  The 16 dropped
 * bits are compared with one half of the kept unit; the carry of a round-up
 * runs into the exponent, which is what IEEE rounding requires (the largest
 * finite values round up to infinity). */
static uint16_t narrow_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if (f != f) {                       /* NaN: keep it a (quiet) NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    }
    uint32_t keep = u >> 16;
    uint32_t drop = u & 0xFFFFu;
    if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) {
        keep += 1u;
    }
    return (uint16_t)keep;
}

void equarx_oracle_bf16_to_f32(const uint16_t *x, int64_t n, float *out)
{
    for (int64_t j = 0; j < n; ++j) out[j] = widen_bf16(x[j]);
}

void equarx_oracle_f32_to_bf16(const float *v, int64_t n, uint16_t *out)
{
    for (int64_t j = 0; j < n; ++j) out[j] = narrow_bf16_rne(v[j]);
}

/* ---- Q_B: block-wise symmetric int8 quantizer (Sec. 3.2) ------------------ */

/* Quantize one block of `len` fp32 values: the scale comes from the block's
 * max-abs; every value is multiplied by the reciprocal scale and rounded to
 * the nearest integer, ties to even. */
static void quantize_block(const float *v, int64_t len, int8_t *code, float *scale_out)
{
    float a = 0.0f;
    for (int64_t j = 0; j < len; ++j) {
        float m = fabsf(v[j]);
        if (m > a) a = m;
    }

    float scale, inv;
    if (a < 127.0f * FLT_MIN) {         /* all-zero (or vanishing) block */
        scale = 0.0f;
        inv = 0.0f;
    } else {
        scale = a / 127.0f;
        inv = 127.0f / a;
    }
    *scale_out = scale;

    for (int64_t j = 0; j < len; ++j) {
        float r = v[j] * inv;           /* rounds once to fp32 */
        r = nearbyintf(r);              /* default mode: to nearest, ties to even */
        if (r > 127.0f) r = 127.0f;
        if (r < -127.0f) r = -127.0f;
        if (r != r) r = 0.0f;           /* NaN input: result unspecified, keep the cast defined */
        code[j] = (int8_t)(int)r;
    }
}

static int64_t block_count(int64_t n, int32_t B)
{
    return (n + B - 1) / B;
}

static int64_t block_len(int64_t n, int32_t B, int64_t b)
{
    int64_t start = b * (int64_t)B;
    int64_t len = n - start;
    return len < B ? len : B;
}

/* Q_B over an fp32 tensor. codes[n], scales[ceil(n/B)]. */
void equarx_oracle_quantize_f32(const float *v, int64_t n, int32_t B, int8_t *codes, float *scales)
{
    int64_t nb = block_count(n, B);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        quantize_block(v + b * (int64_t)B, block_len(n, B, b), codes + b * (int64_t)B, scales + b);
    }
}

/* Q_B over a bf16 tensor (the first element of the chain quantizes the raw
 * shard before it is sent, Sec. 3.1). */
void equarx_oracle_quantize_bf16(const uint16_t *x, int64_t n, int32_t B, int8_t *codes, float *scales)
{
    int64_t nb = block_count(n, B);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        int64_t len = block_len(n, B, b);
        float *v = (float *)malloc((size_t)len * sizeof(float));
        for (int64_t j = 0; j < len; ++j) v[j] = widen_bf16(x[b * (int64_t)B + j]);
        quantize_block(v, len, codes + b * (int64_t)B, scales + b);
        free(v);
    }
}

/* ---- Dq: int8 -> fp32 (Sec. 3.1) ------------------------------------------ */

void equarx_oracle_dequantize_f32(const int8_t *codes, const float *scales, int64_t n, int32_t B, float *out)
{
    for (int64_t j = 0; j < n; ++j) {
        out[j] = (float)codes[j] * scales[j / B];
    }
}

/* Final dequantize of the quantized all-gather (Sec. 3.4): the fp32 product
 * is narrowed to bf16, the tensor's own type. */
void equarx_oracle_dequantize_bf16(const int8_t *codes, const float *scales, int64_t n, int32_t B, uint16_t *out)
{
    for (int64_t j = 0; j < n; ++j) {
        float d = (float)codes[j] * scales[j / B];
        out[j] = narrow_bf16_rne(d);
    }
}

/* ---- one reduce-scatter step on the receiving device (Sec. 3, 3.1) -------- */

/* The received (codes_in, scales_in) are dequantized and added to the local,
 * unquantized bf16 shard in fp32 -- one fused multiply-add per element -- and
 * the partial sum is quantized again for the next send. */
void equarx_oracle_hop(const int8_t *codes_in, const float *scales_in, const uint16_t *local,
                       int64_t n, int32_t B, int8_t *codes_out, float *scales_out)
{
    int64_t nb = block_count(n, B);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        int64_t len = block_len(n, B, b);
        int64_t at = b * (int64_t)B;
        float *t = (float *)malloc((size_t)len * sizeof(float));
        for (int64_t j = 0; j < len; ++j) {
            t[j] = fmaf((float)codes_in[at + j], scales_in[b], widen_bf16(local[at + j]));
        }
        quantize_block(t, len, codes_out + at, scales_out + b);
        free(t);
    }
}

/* ---- the whole adder chain (Sec. 3.3 full-loop, Sec. 3.4) ------------------ */

/* partials[0..P-1] in chain order, each n bf16 values.  out[n] bf16.
 * If wire_codes / wire_scales are non-NULL they receive what is on the wire
 * after every quantization: wire_codes[i*n + j], wire_scales[i*nb + b],
 * i = 0..P-1 (i = P-1 is what the all-gather carries). */
void equarx_oracle_reduce_chain(const uint16_t *const *partials, int32_t P, int64_t n, int32_t B,
                                uint16_t *out, int8_t *wire_codes, float *wire_scales)
{
    int64_t nb = block_count(n, B);
    int8_t *c_prev = (int8_t *)malloc((size_t)(n > 0 ? n : 1));
    int8_t *c_next = (int8_t *)malloc((size_t)(n > 0 ? n : 1));
    float *s_prev = (float *)malloc((size_t)(nb > 0 ? nb : 1) * sizeof(float));
    float *s_next = (float *)malloc((size_t)(nb > 0 ? nb : 1) * sizeof(float));

    equarx_oracle_quantize_bf16(partials[0], n, B, c_prev, s_prev);
    if (wire_codes) memcpy(wire_codes, c_prev, (size_t)n);
    if (wire_scales) memcpy(wire_scales, s_prev, (size_t)nb * sizeof(float));

    for (int32_t i = 1; i < P; ++i) {
        equarx_oracle_hop(c_prev, s_prev, partials[i], n, B, c_next, s_next);
        if (wire_codes) memcpy(wire_codes + (int64_t)i * n, c_next, (size_t)n);
        if (wire_scales) memcpy(wire_scales + (int64_t)i * nb, s_next, (size_t)nb * sizeof(float));
        int8_t *tc = c_prev; c_prev = c_next; c_next = tc;
        float *ts = s_prev; s_prev = s_next; s_next = ts;
    }

    equarx_oracle_dequantize_bf16(c_prev, s_prev, n, B, out);

    free(c_prev); free(c_next); free(s_prev); free(s_next);
}

/* ---- the unquantized sum, for the error columns --------------------------- */

/* Sum of the P partials in fp64, in array order.  bf16 values carry 8
 * significant bits, so this is exact unless the magnitudes span more than
 * about 2^44. */
void equarx_oracle_exact_sum_f64(const uint16_t *const *partials, int32_t P, int64_t n, double *ref)
{
    for (int64_t j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int32_t i = 0; i < P; ++i) acc += (double)widen_bf16(partials[i][j]);
        ref[j] = acc;
    }
}

/* The same sum accumulated in fp32, array order: what an unquantized
 * reduce-scatter with an fp32 accumulator would hold. */
void equarx_oracle_sum_f32(const uint16_t *const *partials, int32_t P, int64_t n, float *ref)
{
    for (int64_t j = 0; j < n; ++j) {
        float acc = widen_bf16(partials[0][j]);
        for (int32_t i = 1; i < P; ++i) acc = acc + widen_bf16(partials[i][j]);
        ref[j] = acc;
    }
}

/* ======================================================================== *
 * Variants of the chain (the paper's knobs and the forms a GPU mesh favours)
 * ======================================================================== */

/* Full-loop chain with the stage-selection knob (Sec. 3.4: the user picks
 * whether the reduce-scatter stage, the all-gather stage, or both are
 * quantized).
 *   quantize_rs: what a device forwards during the reduce-scatter is quantized
 *                (Sec. 3.1); otherwise partial sums travel and add in fp32.
 *   quantize_ag: the finished sum is quantized once more for the all-gather
 *                and dequantized by every receiver (Sec. 3.4); otherwise the
 *                fp32 sum is narrowed to bf16 directly.
 * The owner of a shard adds the last received partial sum to its own shard in
 * fp32; that sum is not quantized by the reduce-scatter, only by the
 * all-gather if that stage is quantized. */
void equarx_oracle_reduce_stages(const uint16_t *const *partials, int32_t P, int64_t n, int32_t B,
                                 int quantize_rs, int quantize_ag, uint16_t *out)
{
    int64_t nb = block_count(n, B);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        int64_t len = block_len(n, B, b);
        int64_t at = b * (int64_t)B;
        float *t = (float *)malloc((size_t)len * sizeof(float));
        int8_t *c = (int8_t *)malloc((size_t)len);
        float s;

        for (int64_t j = 0; j < len; ++j) t[j] = widen_bf16(partials[0][at + j]);
        for (int32_t i = 1; i < P; ++i) {
            if (quantize_rs) {
                quantize_block(t, len, c, &s);                       /* sent to the next device */
                for (int64_t j = 0; j < len; ++j) {
                    t[j] = fmaf((float)c[j], s, widen_bf16(partials[i][at + j]));
                }
            } else {
                for (int64_t j = 0; j < len; ++j) t[j] = t[j] + widen_bf16(partials[i][at + j]);
            }
        }
        if (quantize_ag) {
            quantize_block(t, len, c, &s);
            for (int64_t j = 0; j < len; ++j) out[at + j] = narrow_bf16_rne((float)c[j] * s);
        } else {
            for (int64_t j = 0; j < len; ++j) out[at + j] = narrow_bf16_rne(t[j]);
        }
        free(t); free(c);
    }
}

/* Semi-loop variant (Sec. 3.3): both ring directions are used and the owner
 * of a shard (partials[0] here, the others in ring order around it) receives
 * two partial sums.  With h = P/2:
 *   clockwise chain          x_h -> x_(h-1) -> ... -> x_1 -> owner   (h sends)
 *   counter-clockwise chain  x_(h+1) -> x_(h+2) -> ... -> x_(P-1) -> owner   (P-1-h sends)
 * Every send is quantized; every receiver dequantizes and adds its own shard
 * in fp32.  The shorter, counter-clockwise chain arrives first, so the owner
 * adds it first (the paper's 4-device example: device 3's shard reaches
 * device 0 in the first iteration, device 1's partial sum in the second).
 * quantize_ag as in equarx_oracle_reduce_stages. */
void equarx_oracle_reduce_semi_loop(const uint16_t *const *partials, int32_t P, int64_t n, int32_t B,
                                    int quantize_ag, uint16_t *out)
{
    int64_t nb = block_count(n, B);
    int32_t h = P / 2;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        int64_t len = block_len(n, B, b);
        int64_t at = b * (int64_t)B;
        float *t = (float *)malloc((size_t)len * sizeof(float));
        float *own = (float *)malloc((size_t)len * sizeof(float));
        int8_t *c = (int8_t *)malloc((size_t)len);
        float s;

        for (int64_t j = 0; j < len; ++j) own[j] = widen_bf16(partials[0][at + j]);

        if (h + 1 <= P - 1) {                      /* counter-clockwise: h+1, h+2, ..., P-1, then the owner */
            for (int64_t j = 0; j < len; ++j) t[j] = widen_bf16(partials[h + 1][at + j]);
            for (int32_t i = h + 2; i <= P - 1; ++i) {
                quantize_block(t, len, c, &s);
                for (int64_t j = 0; j < len; ++j) t[j] = fmaf((float)c[j], s, widen_bf16(partials[i][at + j]));
            }
            quantize_block(t, len, c, &s);
            for (int64_t j = 0; j < len; ++j) own[j] = fmaf((float)c[j], s, own[j]);
        }
        if (h >= 1) {                              /* clockwise: h, h-1, ..., 1, then the owner */
            for (int64_t j = 0; j < len; ++j) t[j] = widen_bf16(partials[h][at + j]);
            for (int32_t i = h - 1; i >= 1; --i) {
                quantize_block(t, len, c, &s);
                for (int64_t j = 0; j < len; ++j) t[j] = fmaf((float)c[j], s, widen_bf16(partials[i][at + j]));
            }
            quantize_block(t, len, c, &s);
            for (int64_t j = 0; j < len; ++j) own[j] = fmaf((float)c[j], s, own[j]);
        }

        if (quantize_ag) {
            quantize_block(own, len, c, &s);
            for (int64_t j = 0; j < len; ++j) out[at + j] = narrow_bf16_rne((float)c[j] * s);
        } else {
            for (int64_t j = 0; j < len; ++j) out[at + j] = narrow_bf16_rne(own[j]);
        }
        free(t); free(own); free(c);
    }
}

/* Flat one-shot reduce: the reduce-scatter done as an all-to-all followed by a
 * local reduction (the decomposition Sec. 2 describes for ZeRO++).  Every other
 * device has quantized its shard once (Q_B, as in equarx_oracle_quantize_bf16)
 * and the owner holds R received (codes, scales) pairs plus its own bf16
 * shard.  It dequantizes and accumulates them in fp32, in array order, one
 * fused multiply-add each, then quantizes the sum once for the all-gather.
 *   codes[r], scales[r]: r = 0..R-1, each n codes / nb scales.
 *   codes_out / scales_out (may be NULL): what the all-gather carries.
 *   out: its dequantized bf16 value. */
void equarx_oracle_reduce_flat(const uint16_t *local, const int8_t *const *codes, const float *const *scales,
                               int32_t R, int64_t n, int32_t B, uint16_t *out, int8_t *codes_out, float *scales_out)
{
    int64_t nb = block_count(n, B);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        int64_t len = block_len(n, B, b);
        int64_t at = b * (int64_t)B;
        float *acc = (float *)malloc((size_t)len * sizeof(float));
        int8_t *c = (int8_t *)malloc((size_t)len);
        float s;
        for (int64_t j = 0; j < len; ++j) acc[j] = widen_bf16(local[at + j]);
        for (int32_t r = 0; r < R; ++r) {
            for (int64_t j = 0; j < len; ++j) acc[j] = fmaf((float)codes[r][at + j], scales[r][b], acc[j]);
        }
        quantize_block(acc, len, c, &s);
        for (int64_t j = 0; j < len; ++j) out[at + j] = narrow_bf16_rne((float)c[j] * s);
        if (codes_out) memcpy(codes_out + at, c, (size_t)len);
        if (scales_out) scales_out[b] = s;
        free(acc); free(c);
    }
}
