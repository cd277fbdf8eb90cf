/* A plain C99 client of libequarx: no Python, no torch, no C++.  The GPU tests
 * build it with gcc and run it on inputs they wrote, then compare its output
 * file with the CPU oracle; it shows that the C ABI alone is enough to drive the
 * whole path (device memory from the HIP runtime, plain pointers in, status
 * codes out).
 *
 * usage: abi_client IN.bin OUT.bin P n block
 *   IN.bin   P * n little-endian uint16 (bf16 bit patterns), partial after partial
 *   OUT.bin  n uint16: the result of equarx_reduce_quantized
 * Also runs equarx_reduce_fused and equarx_reduce_quantized_fused_ends on the
 * same inputs and fails (exit 3) unless all three outputs are identical.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "equarx.h"

#define HIP_OK(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                 \
            return 2;                                                                  \
        }                                                                              \
    } while (0)

#define EQ_OK(call)                                                                    \
    do {                                                                               \
        int s_ = (call);                                                               \
        if (s_ != EQUARX_OK) {                                                         \
            fprintf(stderr, "%s: %s\n", #call, equarx_status_string(s_));              \
            return 2;                                                                  \
        }                                                                              \
    } while (0)

int main(int argc, char **argv)
{
    if (argc != 6) {
        fprintf(stderr, "usage: %s IN.bin OUT.bin P n block\n", argv[0]);
        return 1;
    }
    const int P = atoi(argv[3]);
    const long long n = atoll(argv[4]);
    const int block = atoi(argv[5]);
    if (P < 1 || P > EQUARX_MAX_PARTIALS || n < 1) return 1;
    const size_t bytes = (size_t)n * sizeof(uint16_t);

    uint16_t *host = (uint16_t *)malloc(bytes * (size_t)P);
    uint16_t *res[3] = {(uint16_t *)malloc(bytes), (uint16_t *)malloc(bytes), (uint16_t *)malloc(bytes)};
    if (!host || !res[0] || !res[1] || !res[2]) return 2;
    FILE *in = fopen(argv[1], "rb");
    if (!in || fread(host, bytes, (size_t)P, in) != (size_t)P) {
        fprintf(stderr, "cannot read %s\n", argv[1]);
        return 2;
    }
    fclose(in);

    const void *parts[EQUARX_MAX_PARTIALS];
    for (int i = 0; i < P; ++i) {
        void *d = NULL;
        HIP_OK(hipMalloc(&d, bytes));
        HIP_OK(hipMemcpy(d, host + (size_t)i * (size_t)n, bytes, hipMemcpyHostToDevice));
        parts[i] = d;
    }
    void *out = NULL, *work = NULL;
    const size_t work_bytes = equarx_workspace_bytes(P, n, block);
    if (work_bytes == 0) {
        fprintf(stderr, "equarx_workspace_bytes rejected P=%d n=%lld block=%d\n", P, n, block);
        return 2;
    }
    HIP_OK(hipMalloc(&out, bytes));
    HIP_OK(hipMalloc(&work, work_bytes));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    for (int which = 0; which < 3; ++which) {
        HIP_OK(hipMemsetAsync(out, 0xAB, bytes, stream));
        if (which == 0) {
            EQ_OK(equarx_reduce_quantized(parts, P, n, block, out, work, work_bytes, NULL, NULL, stream));
        } else if (which == 1) {
            EQ_OK(equarx_reduce_fused(parts, P, n, block, out, NULL, NULL, stream));
        } else {
            EQ_OK(equarx_reduce_quantized_fused_ends(parts, P, n, block, out, work, work_bytes, stream));
        }
        HIP_OK(hipStreamSynchronize(stream));
        HIP_OK(hipMemcpy(res[which], out, bytes, hipMemcpyDeviceToHost));
    }
    if (memcmp(res[0], res[1], bytes) != 0 || memcmp(res[0], res[2], bytes) != 0) {
        fprintf(stderr, "the three schedules disagree\n");
        return 3;
    }
    /* an invalid call is refused with a status, not a crash */
    if (equarx_reduce_quantized(parts, P, n, 100, out, work, work_bytes, NULL, NULL, stream) != EQUARX_BAD_BLOCK) return 3;

    FILE *fo = fopen(argv[2], "wb");
    if (!fo || fwrite(res[0], bytes, 1, fo) != 1) {
        fprintf(stderr, "cannot write %s\n", argv[2]);
        return 2;
    }
    fclose(fo);
    printf("abi_client ok: P=%d n=%lld block=%d\n", P, n, block);
    return 0;
}
