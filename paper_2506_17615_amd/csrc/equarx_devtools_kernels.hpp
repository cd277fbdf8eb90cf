// Device code of the developer aids of libequarx (declared in equarx_devtools.h):
// self-tests of the kernels' arithmetic shortcuts and the calibration kernels
// the benchmark sets beside the real ones.  Included by one translation unit.
#pragma once

#include "equarx_device.hpp"

namespace equarx {

// ---------------------------------------------------------------- self-tests of the arithmetic

// Compares block_quotients with the IEEE division for the `count` consecutive
// fp32 bit patterns starting at first_bits (grid-stride).  mismatches[0] counts
// differing scales, mismatches[1] differing reciprocals.
__global__ __launch_bounds__(kThreads) void selftest_quotients_kernel(uint32_t first_bits, uint64_t count,
                                                                       unsigned long long *mismatches)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    unsigned bad_scale = 0, bad_inv = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
        const float a = __uint_as_float(first_bits + (uint32_t)i);
        float s0, i0, s1, i1;
        block_quotients(a, s0, i0);
        block_quotients_ieee(a, s1, i1);
        bad_scale += __float_as_uint(s0) != __float_as_uint(s1);
        bad_inv += __float_as_uint(i0) != __float_as_uint(i1);
    }
    if (bad_scale) atomicAdd(&mismatches[0], (unsigned long long)bad_scale);
    if (bad_inv) atomicAdd(&mismatches[1], (unsigned long long)bad_inv);
}

// Compares the code the kernels take from the low byte of p + 1.5 * 2^23 with
// (int8) rint(p), for +p and -p, over `count` consecutive fp32 bit patterns of
// |p| starting at first_bits (grid-stride).  mismatches[0] counts differences.
__global__ __launch_bounds__(kThreads) void selftest_rounding_kernel(uint32_t first_bits, uint64_t count,
                                                                      unsigned long long *mismatches)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    unsigned bad = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
        const float mag = __uint_as_float(first_bits + (uint32_t)i);
#pragma unroll
        for (int sign = 0; sign < 2; ++sign) {
            const float p = sign ? -mag : mag;
            const uint32_t fast = __float_as_uint(p + kRoundMagic) & 0xFFu;
            const uint32_t plain = (uint32_t)(int)__builtin_rintf(p) & 0xFFu;
            bad += fast != plain;
        }
    }
    if (bad) atomicAdd(&mismatches[0], (unsigned long long)bad);
}

// Evaluates block_quotients on caller-chosen values, for comparison with a
// division done on the host.
__global__ __launch_bounds__(kThreads) void eval_quotients_kernel(const float *__restrict__ a, int64_t n,
                                                                   float *__restrict__ scale, float *__restrict__ inv)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        float s, v;
        block_quotients(a[i], s, v);
        scale[i] = s;
        inv[i] = v;
    }
}

// Calibration: a kernel that does nothing, for the time a launch occupies a stream whatever its work.
__global__ __launch_bounds__(kThreads) void empty_kernel(int) {}

// Calibration: plain 16-byte-vector copy.
__global__ __launch_bounds__(kThreads) void copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                        int64_t nvec)
{
    constexpr int K = 4;
    const int64_t at = (int64_t)blockIdx.x * (kThreads * K) + threadIdx.x;
    u32x4 v[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t i = at + k * kThreads;
        if (i < nvec) v[k] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t i = at + k * kThreads;
        if (i < nvec) __builtin_nontemporal_store(v[k], dst + i);
    }
}

// Calibration: the hop's memory traffic without its arithmetic.  Same loads
// and stores per lane as hop_kernel (16 bytes of bf16, 8 bytes of codes, the
// group's scale in; 8 bytes of codes and the group leader's scale out), the
// same tiling; the "result" is an XOR of what was read.
template <int B, int K>
__global__ __launch_bounds__(kThreads) void hop_traffic_kernel(const u32x4 *__restrict__ x, const u32x2 *cin,
                                                               const float *sin, int64_t lanes, u32x2 *cout,
                                                               float *sout)
{
    constexpr int G = B / kLaneElems;
    const int64_t at = (int64_t)blockIdx.x * (kThreads * K) + threadIdx.x;
    u32x4 xv[K];
    u32x2 cv[K];
    float sv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t i = at + k * kThreads;
        if (i < lanes) {
            xv[k] = __builtin_nontemporal_load(x + i);
            cv[k] = cin[i];
            sv[k] = sin[i / G];
        }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t i = at + k * kThreads;
        if (i < lanes) {
            u32x2 w;
            w.x = xv[k].x ^ xv[k].z ^ cv[k].x;
            w.y = xv[k].y ^ xv[k].w ^ cv[k].y;
            cout[i] = w;
            if ((threadIdx.x % G) == 0) sout[i / G] = sv[k];
        }
    }
}

}  // namespace equarx
