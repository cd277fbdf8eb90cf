// Host-side plumbing shared by the translation units of libequarx: the launch
// context every entry point creates (stream, first HIP error, the developer's
// timing hooks), and the argument checks (alignment, shapes, which buffers may
// share memory).  No device code here.
#pragma once

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "equarx.h"

namespace equarx {
namespace host {

constexpr size_t kAlign = 16;           // every data pointer
constexpr size_t kWorkspaceAlign = 256;

inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

inline bool block_ok(int32_t block)
{
    return block == 32 || block == 64 || block == 128 || block == 256 || block == 512;
}

inline int64_t blocks_of(int64_t n, int32_t block) { return (n + block - 1) / block; }

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// The grid is a 32-bit count of workgroups of at least 2048 elements each.
inline bool too_long(int64_t n) { return n > ((int64_t)1 << 40); }

inline int check_shape(int64_t n, int32_t block)
{
    if (!block_ok(block)) return EQUARX_BAD_BLOCK;
    if (n < 0 || too_long(n)) return EQUARX_BAD_SHAPE;
    return EQUARX_OK;
}

// ---------------------------------------------------------------- which buffers may share memory
//
// Every entry point lists the byte ranges it reads and the ones it writes.  A
// written range may not overlap any other range of the call, with one
// exception: where the header allows an output to BE an input (the hop's wire
// in place, a chain's output in place of a partial), the two carry the same
// non-zero tag and may coincide exactly -- same first byte, same length.
// Anything else that overlaps is EQUARX_BAD_SHAPE.  NULL or empty ranges never
// overlap anything.
class Aliasing {
public:
    void reads(const void *p, size_t bytes, int tag = 0) { add(p, bytes, tag, false); }
    void writes(const void *p, size_t bytes, int tag = 0) { add(p, bytes, tag, true); }

    // EQUARX_OK, or EQUARX_BAD_SHAPE if a written range overlaps another range where it may not.
    int check() const
    {
        if (overflow_) return EQUARX_BAD_SHAPE;
        for (int i = 0; i < count_; ++i) {
            if (!r_[i].written) continue;
            for (int j = 0; j < count_; ++j) {
                if (j == i || (r_[j].written && j < i)) continue;      // a pair of outputs is looked at once
                if (!(r_[i].lo < r_[j].hi && r_[j].lo < r_[i].hi)) continue;
                const bool same = r_[i].lo == r_[j].lo && r_[i].hi == r_[j].hi;
                if (same && r_[i].tag != 0 && r_[i].tag == r_[j].tag && !r_[j].written) continue;
                return EQUARX_BAD_SHAPE;
            }
        }
        return EQUARX_OK;
    }

private:
    struct Range {
        uintptr_t lo, hi;
        int tag;
        bool written;
    };
    static constexpr int kMax = 3 * EQUARX_MAX_PARTIALS + 8;

    void add(const void *p, size_t bytes, int tag, bool written)
    {
        if (!p || bytes == 0) return;
        if (count_ == kMax) {
            overflow_ = true;
            return;
        }
        const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
        r_[count_++] = Range{lo, lo + bytes, tag, written};
    }

    Range r_[kMax];
    int count_ = 0;
    bool overflow_ = false;
};

// ---------------------------------------------------------------- launching

// What a developer armed on this thread for its next entry-point call (the
// profiling aids declared in equarx_devtools.h).  An entry point takes the
// hooks over when it starts and drops them when it returns, whether it
// launched anything or failed validation: nothing stays pending.
struct TimingHooks {
    hipEvent_t launch_start = nullptr, launch_stop = nullptr;   // carried by the call's first launch
    hipEvent_t span_start = nullptr, span_stop = nullptr;       // recorded on the stream around launches first..last
    int span_first = 0, span_last = 0;
};

inline thread_local TimingHooks t_pending_hooks;

// One per entry-point call, created before validation.  Launches go through it;
// it remembers the first HIP error any of them returned (taken from the launch
// call's own return value, so an error some earlier, unrelated HIP call left on
// the thread is neither reported nor cleared) and launches nothing further
// after one.
class LaunchCtx {
public:
    explicit LaunchCtx(void *stream) : stream_(static_cast<hipStream_t>(stream)), hooks_(t_pending_hooks)
    {
        t_pending_hooks = TimingHooks{};
    }
    LaunchCtx(const LaunchCtx &) = delete;
    LaunchCtx &operator=(const LaunchCtx &) = delete;

    hipStream_t stream() const { return stream_; }
    int status() const { return error_ == hipSuccess ? EQUARX_OK : EQUARX_DEVICE_ERROR; }

    template <typename... KArgs, typename... Args>
    void launch2d(void (*kernel)(KArgs...), unsigned grid_x, unsigned grid_y, unsigned threads, Args... args)
    {
        launch3d(kernel, grid_x, grid_y, 1u, threads, args...);
    }

    template <typename... KArgs, typename... Args>
    void launch3d(void (*kernel)(KArgs...), unsigned grid_x, unsigned grid_y, unsigned grid_z, unsigned threads,
                  Args... args)
    {
        static_assert(sizeof...(KArgs) == sizeof...(Args), "kernel argument count");
        if (error_ != hipSuccess) return;
        const int index = launches_++;
        if (hooks_.span_start && index == hooks_.span_first) note(hipEventRecord(hooks_.span_start, stream_));
        if (error_ != hipSuccess) return;

        std::tuple<KArgs...> params{static_cast<KArgs>(args)...};       // the kernel's own parameter types
        void *slots[sizeof...(KArgs) > 0 ? sizeof...(KArgs) : 1];
        fill_slots(params, slots, std::index_sequence_for<KArgs...>{});
        hipEvent_t e0 = index == 0 ? hooks_.launch_start : nullptr;
        hipEvent_t e1 = index == 0 ? hooks_.launch_stop : nullptr;
        const void *fn = reinterpret_cast<const void *>(kernel);
        if (e0 || e1) {
            note(hipExtLaunchKernel(fn, dim3(grid_x, grid_y, grid_z), dim3(threads), slots, 0, stream_, e0, e1, 0));
        } else {
            note(hipLaunchKernel(fn, dim3(grid_x, grid_y, grid_z), dim3(threads), slots, 0, stream_));
        }
        if (error_ == hipSuccess && hooks_.span_stop && index == hooks_.span_last) {
            note(hipEventRecord(hooks_.span_stop, stream_));
        }
    }

    template <typename... KArgs, typename... Args>
    void launch(void (*kernel)(KArgs...), unsigned grid, unsigned threads, Args... args)
    {
        launch2d(kernel, grid, 1u, threads, args...);
    }

private:
    template <typename Tuple, size_t... I>
    static void fill_slots(Tuple &params, void **slots, std::index_sequence<I...>)
    {
        ((slots[I] = const_cast<void *>(static_cast<const void *>(&std::get<I>(params)))), ...);
    }

    void note(hipError_t e)
    {
        if (e != hipSuccess && error_ == hipSuccess) {
            error_ = e;
            (void)hipGetLastError();        // this call's own error: reported through the status, not left behind
        }
    }

    hipStream_t stream_;
    TimingHooks hooks_;
    hipError_t error_ = hipSuccess;
    int launches_ = 0;
};

}  // namespace host
}  // namespace equarx
