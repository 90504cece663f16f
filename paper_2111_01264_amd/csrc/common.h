// Shared host-side helpers of the DQN hot-path library: error reporting and launch checks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/dqn_mi355.h"

namespace dqn {

// Thread-local message behind dqn_last_error().
char* error_buffer();
int fail(int code, const char* fmt, ...);

#define DQN_HIP(expr)                                                                        \
    do {                                                                                     \
        hipError_t e__ = (expr);                                                             \
        if (e__ != hipSuccess)                                                               \
            return ::dqn::fail(e__ == hipErrorOutOfMemory ? DQN_ENOMEM : DQN_EHIP,           \
                               "%s failed: %s", #expr, hipGetErrorString(e__));              \
    } while (0)

#define DQN_LAUNCH_CHECK()                                                                   \
    do {                                                                                     \
        hipError_t e__ = hipGetLastError();                                                  \
        if (e__ != hipSuccess)                                                               \
            return ::dqn::fail(DQN_EHIP, "kernel launch failed at %s:%d: %s", __FILE__,      \
                               __LINE__, hipGetErrorString(e__));                            \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Replay internals needed by dqn_sync_target.
int replay_flush_ordered(replay* rb);
hipStream_t replay_sample_stream(replay* rb);
hipStream_t replay_push_stream(replay* rb);

constexpr int kFrameBytes = 84 * 84;          // 7056 = 441 * 16
constexpr int kFrameVec16 = kFrameBytes / 16; // 441
constexpr int kStateBytes = 4 * kFrameBytes;

}  // namespace dqn
