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
constexpr int kMaxLanes = 64;

// A frame is 7056 = 110.25 x 64 bytes, so frames in a [n][84][84] array start at every 16-byte phase of a
// 64-byte line.  A 16-byte store whose group of four lanes straddles a line boundary reaches memory as two
// partial writes (measured: 1.75x the written bytes on average); shifting the vector index by the
// destination's phase makes every group of four lanes cover exactly one line.
__device__ inline int line_phase(const void* p) { return static_cast<int>((reinterpret_cast<uintptr_t>(p) >> 4) & 3); }

__device__ inline void copy_frame(uint8_t* __restrict__ dst, const uint8_t* __restrict__ src)
{
    const uint4* s = reinterpret_cast<const uint4*>(src);
    uint4* d = reinterpret_cast<uint4*>(dst);
    const int ph = line_phase(dst);
    for (int v = static_cast<int>(threadIdx.x) - ph; v < kFrameVec16; v += blockDim.x)
        if (v >= 0) d[v] = s[v];
}

// One experience per lane appended to the temporary buffers (Section 3), as data for a kernel: what
// replay_push_step does, for a caller that folds the append into a launch of its own.
struct PushStepPlan {
    const uint8_t* frames;      // [L][84][84]
    const int32_t* actions;     // [L]
    const float* rewards;       // [L]
    const uint8_t* terminals;   // [L]
    uint8_t* st_frames;
    int32_t* st_actions;
    float* st_rewards;
    uint8_t* st_terminals;
    int64_t S;                  // staging slots per lane
    int32_t L;                  // 0 = nothing to append
    int32_t slot[kMaxLanes];    // staging slot of each lane's new experience
};

// Workgroup `lane` of a push: frame copy by the whole workgroup, the three scalars by thread 0.
__device__ inline void push_step_block(const PushStepPlan& p, int lane)
{
    const int64_t dst = static_cast<int64_t>(lane) * p.S + p.slot[lane];
    copy_frame(p.st_frames + dst * kFrameBytes, p.frames + static_cast<int64_t>(lane) * kFrameBytes);
    if (threadIdx.x == 0) {
        p.st_actions[dst] = p.actions[lane];
        p.st_rewards[dst] = p.rewards[lane];
        p.st_terminals[dst] = p.terminals[lane];
    }
}

// Validates a replay_push_step call and fills `plan` without enqueuing anything; replay_commit_push_step then
// records that the experiences have been appended (call it once the kernel carrying the plan is enqueued).
int replay_plan_push_step(replay* rb, const uint8_t* frames, const int32_t* actions, const float* rewards,
                          const uint8_t* terminals, PushStepPlan* plan);
void replay_commit_push_step(replay* rb);

}  // namespace dqn
