// Shared host-side helpers of the DQN hot-path library: error reporting and launch checks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/dqn_mi355.h"
#include "philox.h"

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
int replay_lanes(const replay* rb);
// Context internals needed by the Algorithm 1 orchestrator.
hipStream_t dqn_ctx_act_stream(dqn_ctx* c);
int dqn_ctx_num_actions(const dqn_ctx* c);
int dqn_ctx_max_envs(const dqn_ctx* c);
int dqn_ctx_max_batch(const dqn_ctx* c);

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

struct LaneTable {
    int32_t head[kMaxLanes];   // next write position inside the lane
    int32_t count[kMaxLanes];  // visible frames in the lane
};

// One replay_sample_gather call as data for a kernel (for a caller that folds the gather into a launch of its own).
struct GatherPlan {
    const uint8_t* frames; const int32_t* actions; const float* rewards; const uint8_t* terminals;   // the ring
    LaneTable tab;
    int32_t L; int64_t M, V;
    uint64_t seed, sample_step;
    const int64_t* idx_in;
    uint8_t* s; uint8_t* s2; int32_t* a; float* r; float* done; int64_t* idx_out;
    int32_t B;                  // 0 = nothing to gather
};

// Global index of the transition that draw b of the call selects (or that idx_in names).
__device__ inline int64_t sampled_index(const GatherPlan& p, int b)
{
    if (p.idx_in) return p.idx_in[b];
    const Philox4 d = philox_draw(p.seed, kTagSample, p.sample_step, static_cast<uint32_t>(b));
    const uint64_t u = (static_cast<uint64_t>(d.x[1]) << 32) | d.x[0];
    int64_t k = static_cast<int64_t>(__umul64hi(u, static_cast<uint64_t>(p.V)));
    int lane = 0;
    for (;;) {
        const int64_t v = p.tab.count[lane] > 4 ? p.tab.count[lane] - 4 : 0;
        if (k < v || lane == p.L - 1) break;
        k -= v;
        ++lane;
    }
    return lane * p.M + 3 + k;
}

// The minibatch row of sample b as a DESCRIPTOR instead of copied frames: desc[0..3] = replay slots of the four frames
// of s, desc[4..7] = those of s', -1 for a frame that is all zeros (a terminal flag lies between it and the stack's
// newest frame, or the index is invalid); a, r, done (and idx_out) are written as gather_block writes them.  A kernel
// that consumes states can then read the frames straight from the replay memory (Section 2.1: states are stacks of
// the four latest frames), and the 56 KB per sample that a materialised (s, s') pair costs are never written.
constexpr int kDescInts = 8;
__device__ inline void sample_desc(const GatherPlan& p, int b, int32_t* __restrict__ desc)
{
    const int64_t idx = sampled_index(p, b);
    bool ok = idx >= 0 && idx < static_cast<int64_t>(p.L) * p.M;
    int lane = 0;
    int64_t j = 0;
    if (ok) {
        lane = static_cast<int>(idx / p.M);
        j = idx % p.M;
        ok = j >= 3 && j <= static_cast<int64_t>(p.tab.count[lane]) - 2;
    }
    if (p.idx_out) p.idx_out[b] = idx;
    if (!ok) {
#pragma unroll
        for (int f = 0; f < kDescInts; ++f) desc[f] = -1;
        p.a[b] = -1; p.r[b] = 0.f; p.done[b] = 0.f;
        return;
    }
    const int64_t base = static_cast<int64_t>(p.tab.head[lane]) - p.tab.count[lane] + p.M;  // >= 0
    const int64_t lane0 = lane * p.M;
    uint32_t t[4];   // terminal flags of ages j-3 .. j
#pragma unroll
    for (int u = 0; u < 4; ++u) t[u] = p.terminals[lane0 + (base + j - 3 + u) % p.M];
    int32_t slot[5];
#pragma unroll
    for (int f = 0; f < 5; ++f) slot[f] = static_cast<int32_t>(lane0 + (base + j - 3 + f) % p.M);
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        uint32_t any_s = 0, any_s2 = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u >= f && u <= 2) any_s |= t[u];          // frame f of s: ages j-3+f .. j-1
            if (u >= f + 1) any_s2 |= t[u];               // frame f of s' is window frame f+1: ages j-2+f .. j
        }
        desc[f] = any_s ? -1 : slot[f];
        desc[4 + f] = any_s2 ? -1 : slot[f + 1];
    }
    const int64_t tslot = lane0 + (base + j) % p.M;
    p.a[b] = p.actions[tslot];
    p.r[b] = p.rewards[tslot];
    p.done[b] = t[3] ? 1.f : 0.f;
}

// Workgroup (frame f of the five-frame window ages j-3 .. j+1, sample b), 256 threads.  The frame is read once and
// written into s (position f, f <= 3) and s2 (position f-1, f >= 1), each zeroed if a terminal flag lies between
// the frame and the newest frame of that stack (Section 2.1: states are stacks of the four latest frames).
__device__ inline void gather_block(const GatherPlan& p, int f, int b)
{
    const uint8_t* __restrict__ frames = p.frames; const int32_t* __restrict__ actions = p.actions;
    const float* __restrict__ rewards = p.rewards; const uint8_t* __restrict__ terminals = p.terminals;
    const LaneTable& tab = p.tab;
    const int32_t L = p.L; const int64_t M = p.M, V = p.V; const uint64_t seed = p.seed, sample_step = p.sample_step;
    const int64_t* __restrict__ idx_in = p.idx_in; uint8_t* __restrict__ s = p.s; uint8_t* __restrict__ s2 = p.s2;
    int32_t* __restrict__ a = p.a; float* __restrict__ r = p.r; float* __restrict__ done = p.done; int64_t* __restrict__ idx_out = p.idx_out;
    const int64_t idx = sampled_index(p, b);
    bool ok = idx >= 0 && idx < static_cast<int64_t>(L) * M;
    int lane = 0;
    int64_t j = 0;
    if (ok) {
        lane = static_cast<int>(idx / M);
        j = idx % M;
        ok = j >= 3 && j <= static_cast<int64_t>(tab.count[lane]) - 2;
    }
    uint4* ds = (f <= 3) ? reinterpret_cast<uint4*>(s + (static_cast<int64_t>(b) * 4 + f) * kFrameBytes) : nullptr;
    uint4* ds2 = (f >= 1) ? reinterpret_cast<uint4*>(s2 + (static_cast<int64_t>(b) * 4 + f - 1) * kFrameBytes) : nullptr;
    const int ph = ds ? line_phase(ds) : 0, ph2 = ds2 ? line_phase(ds2) : 0;   // see copy_frame
    if (!ok) {
        const uint4 z = make_uint4(0, 0, 0, 0);
        for (int v = threadIdx.x; v < kFrameVec16 + 3; v += blockDim.x) {
            if (ds && v - ph >= 0 && v - ph < kFrameVec16) ds[v - ph] = z;
            if (ds2 && v - ph2 >= 0 && v - ph2 < kFrameVec16) ds2[v - ph2] = z;
        }
        if (f == 0 && threadIdx.x == 0) {
            a[b] = -1; r[b] = 0.f; done[b] = 0.f;
            if (idx_out) idx_out[b] = idx;
        }
        return;
    }
    const int64_t base = static_cast<int64_t>(tab.head[lane]) - tab.count[lane] + M;  // >= 0
    const int64_t lane0 = lane * M;
    // terminal flags of ages j-3 .. j
    uint32_t t[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) t[u] = terminals[lane0 + (base + j - 3 + u) % M];
    uint32_t any_s = 0, any_s2 = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (u >= f && u <= 2) any_s |= t[u];
        if (u >= f) any_s2 |= t[u];
    }
    const int64_t slot = lane0 + (base + j - 3 + f) % M;
    const uint4* src = reinterpret_cast<const uint4*>(frames + slot * kFrameBytes);
    // a frame behind a terminal flag is zeroed with a mask (a choice between the loaded vector and a zero vector made the
    // compiler keep the zero vector in scratch memory and load through a pointer)
    const uint32_t keep_s = any_s ? 0u : 0xFFFFFFFFu, keep_s2 = any_s2 ? 0u : 0xFFFFFFFFu;
    // each destination with its own phase shift; the second read of the frame comes from cache
    for (int v = threadIdx.x; v < kFrameVec16 + 3; v += blockDim.x) {
        const int v1 = v - ph, v2 = v - ph2;
        if (ds && v1 >= 0 && v1 < kFrameVec16) { uint4 w = src[v1]; w.x &= keep_s; w.y &= keep_s; w.z &= keep_s; w.w &= keep_s; ds[v1] = w; }
        if (ds2 && v2 >= 0 && v2 < kFrameVec16) { uint4 w = src[v2]; w.x &= keep_s2; w.y &= keep_s2; w.z &= keep_s2; w.w &= keep_s2; ds2[v2] = w; }
    }
    if (f == 0 && threadIdx.x == 0) {
        const int64_t tslot = lane0 + (base + j) % M;
        a[b] = actions[tslot];
        r[b] = rewards[tslot];
        done[b] = t[3] ? 1.f : 0.f;
        if (idx_out) idx_out[b] = idx;
    }
}

// Validates a replay_sample_gather call and fills `plan` without enqueuing anything.
int replay_plan_sample_gather(replay* rb, int32_t B, uint64_t sample_step, const int64_t* idx_in, uint8_t* s, uint8_t* s2,
                              int32_t* a, float* r, float* done, int64_t* idx_out, GatherPlan* plan);
// Changes with every flush (and differs between replay memories): two gathers of the same sample step read the same
// minibatch iff their epochs are equal.
uint64_t replay_epoch(const replay* rb);
// The ring's frame array [capacity][84][84] (device memory owned by rb).
const uint8_t* replay_ring_frames(const replay* rb);

// Validates a replay_push_step call and fills `plan` without enqueuing anything; replay_commit_push_step then
// records that the experiences have been appended (call it once the kernel carrying the plan is enqueued).
int replay_plan_push_step(replay* rb, const uint8_t* frames, const int32_t* actions, const float* rewards,
                          const uint8_t* terminals, PushStepPlan* plan);
void replay_commit_push_step(replay* rb);

}  // namespace dqn
