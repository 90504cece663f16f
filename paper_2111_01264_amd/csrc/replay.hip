// Replay memory D as a uint8 frame ring in HBM: per-lane rings, temporary buffers that are only
// merged at the synchronisation point (Section 3), uniform sampling (Section 2.1) and the fused
// sample + frame-stack gather with terminal masking.  All of it is byte/index work bound by HBM
// bandwidth: frames move as 16-byte vectors (7056 = 441 * 16), one frame per workgroup.
#include <atomic>
#include <new>

#include "common.h"

namespace dqn {

struct FlushTable {
    int32_t head[kMaxLanes];
    int32_t first[kMaxLanes + 1];  // prefix sums of the staged counts
};

}  // namespace dqn

struct replay {
    int64_t N, M, S;
    int32_t L;
    uint64_t seed;
    hipStream_t push_stream, sample_stream;
    uint8_t* frames;
    int32_t* actions;
    float* rewards;
    uint8_t* terminals;
    uint8_t* st_frames;
    int32_t* st_actions;
    float* st_rewards;
    uint8_t* st_terminals;
    int64_t head[dqn::kMaxLanes], count[dqn::kMaxLanes], staged[dqn::kMaxLanes];
    hipEvent_t ev_push, ev_flush;
    uint64_t epoch;   // (creation serial << 32) + flushes so far
};

namespace dqn {

// Temporary buffer append: frame i of the call goes to staging slot first + i of its lane.
__global__ __launch_bounds__(256) void push_kernel(
    const uint8_t* __restrict__ frames, const int32_t* __restrict__ actions,
    const float* __restrict__ rewards, const uint8_t* __restrict__ terminals,
    uint8_t* __restrict__ st_frames, int32_t* __restrict__ st_actions, float* __restrict__ st_rewards,
    uint8_t* __restrict__ st_terminals, int64_t first)
{
    const int64_t i = blockIdx.x;
    copy_frame(st_frames + (first + i) * kFrameBytes, frames + i * kFrameBytes);
    if (threadIdx.x == 0) {
        st_actions[first + i] = actions[i];
        st_rewards[first + i] = rewards[i];
        st_terminals[first + i] = terminals[i];
    }
}

// One experience per lane: row l of the call goes to staging slot l * S + staged[l].
__global__ __launch_bounds__(256) void push_step_kernel(PushStepPlan plan) { push_step_block(plan, blockIdx.x); }

// Flush: staged experience number blockIdx.x (lanes concatenated) moves to its ring slot.
__global__ __launch_bounds__(256) void flush_kernel(
    const uint8_t* __restrict__ st_frames, const int32_t* __restrict__ st_actions,
    const float* __restrict__ st_rewards, const uint8_t* __restrict__ st_terminals,
    uint8_t* __restrict__ frames, int32_t* __restrict__ actions, float* __restrict__ rewards,
    uint8_t* __restrict__ terminals, FlushTable tab, int32_t L, int64_t M, int64_t S)
{
    const int32_t g = blockIdx.x;
    int lane = 0;
    while (lane + 1 < L && g >= tab.first[lane + 1]) ++lane;
    const int64_t i = g - tab.first[lane];
    const int64_t src = lane * S + i;
    const int64_t dst = lane * M + (tab.head[lane] + i) % M;
    copy_frame(frames + dst * kFrameBytes, st_frames + src * kFrameBytes);
    if (threadIdx.x == 0) {
        actions[dst] = st_actions[src];
        rewards[dst] = st_rewards[src];
        terminals[dst] = st_terminals[src];
    }
}

// One workgroup per (sample b, frame f of the five-frame window): see gather_block.
__global__ __launch_bounds__(256) void sample_gather_kernel(GatherPlan plan) { gather_block(plan, blockIdx.x, blockIdx.y); }

// ---- seeded synthetic inputs ------------------------------------------------------------------
__host__ __device__ inline uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

// One thread per 16 output bytes = eight 64-bit words of the generator.
__global__ __launch_bounds__(256) void synth_frames_kernel(
    uint8_t* __restrict__ dst, int64_t n, uint64_t id0, uint64_t id_step, uint64_t stream_key,
    uint32_t pix_threshold, uint32_t background)
{
    const int64_t total = n * kFrameVec16;
    for (int64_t v = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; v < total;
         v += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int64_t fr = v / kFrameVec16;
        const uint32_t chunk = static_cast<uint32_t>(v % kFrameVec16);
        const uint64_t fkey = mix64(stream_key + (id0 + static_cast<uint64_t>(fr) * id_step));
        uint32_t out[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t packed = 0;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint64_t g = static_cast<uint64_t>(chunk) * 8 + q * 2 + h;
                const uint64_t w = mix64(fkey + kGamma * (g + 1));
                const uint32_t lo = static_cast<uint32_t>(w), hi = static_cast<uint32_t>(w >> 32);
                const uint32_t p0 = (lo >> 8) < pix_threshold ? (lo & 0xFFu) : background;
                const uint32_t p1 = (hi >> 8) < pix_threshold ? (hi & 0xFFu) : background;
                packed |= (p0 | (p1 << 8)) << (16 * h);
            }
            out[q] = packed;
        }
        reinterpret_cast<uint4*>(dst)[v] = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

__global__ __launch_bounds__(256) void synth_transitions_kernel(
    int32_t* __restrict__ actions, float* __restrict__ rewards, uint8_t* __restrict__ terminals,
    int64_t n, uint64_t id0, uint64_t id_step, uint64_t stream_key, uint32_t num_actions,
    uint32_t t_neg, uint32_t t_pos, uint32_t t_term)
{
    const int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
    if (i >= n) return;
    const uint64_t fkey = mix64(stream_key + (id0 + static_cast<uint64_t>(i) * id_step));
    const uint64_t w = mix64(fkey + kGamma);
    const uint32_t rb = static_cast<uint32_t>(w & 0xFFFFFFu);
    const uint32_t tb = static_cast<uint32_t>((w >> 24) & 0xFFFFFFu);
    const uint32_t ab = static_cast<uint32_t>(w >> 48);
    rewards[i] = rb < t_neg ? -1.f : (rb >= (1u << 24) - t_pos ? 1.f : 0.f);
    terminals[i] = tb < t_term ? 1 : 0;
    actions[i] = static_cast<int32_t>((ab * num_actions) >> 16);
}

}  // namespace dqn

using namespace dqn;

extern "C" {

int replay_create(int64_t capacity_frames, int32_t lanes, int64_t staging_per_lane, uint64_t seed,
                  void* push_stream, void* sample_stream, replay** host_out)
{
    if (!host_out) return fail(DQN_EINVAL, "replay_create: host_out is null");
    *host_out = nullptr;
    if (lanes < 1 || lanes > kMaxLanes) return fail(DQN_EINVAL, "replay_create: lanes %d outside 1..%d", lanes, kMaxLanes);
    if (capacity_frames < lanes || capacity_frames % lanes != 0)
        return fail(DQN_EINVAL, "replay_create: capacity %lld is not a positive multiple of lanes %d",
                    (long long)capacity_frames, lanes);
    const int64_t M = capacity_frames / lanes;
    if (M > 0x7FFFFFF0ll) return fail(DQN_EINVAL, "replay_create: lane length %lld too large", (long long)M);
    if (staging_per_lane < 1 || staging_per_lane > M)
        return fail(DQN_EINVAL, "replay_create: staging_per_lane %lld outside 1..%lld",
                    (long long)staging_per_lane, (long long)M);
    replay* rb = new (std::nothrow) replay();
    if (!rb) return fail(DQN_ENOMEM, "replay_create: host allocation failed");
    rb->N = capacity_frames; rb->M = M; rb->S = staging_per_lane; rb->L = lanes; rb->seed = seed;
    {   // epochs of different replay memories never coincide (a new one may reuse the address of a destroyed one)
        static std::atomic<uint64_t> serial{1};
        rb->epoch = serial.fetch_add(1) << 32;
    }
    rb->push_stream = static_cast<hipStream_t>(push_stream);
    rb->sample_stream = static_cast<hipStream_t>(sample_stream);
    const int64_t SN = staging_per_lane * lanes;
    hipError_t e = hipSuccess;
    auto alloc = [&](void** p, size_t bytes) { if (e == hipSuccess) e = hipMalloc(p, bytes); };
    alloc((void**)&rb->frames, (size_t)capacity_frames * kFrameBytes);
    alloc((void**)&rb->actions, (size_t)capacity_frames * 4);
    alloc((void**)&rb->rewards, (size_t)capacity_frames * 4);
    alloc((void**)&rb->terminals, (size_t)capacity_frames);
    alloc((void**)&rb->st_frames, (size_t)SN * kFrameBytes);
    alloc((void**)&rb->st_actions, (size_t)SN * 4);
    alloc((void**)&rb->st_rewards, (size_t)SN * 4);
    alloc((void**)&rb->st_terminals, (size_t)SN);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&rb->ev_push, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&rb->ev_flush, hipEventDisableTiming);
    if (e != hipSuccess) {
        const int code = e == hipErrorOutOfMemory ? DQN_ENOMEM : DQN_EHIP;
        fail(code, "replay_create: %s", hipGetErrorString(e));
        replay_destroy(rb);
        return code;
    }
    *host_out = rb;
    return DQN_OK;
}

int replay_destroy(replay* rb)
{
    if (!rb) return DQN_OK;
    (void)hipStreamSynchronize(rb->push_stream);
    (void)hipStreamSynchronize(rb->sample_stream);
    (void)hipFree(rb->frames); (void)hipFree(rb->actions); (void)hipFree(rb->rewards); (void)hipFree(rb->terminals);
    (void)hipFree(rb->st_frames); (void)hipFree(rb->st_actions); (void)hipFree(rb->st_rewards); (void)hipFree(rb->st_terminals);
    if (rb->ev_push) (void)hipEventDestroy(rb->ev_push);
    if (rb->ev_flush) (void)hipEventDestroy(rb->ev_flush);
    delete rb;
    return DQN_OK;
}

int replay_push(replay* rb, int32_t lane, const uint8_t* frames, const int32_t* actions,
                const float* rewards, const uint8_t* terminals, int32_t n)
{
    if (!rb) return fail(DQN_EINVAL, "replay_push: rb is null");
    if (lane < 0 || lane >= rb->L) return fail(DQN_EINVAL, "replay_push: lane %d outside 0..%d", lane, rb->L - 1);
    if (n < 0) return fail(DQN_EINVAL, "replay_push: n = %d", n);
    if (n == 0) return DQN_OK;
    if (!frames || !actions || !rewards || !terminals) return fail(DQN_EINVAL, "replay_push: null pointer");
    if (!aligned16(frames)) return fail(DQN_EINVAL, "replay_push: frames not 16-byte aligned");
    if (rb->staged[lane] + n > rb->S)
        return fail(DQN_ESTATE, "replay_push: lane %d buffer would hold %lld > %lld experiences; flush first",
                    lane, (long long)(rb->staged[lane] + n), (long long)rb->S);
    const int64_t first = lane * rb->S + rb->staged[lane];
    hipLaunchKernelGGL(push_kernel, dim3(n), dim3(256), 0, rb->push_stream, frames, actions, rewards,
                       terminals, rb->st_frames, rb->st_actions, rb->st_rewards, rb->st_terminals, first);
    DQN_LAUNCH_CHECK();
    rb->staged[lane] += n;
    return DQN_OK;
}

int replay_push_step(replay* rb, const uint8_t* frames, const int32_t* actions, const float* rewards,
                     const uint8_t* terminals)
{
    PushStepPlan plan;
    const int rc = replay_plan_push_step(rb, frames, actions, rewards, terminals, &plan);
    if (rc != DQN_OK) return rc;
    hipLaunchKernelGGL(push_step_kernel, dim3(rb->L), dim3(256), 0, rb->push_stream, plan);
    DQN_LAUNCH_CHECK();
    replay_commit_push_step(rb);
    return DQN_OK;
}

// Enqueues the flush on sample_stream; the caller has already made sample_stream wait for the pushes.
static int flush_enqueue(replay* rb)
{
    FlushTable tab;
    int64_t total = 0;
    for (int l = 0; l < rb->L; ++l) {
        tab.head[l] = (int32_t)rb->head[l];
        tab.first[l] = (int32_t)total;
        total += rb->staged[l];
    }
    tab.first[rb->L] = (int32_t)total;
    if (total > 0x7FFFFFFFll) return fail(DQN_ESTATE, "replay_flush: too many staged experiences");
    if (total > 0) {
        hipLaunchKernelGGL(flush_kernel, dim3((unsigned)total), dim3(256), 0, rb->sample_stream,
                           rb->st_frames, rb->st_actions, rb->st_rewards, rb->st_terminals, rb->frames,
                           rb->actions, rb->rewards, rb->terminals, tab, rb->L, rb->M, rb->S);
        DQN_LAUNCH_CHECK();
    }
    for (int l = 0; l < rb->L; ++l) {
        rb->head[l] = (rb->head[l] + rb->staged[l]) % rb->M;
        rb->count[l] = rb->count[l] + rb->staged[l] > rb->M ? rb->M : rb->count[l] + rb->staged[l];
        rb->staged[l] = 0;
    }
    ++rb->epoch;
    return DQN_OK;
}

}  // extern "C"

namespace dqn {
int replay_plan_push_step(replay* rb, const uint8_t* frames, const int32_t* actions, const float* rewards,
                          const uint8_t* terminals, PushStepPlan* plan)
{
    if (!rb) return fail(DQN_EINVAL, "replay_push_step: rb is null");
    if (!frames || !actions || !rewards || !terminals) return fail(DQN_EINVAL, "replay_push_step: null pointer");
    if (!aligned16(frames)) return fail(DQN_EINVAL, "replay_push_step: frames not 16-byte aligned");
    for (int l = 0; l < rb->L; ++l) {
        if (rb->staged[l] + 1 > rb->S)
            return fail(DQN_ESTATE, "replay_push_step: lane %d buffer is full (%lld experiences); flush first", l,
                        (long long)rb->S);
        plan->slot[l] = (int32_t)rb->staged[l];
    }
    plan->frames = frames; plan->actions = actions; plan->rewards = rewards; plan->terminals = terminals;
    plan->st_frames = rb->st_frames; plan->st_actions = rb->st_actions; plan->st_rewards = rb->st_rewards;
    plan->st_terminals = rb->st_terminals;
    plan->S = rb->S; plan->L = rb->L;
    return DQN_OK;
}

void replay_commit_push_step(replay* rb)
{
    for (int l = 0; l < rb->L; ++l) rb->staged[l] += 1;
}

// Used by dqn_sync_target as well: orders push_stream -> flush (sample_stream) -> push_stream.
int replay_flush_ordered(replay* rb)
{
    DQN_HIP(hipEventRecord(rb->ev_push, rb->push_stream));
    DQN_HIP(hipStreamWaitEvent(rb->sample_stream, rb->ev_push, 0));
    const int rc = flush_enqueue(rb);
    if (rc != DQN_OK) return rc;
    DQN_HIP(hipEventRecord(rb->ev_flush, rb->sample_stream));
    DQN_HIP(hipStreamWaitEvent(rb->push_stream, rb->ev_flush, 0));
    return DQN_OK;
}

int replay_plan_sample_gather(replay* rb, int32_t B, uint64_t sample_step, const int64_t* idx_in, uint8_t* s, uint8_t* s2,
                              int32_t* a, float* r, float* done, int64_t* idx_out, GatherPlan* plan)
{
    if (!rb) return fail(DQN_EINVAL, "replay_sample_gather: rb is null");
    if (B < 1 || B > 65535) return fail(DQN_EINVAL, "replay_sample_gather: B = %d outside 1..65535", B);
    if (!s || !s2 || !a || !r || !done) return fail(DQN_EINVAL, "replay_sample_gather: null output pointer");
    if (!aligned16(s) || !aligned16(s2)) return fail(DQN_EINVAL, "replay_sample_gather: s/s2 not 16-byte aligned");
    const int64_t V = replay_num_valid(rb);
    if (V <= 0) return fail(DQN_ESTATE, "replay_sample_gather: replay memory holds no complete transition");
    plan->frames = rb->frames; plan->actions = rb->actions; plan->rewards = rb->rewards; plan->terminals = rb->terminals;
    for (int l = 0; l < rb->L; ++l) { plan->tab.head[l] = (int32_t)rb->head[l]; plan->tab.count[l] = (int32_t)rb->count[l]; }
    plan->L = rb->L; plan->M = rb->M; plan->V = V; plan->seed = rb->seed; plan->sample_step = sample_step;
    plan->idx_in = idx_in; plan->s = s; plan->s2 = s2; plan->a = a; plan->r = r; plan->done = done; plan->idx_out = idx_out;
    plan->B = B;
    return DQN_OK;
}

uint64_t replay_epoch(const replay* rb) { return rb->epoch; }
const uint8_t* replay_ring_frames(const replay* rb) { return rb->frames; }

hipStream_t replay_sample_stream(replay* rb) { return rb->sample_stream; }
hipStream_t replay_push_stream(replay* rb) { return rb->push_stream; }
int replay_lanes(const replay* rb) { return rb->L; }
}  // namespace dqn

extern "C" {

int replay_flush(replay* rb, int32_t blocking)
{
    if (!rb) return fail(DQN_EINVAL, "replay_flush: rb is null");
    const int rc = replay_flush_ordered(rb);
    if (rc != DQN_OK) return rc;
    if (blocking) DQN_HIP(hipStreamSynchronize(rb->sample_stream));
    return DQN_OK;
}

int64_t replay_num_valid(const replay* rb)
{
    if (!rb) return 0;
    int64_t V = 0;
    for (int l = 0; l < rb->L; ++l) V += rb->count[l] > 4 ? rb->count[l] - 4 : 0;
    return V;
}

int replay_sample_gather(replay* rb, int32_t B, uint64_t sample_step, const int64_t* idx_in,
                         uint8_t* s, uint8_t* s2, int32_t* a, float* r, float* done, int64_t* idx_out)
{
    GatherPlan plan;
    const int rc = replay_plan_sample_gather(rb, B, sample_step, idx_in, s, s2, a, r, done, idx_out, &plan);
    if (rc != DQN_OK) return rc;
    hipLaunchKernelGGL(sample_gather_kernel, dim3(5, B), dim3(256), 0, rb->sample_stream, plan);
    DQN_LAUNCH_CHECK();
    return DQN_OK;
}

int synth_frames(uint8_t* dst, int64_t n, uint64_t id0, uint64_t id_step, uint64_t seed,
                 uint32_t stream_tag, uint32_t pix_threshold, uint32_t background, void* stream)
{
    if (n < 0) return fail(DQN_EINVAL, "synth_frames: n < 0");
    if (n == 0) return DQN_OK;
    if (!dst || !aligned16(dst)) return fail(DQN_EINVAL, "synth_frames: dst null or not 16-byte aligned");
    if (background > 255) return fail(DQN_EINVAL, "synth_frames: background > 255");
    const uint64_t key = mix64(seed + kGamma * (static_cast<uint64_t>(stream_tag) + 1));
    const int64_t total = n * kFrameVec16;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(synth_frames_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       dst, n, id0, id_step, key, pix_threshold, background);
    DQN_LAUNCH_CHECK();
    return DQN_OK;
}

int synth_transitions(int32_t* actions, float* rewards, uint8_t* terminals, int64_t n, uint64_t id0,
                      uint64_t id_step, uint64_t seed, int32_t num_actions, uint32_t t_neg, uint32_t t_pos,
                      uint32_t t_term, void* stream)
{
    if (n < 0) return fail(DQN_EINVAL, "synth_transitions: n < 0");
    if (n == 0) return DQN_OK;
    if (!actions || !rewards || !terminals) return fail(DQN_EINVAL, "synth_transitions: null pointer");
    if (num_actions < 1 || num_actions > 65535) return fail(DQN_EINVAL, "synth_transitions: num_actions");
    if (n > 0x7FFFFFFFll * 256) return fail(DQN_EINVAL, "synth_transitions: n too large");
    const uint64_t key = mix64(seed + kGamma * 2ull);   // stream tag 1
    hipLaunchKernelGGL(synth_transitions_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), actions, rewards, terminals, n, id0, id_step, key,
                       (uint32_t)num_actions, t_neg, t_pos, t_term);
    DQN_LAUNCH_CHECK();
    return DQN_OK;
}

}  // extern "C"
