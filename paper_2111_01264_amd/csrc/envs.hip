// Synchronized Execution's shared arrays (Section 4) between the caller's sampler threads and the device.
//
// The W sampler threads and the kernels address the same pinned host arrays: the act step's last kernel stores the W
// actions (and, on request, the Q rows) into them, and after the samplers' step one small kernel reads the W new
// observations, rewards and terminal flags out of them -- no copy commands, two bus crossings per act step whatever W
// is.  The frame stacks stay on the device: that kernel shifts each stack and appends the new observation, clearing
// what belongs to a finished episode (the rule the replay gather applies, so the states acted from are the states
// training later rebuilds), and appends the experience of the step just taken -- whose observation is still the
// stack's newest frame at that moment -- to the replay memory's temporary buffers.
#include <new>

#include "envs.h"

namespace dqn {
namespace {

struct ObserveArgs {
    uint8_t* states;                 // [W][4][84][84]
    const uint8_t* host_obs;         // [W][84*84]  next observations
    const int32_t* host_actions;     // [W]         actions of the step just taken
    const float* host_rewards;       // [W]
    const uint8_t* host_terminals;   // [W]
    int32_t start;                   // 1: episode start for every environment (stack keeps only the observation, nothing is stored)
    PushStepPlan push;               // push.L == 0: nothing is stored
};

// Workgroup j serves environment j; thread -> 16-byte vectors of a frame (441 vectors, 256 threads).
__global__ __launch_bounds__(256) void envs_observe_kernel(const ObserveArgs a)
{
    const int j = blockIdx.x;
    uint4* st = reinterpret_cast<uint4*>(a.states + static_cast<size_t>(j) * kStateBytes);
    const uint4* nf = reinterpret_cast<const uint4*>(a.host_obs + static_cast<size_t>(j) * kFrameBytes);
    // every read that crosses the bus is requested here, before anything waits: a bus round trip is 2-3 us, and a read
    // requested later (the three scalars, by one thread, at the end) would add another one to the kernel
    uint4 fresh[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int v = threadIdx.x + i * 256;
        fresh[i] = nf[v < kFrameVec16 ? v : kFrameVec16 - 1];
    }
    const uint32_t term_in = a.host_terminals[j];
    const int32_t act_in = a.host_actions[j];
    const float rew_in = a.host_rewards[j];
    const bool store = !a.start && a.push.L > 0;
    const uint32_t term = a.start ? 1u : term_in;
    const uint32_t keep_old = term ? 0u : 0xFFFFFFFFu;
    const int64_t dst = store ? static_cast<int64_t>(j) * a.push.S + a.push.slot[j] : 0;
    uint4* staged = reinterpret_cast<uint4*>(a.push.st_frames + dst * kFrameBytes);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int v = threadIdx.x + i * 256;
        if (v >= kFrameVec16) break;
        uint4 f1 = st[kFrameVec16 + v], f2 = st[2 * kFrameVec16 + v], f3 = st[3 * kFrameVec16 + v];
        if (store) staged[v] = f3;   // the observation the action was taken on
        f1.x &= keep_old; f1.y &= keep_old; f1.z &= keep_old; f1.w &= keep_old;
        f2.x &= keep_old; f2.y &= keep_old; f2.z &= keep_old; f2.w &= keep_old;
        f3.x &= keep_old; f3.y &= keep_old; f3.z &= keep_old; f3.w &= keep_old;
        st[v] = f1; st[kFrameVec16 + v] = f2; st[2 * kFrameVec16 + v] = f3;
        st[3 * kFrameVec16 + v] = fresh[i];
    }
    if (store && threadIdx.x == 0) {
        a.push.st_actions[dst] = act_in;
        a.push.st_rewards[dst] = rew_in;
        a.push.st_terminals[dst] = static_cast<uint8_t>(term != 0);
    }
}

template <typename T>
int pinned(T** host, T** device, size_t n)
{
    DQN_HIP(hipHostMalloc(reinterpret_cast<void**>(host), n * sizeof(T), hipHostMallocDefault));
    DQN_HIP(hipHostGetDevicePointer(reinterpret_cast<void**>(device), *host, 0));
    return DQN_OK;
}

}  // namespace
}  // namespace dqn

using namespace dqn;

extern "C" {

int dqn_envs_create(dqn_ctx* ctx, replay* rb, int32_t W, dqn_envs** out)
{
    if (!ctx || !out) return fail(DQN_EINVAL, "dqn_envs_create: null pointer");
    if (W < 1 || W > dqn_ctx_max_envs(ctx) || W > kMaxLanes)
        return fail(DQN_EINVAL, "dqn_envs_create: W = %d outside 1..%d", W, dqn_ctx_max_envs(ctx) < kMaxLanes ? dqn_ctx_max_envs(ctx) : kMaxLanes);
    if (rb && replay_lanes(rb) != W)
        return fail(DQN_EINVAL, "dqn_envs_create: the replay memory needs one lane per environment (%d lanes, W = %d)", replay_lanes(rb), W);
    if (rb && replay_push_stream(rb) != dqn_ctx_act_stream(ctx))
        return fail(DQN_EINVAL, "dqn_envs_create: the replay's push stream must be the act stream");
    dqn_envs* e = new (std::nothrow) dqn_envs();
    if (!e) return fail(DQN_ENOMEM, "dqn_envs_create: host allocation failed");
    e->ctx = ctx; e->rb = rb; e->W = W; e->A = dqn_ctx_num_actions(ctx); e->act_stream = dqn_ctx_act_stream(ctx);
    auto body = [&]() -> int {
        int rc;
        if ((rc = pinned(&e->h_obs, &e->hd_obs, static_cast<size_t>(W) * kFrameBytes)) != DQN_OK) return rc;
        if ((rc = pinned(&e->h_actions, &e->hd_actions, W)) != DQN_OK) return rc;
        if ((rc = pinned(&e->h_rewards, &e->hd_rewards, W)) != DQN_OK) return rc;
        if ((rc = pinned(&e->h_terminals, &e->hd_terminals, W)) != DQN_OK) return rc;
        if ((rc = pinned(&e->h_q, &e->hd_q, static_cast<size_t>(W) * e->A)) != DQN_OK) return rc;
        DQN_HIP(hipMalloc(reinterpret_cast<void**>(&e->d_states), static_cast<size_t>(W) * kStateBytes));
        DQN_HIP(hipMemsetAsync(e->d_states, 0, static_cast<size_t>(W) * kStateBytes, e->act_stream));
        DQN_HIP(hipStreamSynchronize(e->act_stream));
        return DQN_OK;
    };
    const int rc = body();
    if (rc != DQN_OK) {
        char saved[512];
        snprintf(saved, sizeof(saved), "%s", error_buffer());
        dqn_envs_destroy(e);
        return fail(rc, "dqn_envs_create: %s", saved);
    }
    *out = e;
    return DQN_OK;
}

int dqn_envs_destroy(dqn_envs* e)
{
    if (!e) return DQN_OK;
    if (e->act_stream || e->d_states) (void)hipStreamSynchronize(e->act_stream);
    (void)hipHostFree(e->h_obs); (void)hipHostFree(e->h_actions); (void)hipHostFree(e->h_rewards);
    (void)hipHostFree(e->h_terminals); (void)hipHostFree(e->h_q);
    (void)hipFree(e->d_states);
    delete e;
    return DQN_OK;
}

int dqn_envs_arrays(dqn_envs* e, uint8_t** host_observations, int32_t** host_actions, float** host_rewards,
                    uint8_t** host_terminals, float** host_q)
{
    if (!e) return fail(DQN_EINVAL, "dqn_envs_arrays: handle is null");
    if (host_observations) *host_observations = e->h_obs;
    if (host_actions) *host_actions = e->h_actions;
    if (host_rewards) *host_rewards = e->h_rewards;
    if (host_terminals) *host_terminals = e->h_terminals;
    if (host_q) *host_q = e->h_q;
    return DQN_OK;
}

int dqn_envs_reset(dqn_envs* e)
{
    if (!e) return fail(DQN_EINVAL, "dqn_envs_reset: handle is null");
    ObserveArgs a{};
    a.states = e->d_states; a.host_obs = e->hd_obs; a.host_actions = e->hd_actions; a.host_rewards = e->hd_rewards;
    a.host_terminals = e->hd_terminals; a.start = 1; a.push.L = 0;
    hipLaunchKernelGGL(envs_observe_kernel, dim3(e->W), dim3(256), 0, e->act_stream, a);
    DQN_LAUNCH_CHECK();
    e->started = true;
    return DQN_OK;
}

int dqn_envs_act(dqn_envs* e, float epsilon, uint64_t act_step, int32_t use_target, int32_t want_q)
{
    if (!e) return fail(DQN_EINVAL, "dqn_envs_act: handle is null");
    if (!e->started) return fail(DQN_ESTATE, "dqn_envs_act: dqn_envs_reset has not been called");
    const int rc = dqn_act(e->ctx, e->d_states, e->W, epsilon, act_step, use_target, e->hd_actions, want_q ? e->hd_q : nullptr);
    if (rc != DQN_OK) return rc;
    DQN_HIP(hipStreamSynchronize(e->act_stream));
    return DQN_OK;
}

int dqn_envs_observe(dqn_envs* e)
{
    if (!e) return fail(DQN_EINVAL, "dqn_envs_observe: handle is null");
    if (!e->started) return fail(DQN_ESTATE, "dqn_envs_observe: dqn_envs_reset has not been called");
    ObserveArgs a{};
    a.states = e->d_states; a.host_obs = e->hd_obs; a.host_actions = e->hd_actions; a.host_rewards = e->hd_rewards;
    a.host_terminals = e->hd_terminals; a.start = 0; a.push.L = 0;
    if (e->rb) {
        // slots and capacity check of one experience per lane; the source pointers of the plan are not used by this kernel
        const int rc = replay_plan_push_step(e->rb, e->d_states, e->hd_actions, e->hd_rewards, e->hd_terminals, &a.push);
        if (rc != DQN_OK) return rc;
    }
    hipLaunchKernelGGL(envs_observe_kernel, dim3(e->W), dim3(256), 0, e->act_stream, a);
    DQN_LAUNCH_CHECK();
    if (e->rb) replay_commit_push_step(e->rb);
    return DQN_OK;
}

}  // extern "C"
