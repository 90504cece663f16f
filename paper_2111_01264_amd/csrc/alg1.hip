// Algorithm 1 (DQN with Concurrent Training and Synchronized Execution, main thread) as a native host orchestrator:
// W sampler threads and one trainer thread around the hot-path calls of this library.
//
//   * every C timesteps: wait for the trainer and the samplers, append what is pending, flush the temporary buffers
//     into D, theta^- <- theta (dqn_sync_target), dispatch the trainer thread for C / F minibatches;
//   * every W timesteps: wait for the samplers, evaluate Q(s^(j), .) for all W states in one minibatch (Section 4) --
//     with the previous step's experiences riding in the same launches --, hand every sampler its action;
//   * a sampler thread takes one step in its environment with that action.
//
// The environments are synthetic (a seeded frame generator stands in for the Atari emulator, see the header): they
// live on the host, as an emulator would, one per sampler thread.  States, actions, rewards and terminal flags cross
// the bus through pinned "shared arrays" (Section 4) that both the threads and the kernels address directly: the act
// step's last kernel stores the W actions into the pinned array, and after the samplers' step one small kernel reads
// the W new observations, rewards and flags out of the pinned arrays -- no copy commands, two bus crossings per act
// step whatever W is.  The frame stacks themselves stay on the device: that kernel shifts each stack and appends the
// new frame, clearing what belongs to a finished episode (the rule the replay gather applies, so the states acted from
// are the states training later rebuilds), and keeps device copies of what the next append needs.
//
// The ablation of Section 5.1 switches the two techniques off independently.  Without Synchronized Execution every
// sampler thread queries the network by itself (its own batch-1 dqn_act, its own transfers, its own append), the calls
// serialised by a mutex as a single device serialises them; without Concurrent Training the loop is standard DQN: the
// policy reads theta, every round's experiences are flushed into D at once and the calling thread itself makes the train
// steps that have become due (one per F timesteps) before the next round.
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "common.h"

namespace dqn {

namespace {

constexpr uint64_t kGammaEnv = 0x9E3779B97F4A7C15ull;
inline uint64_t mix64_host(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}
constexpr uint32_t kStreamEnv = 3, kStreamEnvMeta = 4;   // stream tags of the synthetic environments
constexpr uint32_t kPixThreshold = 838861;               // ceil(0.05 * 2^24)
constexpr uint32_t kBackground = 40;
constexpr std::chrono::microseconds kSpin(200);          // how long a thread polls for its next task before it blocks

// Observation `id` of the environment stream: the frame generator of the header, on the host.
void env_frame_host(uint64_t stream_key, uint64_t id, uint8_t* dst)
{
    const uint64_t fkey = mix64_host(stream_key + id);
    for (uint32_t g = 0; g < kFrameBytes / 2; ++g) {
        const uint64_t w = mix64_host(fkey + kGammaEnv * (static_cast<uint64_t>(g) + 1));
        const uint32_t lo = static_cast<uint32_t>(w), hi = static_cast<uint32_t>(w >> 32);
        dst[2 * g] = static_cast<uint8_t>((lo >> 8) < kPixThreshold ? (lo & 0xFFu) : kBackground);
        dst[2 * g + 1] = static_cast<uint8_t>((hi >> 8) < kPixThreshold ? (hi & 0xFFu) : kBackground);
    }
}

// Shift every environment's frame stack by one and append its new observation; a stack whose previous step ended
// an episode keeps only the new observation.  One workgroup per environment, thread -> 16-byte vector of a frame.
__global__ __launch_bounds__(256) void env_advance_kernel(uint8_t* __restrict__ states, const uint8_t* __restrict__ new_frames,
                                                          const uint8_t* __restrict__ terminals)
{
    const int j = blockIdx.x;
    uint4* st = reinterpret_cast<uint4*>(states + static_cast<size_t>(j) * kStateBytes);
    const uint4* nf = reinterpret_cast<const uint4*>(new_frames + static_cast<size_t>(j) * kFrameBytes);
    const bool reset = terminals[j] != 0;
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (int v = threadIdx.x; v < kFrameVec16; v += blockDim.x) {
        const uint4 f1 = st[kFrameVec16 + v], f2 = st[2 * kFrameVec16 + v], f3 = st[3 * kFrameVec16 + v];
        st[v] = reset ? z : f1;
        st[kFrameVec16 + v] = reset ? z : f2;
        st[2 * kFrameVec16 + v] = reset ? z : f3;
        st[3 * kFrameVec16 + v] = nf[v];
    }
}

// The same for a synchronized round, fed straight from the pinned host arrays: workgroup j reads environment j's new
// observation once over the bus, appends it to the stack and keeps a device copy of it (it is the frame of the next
// experience to be appended), and thread 0 keeps device copies of (a, r, d) of the step just taken.
__global__ __launch_bounds__(256) void env_round_kernel(uint8_t* __restrict__ states, const uint8_t* __restrict__ host_frames,
                                                        const float* __restrict__ host_rewards, const uint8_t* __restrict__ host_terminals,
                                                        const int32_t* __restrict__ host_actions, uint8_t* __restrict__ frames_out,
                                                        float* __restrict__ rewards_out, uint8_t* __restrict__ terminals_out,
                                                        int32_t* __restrict__ actions_out)
{
    const int j = blockIdx.x;
    uint4* st = reinterpret_cast<uint4*>(states + static_cast<size_t>(j) * kStateBytes);
    const uint4* nf = reinterpret_cast<const uint4*>(host_frames + static_cast<size_t>(j) * kFrameBytes);
    uint4* keep = reinterpret_cast<uint4*>(frames_out + static_cast<size_t>(j) * kFrameBytes);
    uint4 fresh[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {   // 441 vectors, 256 threads: both bus reads in flight before anything else
        const int v = threadIdx.x + i * 256;
        fresh[i] = nf[v < kFrameVec16 ? v : kFrameVec16 - 1];
    }
    const uint8_t term = host_terminals[j];
    const uint32_t keep_old = term ? 0u : 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int v = threadIdx.x + i * 256;
        if (v >= kFrameVec16) break;
        uint4 f1 = st[kFrameVec16 + v], f2 = st[2 * kFrameVec16 + v], f3 = st[3 * kFrameVec16 + v];
        f1.x &= keep_old; f1.y &= keep_old; f1.z &= keep_old; f1.w &= keep_old;
        f2.x &= keep_old; f2.y &= keep_old; f2.z &= keep_old; f2.w &= keep_old;
        f3.x &= keep_old; f3.y &= keep_old; f3.z &= keep_old; f3.w &= keep_old;
        st[v] = f1; st[kFrameVec16 + v] = f2; st[2 * kFrameVec16 + v] = f3;
        st[3 * kFrameVec16 + v] = fresh[i];
        keep[v] = fresh[i];
    }
    if (threadIdx.x == 0) {
        terminals_out[j] = term;
        rewards_out[j] = host_rewards[j];
        actions_out[j] = host_actions[j];
    }
}

}  // namespace
}  // namespace dqn

using namespace dqn;

struct dqn_alg1 {
    dqn_ctx* ctx = nullptr;
    replay* rb = nullptr;
    dqn_alg1_config cfg{};
    int A = 0;
    hipStream_t act_stream = nullptr;
    uint64_t key_env = 0, key_meta = 0;
    uint32_t t_neg = 0, t_pos = 0, t_term = 0;
    // pinned host arrays shared between the main thread and the sampler threads
    uint8_t* h_frames[2] = {nullptr, nullptr};   // [W][84*84]: observations o_n / o_{n+1}, alternating
    int32_t* h_actions = nullptr;
    float* h_rewards = nullptr;
    uint8_t* h_terminals = nullptr;
    // the pinned arrays as the device addresses them
    uint8_t* hd_frames[2] = {nullptr, nullptr};
    int32_t* hd_actions = nullptr;
    float* hd_rewards = nullptr;
    uint8_t* hd_terminals = nullptr;
    // device side of the same
    uint8_t* d_frames[2] = {nullptr, nullptr};
    uint8_t* d_states = nullptr;                 // [W][4][84][84]
    int32_t* d_actions = nullptr;
    float* d_rewards = nullptr;
    uint8_t* d_terminals = nullptr;
    // progress
    int64_t n = 0;            // steps every environment has taken
    int cur = 0;              // d_frames[cur] holds o_n
    bool started = false;     // o_0 generated, states initialised
    bool pending = false;     // experience n-1 is complete on the device and not yet appended
    int64_t t = 0, act_steps = 0, train_steps = 0, episodes = 0;
    double reward_sum = 0.0;
    // worker threads: tasks are handed out by generation number
    std::mutex mu;
    std::condition_variable cv_work, cv_done;
    std::atomic<uint64_t> sampler_gen{0};   // written under mu; the samplers first spin on it, then block on cv_work
    uint64_t trainer_gen = 0;
    int sampler_task = 0;     // 0: observation o_0, 1: one environment step, 2: own network query + environment step
    float task_epsilon = 0.f; // task 2: exploration rate and parameter set of the query
    int task_use_target = 1;
    std::atomic<int> samplers_done{0};
    int sampler_rc = DQN_OK;  // first error of a sampler thread's device calls
    char sampler_err[256] = {0};
    std::mutex gpu_mu;        // serialises the sampler threads' device calls (task 2)
    hipEvent_t ev_query[kMaxLanes] = {};
    bool trainer_busy = false;
    std::atomic<bool> stop{false};
    int trainer_rc = DQN_OK;
    char trainer_err[256] = {0};
    int64_t trainer_first = 0;
    int trainer_count = 0;
    std::vector<std::thread> samplers;
    std::thread trainer;
};

namespace {

// One step of environment j with the action in the shared array: (r_n, d_n) and o_{n+1} into the shared arrays.
void sampler_env_step(dqn_alg1* h, int j, int64_t n, int nb)
{
    const int W = h->cfg.W;
    const auto t0 = std::chrono::steady_clock::now();
    const uint64_t id = static_cast<uint64_t>(n) * W + j;
    const uint64_t w = mix64_host(mix64_host(h->key_meta + id) + kGammaEnv);
    const uint32_t rbits = static_cast<uint32_t>(w & 0xFFFFFFu), tbits = static_cast<uint32_t>((w >> 24) & 0xFFFFFFu);
    const uint32_t abits = static_cast<uint32_t>((w >> 48) & 0xFFFFu);
    const int good = static_cast<int>((abits * static_cast<uint32_t>(h->A)) >> 16);
    float r = rbits < h->t_neg ? -1.f : (rbits >= (1u << 24) - h->t_pos ? 1.f : 0.f);
    if (h->h_actions[j] != good) r = 0.f;
    h->h_rewards[j] = r;
    h->h_terminals[j] = tbits < h->t_term ? 1 : 0;
    env_frame_host(h->key_env, id + W, h->h_frames[nb] + static_cast<size_t>(j) * kFrameBytes);
    if (h->cfg.env_step_ns) {   // stand-in for the emulator's own time per step
        const auto until = t0 + std::chrono::nanoseconds(h->cfg.env_step_ns);
        while (std::chrono::steady_clock::now() < until) {}
    }
}

// Without Synchronized Execution: sampler j evaluates its own state (a minibatch of one) and fetches its action.
int sampler_query(dqn_alg1* h, int j, int64_t n)
{
    {
        std::lock_guard<std::mutex> g(h->gpu_mu);
        const int rc = dqn_act(h->ctx, h->d_states + static_cast<size_t>(j) * kStateBytes, 1, h->task_epsilon,
                               static_cast<uint64_t>(h->act_steps) * h->cfg.W + j, h->task_use_target, h->d_actions + j, nullptr);
        if (rc != DQN_OK) return rc;
        DQN_HIP(hipMemcpyAsync(h->h_actions + j, h->d_actions + j, sizeof(int32_t), hipMemcpyDeviceToHost, h->act_stream));
        DQN_HIP(hipEventRecord(h->ev_query[j], h->act_stream));
    }
    (void)n;
    DQN_HIP(hipEventSynchronize(h->ev_query[j]));
    return DQN_OK;
}

// ... and hands its experience and its next observation to the device by itself.
int sampler_commit(dqn_alg1* h, int j, int nb)
{
    std::lock_guard<std::mutex> g(h->gpu_mu);
    uint8_t* stack = h->d_states + static_cast<size_t>(j) * kStateBytes;
    uint8_t* fresh = h->d_frames[nb] + static_cast<size_t>(j) * kFrameBytes;
    DQN_HIP(hipMemcpyAsync(fresh, h->h_frames[nb] + static_cast<size_t>(j) * kFrameBytes, kFrameBytes, hipMemcpyHostToDevice, h->act_stream));
    DQN_HIP(hipMemcpyAsync(h->d_rewards + j, h->h_rewards + j, sizeof(float), hipMemcpyHostToDevice, h->act_stream));
    DQN_HIP(hipMemcpyAsync(h->d_terminals + j, h->h_terminals + j, 1, hipMemcpyHostToDevice, h->act_stream));
    // the newest frame of the stack is the observation the action was taken on
    const int rc = replay_push(h->rb, j, stack + 3 * kFrameBytes, h->d_actions + j, h->d_rewards + j, h->d_terminals + j, 1);
    if (rc != DQN_OK) return rc;
    hipLaunchKernelGGL(env_advance_kernel, dim3(1), dim3(256), 0, h->act_stream, stack, fresh, h->d_terminals + j);
    DQN_LAUNCH_CHECK();
    return DQN_OK;
}

void sampler_main(dqn_alg1* h, int j)
{
    uint64_t seen = 0;
    for (;;) {
        int task;
        int64_t n;
        int nb;
        {
            // a round follows the last one within tens of microseconds: spin that long before going to sleep
            const auto t0 = std::chrono::steady_clock::now();
            bool go = false;
            while (!(go = h->stop.load(std::memory_order_acquire) || h->sampler_gen.load(std::memory_order_acquire) != seen)) {
                __builtin_ia32_pause();
                if (std::chrono::steady_clock::now() - t0 > kSpin) break;
            }
            if (!go) {
                std::unique_lock<std::mutex> lk(h->mu);
                h->cv_work.wait(lk, [&] { return h->stop.load() || h->sampler_gen.load() != seen; });
            }
            if (h->stop.load(std::memory_order_acquire)) return;
            seen = h->sampler_gen.load(std::memory_order_acquire);
            task = h->sampler_task; n = h->n; nb = h->cur ^ 1;   // written before the generation was published
        }
        const int W = h->cfg.W;
        int rc = DQN_OK;
        if (task == 0) {
            env_frame_host(h->key_env, static_cast<uint64_t>(j), h->h_frames[h->cur] + static_cast<size_t>(j) * kFrameBytes);
        } else {
            if (task == 2) rc = sampler_query(h, j, n);
            if (rc == DQN_OK) {
                sampler_env_step(h, j, n, nb);
                if (task == 2) rc = sampler_commit(h, j, nb);
            }
        }
        if (rc != DQN_OK) {
            std::lock_guard<std::mutex> lk(h->mu);
            if (h->sampler_rc == DQN_OK) {
                h->sampler_rc = rc;
                snprintf(h->sampler_err, sizeof(h->sampler_err), "%s", dqn_last_error());
            }
        }
        if (h->samplers_done.fetch_add(1, std::memory_order_acq_rel) + 1 == W) {
            { std::lock_guard<std::mutex> lk(h->mu); }   // the main thread is either still spinning or already inside wait()
            h->cv_done.notify_all();
        }
    }
}

void trainer_main(dqn_alg1* h)
{
    uint64_t seen = 0;
    for (;;) {
        int64_t first;
        int count;
        {
            std::unique_lock<std::mutex> lk(h->mu);
            h->cv_work.wait(lk, [&] { return h->stop.load() || h->trainer_gen != seen; });
            if (h->stop.load()) return;
            seen = h->trainer_gen;
            first = h->trainer_first; count = h->trainer_count;
        }
        int rc = DQN_OK;
        for (int i = 0; i < count && rc == DQN_OK; ++i)
            rc = dqn_train_step_sampled(h->ctx, h->rb, h->cfg.B, static_cast<uint64_t>(first + i), i + 1 < count, nullptr);
        {
            std::lock_guard<std::mutex> lk(h->mu);
            h->trainer_rc = rc;
            if (rc != DQN_OK) snprintf(h->trainer_err, sizeof(h->trainer_err), "%s", dqn_last_error());
            h->trainer_busy = false;
            h->cv_done.notify_all();
        }
    }
}

void run_samplers(dqn_alg1* h, int task)
{
    const int W = h->cfg.W;
    {
        std::lock_guard<std::mutex> lk(h->mu);
        h->sampler_task = task;
        h->samplers_done.store(0, std::memory_order_relaxed);
        h->sampler_gen.fetch_add(1, std::memory_order_release);
    }
    h->cv_work.notify_all();
    const auto t0 = std::chrono::steady_clock::now();
    while (h->samplers_done.load(std::memory_order_acquire) != W) {
        __builtin_ia32_pause();
        if (std::chrono::steady_clock::now() - t0 > kSpin) {
            std::unique_lock<std::mutex> lk(h->mu);
            h->cv_done.wait(lk, [&] { return h->samplers_done.load(std::memory_order_acquire) == W; });
            break;
        }
    }
}

int wait_trainer(dqn_alg1* h)
{
    std::unique_lock<std::mutex> lk(h->mu);
    h->cv_done.wait(lk, [&] { return !h->trainer_busy; });
    if (h->trainer_rc != DQN_OK) {
        const int rc = h->trainer_rc;
        h->trainer_rc = DQN_OK;
        return fail(rc, "trainer thread: %s", h->trainer_err);
    }
    return DQN_OK;
}

// Hands what the samplers just produced for step n (a_n, r_n, d_n, o_{n+1}) to the device and advances the frame stacks.
int advance_round(dqn_alg1* h)
{
    const int W = h->cfg.W, nb = h->cur ^ 1;
    hipLaunchKernelGGL(env_round_kernel, dim3(W), dim3(256), 0, h->act_stream, h->d_states, h->hd_frames[nb], h->hd_rewards, h->hd_terminals,
                       h->hd_actions, h->d_frames[nb], h->d_rewards, h->d_terminals, h->d_actions);
    DQN_LAUNCH_CHECK();
    return DQN_OK;
}

int start_envs(dqn_alg1* h)
{
    const int W = h->cfg.W;
    run_samplers(h, 0);   // o_0 of every environment into h_frames[cur]
    for (int j = 0; j < W; ++j) h->h_terminals[j] = 1;   // "episode start": the stack keeps only the new observation
    DQN_HIP(hipMemcpyAsync(h->d_frames[h->cur], h->h_frames[h->cur], static_cast<size_t>(W) * kFrameBytes, hipMemcpyHostToDevice, h->act_stream));
    DQN_HIP(hipMemcpyAsync(h->d_terminals, h->h_terminals, W, hipMemcpyHostToDevice, h->act_stream));
    hipLaunchKernelGGL(env_advance_kernel, dim3(W), dim3(256), 0, h->act_stream, h->d_states, h->d_frames[h->cur], h->d_terminals);
    DQN_LAUNCH_CHECK();
    DQN_HIP(hipStreamSynchronize(h->act_stream));   // h_terminals is reused by the samplers
    h->started = true;
    return DQN_OK;
}

int sampler_error(dqn_alg1* h)
{
    std::lock_guard<std::mutex> lk(h->mu);
    if (h->sampler_rc == DQN_OK) return DQN_OK;
    const int rc = h->sampler_rc;
    h->sampler_rc = DQN_OK;
    return fail(rc, "sampler thread: %s", h->sampler_err);
}

// One round without Synchronized Execution: every sampler thread queries the network for its own state, steps its
// environment and hands the experience and the next observation to the device itself.
int round_unsynchronized(dqn_alg1* h, float epsilon, int use_target)
{
    const int W = h->cfg.W;
    h->task_epsilon = epsilon;
    h->task_use_target = use_target;
    run_samplers(h, 2);
    const int rc = sampler_error(h);
    if (rc != DQN_OK) return rc;
    for (int j = 0; j < W; ++j) { h->reward_sum += h->h_rewards[j]; h->episodes += h->h_terminals[j]; }
    ++h->act_steps;
    h->cur ^= 1;
    ++h->n;
    h->t += W;
    return DQN_OK;
}

// One act step: Q for all W states in one minibatch, actions to the samplers, one environment step each.
int act_step(dqn_alg1* h, float epsilon, int use_target)
{
    if (!h->cfg.synchronized) return round_unsynchronized(h, epsilon, use_target);
    const int W = h->cfg.W;
    int rc;
    if (h->pending) {
        // experience n-1 = (o_{n-1}, a_{n-1}, r_{n-1}, d_{n-1}) rides in this step's launches, from the device copies the last
        // round left; the new actions go straight into the pinned array
        rc = dqn_act_push_step(h->ctx, h->rb, h->d_frames[h->cur ^ 1], h->d_actions, h->d_rewards, h->d_terminals, h->d_states, W, epsilon,
                               static_cast<uint64_t>(h->act_steps), use_target, h->hd_actions, nullptr);
        h->pending = false;
    } else {
        rc = dqn_act(h->ctx, h->d_states, W, epsilon, static_cast<uint64_t>(h->act_steps), use_target, h->hd_actions, nullptr);
    }
    if (rc != DQN_OK) return rc;
    DQN_HIP(hipStreamSynchronize(h->act_stream));
    ++h->act_steps;
    run_samplers(h, 1);
    for (int j = 0; j < W; ++j) { h->reward_sum += h->h_rewards[j]; h->episodes += h->h_terminals[j]; }
    rc = advance_round(h);
    if (rc != DQN_OK) return rc;
    h->cur ^= 1;
    ++h->n;
    h->pending = true;
    h->t += W;
    return DQN_OK;
}

// Appends the pending experience by itself (in front of a flush).
int append_pending(dqn_alg1* h)
{
    if (!h->pending) return DQN_OK;
    const int rc = replay_push_step(h->rb, h->d_frames[h->cur ^ 1], h->d_actions, h->d_rewards, h->d_terminals);
    if (rc != DQN_OK) return rc;
    h->pending = false;
    return DQN_OK;
}

}  // namespace

extern "C" {

int dqn_alg1_create(dqn_ctx* ctx, replay* rb, const dqn_alg1_config* cfg, dqn_alg1** out)
{
    if (!ctx || !rb || !cfg || !out) return fail(DQN_EINVAL, "dqn_alg1_create: null pointer");
    const int W = cfg->W;
    if (W < 1 || W > dqn_ctx_max_envs(ctx) || W > kMaxLanes) return fail(DQN_EINVAL, "dqn_alg1_create: W = %d outside 1..%d", W, dqn_ctx_max_envs(ctx));
    if (replay_lanes(rb) != W) return fail(DQN_EINVAL, "dqn_alg1_create: the replay memory needs one lane per sampler (%d lanes, W = %d)", replay_lanes(rb), W);
    if (replay_push_stream(rb) != dqn_ctx_act_stream(ctx)) return fail(DQN_EINVAL, "dqn_alg1_create: the replay's push stream must be the act stream");
    if (cfg->C < 1 || cfg->F < 1 || cfg->C % W != 0 || cfg->C % cfg->F != 0)
        return fail(DQN_EINVAL, "dqn_alg1_create: C = %d must be a positive multiple of W = %d and of F = %d", cfg->C, W, cfg->F);
    if (cfg->B < 1 || cfg->B > dqn_ctx_max_batch(ctx)) return fail(DQN_EINVAL, "dqn_alg1_create: B = %d outside 1..%d", cfg->B, dqn_ctx_max_batch(ctx));
    if (!(cfg->epsilon >= 0.f && cfg->epsilon <= 1.f)) return fail(DQN_EINVAL, "dqn_alg1_create: epsilon outside [0,1]");
    if (cfg->t_reward_neg > (1u << 24) || cfg->t_reward_pos > (1u << 24) || cfg->t_term > (1u << 24) ||
        static_cast<uint64_t>(cfg->t_reward_neg) + cfg->t_reward_pos > (1u << 24))
        return fail(DQN_EINVAL, "dqn_alg1_create: environment thresholds exceed 2^24");
    if ((cfg->concurrent != 0 && cfg->concurrent != 1) || (cfg->synchronized != 0 && cfg->synchronized != 1))
        return fail(DQN_EINVAL, "dqn_alg1_create: concurrent and synchronized must be 0 or 1");
    dqn_alg1* h = new (std::nothrow) dqn_alg1();
    if (!h) return fail(DQN_ENOMEM, "dqn_alg1_create: host allocation failed");
    h->ctx = ctx; h->rb = rb; h->cfg = *cfg; h->A = dqn_ctx_num_actions(ctx); h->act_stream = dqn_ctx_act_stream(ctx);
    h->key_env = mix64_host(cfg->env_seed + kGammaEnv * (kStreamEnv + 1ull));
    h->key_meta = mix64_host(cfg->env_seed + kGammaEnv * (kStreamEnvMeta + 1ull));
    h->t_neg = cfg->t_reward_neg; h->t_pos = cfg->t_reward_pos; h->t_term = cfg->t_term;
    auto body = [&]() -> int {
        const size_t fb = static_cast<size_t>(W) * kFrameBytes;
        for (int i = 0; i < 2; ++i) {
            DQN_HIP(hipHostMalloc(reinterpret_cast<void**>(&h->h_frames[i]), fb, hipHostMallocDefault));
            DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_frames[i]), fb));
        }
        DQN_HIP(hipHostMalloc(reinterpret_cast<void**>(&h->h_actions), W * sizeof(int32_t), hipHostMallocDefault));
        DQN_HIP(hipHostMalloc(reinterpret_cast<void**>(&h->h_rewards), W * sizeof(float), hipHostMallocDefault));
        DQN_HIP(hipHostMalloc(reinterpret_cast<void**>(&h->h_terminals), W, hipHostMallocDefault));
        DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_states), static_cast<size_t>(W) * kStateBytes));
        DQN_HIP(hipMemset(h->d_states, 0, static_cast<size_t>(W) * kStateBytes));
        DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_actions), W * sizeof(int32_t)));
        DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_rewards), W * sizeof(float)));
        DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_terminals), W));
        for (int i = 0; i < 2; ++i) DQN_HIP(hipHostGetDevicePointer(reinterpret_cast<void**>(&h->hd_frames[i]), h->h_frames[i], 0));
        DQN_HIP(hipHostGetDevicePointer(reinterpret_cast<void**>(&h->hd_actions), h->h_actions, 0));
        DQN_HIP(hipHostGetDevicePointer(reinterpret_cast<void**>(&h->hd_rewards), h->h_rewards, 0));
        DQN_HIP(hipHostGetDevicePointer(reinterpret_cast<void**>(&h->hd_terminals), h->h_terminals, 0));
        for (int j = 0; j < W; ++j) DQN_HIP(hipEventCreateWithFlags(&h->ev_query[j], hipEventDisableTiming));
        DQN_HIP(hipDeviceSynchronize());
        return DQN_OK;
    };
    const int rc = body();
    if (rc != DQN_OK) {
        char saved[512];
        snprintf(saved, sizeof(saved), "%s", error_buffer());
        dqn_alg1_destroy(h);
        return fail(rc, "dqn_alg1_create: %s", saved);
    }
    for (int j = 0; j < W; ++j) h->samplers.emplace_back(sampler_main, h, j);
    h->trainer = std::thread(trainer_main, h);
    *out = h;
    return DQN_OK;
}

int dqn_alg1_destroy(dqn_alg1* h)
{
    if (!h) return DQN_OK;
    {
        std::unique_lock<std::mutex> lk(h->mu);
        h->cv_done.wait(lk, [&] { return !h->trainer_busy; });
        h->stop.store(true, std::memory_order_release);
        h->cv_work.notify_all();
    }
    for (std::thread& t : h->samplers) t.join();
    if (h->trainer.joinable()) h->trainer.join();
    if (h->act_stream) (void)hipStreamSynchronize(h->act_stream);
    for (int i = 0; i < 2; ++i) { (void)hipHostFree(h->h_frames[i]); (void)hipFree(h->d_frames[i]); }
    for (int j = 0; j < kMaxLanes; ++j)
        if (h->ev_query[j]) (void)hipEventDestroy(h->ev_query[j]);
    (void)hipHostFree(h->h_actions); (void)hipHostFree(h->h_rewards); (void)hipHostFree(h->h_terminals);
    (void)hipFree(h->d_states); (void)hipFree(h->d_actions); (void)hipFree(h->d_rewards); (void)hipFree(h->d_terminals);
    delete h;
    return DQN_OK;
}

int dqn_alg1_prepopulate(dqn_alg1* h, int64_t timesteps)
{
    if (!h) return fail(DQN_EINVAL, "dqn_alg1_prepopulate: handle is null");
    if (timesteps < 0 || timesteps % h->cfg.W != 0) return fail(DQN_EINVAL, "dqn_alg1_prepopulate: timesteps must be a multiple of W");
    int rc = wait_trainer(h);
    if (rc != DQN_OK) return rc;
    if (!h->started && (rc = start_envs(h)) != DQN_OK) return rc;
    const int64_t t0 = h->t;
    for (int64_t k = 0; k < timesteps / h->cfg.W; ++k)
        if ((rc = act_step(h, 1.f, 1)) != DQN_OK) return rc;
    h->t = t0;   // prepopulation does not count as timesteps of the algorithm
    if ((rc = append_pending(h)) != DQN_OK) return rc;
    return replay_flush(h->rb, 1);
}

int dqn_alg1_run(dqn_alg1* h, int64_t timesteps)
{
    if (!h) return fail(DQN_EINVAL, "dqn_alg1_run: handle is null");
    if (timesteps < 0 || timesteps % h->cfg.C != 0) return fail(DQN_EINVAL, "dqn_alg1_run: timesteps must be a multiple of C");
    int rc;
    if (!h->started && (rc = start_envs(h)) != DQN_OK) return rc;
    const int W = h->cfg.W, C = h->cfg.C, F = h->cfg.F;
    for (int64_t block = 0; block < timesteps / C; ++block) {
        // t mod C == 0: the samplers are idle (they only run inside act_step); wait for the trainer, then synchronise
        if ((rc = wait_trainer(h)) != DQN_OK) return rc;
        if ((rc = append_pending(h)) != DQN_OK) return rc;
        if ((rc = dqn_sync_target(h->ctx, h->rb, 0)) != DQN_OK) return rc;
        if (h->cfg.concurrent) {
            {
                std::lock_guard<std::mutex> lk(h->mu);
                h->trainer_first = h->train_steps;
                h->trainer_count = C / F;
                h->trainer_busy = true;
                ++h->trainer_gen;
                h->cv_work.notify_all();
            }
            h->train_steps += C / F;
            for (int k = 0; k < C / W; ++k)
                if ((rc = act_step(h, h->cfg.epsilon, 1)) != DQN_OK) return rc;
            continue;
        }
        // standard DQN (Section 2.1): act from theta; the round's experiences enter D at once; then the train steps that
        // have become due, on this thread -- the next round's Q evaluation waits for them on the device
        for (int k = 0; k < C / W; ++k) {
            if ((rc = act_step(h, h->cfg.epsilon, 0)) != DQN_OK) return rc;
            if ((rc = append_pending(h)) != DQN_OK) return rc;
            if ((rc = replay_flush(h->rb, 0)) != DQN_OK) return rc;
            while (h->train_steps < h->t / F) {
                if ((rc = dqn_train_step_sampled(h->ctx, h->rb, h->cfg.B, static_cast<uint64_t>(h->train_steps), 0, nullptr)) != DQN_OK) return rc;
                ++h->train_steps;
            }
        }
    }
    return wait_trainer(h);   // every launch of the last block has been issued when this returns
}

int dqn_alg1_flush(dqn_alg1* h)
{
    if (!h) return fail(DQN_EINVAL, "dqn_alg1_flush: handle is null");
    int rc = wait_trainer(h);
    if (rc != DQN_OK) return rc;
    if ((rc = append_pending(h)) != DQN_OK) return rc;
    return replay_flush(h->rb, 1);
}

int dqn_alg1_stats(const dqn_alg1* h, int64_t* host_t, int64_t* host_act_steps, int64_t* host_train_steps, double* host_reward_sum,
                   int64_t* host_episodes)
{
    if (!h) return fail(DQN_EINVAL, "dqn_alg1_stats: handle is null");
    if (host_t) *host_t = h->t;
    if (host_act_steps) *host_act_steps = h->act_steps;
    if (host_train_steps) *host_train_steps = h->train_steps;
    if (host_reward_sum) *host_reward_sum = h->reward_sum;
    if (host_episodes) *host_episodes = h->episodes;
    return DQN_OK;
}

}  // extern "C"
