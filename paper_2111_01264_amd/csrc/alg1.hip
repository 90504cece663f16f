// Algorithm 1 (DQN with Concurrent Training and Synchronized Execution, main thread) as a native host orchestrator:
// W sampler threads and one trainer thread around the hot-path calls of this library.
//
//   * every C timesteps: wait for the trainer and the samplers, flush the temporary buffers into D, theta^- <- theta
//     (dqn_sync_target), dispatch the trainer thread for C / F minibatches;
//   * every W timesteps: wait for the samplers, evaluate Q(s^(j), .) for all W states in one minibatch (Section 4),
//     hand every sampler its action;
//   * a sampler thread takes one step in its environment with that action.
//
// The environments are synthetic (a seeded frame generator stands in for the Atari emulator, see the header): they
// live on the host, as an emulator would, one per sampler thread, and talk to the device through the shared arrays of
// dqn_envs (pinned memory that threads and kernels both address; the frame stacks stay on the device).
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

#include "envs.h"

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
constexpr std::chrono::microseconds kSpin(200);          // how long a thread polls for its next task before it blocks ...
constexpr int kSpinMaxSamplers = 12;                     // ... if the sampler threads are few enough to have a core each while polling

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

// Without Synchronized Execution: shift ONE environment's frame stack and append its new observation from a device
// copy; a stack whose previous step ended an episode keeps only the new observation.
__global__ __launch_bounds__(256) void env_advance_kernel(uint8_t* __restrict__ stack, const uint8_t* __restrict__ new_frame,
                                                          const uint8_t* __restrict__ terminal)
{
    uint4* st = reinterpret_cast<uint4*>(stack);
    const uint4* nf = reinterpret_cast<const uint4*>(new_frame);
    const uint32_t keep_old = terminal[0] ? 0u : 0xFFFFFFFFu;
    for (int v = threadIdx.x; v < kFrameVec16; v += blockDim.x) {
        uint4 f1 = st[kFrameVec16 + v], f2 = st[2 * kFrameVec16 + v], f3 = st[3 * kFrameVec16 + v];
        f1.x &= keep_old; f1.y &= keep_old; f1.z &= keep_old; f1.w &= keep_old;
        f2.x &= keep_old; f2.y &= keep_old; f2.z &= keep_old; f2.w &= keep_old;
        f3.x &= keep_old; f3.y &= keep_old; f3.z &= keep_old; f3.w &= keep_old;
        st[v] = f1; st[kFrameVec16 + v] = f2; st[2 * kFrameVec16 + v] = f3;
        st[3 * kFrameVec16 + v] = nf[v];
    }
}

}  // namespace
}  // namespace dqn

using namespace dqn;

struct dqn_alg1 {
    dqn_ctx* ctx = nullptr;
    replay* rb = nullptr;
    dqn_envs* envs = nullptr;   // shared arrays and frame stacks
    dqn_alg1_config cfg{};
    int A = 0;
    hipStream_t act_stream = nullptr;
    uint64_t key_env = 0, key_meta = 0;
    uint32_t t_neg = 0, t_pos = 0, t_term = 0;
    // without Synchronized Execution every sampler moves its own data with copy commands: device staging for them
    uint8_t* d_frames = nullptr;   // [W][84*84]
    int32_t* d_actions = nullptr;
    float* d_rewards = nullptr;
    uint8_t* d_terminals = nullptr;
    hipEvent_t ev_query[kMaxLanes] = {};
    std::mutex gpu_mu;        // serialises the sampler threads' device calls
    // progress
    int64_t n = 0;            // steps every environment has taken
    bool started = false;     // o_0 generated, stacks initialised
    int64_t t = 0, act_steps = 0, train_steps = 0, episodes = 0;
    double reward_sum = 0.0;
    // worker threads: tasks are handed out by generation number
    std::mutex mu;
    std::condition_variable cv_work, cv_done;
    std::atomic<uint64_t> sampler_gen{0};   // written under mu; the samplers first poll it, then block on cv_work
    uint64_t trainer_gen = 0;
    int sampler_task = 0;     // 0: observation o_0, 1: one environment step, 2: own network query + environment step
    float task_epsilon = 0.f; // task 2: exploration rate and parameter set of the query
    int task_use_target = 1;
    std::atomic<int> samplers_done{0};
    int sampler_rc = DQN_OK;  // first error of a sampler thread's device calls
    char sampler_err[256] = {0};
    bool trainer_busy = false;
    std::atomic<bool> stop{false};
    std::chrono::microseconds spin{0};   // polling time before a thread blocks (0: block at once)
    int trainer_rc = DQN_OK;
    char trainer_err[256] = {0};
    int64_t trainer_first = 0;
    int trainer_count = 0;
    std::vector<std::thread> samplers;
    std::thread trainer;
};

namespace {

// One step of environment j with the action in the shared array: (r_n, d_n) and o_{n+1} into the shared arrays.
void sampler_env_step(dqn_alg1* h, int j, int64_t n)
{
    const int W = h->cfg.W;
    dqn_envs* e = h->envs;
    const auto t0 = std::chrono::steady_clock::now();
    const uint64_t id = static_cast<uint64_t>(n) * W + j;
    const uint64_t w = mix64_host(mix64_host(h->key_meta + id) + kGammaEnv);
    const uint32_t rbits = static_cast<uint32_t>(w & 0xFFFFFFu), tbits = static_cast<uint32_t>((w >> 24) & 0xFFFFFFu);
    const uint32_t abits = static_cast<uint32_t>((w >> 48) & 0xFFFFu);
    const int good = static_cast<int>((abits * static_cast<uint32_t>(h->A)) >> 16);
    float r = rbits < h->t_neg ? -1.f : (rbits >= (1u << 24) - h->t_pos ? 1.f : 0.f);
    if (e->h_actions[j] != good) r = 0.f;
    e->h_rewards[j] = r;
    e->h_terminals[j] = tbits < h->t_term ? 1 : 0;
    env_frame_host(h->key_env, id + W, e->h_obs + static_cast<size_t>(j) * kFrameBytes);
    if (h->cfg.env_step_ns) {   // stand-in for the emulator's own time per step
        const auto until = t0 + std::chrono::nanoseconds(h->cfg.env_step_ns);
        while (std::chrono::steady_clock::now() < until) {}
    }
}

// Without Synchronized Execution: sampler j evaluates its own state (a minibatch of one) and fetches its action.
int sampler_query(dqn_alg1* h, int j)
{
    dqn_envs* e = h->envs;
    {
        std::lock_guard<std::mutex> g(h->gpu_mu);
        const int rc = dqn_act(h->ctx, e->d_states + static_cast<size_t>(j) * kStateBytes, 1, h->task_epsilon,
                               static_cast<uint64_t>(h->act_steps) * h->cfg.W + j, h->task_use_target, h->d_actions + j, nullptr);
        if (rc != DQN_OK) return rc;
        DQN_HIP(hipMemcpyAsync(e->h_actions + j, h->d_actions + j, sizeof(int32_t), hipMemcpyDeviceToHost, h->act_stream));
        DQN_HIP(hipEventRecord(h->ev_query[j], h->act_stream));
    }
    DQN_HIP(hipEventSynchronize(h->ev_query[j]));
    return DQN_OK;
}

// ... and hands its experience and its next observation to the device by itself.
int sampler_commit(dqn_alg1* h, int j)
{
    dqn_envs* e = h->envs;
    std::lock_guard<std::mutex> g(h->gpu_mu);
    uint8_t* stack = e->d_states + static_cast<size_t>(j) * kStateBytes;
    uint8_t* fresh = h->d_frames + static_cast<size_t>(j) * kFrameBytes;
    DQN_HIP(hipMemcpyAsync(fresh, e->h_obs + static_cast<size_t>(j) * kFrameBytes, kFrameBytes, hipMemcpyHostToDevice, h->act_stream));
    DQN_HIP(hipMemcpyAsync(h->d_rewards + j, e->h_rewards + j, sizeof(float), hipMemcpyHostToDevice, h->act_stream));
    DQN_HIP(hipMemcpyAsync(h->d_terminals + j, e->h_terminals + j, 1, hipMemcpyHostToDevice, h->act_stream));
    // the newest frame of the stack is the observation the action was taken on
    const int rc = replay_push(h->rb, j, stack + 3 * kFrameBytes, h->d_actions + j, h->d_rewards + j, h->d_terminals + j, 1);
    if (rc != DQN_OK) return rc;
    hipLaunchKernelGGL(env_advance_kernel, dim3(1), dim3(256), 0, h->act_stream, stack, fresh, h->d_terminals + j);
    DQN_LAUNCH_CHECK();
    // the pinned arrays are rewritten in the next round: the copies out of them must have been made by then
    DQN_HIP(hipEventRecord(h->ev_query[j], h->act_stream));
    return DQN_OK;
}

void sampler_main(dqn_alg1* h, int j)
{
    uint64_t seen = 0;
    for (;;) {
        int task;
        int64_t n;
        {
            // a round follows the last one within tens of microseconds: poll that long before going to sleep
            const auto t0 = std::chrono::steady_clock::now();
            bool go = false;
            while (!(go = h->stop.load(std::memory_order_acquire) || h->sampler_gen.load(std::memory_order_acquire) != seen)) {
                __builtin_ia32_pause();
                if (std::chrono::steady_clock::now() - t0 > h->spin) break;
            }
            if (!go) {
                std::unique_lock<std::mutex> lk(h->mu);
                h->cv_work.wait(lk, [&] { return h->stop.load() || h->sampler_gen.load() != seen; });
            }
            if (h->stop.load(std::memory_order_acquire)) return;
            seen = h->sampler_gen.load(std::memory_order_acquire);
            task = h->sampler_task; n = h->n;   // written before the generation was published
        }
        const int W = h->cfg.W;
        int rc = DQN_OK;
        if (task == 0) {
            env_frame_host(h->key_env, static_cast<uint64_t>(j), h->envs->h_obs + static_cast<size_t>(j) * kFrameBytes);
        } else {
            if (task == 2) rc = sampler_query(h, j);
            if (rc == DQN_OK) {
                sampler_env_step(h, j, n);
                if (task == 2) rc = sampler_commit(h, j);
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
            { std::lock_guard<std::mutex> lk(h->mu); }   // the main thread is either still polling or already inside wait()
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
        if (std::chrono::steady_clock::now() - t0 > h->spin) {
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

int sampler_error(dqn_alg1* h)
{
    std::lock_guard<std::mutex> lk(h->mu);
    if (h->sampler_rc == DQN_OK) return DQN_OK;
    const int rc = h->sampler_rc;
    h->sampler_rc = DQN_OK;
    return fail(rc, "sampler thread: %s", h->sampler_err);
}

int start_envs(dqn_alg1* h)
{
    run_samplers(h, 0);   // o_0 of every environment into the shared array
    const int rc = dqn_envs_reset(h->envs);
    if (rc != DQN_OK) return rc;
    DQN_HIP(hipStreamSynchronize(h->act_stream));   // the shared array is rewritten by the first step
    h->started = true;
    return DQN_OK;
}

// One round of W timesteps: an action for every environment, one environment step each, the experiences and the next
// observations handed to the device.
int act_step(dqn_alg1* h, float epsilon, int use_target)
{
    const int W = h->cfg.W;
    dqn_envs* e = h->envs;
    int rc;
    if (h->cfg.synchronized) {
        // Q for all W stacks in one minibatch; returns when the actions are in the shared array
        if ((rc = dqn_envs_act(e, epsilon, static_cast<uint64_t>(h->act_steps), use_target, 0)) != DQN_OK) return rc;
        run_samplers(h, 1);
        if ((rc = dqn_envs_observe(e)) != DQN_OK) return rc;
    } else {
        // every sampler thread queries the network for its own state, steps its environment and hands the experience
        // and the next observation to the device itself
        h->task_epsilon = epsilon;
        h->task_use_target = use_target;
        run_samplers(h, 2);
        if ((rc = sampler_error(h)) != DQN_OK) return rc;
        for (int j = 0; j < W; ++j) DQN_HIP(hipEventSynchronize(h->ev_query[j]));
    }
    for (int j = 0; j < W; ++j) { h->reward_sum += e->h_rewards[j]; h->episodes += e->h_terminals[j]; }
    ++h->act_steps;
    ++h->n;
    h->t += W;
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
    h->spin = W <= kSpinMaxSamplers ? kSpin : std::chrono::microseconds(0);
    auto body = [&]() -> int {
        const int rc = dqn_envs_create(ctx, rb, W, &h->envs);
        if (rc != DQN_OK) return rc;
        if (!cfg->synchronized) {
            DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_frames), static_cast<size_t>(W) * kFrameBytes));
            DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_actions), W * sizeof(int32_t)));
            DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_rewards), W * sizeof(float)));
            DQN_HIP(hipMalloc(reinterpret_cast<void**>(&h->d_terminals), W));
            for (int j = 0; j < W; ++j) DQN_HIP(hipEventCreateWithFlags(&h->ev_query[j], hipEventDisableTiming));
        }
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
    (void)dqn_envs_destroy(h->envs);
    (void)hipFree(h->d_frames); (void)hipFree(h->d_actions); (void)hipFree(h->d_rewards); (void)hipFree(h->d_terminals);
    for (int j = 0; j < kMaxLanes; ++j)
        if (h->ev_query[j]) (void)hipEventDestroy(h->ev_query[j]);
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
    const int rc = wait_trainer(h);
    if (rc != DQN_OK) return rc;
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
