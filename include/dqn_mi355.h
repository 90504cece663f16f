/*
 * dqn_mi355.h -- C boundary of the MI355X (gfx950) DQN hot-path library.
 *
 * The calls follow the problem statement of "Human-Level Control without Server-Grade Hardware"
 * (Daley & Amato): Section 2.1 (Q-network, Eq. 1, replay memory D, target network, epsilon-greedy),
 * Section 3 (Concurrent Training: actions from the target parameters, experiences buffered until
 * the synchronisation point), Section 4 (Synchronized Execution: one minibatch of W states per act
 * step), Algorithm 1 (flush + target update every C timesteps), Appendix B / Table 5 (RMSProp
 * constants, gamma, minibatch size).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name starts with host_.  The caller owns every
 *     buffer it passes in; the library owns what lives inside the opaque handles.
 *   - Streams are hipStream_t values passed as void*.  Calls only ENQUEUE work on their stream and
 *     return; they do not synchronise with the host, except dqn_get_params, dqn_get_train_q,
 *     dqn_set_params, and dqn_sync_target / replay_flush with blocking != 0.
 *   - Every call returns DQN_OK or a negative code, never throws, aborts or prints;
 *     dqn_last_error() returns a thread-local message for the last failing call.  Arguments are
 *     validated on the host before anything is launched; a failing call launches nothing.
 *   - Image tensors are uint8 [n, 4, 84, 84] (stacked states) or [n, 84, 84] (single frames),
 *     densely packed, 16-byte aligned.
 *   - Parameter blobs are flat float32 in this order and layout:
 *       conv1.w [32,4,8,8], conv1.b [32], conv2.w [64,32,4,4], conv2.b [64], conv3.w [64,64,3,3],
 *       conv3.b [64], fc1.w [512,3136] (input index = c*49 + h*7 + w), fc1.b [512],
 *       fc2.w [A,512], fc2.b [A].
 */
#ifndef DQN_MI355_H
#define DQN_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#pragma GCC visibility push(default)
#endif

enum { DQN_OK = 0, DQN_EINVAL = -1, DQN_EHIP = -2, DQN_ENOMEM = -3, DQN_ESTATE = -4 };

enum { DQN_PRECISION_FP32 = 0, DQN_PRECISION_BF16 = 1 };

/* dqn_get_params / dqn_set_params selector */
enum {
    DQN_PARAMS_ONLINE = 0,   /* theta                                   */
    DQN_PARAMS_TARGET = 1,   /* theta^-                                 */
    DQN_PARAMS_RMS_V = 2,    /* RMSProp second-moment accumulator       */
    DQN_PARAMS_RMS_M = 3,    /* RMSProp first-moment accumulator        */
    DQN_PARAMS_GRAD = 4      /* gradient of the last train step (get only) */
};

typedef struct dqn_ctx dqn_ctx;
typedef struct replay replay;

typedef struct {
    int32_t num_actions;   /* A, 1..32 (the paper's games use 4..18)                              */
    int32_t max_batch;     /* largest minibatch dqn_train_step will see (Table 5: 32)              */
    int32_t max_envs;      /* largest W dqn_act will see (Section 4)                              */
    int32_t precision;     /* DQN_PRECISION_FP32: fp32 operands on fp32 MFMA;
                              DQN_PRECISION_BF16: bf16 operands on bf16 MFMA, fp32 accumulation,
                              fp32 master parameters and optimiser state                           */
    int32_t double_dqn;    /* 0: Eq. 1 (max over theta^-); 1: argmax from theta, value from theta^- */
    int32_t centered;      /* 1: centered RMSProp (Appendix B); 0: plain RMSProp                   */
    float gamma;           /* discount, Table 5: 0.99                                              */
    float huber_delta;     /* error-clipping threshold of the adopted setup: 1                     */
    float lr;              /* Appendix B: 2.5e-4                                                   */
    float rms_alpha;       /* Appendix B: 0.95 for both moments                                    */
    float rms_eps;         /* Appendix B: 0.01, added to the denominator outside the square root   */
    uint64_t seed;         /* key of the counter-based generator used by the epsilon-greedy draws  */
} dqn_config;

/* ---- lifetime ------------------------------------------------------------------------------- */

/* Creates a context on the current device.  Parameters start at zero; load them with
 * dqn_set_params.  act_stream carries dqn_act, train_stream carries dqn_train_step (Section 3:
 * the two run concurrently between synchronisation points).  Errors: DQN_EINVAL (bad config,
 * null pointer), DQN_ENOMEM, DQN_EHIP. */
int dqn_create(const dqn_config* host_cfg, void* act_stream, void* train_stream, dqn_ctx** host_out);
int dqn_destroy(dqn_ctx* ctx);

size_t dqn_num_params(const dqn_ctx* ctx);

/* Copies a float32 blob (layout above) from / to host memory.  n must equal dqn_num_params().
 * Both wait for the context's two streams first.  Setting DQN_PARAMS_ONLINE or DQN_PARAMS_TARGET
 * also refreshes that network's low-precision operand copy.  DQN_PARAMS_GRAD cannot be set. */
int dqn_set_params(dqn_ctx* ctx, int which, const float* host_src, size_t n);
int dqn_get_params(dqn_ctx* ctx, int which, float* host_dst, size_t n);

/* ---- act step (Sections 3 and 4, Algorithm 1's batched Q evaluation) --------------------- */

/* Evaluates Q(s^(j), .) for the W states in one minibatch and picks one action per environment:
 * with probability epsilon a uniformly random action, otherwise argmax_a Q (lowest index on
 * ties).  Environment j at call counter act_step uses the Philox4x32-10 outputs (x0, x1, ..) for
 * key = (seed lo, seed hi), counter = (j, 1, act_step lo, act_step hi): it explores iff
 * float(x0 >> 8) * 2^-24 < epsilon (float32 compare), and the random action is (x1 * A) >> 32.
 *   states   [W,4,84,84] uint8, scaled by 1/255 inside.
 *   use_target  1: parameters theta^- (Concurrent Training, Section 3); 0: theta (standard DQN);
 *               with 0 the call first waits, on the device, for the last enqueued train step; if another host
 *               thread is enqueuing a train step at that moment, the two calls take turns (a host-side lock),
 *               so the policy never reads parameters that a running update is overwriting.
 *   actions  [W] int32 out.   q_out  [W,A] float32 out, or NULL.
 * Runs on act_stream.  Errors: DQN_EINVAL (W < 1, W > max_envs, null/misaligned pointer,
 * epsilon outside [0,1]). */
int dqn_act(dqn_ctx* ctx, const uint8_t* states, int32_t W, float epsilon, uint64_t act_step,
            int32_t use_target, int32_t* actions, float* q_out);

/* For callers that cannot allocate device memory or keep a workspace of their own alive: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as dqn_act,
 * but every intermediate of the call (the activations between the layers and fc1's partial sums) lives in ONE
 * fixed array inside the library's device image (about 3 MiB per GPU, held until the process ends) instead of in
 * the buffers dqn_create allocated; the call itself allocates and frees nothing.  W <= DQN_ACT_STATIC_MAX_ENVS
 * (and <= max_envs), else DQN_EINVAL.  Every call on a GPU, from any context, shares that GPU's array: two such
 * calls that overlap on one GPU (different contexts or streams) race on it; calls on one act stream are ordered
 * by the stream.  Nothing in the array needs clearing between calls (every element read was written by the same
 * call).  ctx must have been created with the current device current. */
#define DQN_ACT_STATIC_MAX_ENVS 32
int dqn_act_static(dqn_ctx* ctx, const uint8_t* states, int32_t W, float epsilon, uint64_t act_step,
                   int32_t use_target, int32_t* actions, float* q_out);

/* ---- minibatch train step (Section 2.1, Eq. 1; Appendix B) -------------------------------- */

/* One gradient update of theta on a minibatch of B transitions:
 *   y_b = r_b + gamma (1 - done_b) max_a' Q(s2_b, a'; theta^-)        (double_dqn: Q(s2_b, a*; theta^-),
 *                                                                        a* = argmax_a Q(s2_b, a; theta))
 *   delta_b = Q(s_b, a_b; theta) - y_b;  loss = mean_b huber(delta_b);  no gradient through y
 *   theta <- RMSProp(theta, dloss/dtheta).   theta^- is not touched.
 *   s, s2 [B,4,84,84] uint8;  a [B] int32 in [0,A);  r, done [B] float32 (done is 0 or 1);
 *   loss_out: device float32 scalar, or NULL.
 * A row whose action lies outside [0,A) (replay_sample_gather marks a row it could not assemble with -1) is
 * checked on the device and contributes nothing: loss term 0, gradient 0; the mean still divides by B.
 * Runs on train_stream.  Errors: DQN_EINVAL (B < 1, B > max_batch, null/misaligned pointer). */
int dqn_train_step(dqn_ctx* ctx, const uint8_t* s, const int32_t* a, const float* r,
                   const uint8_t* s2, const float* done, int32_t B, float* loss_out);

/* Q rows computed inside the last dqn_train_step, copied to host memory after waiting for
 * train_stream: host_q_online [B,A] = Q(s,.;theta) (before the update), host_q_next_target [B,A] =
 * Q(s2,.;theta^-), host_q_next_online [B,A] = Q(s2,.;theta) (double_dqn only, else untouched).
 * Any pointer may be NULL.  Errors: DQN_ESTATE if no train step has run. */
int dqn_get_train_q(dqn_ctx* ctx, float* host_q_online, float* host_q_next_target,
                    float* host_q_next_online);

/* ---- synchronisation point (Algorithm 1: wait, flush, theta^- <- theta) ------------------- */

/* On the device: train_stream waits for everything enqueued on act_stream (and on rb's push
 * stream), then rb's staged experiences are flushed into D (if rb != NULL), then theta^- <- theta
 * (bitwise, plus the operand copy); act_stream (and rb's push stream) then wait for that.
 * blocking != 0 additionally waits on the host.  Must not be called concurrently with another
 * call on the same ctx / rb. */
int dqn_sync_target(dqn_ctx* ctx, replay* rb, int32_t blocking);

/* ---- replay memory D (Section 2.1; buffering of Section 3) -------------------------------- */

/* D holds capacity_frames single frames with (action, reward, terminal) each, split into `lanes`
 * equal rings (one per sampler; capacity_frames % lanes == 0, 1 <= lanes <= 64).  A terminal flag
 * means the episode ended after that frame's action.  staging_per_lane (1..capacity_frames/lanes)
 * is the number of experiences a lane can buffer between two flushes.  push_stream carries
 * replay_push, sample_stream carries replay_sample_gather and the flush.  seed keys the sampling
 * generator. */
int replay_create(int64_t capacity_frames, int32_t lanes, int64_t staging_per_lane, uint64_t seed,
                  void* push_stream, void* sample_stream, replay** host_out);
int replay_destroy(replay* rb);

/* Appends n experiences of one lane to that lane's temporary buffer; they stay invisible to
 * sampling until the next flush (Section 3).  frames [n,84,84] uint8; actions [n] int32;
 * rewards [n] float32; terminals [n] uint8.  Errors: DQN_EINVAL (lane out of range, n < 0,
 * null/misaligned pointer), DQN_ESTATE (temporary buffer would overflow). */
int replay_push(replay* rb, int32_t lane, const uint8_t* frames, const int32_t* actions,
                const float* rewards, const uint8_t* terminals, int32_t n);

/* Synchronized Execution (Section 4): all W = lanes samplers have stepped once; appends one
 * experience to every lane's temporary buffer in a single launch.  frames [lanes,84,84] uint8 (row l
 * goes to lane l); actions [lanes] int32; rewards [lanes] float32; terminals [lanes] uint8.
 * Errors as replay_push. */
int replay_push_step(replay* rb, const uint8_t* frames, const int32_t* actions, const float* rewards,
                     const uint8_t* terminals);

/* One synchronized step of the samplers as a single launch sequence (Section 4: one device
 * transaction per step for all W environments): exactly replay_push_step(rb, push_frames, push_actions,
 * push_rewards, push_terminals) -- the experiences the previous step produced -- followed by
 * dqn_act(ctx, states, W, epsilon, act_step, use_target, actions, q_out) on the states that step led
 * to; in the reduced-precision mode the append rides in the first kernel of the act step instead of
 * costing a dependent launch of its own.  push_actions may be the `actions` buffer of the previous
 * call (it is read before this call's actions are written).  The replay memory's push stream must be
 * the context's act stream.  Arguments, results and errors as for the two calls; DQN_EINVAL also if
 * the streams differ. */
int dqn_act_push_step(dqn_ctx* ctx, replay* rb, const uint8_t* push_frames, const int32_t* push_actions,
                      const float* push_rewards, const uint8_t* push_terminals, const uint8_t* states,
                      int32_t W, float epsilon, uint64_t act_step, int32_t use_target, int32_t* actions,
                      float* q_out);

/* Moves every lane's buffered experiences into D in push order, overwriting the oldest. */
int replay_flush(replay* rb, int32_t blocking);

/* Number of transitions that can currently be sampled (host-side bookkeeping, no device work). */
int64_t replay_num_valid(const replay* rb);

/* Draws B transitions uniformly with replacement (or takes them from idx_in) and assembles the
 * minibatch.  Indexing: within lane l the visible frames are numbered by age j = 0 (oldest) ..
 * count_l - 1; the global index of a transition is l * (capacity_frames / lanes) + j, valid iff
 * 3 <= j <= count_l - 2.  Draw i at counter sample_step uses the Philox4x32-10 outputs for
 * key = (seed lo, seed hi), counter = (i, 2, sample_step lo, sample_step hi):
 * k = ((x1:x0) * V) >> 64 with V the number of valid transitions, lanes walked in order.
 *   s  [B,4,84,84]: frames of ages j-3..j;  s2: ages j-2..j+1;  a stacked frame is all zeros if a
 *   terminal flag lies between it (inclusive) and the stack's newest frame (exclusive).
 *   a [B] int32, r [B] float32, done [B] float32 (0/1) of the frame at age j.
 *   idx_in [B] int64 or NULL;  idx_out [B] int64 or NULL.
 * Runs on sample_stream.  Errors: DQN_EINVAL (B < 1, null/misaligned pointer), DQN_ESTATE (no
 * valid transition).  Indices passed through idx_in are range-checked on the device: an invalid
 * one yields all-zero stacks and a = -1 for that row instead of an out-of-range read. */
int replay_sample_gather(replay* rb, int32_t B, uint64_t sample_step, const int64_t* idx_in,
                         uint8_t* s, uint8_t* s2, int32_t* a, float* r, float* done,
                         int64_t* idx_out);

/* replay_sample_gather(rb, B, sample_step, NULL, ...) followed by dqn_train_step on that minibatch -- with the
 * assembly of the minibatch taken out of the chain of dependent launches: if prefetch_next != 0, workgroups
 * riding in one of this step's kernels already prepare the minibatch of sample_step + 1 (the replay memory is
 * constant between synchronisation points, Section 3 / Algorithm 1), and the next call, if it asks for exactly
 * that minibatch (same rb, B, sample_step + 1, and no replay_flush / dqn_sync_target in between), finds it
 * prepared.  Any other call prepares it first, as the two separate calls would: results are identical to
 * theirs in every case.  "Prepared" means, in the reduced-precision mode at B >= 96: DESCRIBED -- the replay
 * slots of the eight frames of (s, s') per sample, with a, r, done -- and the kernels that consume states read
 * the frames straight from D, so the 56 KB per sample of an assembled (s, s') pair are never written; otherwise:
 * assembled into one of two buffer sets owned by ctx (in the full-precision mode only up to B = 256: beyond it
 * no kernel of the step is long enough to ride in, and every call assembles first).  The replay's
 * sample_stream must be ctx's train_stream.  Errors: those of the two calls. */
int dqn_train_step_sampled(dqn_ctx* ctx, replay* rb, int32_t B, uint64_t sample_step,
                           int32_t prefetch_next, float* loss_out);

/* ---- seeded synthetic inputs (benchmark support; stands in for emulator output) ----------- */

/* Frame i of the call gets id = id0 + i * id_step and is written to dst[i] ([n,84,84] uint8):
 * with mix64 the SplitMix64 output function, GAMMA = 0x9E3779B97F4A7C15 and
 * word(id, g) = mix64(mix64(mix64(seed + GAMMA*(stream_tag+1)) + id) + GAMMA*(g+1)), pixel p takes
 * w32 = 32-bit half (p & 1) of word(id, p >> 1) and is (w32 & 255) if (w32 >> 8) < pix_threshold,
 * else `background`. */
int synth_frames(uint8_t* dst, int64_t n, uint64_t id0, uint64_t id_step, uint64_t seed,
                 uint32_t stream_tag, uint32_t pix_threshold, uint32_t background, void* stream);

/* Transition i (id as above): w = word(id, 0) with stream_tag 1;  rb = w & 0xFFFFFF,
 * tb = (w >> 24) & 0xFFFFFF, ab = w >> 48;  reward = -1 if rb < t_neg, +1 if rb >= 2^24 - t_pos,
 * else 0;  terminal = tb < t_term;  action = (ab * num_actions) >> 16. */
int synth_transitions(int32_t* actions, float* rewards, uint8_t* terminals, int64_t n,
                      uint64_t id0, uint64_t id_step, uint64_t seed, int32_t num_actions,
                      uint32_t t_neg, uint32_t t_pos, uint32_t t_term, void* stream);

/* ---- shared arrays of the synchronized samplers (Section 4) --------------------------------- */

/* W environments stepped by the CALLER's sampler threads (an emulator each), acting through one
 * minibatch per step.  The handle owns (a) pinned host arrays that the sampler threads and the
 * kernels both address -- observations [W,84,84] uint8, actions [W] int32, rewards [W] float32,
 * terminals [W] uint8, q [W,A] float32 -- so that an act step crosses the bus twice whatever W is and
 * needs no copy command, and (b) the W frame stacks [W,4,84,84] on the device.  The state of
 * environment j is the stack of its four latest observations, those from before its latest episode
 * start replaced by zeros (the states replay_sample_gather later rebuilds).  Protocol:
 *     write o_0 of every environment into observations;  dqn_envs_reset
 *     loop:  dqn_envs_act          -> actions (and q) are in the arrays when it returns
 *            every sampler j steps its environment with actions[j] and writes rewards[j],
 *            terminals[j] (1: the episode ended with this step) and its next observation
 *            (the first observation of the next episode after a terminal step) into observations[j]
 *            dqn_envs_observe      -> experiences appended, stacks advanced (enqueued)
 * The arrays must not be written between dqn_envs_observe / dqn_envs_reset and the return of the next
 * dqn_envs_act (the kernels that read them have finished by then).
 * rb (may be NULL: nothing is stored) needs W lanes and the context's act stream as push stream;
 * W <= max_envs.  All device work runs on the act stream.  Errors: DQN_EINVAL, DQN_ENOMEM, DQN_EHIP. */
typedef struct dqn_envs dqn_envs;
int dqn_envs_create(dqn_ctx* ctx, replay* rb, int32_t W, dqn_envs** host_out);
int dqn_envs_destroy(dqn_envs* e);

/* Host addresses of the shared arrays (owned by e, valid until dqn_envs_destroy); any argument may be
 * NULL. */
int dqn_envs_arrays(dqn_envs* e, uint8_t** host_observations, int32_t** host_actions,
                    float** host_rewards, uint8_t** host_terminals, float** host_q);

/* Every environment starts an episode with the observation in the shared array: stack j becomes
 * (0, 0, 0, observations[j]); nothing is stored.  Enqueues only. */
int dqn_envs_reset(dqn_envs* e);

/* dqn_act on the W stacks (same epsilon-greedy definition and counters) with the actions -- and the Q
 * rows if want_q != 0 -- stored into the shared arrays; waits for the act stream, so they are there on
 * return.  Errors: those of dqn_act; DQN_ESTATE before dqn_envs_reset. */
int dqn_envs_act(dqn_envs* e, float epsilon, uint64_t act_step, int32_t use_target, int32_t want_q);

/* After every sampler has stepped: for each environment j, appends the experience (the observation the
 * action was taken on, actions[j], rewards[j], terminals[j]) to lane j of rb's temporary buffers (what
 * replay_push_step does; the action is read from the shared array, so a sampler that overrode it
 * stores what it actually did), then shifts stack j by one and appends observations[j], keeping only
 * that observation if terminals[j] is set.  One launch; enqueues only.  Errors: DQN_ESTATE (a
 * temporary buffer is full, or dqn_envs_reset has not run). */
int dqn_envs_observe(dqn_envs* e);

/* ---- Algorithm 1: the main loop around the calls above (Sections 3 and 4) ------------------- */

/* The paper's host program: W sampler threads, one trainer thread and the main thread that
 * synchronises them.  The samplers step W synthetic environments that live on the host like an emulator
 * would (seeded stand-ins for it, defined below); everything else is the calls above.
 *   every C timesteps   wait for trainer and samplers; flush the temporary buffers into D;
 *                       theta^- <- theta (dqn_sync_target); hand the trainer thread C / F minibatches
 *                       (dqn_train_step_sampled, sample_step = train steps so far);
 *   every W timesteps   dqn_envs_act for all W states from theta^- at the given epsilon (act_step =
 *                       act steps so far), each sampler thread steps its environment,
 *                       dqn_envs_observe.
 * Timesteps count single environment steps, so one act step advances t by W (Section 4); the
 * synchronisation happens when t mod C == 0 with t counted from 0.
 *
 * Synthetic environment j (j < W), with word() the generator of synth_frames below and stream tags 3
 * (observations) and 4 (outcomes): its n-th observation o_n is frame id n*W + j of stream 3 (pixel
 * threshold 838861, background 40).  Its n-th step under action a returns, from w = word(id n*W + j, 0)
 * of stream 4: reward = (-1 if (w & 0xFFFFFF) < t_reward_neg, +1 if (w & 0xFFFFFF) >= 2^24 -
 * t_reward_pos, else 0) if a == (((w >> 48) & 0xFFFF) * A) >> 16, else 0; terminal = ((w >> 24) &
 * 0xFFFFFF) < t_term.  The state handed to the network is the stack (o_{n-3}, .., o_n) with the
 * observations from before the latest terminal step replaced by zeros (and zeros before o_0): the states
 * acted from are the states replay_sample_gather later rebuilds.  Environment j writes lane j of D with
 * the experience (o_n, a_n, r_n, terminal_n). */
typedef struct {
    int32_t W;             /* sampler threads = environments = replay lanes (Section 4)            */
    int32_t C;             /* target update period in timesteps; multiple of W and of F (Table 5)  */
    int32_t F;             /* timesteps per train step (Table 5: 4)                                */
    int32_t B;             /* minibatch size (Table 5: 32)                                         */
    float epsilon;         /* exploration rate of dqn_alg1_run                                     */
    uint32_t t_reward_neg, t_reward_pos, t_term;   /* thresholds on 24-bit draws, see above        */
    int32_t concurrent;    /* 1: Concurrent Training (Section 3); 0: standard DQN, see below       */
    int32_t synchronized;  /* 1: Synchronized Execution (Section 4); 0: one query per sampler      */
    uint32_t env_step_ns;  /* extra busy time per environment step standing in for an emulator's
                              own cost (0: none); changes timing only                              */
    uint32_t reserved;     /* 0                                                                    */
    uint64_t env_seed;     /* seed of the synthetic environments                                   */
} dqn_alg1_config;

/* The ablation of Section 5.1.  synchronized = 0: in every round of W timesteps each sampler thread makes
 * its own dqn_act call on its own state (W = 1; environment j at round k uses act_step = k * W + j), its
 * own download of the action, and after its environment step its own upload and replay_push (copy
 * commands instead of shared arrays); the threads' calls are serialised by a mutex.  concurrent = 0: the
 * policy reads theta (use_target = 0); after every round the experiences are flushed into D (replay_flush) and the calling
 * thread makes the train steps that have become due -- t / F train steps have been made once the
 * timestep counter stands at t -- before the next round; theta^- <- theta still every C timesteps; the
 * trainer thread stays idle. */

typedef struct dqn_alg1 dqn_alg1;

/* ctx and rb stay owned by the caller and must outlive the handle; rb needs W lanes, its push stream
 * must be ctx's act stream and its sample stream ctx's train stream, and staging_per_lane >= C / W
 * (and >= the prepopulation's timesteps / W).  Allocates pinned host arrays and device buffers for W
 * observations, stacks, actions, rewards and flags, and starts the W + 1 threads (idle until a call
 * below).  While a call below runs, no other thread may use ctx or rb.  Errors: DQN_EINVAL, DQN_ENOMEM,
 * DQN_EHIP. */
int dqn_alg1_create(dqn_ctx* ctx, replay* rb, const dqn_alg1_config* host_cfg, dqn_alg1** host_out);
/* Waits for the threads, frees the buffers; does not touch ctx or rb. */
int dqn_alg1_destroy(dqn_alg1* h);

/* Fills D with experiences collected at random: timesteps / W act steps at epsilon = 1 without training,
 * then a blocking flush.  These steps advance the environments and the act-step counter but not t.
 * timesteps must be a multiple of W. */
int dqn_alg1_prepopulate(dqn_alg1* h, int64_t timesteps);

/* Runs timesteps (a multiple of C) of the loop above, continuing from where the last call stopped.
 * Returns when every launch has been enqueued and the trainer thread is idle; the experiences of the
 * last block are still in the temporary buffers, as they would be at that instant of the paper's loop.  An error inside the trainer thread is reported by the next
 * synchronisation point or by this call's return. */
int dqn_alg1_run(dqn_alg1* h, int64_t timesteps);

/* Flushes the temporary buffers into D (blocking), so that D can be inspected; the next dqn_alg1_run starts with its own synchronisation point as usual. */
int dqn_alg1_flush(dqn_alg1* h);

/* Host-side counters (any pointer may be NULL): timesteps of dqn_alg1_run so far, act steps and train
 * steps issued, sum of rewards and number of finished episodes over all environments (prepopulation
 * included). */
int dqn_alg1_stats(const dqn_alg1* h, int64_t* host_t, int64_t* host_act_steps, int64_t* host_train_steps,
                   double* host_reward_sum, int64_t* host_episodes);

/* ---- per-kernel timing (measurement support) ------------------------------------------------- */

/* Number of distinct kernels a train step launches, and their names (id 1 .. count).  The id named
 * "event_pair" is not a kernel: selecting it times a pair of event records with nothing in between (what an
 * event bracket around a launch would add; the timing below does not use brackets). */
int dqn_profile_kernel_count(void);
const char* dqn_profile_kernel_name(int kernel_id);

/* Selects one kernel of dqn_train_step (0 = none): from now on each of its launches carries a pair of HIP
 * events bound to the kernel's own dispatch (hipExtLaunchKernel), so that the time between them is the
 * kernel's begin-to-end time on the GPU -- the duration a kernel trace reports for it (up to 4096 launches
 * are kept, later ones are not timed).  Selecting resets the collected data. */
int dqn_profile_select(dqn_ctx* ctx, int kernel_id);

/* The same with only every `every`-th launch of the kernel timed (every >= 1), so that the 4096 kept
 * samples span a long run. */
int dqn_profile_select_every(dqn_ctx* ctx, int kernel_id, int32_t every);

/* Waits for train_stream, then returns the summed duration in milliseconds and the number of
 * timed launches of the selected kernel since dqn_profile_select. */
int dqn_profile_read(dqn_ctx* ctx, double* host_total_ms, int64_t* host_launches);

const char* dqn_last_error(void);

#ifdef __cplusplus
#pragma GCC visibility pop
}
#endif
#endif /* DQN_MI355_H */
