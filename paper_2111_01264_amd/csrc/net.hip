// The Q-network side of the hot path: batched act step (Sections 3, 4), minibatch train step
// (Section 2.1, Eq. 1; Appendix B) and the synchronisation point (Algorithm 1), as sequences of
// hand-written gfx950 kernels on two HIP streams.
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"
#include <type_traits>

#include "conv_tower.h"
#include "conv_tower_bwd.h"
#include "fc_as.h"
#include "wgrad_all.h"
#include "head_kernels.h"
#include "layers.h"

namespace dqn {

enum KernelId {
    K_NONE = 0, K_CONV1_FWD, K_CONV2_FWD, K_CONV3_FWD, K_FC1_FWD, K_FC2_TD, K_TD_HEAD_BWD, K_FC1_WGRAD,
    K_FC1_DGRAD, K_CONV3_WGRAD, K_CONV3_DGRAD, K_CONV2_WGRAD, K_CONV2_DGRAD, K_CONV1_WGRAD, K_BIAS_GRAD,
    K_RMSPROP, K_WGRAD_ALL, K_EVENT_PAIR, K_TOWER_BWD, K_COUNT
};
static const char* const kKernelNames[K_COUNT] = {
    "none", "conv_tower", "(conv2_fwd)", "(conv3_fwd)", "fc1_fwd", "head_td", "(unused)", "fc1_wgrad",
    "fc1_dgrad", "conv3_wgrad", "conv3_dgrad", "conv2_wgrad", "conv2_dgrad", "conv1_wgrad", "small_grads",
    "rmsprop", "wgrad_all", "event_pair", "conv_tower_bwd"};
constexpr size_t kProfPairs = 4096;

// Layer geometries (Section 5: the Nature-DQN network).
template <typename T> using Conv2Geo = FwdGeo<T, 32, 20, 20, 64, 9, 9, 4, 2>;
template <typename T> using Conv3Geo = FwdGeo<T, 64, 9, 9, 64, 7, 7, 3, 1>;
template <typename T> using Conv3DgradGeo = DgradGeo<T, 64, 9, 9, 64, 7, 7, 3, 1>;
template <typename T> using Conv2DgradGeo = DgradGeo<T, 32, 20, 20, 64, 9, 9, 4, 2>;

}  // namespace dqn

using namespace dqn;

// Activations of one forward workspace, sized for `cap` samples in each of `groups` groups.
struct Workspace {
    void* act1 = nullptr;   // [G*cap][20][20][32]
    void* act2 = nullptr;   // [G*cap][9][9][64]
    void* act3 = nullptr;   // [G*cap][7][7][64]
    void* h = nullptr;      // [cap][512]: fc1 output of the online pass on s (kept for the backward pass)
    float* q = nullptr;     // [G*cap][A]
    float* partial = nullptr;   // fc1 k-slices
    size_t partial_cap = 0;

};

// ---- dqn_act_static: the act step's intermediates in a fixed array of the device image ------------------------
// Sub-buffers for up to kActStaticMaxEnvs states in either precision (fp32 sizes; the 16-bit mode uses half of the
// activation bytes): act1, act2, act3 and the seven fc1 k-slices of a minibatch of at most 32 rows.
constexpr int kActStaticMaxEnvs = DQN_ACT_STATIC_MAX_ENVS;
constexpr size_t align256(size_t n) { return (n + 255) / 256 * 256; }
constexpr size_t kActStaticAct1 = 0;
constexpr size_t kActStaticAct2 = kActStaticAct1 + align256(static_cast<size_t>(kActStaticMaxEnvs) * 12800 * 4);
constexpr size_t kActStaticAct3 = kActStaticAct2 + align256(static_cast<size_t>(kActStaticMaxEnvs) * 5184 * 4);
constexpr size_t kActStaticPartial = kActStaticAct3 + align256(static_cast<size_t>(kActStaticMaxEnvs) * 3136 * 4);
constexpr size_t kActStaticBytes = kActStaticPartial + align256(static_cast<size_t>(7) * kActStaticMaxEnvs * 512 * 4);
static_assert(kActStaticMaxEnvs <= 32, "the k-slice area assumes the small-batch fc1 kernel (seven slices)");
static __device__ __align__(256) unsigned char scratch[kActStaticBytes];   // about 3 MiB per GPU, for the life of the process

// In host code `scratch` is only a handle for the symbol: its device address differs per GPU and is looked up once
// per device, with that device current (dqn_create does it for the device it runs on).
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

static hipError_t static_scratch_of(int device, void** out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        int current = -1;
        hipError_t e = hipGetDevice(&current);
        if (e != hipSuccess) return e;
        if (current != device) return hipErrorInvalidDevice;   // resolved for the current device only
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

struct dqn_ctx {
    dqn_config cfg;
    int device = 0;
    int A;
    Offsets off;
    size_t esize;           // bytes per operand element
    hipStream_t act_stream, train_stream;
    float *theta = nullptr, *theta_t = nullptr, *v = nullptr, *m = nullptr, *grad = nullptr;
    void *sh = nullptr, *sh_t = nullptr;   // forward operand copies; alias theta / theta_t in fp32 mode
    void* bsh = nullptr;                   // backward operand copies of theta
    Workspace train_ws, act_ws;
    void *dzh = nullptr, *dz3 = nullptr, *dz2 = nullptr, *dz1 = nullptr;
    float *dqv = nullptr, *lossv = nullptr, *loss_keep = nullptr;
    float* bias_partial = nullptr;
    float* wg_partial = nullptr;
    hipEvent_t ev_train = nullptr, ev_act = nullptr, ev_sync = nullptr;
    std::atomic<bool> train_unrecorded{false};   // a train step has been enqueued since ev_train was last recorded
    // Held while a train step is being enqueued, and by an act step that reads theta (use_target = 0) from its wait for
    // the train stream to the record of its own event: such an act step then sees whole train steps only, also when
    // another host thread drives the train stream.  Act steps on theta^- (Concurrent Training) never take it.
    std::mutex online_mu;
    std::atomic<bool> act_reads_online{false};   // an act step with use_target = 0 has been enqueued since the train stream last waited for ev_act
    // dqn_train_step_sampled: two sets of minibatch buffers; `pre_*` describes the minibatch gathered ahead, if any
    uint8_t* mb_s[2] = {nullptr, nullptr};
    uint8_t* mb_s2[2] = {nullptr, nullptr};
    int32_t* mb_a[2] = {nullptr, nullptr};
    float* mb_r[2] = {nullptr, nullptr};
    float* mb_d[2] = {nullptr, nullptr};
    int32_t* mb_desc[2] = {nullptr, nullptr};   // reduced precision: the minibatch as per-sample descriptors (sample_desc)
    bool pre_valid = false;
    const replay* pre_rb = nullptr;
    int pre_B = 0, pre_buf = 0;
    uint64_t pre_step = 0, pre_epoch = 0;
    int last_B = 0;
    int num_cus = 256;
    // per-kernel timing (dqn_profile_*)
    int prof_id = 0;
    std::vector<hipEvent_t> prof_events;   // pairs
    size_t prof_used = 0;                  // pairs recorded since the last select
    int prof_every = 1;                    // every prof_every-th launch of the selected kernel is bracketed
    int64_t prof_seen = 0;                 // its launches since the last select
};

namespace dqn {

constexpr int kMaxFc1Slices = 49;
// deferred split-K scratch of the three conv weight gradients
constexpr size_t kWgMaxSplits = 64, kWgMaxSplits1 = 128;   // conv1's gradient is small: more slices are cheap
constexpr size_t kWgFp32Splits = 32;                       // fp32 mode (separate launches per layer)
// Reduced precision: slices per conv layer at most (conv2 / conv3 run 2 / 3 workgroups per slice, one per column block).
// 44 and not the 64 the buffers allow: with 128 + 2 * 64 + 3 * 64 conv workgroups next to fc1's 200 tiles the grid was far
// beyond the 512 workgroups that are resident at once and fc1's tiles started when the first conv workgroups left;
// 128 + 2 * 43 + 3 * 43 leaves them room from the start (batch 256: 90.4 -> 87.5 us per train step, batch 128: 74.3 -> 70.1).
constexpr int kWgSlices1 = 128, kWgSlices23 = 44;
// Smallest minibatch handled through descriptors.  Below it the assembled states are the faster form: the byte gather
// rides for free in the previous step's head kernel (which leaves most of the chip idle at small batches), and the
// fused conv kernel starts on states that are contiguous and cache-warm instead of after a descriptor round trip
// (per train step through descriptors / through assembled states: batch 32: 52.4 / 51.8 us, batch 64: 62.8 / 62.9,
// batch 96: 64.9 / 67.1, batch 128: 68.1 / 72.0).
constexpr int kDescMinBatch = 96;
constexpr size_t kWgOff1 = 0, kWgOff2 = kWgMaxSplits1 * 32 * 256, kWgOff3 = kWgOff2 + kWgMaxSplits * 64 * 512;
constexpr size_t kWgTotal = kWgOff3 + kWgMaxSplits * 64 * 576;

static int alloc_ws(Workspace& ws, int cap, int groups, int A, size_t esize, bool training)
{
    const size_t n = static_cast<size_t>(cap) * groups;
    DQN_HIP(hipMalloc(&ws.act1, n * 12800 * esize));
    DQN_HIP(hipMalloc(&ws.act2, n * 5184 * esize));
    DQN_HIP(hipMalloc(&ws.act3, n * 3136 * esize));
    DQN_HIP(hipMalloc(&ws.h, static_cast<size_t>(cap) * 512 * esize));
    DQN_HIP(hipMalloc((void**)&ws.q, n * A * sizeof(float)));
    ws.partial_cap = n * kMaxFc1Slices * 512;
    const size_t wgrad = static_cast<size_t>(256) * 64 * 576;   // up to 256 split-K slices of the largest filter
    if (training && ws.partial_cap < wgrad) ws.partial_cap = wgrad;
    DQN_HIP(hipMalloc((void**)&ws.partial, ws.partial_cap * sizeof(float)));
    return DQN_OK;
}

static void free_ws(Workspace& ws)
{
    (void)hipFree(ws.act1); (void)hipFree(ws.act2); (void)hipFree(ws.act3); (void)hipFree(ws.h);
    (void)hipFree(ws.q); (void)hipFree(ws.partial);
}

// The two fused conv kernels need more dynamic LDS than the default limit: raised once per process, whichever host
// thread gets there first (the act and the train thread may both be on their first call).
static hipError_t raise_lds_limits()
{
    static std::once_flag once;
    static hipError_t result = hipSuccess;
    std::call_once(once, [] {
        result = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_tower_kernel<false, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, kTowerSmem);
        if (result == hipSuccess)
            result = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_tower_kernel<false, 3>), hipFuncAttributeMaxDynamicSharedMemorySize, kTowerSmem);
        if (result == hipSuccess)
            result = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_tower_kernel<false, 7>), hipFuncAttributeMaxDynamicSharedMemorySize, kTowerSmem);
        if (result == hipSuccess)
            result = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_tower_kernel<true, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, kTowerSmem);
        if (result == hipSuccess)
            result = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_tower_bwd_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, kTowerBwdSmem);
        if (result == hipSuccess)
            result = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_tower_bwd_kernel<5>), hipFuncAttributeMaxDynamicSharedMemorySize, kTowerBwdSmem);
    });
    return result;
}

// Event pair for a launch of kernel `id`, or nulls if that kernel is not the selected one.
struct ProfPair { hipEvent_t begin = nullptr, end = nullptr; };
static ProfPair prof_pair(dqn_ctx* c, int id)
{
    ProfPair p;
    if (c->prof_id == id && c->prof_seen++ % c->prof_every == 0 && c->prof_used < c->prof_events.size() / 2) {
        p.begin = c->prof_events[2 * c->prof_used];
        p.end = c->prof_events[2 * c->prof_used + 1];
        ++c->prof_used;
    }
    return p;
}

static int pick_splits(int tiles, int K, int BK, int max_splits)
{
    const int target = 512;   // about two workgroups per compute unit
    int s = target / (tiles > 0 ? tiles : 1);
    const int by_k = K / (2 * BK) > 0 ? K / (2 * BK) : 1;
    if (s > by_k) s = by_k;
    if (s > max_splits) s = max_splits;
    return s < 1 ? 1 : s;
}

// Split-K factor of a conv weight gradient with K contraction rows and `n_blocks` column blocks:
// up to 256 workgroups in total, at least two 32-row k-tiles each, at most max_splits slices (every
// slice is a full copy of the gradient that the optimiser kernel has to read back).
static int wgrad_splits(int K, int n_blocks, int max_splits)
{
    int s = 256 / n_blocks;
    const int by_k = K / 64 > 0 ? K / 64 : 1;
    if (s > by_k) s = by_k;
    if (s > max_splits) s = max_splits;
    return s < 1 ? 1 : s;
}

// Number of fc1 k-slices for n rows per group: enough workgroups to fill the chip, few enough that
// the consumer's slice sum stays small.
static int fc1_slices(int n, int groups)
{
    const int row_tiles = (n + 31) / 32;
    const int blocks = 4 * row_tiles * groups;
    int s = 64 / blocks;         // few slices: the head kernel re-reads every slice
    if (s < 7) s = 7;            // 3136 / 7 = 448 columns of X per workgroup fit in LDS
    if (s > kMaxFc1Slices) s = kMaxFc1Slices;
    return s;
}

// A minibatch given by descriptors (sample_desc) instead of assembled states: the fused conv kernel reads the frames
// from the replay memory's frame array itself and leaves the state of the online pass in s_out.
struct StateSource {
    const int32_t* desc;
    const uint8_t* ring;
    uint8_t* s_out;
};

__global__ __launch_bounds__(256) void sample_desc_kernel(GatherPlan plan, int32_t* desc)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b < plan.B) sample_desc(plan, b, desc + static_cast<size_t>(b) * kDescInts);
}

// Forward pass of `groups` independent (input, parameter set) pairs with n samples each, up to the
// fc1 k-slices; the number of slices comes back through *slices_out.
template <typename T>
static int forward_to_fc1(dqn_ctx* c, hipStream_t st, Workspace& ws, int groups, const uint8_t* const* x,
                          const void* const* shadow, const float* const* master, int n, bool timed, int* slices_out,
                          const PushStepPlan* push = nullptr, const StateSource* src = nullptr)
{
    const Offsets& o = c->off;
    auto pp = [&](int id) { return timed ? prof_pair(c, id) : ProfPair(); };
    const size_t e_act3 = static_cast<size_t>(n) * 3136;
    T* act1 = static_cast<T*>(ws.act1); T* act2 = static_cast<T*>(ws.act2); T* act3 = static_cast<T*>(ws.act3);
    if constexpr (std::is_same<T, bf16_t>::value) {
        // conv1 -> conv2 -> conv3 fused; only group 0 of a train step keeps act1 / act2 (the backward pass reads them)
        TowerArgs a{};
        for (int g = 0; g < groups; ++g) {
            a.x[g] = x[g];
            a.w1[g] = reinterpret_cast<const _Float16*>(static_cast<const T*>(shadow[g]) + o.w1); a.b1[g] = master[g] + o.b1;
            a.w2[g] = static_cast<const T*>(shadow[g]) + o.w2; a.b2[g] = master[g] + o.b2;
            a.w3[g] = static_cast<const T*>(shadow[g]) + o.w3; a.b3[g] = master[g] + o.b3;
            a.act1[g] = (timed && g == 0) ? act1 : nullptr;
            a.act2[g] = (timed && g == 0) ? act2 : nullptr;
            a.act3[g] = act3 + g * e_act3;
        }
        a.n = n; a.groups = groups;
        if (src) { a.desc = src->desc; a.ring = src->ring; a.s_out = src->s_out; }
        DQN_HIP(raise_lds_limits());
        // Few items (a round of synchronized samplers, a minibatch of 32): seven or three workgroups per item, a seventh or
        // a third of its output rows each, while that still fits the chip -- the chain of layers of one sample is what the
        // launch waits for
        const int total = n * groups;
        const int parts = a.desc ? 1 : (7 * total <= c->num_cus ? 7 : (3 * total <= c->num_cus ? 3 : 1));
        const int grid = parts > 1 ? parts * total : (total < c->num_cus ? total : c->num_cus);
        a.per = parts > 1 ? 1 : (total + grid - 1) / grid;
        a.tower_blocks = grid;
        a.push.L = 0;
        if (push) a.push = *push;
        const ProfPair pr = pp(K_CONV1_FWD);
        // (the leading arguments repeat the fields a workgroup needs first: see the kernel)
        const dim3 g3(grid + a.push.L), b3(kTowerThreads);
        if (a.desc) launch_timed(conv_tower_kernel<true, 1>, g3, b3, kTowerSmem, st, pr.begin, pr.end, a.n, a.groups, a.per, a.tower_blocks, a.x[0], a.x[1], a.desc, a.ring, a.w1[0], a);
        else if (parts == 7) launch_timed(conv_tower_kernel<false, 7>, g3, b3, kTowerSmem, st, pr.begin, pr.end, a.n, a.groups, a.per, a.tower_blocks, a.x[0], a.x[1], a.desc, a.ring, a.w1[0], a);
        else if (parts == 3) launch_timed(conv_tower_kernel<false, 3>, g3, b3, kTowerSmem, st, pr.begin, pr.end, a.n, a.groups, a.per, a.tower_blocks, a.x[0], a.x[1], a.desc, a.ring, a.w1[0], a);
        else launch_timed(conv_tower_kernel<false, 1>, g3, b3, kTowerSmem, st, pr.begin, pr.end, a.n, a.groups, a.per, a.tower_blocks, a.x[0], a.x[1], a.desc, a.ring, a.w1[0], a);
        DQN_LAUNCH_CHECK();
    } else {
        // fp32 mode: layer by layer; the event pair brackets all three launches
        const size_t e_act1 = static_cast<size_t>(n) * 12800, e_act2 = static_cast<size_t>(n) * 5184;
        const ProfPair pr = pp(K_CONV1_FWD);
        {   // conv1 on the uint8 state, 1/255 folded into the epilogue
            ConvWsArgs<T, Conv1Geo<T>> a{};
            for (int g = 0; g < groups; ++g) {
                a.x[g] = x[g];
                a.w[g] = static_cast<const T*>(shadow[g]) + o.w1;
                a.bias[g] = master[g] + o.b1;
                a.out[g] = act1 + g * e_act1;
            }
            a.M = n * 400; a.scale = 1.f / 255.f;
            DQN_HIP((launch_conv_ws<T, Conv1Geo<T>, kEpiBiasRelu>(st, a, groups, pr.begin, nullptr)));
        }
        {
            ConvWsArgs<T, Conv2Geo<T>> a{};
            for (int g = 0; g < groups; ++g) {
                a.x[g] = act1 + g * e_act1;
                a.w[g] = static_cast<const T*>(shadow[g]) + o.w2;
                a.bias[g] = master[g] + o.b2;
                a.out[g] = act2 + g * e_act2;
            }
            a.M = n * 81; a.scale = 1.f;
            DQN_HIP((launch_conv_ws<T, Conv2Geo<T>, kEpiBiasRelu>(st, a, groups)));
        }
        {
            ConvWsArgs<T, Conv3Geo<T>> a{};
            for (int g = 0; g < groups; ++g) {
                a.x[g] = act2 + g * e_act2;
                a.w[g] = static_cast<const T*>(shadow[g]) + o.w3;
                a.bias[g] = master[g] + o.b3;
                a.out[g] = act3 + g * e_act3;
            }
            a.M = n * 49; a.scale = 1.f;
            DQN_HIP((launch_conv_ws<T, Conv3Geo<T>, kEpiBiasRelu>(st, a, groups, nullptr, pr.end)));
        }
    }
    // fc1 as k-slices of fp32 partial sums [groups][slices][n][512]; the head kernel adds them
    if (n <= 32) {
        FcSkArgs<T> a{};
        for (int g = 0; g < groups; ++g) {
            a.x[g] = act3 + g * e_act3;
            a.w[g] = static_cast<const T*>(shadow[g]) + o.wf1;
        }
        a.partial = ws.partial;
        a.M = n; a.N = 512; a.ldx = 3136; a.ldw = 3136;
        const ProfPair pr = pp(K_FC1_FWD);
        launch_timed(fc_sk_kernel<T, kFcPartial, 7, 7>, dim3(16, groups, 7), dim3(256), 0, st, pr.begin, pr.end, a.x[0], a.x[1], a.w[0], a.w[1], a.M, a.N,
                     a.ldx, a.ldw, a.partial, a);
        DQN_LAUNCH_CHECK();
        *slices_out = 7;
    } else {
        FcAsArgs<T> a{};
        for (int g = 0; g < groups; ++g) {
            a.x[g] = act3 + g * e_act3;
            a.w[g] = static_cast<const T*>(shadow[g]) + o.wf1;
        }
        a.partial = ws.partial;
        a.M = n; a.N = 512; a.ldx = 3136; a.ldw = 3136;
        const ProfPair pr = pp(K_FC1_FWD);
        int used = 0;
        DQN_HIP((launch_fc_as<T, kFcPartial>(st, a, 3136, groups, fc1_slices(n, groups), &used, pr.begin, pr.end)));
        *slices_out = used;
    }
    return DQN_OK;
}

// act_stream waits for every train step enqueued so far.  The event is recorded here, by the reader, and not
// after every train step: an event record costs the train stream several microseconds per step, and with the
// target parameters (Concurrent Training, Section 3) nobody ever waits for it.
static hipError_t wait_for_train(dqn_ctx* c)
{
    if (c->train_unrecorded.exchange(false, std::memory_order_acq_rel)) {
        const hipError_t e = hipEventRecord(c->ev_train, c->train_stream);
        if (e != hipSuccess) return e;
    }
    return hipStreamWaitEvent(c->act_stream, c->ev_train, 0);
}

// train_stream waits for the last act step that read theta (use_target = 0): it must finish before theta is overwritten.
static hipError_t wait_for_online_act(dqn_ctx* c)
{
    if (!c->act_reads_online.exchange(false, std::memory_order_acq_rel)) return hipSuccess;
    return hipStreamWaitEvent(c->train_stream, c->ev_act, 0);
}

template <typename T>
static int act_impl(dqn_ctx* c, Workspace& ws, const uint8_t* states, int W, float epsilon, uint64_t act_step, int use_target,
                    int32_t* actions, float* q_out, const PushStepPlan* push = nullptr)
{
    const uint8_t* x[1] = {states};
    const void* shadow[1] = {use_target ? c->sh_t : c->sh};
    const float* master[1] = {use_target ? c->theta_t : c->theta};
    int slices = 0;
    const int rc = forward_to_fc1<T>(c, c->act_stream, ws, 1, x, shadow, master, W, false, &slices, push);
    if (rc != DQN_OK) return rc;
    HeadArgs ha{};
    ha.partial = ws.partial; ha.slices = slices; ha.rows = W; ha.A = c->A; ha.groups = 1;
    ha.b1[0] = master[0] + c->off.bf1; ha.w2[0] = static_cast<const T*>(shadow[0]) + c->off.wf2; ha.b2[0] = master[0] + c->off.bf2;
    ha.epsilon = epsilon; ha.seed = c->cfg.seed; ha.act_step = act_step; ha.actions = actions; ha.q_out = q_out;
    ha.head_blocks = (W + kHeadRows - 1) / kHeadRows;
    ha.gather.B = 0;
    hipLaunchKernelGGL((head_fwd_kernel<T, kHeadAct>), dim3(ha.head_blocks), dim3(256), 0, c->act_stream, ha.partial, ha.slices, ha.rows, ha.A, ha.groups,
                       ha.head_blocks, ha.w2[0], ha.b1[0], ha.b2[0], ha.epsilon, ha);
    DQN_LAUNCH_CHECK();
    return DQN_OK;
}

template <typename T, bool SHADOW>
static int train_impl(dqn_ctx* c, const uint8_t* s, const int32_t* a, const float* r, const uint8_t* s2,
                      const float* done, int B, float* loss_out, const GatherPlan* ride = nullptr, int32_t* ride_desc = nullptr,
                      const StateSource* src = nullptr)
{
    const Offsets& o = c->off;
    hipStream_t st = c->train_stream;
    Workspace& ws = c->train_ws;
    const int groups = c->cfg.double_dqn ? 3 : 2;
    const uint8_t* x[3] = {s, s2, s2};
    const void* shadow[3] = {c->sh, c->sh_t, c->sh};
    const float* master[3] = {c->theta, c->theta_t, c->theta};
    {   // "event_pair": an empty bracket, i.e. what a pair of event records costs by itself on this stream
        const ProfPair pr = prof_pair(c, K_EVENT_PAIR);
        if (pr.begin) { (void)hipEventRecord(pr.begin, st); (void)hipEventRecord(pr.end, st); }
    }
    int slices = 0;
    int rc = forward_to_fc1<T>(c, st, ws, groups, x, shadow, master, B, true, &slices, nullptr, src);
    if (rc != DQN_OK) return rc;

    const T* sh = static_cast<const T*>(c->sh);
    const T* sh_t = static_cast<const T*>(c->sh_t);
    const T* bsh = static_cast<const T*>(c->bsh);
    const T* act1 = static_cast<const T*>(ws.act1); const T* act2 = static_cast<const T*>(ws.act2);
    const T* act3 = static_cast<const T*>(ws.act3); T* h = static_cast<T*>(ws.h);
    T* dzh = static_cast<T*>(c->dzh); T* dz3 = static_cast<T*>(c->dz3);
    T* dz2 = static_cast<T*>(c->dz2); T* dz1 = static_cast<T*>(c->dz1);

    int wg_splits[3] = {1, 1, 1};
    {
        const ProfPair pr = prof_pair(c, K_FC2_TD);
        HeadArgs ha{};
        ha.partial = ws.partial; ha.slices = slices; ha.rows = B; ha.A = c->A; ha.groups = groups;
        for (int g = 0; g < groups; ++g) {
            ha.b1[g] = master[g] + o.bf1; ha.w2[g] = static_cast<const T*>(shadow[g]) + o.wf2; ha.b2[g] = master[g] + o.bf2;
        }
        ha.double_dqn = c->cfg.double_dqn; ha.act = a; ha.rew = r; ha.done = done;
        ha.gamma = c->cfg.gamma; ha.huber = c->cfg.huber_delta;
        ha.h_online = h; ha.dzh = dzh; ha.q_all = ws.q; ha.dqv = c->dqv; ha.lossv = c->lossv;
        ha.head_blocks = (B + kHeadRows - 1) / kHeadRows;
        // the next minibatch rides along: as a descriptor table (ride_desc, a few workgroups) or as assembled states (5 per sample)
        ha.gather.B = 0;
        ha.desc_out = ride_desc;
        if (ride) ha.gather = *ride;
        const int riders = !ride ? 0 : (ride_desc ? (ride->B + 255) / 256 : 5 * ride->B);
        launch_timed(head_fwd_kernel<T, kHeadTrain>, dim3(ha.head_blocks + riders), dim3(256), 0, st, pr.begin, pr.end, ha.partial, ha.slices, ha.rows, ha.A,
                     ha.groups, ha.head_blocks, ha.w2[0], ha.b1[0], ha.b2[0], ha.epsilon, ha);
        DQN_LAUNCH_CHECK();
    }
    // ---- data-gradient chain: fc1 -> conv3 -> conv2 ------------------------------------------------
    if (B <= 32) {   // fc1 data gradient through conv3's ReLU: dz3[b][f] = [act3 > 0] sum_o dZ[b][o] W1[o][f]
        FcSkArgs<T> fa{};
        fa.x[0] = dzh; fa.w[0] = bsh + kBshWf1; fa.dz = dz3; fa.mask = act3;
        fa.M = B; fa.N = 3136; fa.ldx = 512; fa.ldw = 512;
        const ProfPair pr = prof_pair(c, K_FC1_DGRAD);
        launch_timed(fc_sk_kernel<T, kFcReluMask, 8, 1>, dim3(98, 1, 1), dim3(256), 0, st, pr.begin, pr.end, fa.x[0], fa.x[1], fa.w[0], fa.w[1], fa.M, fa.N,
                     fa.ldx, fa.ldw, fa.partial, fa);
        DQN_LAUNCH_CHECK();
    } else {
        FcAsArgs<T> fa{};
        fa.x[0] = dzh; fa.w[0] = bsh + kBshWf1;
        fa.dz = dz3; fa.mask = act3;
        fa.M = B; fa.N = 3136; fa.ldx = 512; fa.ldw = 512;
        const ProfPair pr = prof_pair(c, K_FC1_DGRAD);
        int used = 0;
        DQN_HIP((launch_fc_as<T, kFcReluMask>(st, fa, 512, 1, 1, &used, pr.begin, pr.end)));
    }
    if constexpr (std::is_same<T, bf16_t>::value) {
        // conv3 and conv2 data gradients in one persistent launch, dz2 handed over in LDS
        TowerBwdArgs ta{};
        ta.dz3 = dz3; ta.act2 = act2; ta.act1 = act1; ta.w3d = bsh + kBshW3; ta.w2d = bsh + kBshW2;
        ta.dz2 = dz2; ta.dz1 = dz1; ta.n = B;
        DQN_HIP(raise_lds_limits());
        // small minibatches: five workgroups per sample (a fifth of its rows each) while that fits the chip
        const bool fifths = 5 * B <= c->num_cus;
        const int grid = fifths ? 5 * B : (B < c->num_cus ? B : c->num_cus);
        ta.per = fifths ? 1 : (B + grid - 1) / grid;
        const ProfPair pr = prof_pair(c, K_TOWER_BWD);
        if (fifths)
            launch_timed(conv_tower_bwd_kernel<5>, dim3(grid), dim3(kTowerThreads), kTowerBwdSmem, st, pr.begin, pr.end, ta.n, ta.per, ta.dz3, ta.w3d, ta.w2d,
                         ta.act2, ta.act1, ta.dz2, ta.dz1);
        else
            launch_timed(conv_tower_bwd_kernel<1>, dim3(grid), dim3(kTowerThreads), kTowerBwdSmem, st, pr.begin, pr.end, ta.n, ta.per, ta.dz3, ta.w3d, ta.w2d,
                         ta.act2, ta.act1, ta.dz2, ta.dz1);
        DQN_LAUNCH_CHECK();
    } else {
        {   // conv3 data gradient through conv2's ReLU
            ConvWsArgs<T, Conv3DgradGeo<T>> ca{};
            ca.x[0] = dz3; ca.w[0] = bsh + kBshW3; ca.out[0] = dz2; ca.mask = act2;
            ca.M = B * 81; ca.scale = 1.f;
            const ProfPair pr = prof_pair(c, K_CONV3_DGRAD);
            DQN_HIP((launch_conv_ws<T, Conv3DgradGeo<T>, kEpiReluMask>(st, ca, 1, pr.begin, pr.end)));
        }
        {   // conv2 data gradient through conv1's ReLU: one problem per stride-parity class
            ConvWsArgs<T, Conv2DgradGeo<T>> ca{};
            for (int g = 0; g < 4; ++g) {
                ca.x[g] = dz2; ca.w[g] = bsh + kBshW2 + static_cast<size_t>(g) * 32 * 256; ca.out[g] = dz1;
            }
            ca.mask = act1; ca.M = B * 100; ca.scale = 1.f;
            const ProfPair pr = prof_pair(c, K_CONV2_DGRAD);
            DQN_HIP((launch_conv_ws<T, Conv2DgradGeo<T>, kEpiReluMask>(st, ca, 4, pr.begin, pr.end)));
        }
    }

    // ---- weight gradients and small reductions ------------------------------------------------------
    int bias_chunks[4], bias_first[4];
    BiasGradArgs bg;
    bg.dz[0] = dz1; bg.rows[0] = B * 400; bg.chans[0] = 32;
    bg.dz[1] = dz2; bg.rows[1] = B * 81;  bg.chans[1] = 64;
    bg.dz[2] = dz3; bg.rows[2] = B * 49;  bg.chans[2] = 64;
    bg.dz[3] = dzh; bg.rows[3] = B;       bg.chans[3] = 512;
    // reduced precision: the conv layers' bias gradients come out of their weight-gradient workgroups (dZ is in LDS there)
    if (std::is_same<T, bf16_t>::value) bg.rows[0] = bg.rows[1] = bg.rows[2] = 0;
    bg.first_block[0] = 0;
    {
        int pofs = 0;
        for (int l = 0; l < 4; ++l) {
            // fc1's dZ is [B][512]: a workgroup covers four rows per pass, so 64 rows per chunk are one round trip of 16 loads in flight
            bg.chunk_rows[l] = l == 3 ? 64 : kBiasRows;
            bg.chunks[l] = (bg.rows[l] + bg.chunk_rows[l] - 1) / bg.chunk_rows[l];
            bg.first_block[l + 1] = bg.first_block[l] + bg.chunks[l];
            bg.first_partial[l] = pofs;
            pofs += bg.chunks[l] * bg.chans[l];
            bias_chunks[l] = bg.chunks[l];
            bias_first[l] = bg.first_partial[l];
        }
    }
    bg.partial = c->bias_partial;
    bg.h = h; bg.act = a; bg.dqv = c->dqv; bg.lossv = c->lossv; bg.B = B; bg.A = c->A;
    bg.g_w2 = c->grad + o.wf2; bg.g_b2 = c->grad + o.bf2; bg.loss_out = loss_out; bg.loss_keep = c->loss_keep;
    const int small_blocks = bg.first_block[4] + kSmallGradsExtraBlocks;

    RmsArgs ra;
    ra.theta = c->theta; ra.grad = c->grad; ra.v = c->v; ra.m = c->m;
    ra.sh = SHADOW ? c->sh : nullptr; ra.bsh = c->bsh; ra.off = o;
    ra.lr = c->cfg.lr; ra.alpha = c->cfg.rms_alpha; ra.eps = c->cfg.rms_eps; ra.centered = c->cfg.centered;
    {
        const size_t n_flat = o.total - static_cast<size_t>(512) * 3136;
        ra.flat_blocks = static_cast<int>((n_flat / 4 + 4 + 255) / 256);
    }
    ra.fc1_tiles = 16 * 49;
    ra.bias_partial = c->bias_partial;
    ra.wg_partial[0] = c->wg_partial + kWgOff1; ra.wg_partial[1] = c->wg_partial + kWgOff2;
    ra.wg_partial[2] = c->wg_partial + kWgOff3;
    for (int l = 0; l < 3; ++l) { ra.wg_splits[l] = 1; ra.wg_scale[l] = 1.f; }
    ra.wg_scale[0] = 1.f / 255.f;   // conv1 reads raw bytes: the input scale is applied to its gradient by the optimiser
    for (int l = 0; l < 4; ++l) { ra.bias_chunks[l] = 0; ra.bias_first[l] = 0; }

    if constexpr (std::is_same<T, bf16_t>::value) {
        // one launch: conv1/conv2/conv3/fc1 weight gradients and the small reductions
        WgradAllArgs wa{};
        // conv layers: split-K over samples, workgroup j writes slice j (conv1's unit is half a sample)
        // (items per workgroup: one, or an even number, because the kernel walks several in pairs -- an odd range costs a padding item)
        auto split = [](int items, int max_slices, int* per, int* slices) {
            *per = (items + max_slices - 1) / max_slices;
            if (*per > 1) *per = (*per + 1) / 2 * 2;
            *slices = (items + *per - 1) / *per;
        };
        int n1 = 0, n2 = 0, n3 = 0;
        wa.c1.dz = dz1; wa.c1.in = s; wa.c1.partial = c->wg_partial + kWgOff1; wa.c1.n = B;
        wa.c1.desc = src ? src->desc : nullptr; wa.c1.ring = src ? src->ring : nullptr;
        split(2 * B, kWgSlices1, &wa.c1.per, &n1);
        wa.c2.dz = dz2; wa.c2.in = act1; wa.c2.partial = c->wg_partial + kWgOff2; wa.c2.n = B;
        split(B, kWgSlices23, &wa.c2.per, &n2);
        wa.c3.dz = dz3; wa.c3.in = act2; wa.c3.partial = c->wg_partial + kWgOff3; wa.c3.n = B;
        split(B, kWgSlices23, &wa.c3.per, &n3);
        wg_splits[0] = n1; wg_splits[1] = n2; wg_splits[2] = n3;
        // their bias gradients: one partial row [C_out] per slice, added in slice order by the optimiser kernel
        constexpr int kConvBiasOff = 16384;
        bias_chunks[0] = n1; bias_first[0] = kConvBiasOff;
        bias_chunks[1] = n2; bias_first[1] = bias_first[0] + kWgSlices1 * 32;
        bias_chunks[2] = n3; bias_first[2] = bias_first[1] + kWgSlices23 * 64;
        static_assert(kConvBiasOff + kWgSlices1 * 32 + 2 * kWgSlices23 * 64 <= 65536, "bias partials fit their buffer");
        wa.c1.bias_partial = c->bias_partial + bias_first[0];
        wa.c2.bias_partial = c->bias_partial + bias_first[1];
        wa.c3.bias_partial = c->bias_partial + bias_first[2];
        wa.f1.dz = dzh; wa.f1.x = act3; wa.f1.B = B; wa.f1.grad = c->grad + o.wf1;
        wa.small = bg;
        wa.first[0] = 0;
        wa.first[1] = wa.first[0] + n1;
        wa.first[2] = wa.first[1] + n2 * WgConv2::CS;
        wa.first[3] = wa.first[2] + n3 * WgConv3::CS;
        wa.first[4] = wa.first[3] + kWgF1Cols * kWgF1Rows;
        wa.first[5] = wa.first[4] + small_blocks;
        const ProfPair pr = prof_pair(c, K_WGRAD_ALL);
        launch_timed(wgrad_all_kernel, dim3(wa.first[5]), dim3(256), kWgradAllSmem, st, pr.begin, pr.end, wa.first[1], wa.first[2], wa.first[3], wa.first[4],
                     wa.c1.dz, wa.c1.in, wa.c1.n, wa.c1.per, wa.c1.desc, wa.c1.ring, wa);
        DQN_LAUNCH_CHECK();
    } else {
        {   // fc1 weight gradient: dW[o][f] = sum_b dZ[b][o] act3[b][f]
            DenseM<T> al{}; DenseM<T> bl{}; EpiGrad ep{c->grad + o.wf1, 3136, 1.f};
            al.p[0] = dzh; al.ld = 512; bl.p[0] = act3; bl.ld = 3136;
            const ProfPair pr = prof_pair(c, K_FC1_WGRAD);
            DQN_HIP((launch_gemm<T, 64, 128, 32, 2>(st, al, bl, ep, 512, 3136, B, 1, 1, ws.partial, ws.partial_cap, pr.begin, pr.end)));
        }
        {   // conv3 weight gradient
            DenseM<T> al{}; WgradB<T, 64, 9, 9, 7, 7, 3, 1> bl{act2}; EpiGrad ep{c->grad + o.w3, 576, 1.f};
            al.p[0] = dz3; al.ld = 64;
            const ProfPair pr = prof_pair(c, K_CONV3_WGRAD);
            DQN_HIP((launch_gemm<T, 64, 64, 32, 2>(st, al, bl, ep, 64, 576, B * 49, 1, pick_splits(9, B * 49, 32, kWgFp32Splits),
                                                    c->wg_partial + kWgOff3, kWgMaxSplits * 64 * 576, pr.begin, pr.end, &wg_splits[2])));
        }
        {   // conv2 weight gradient
            DenseM<T> al{}; WgradB<T, 32, 20, 20, 9, 9, 4, 2> bl{act1}; EpiGrad ep{c->grad + o.w2, 512, 1.f};
            al.p[0] = dz2; al.ld = 64;
            const ProfPair pr = prof_pair(c, K_CONV2_WGRAD);
            DQN_HIP((launch_gemm<T, 64, 64, 32, 2>(st, al, bl, ep, 64, 512, B * 81, 1, pick_splits(8, B * 81, 32, kWgFp32Splits),
                                                    c->wg_partial + kWgOff2, kWgMaxSplits * 64 * 512, pr.begin, pr.end, &wg_splits[1])));
        }
        {   // conv1 weight gradient (the input scale 1/255 is applied by the optimiser kernel)
            DenseM<T> al{}; Conv1WgradB<T> bl{s}; EpiGrad ep{c->grad + o.w1, 256, 1.f};
            al.p[0] = dz1; al.ld = 32;
            const ProfPair pr = prof_pair(c, K_CONV1_WGRAD);
            DQN_HIP((launch_gemm<T, 32, 128, 32, 1>(st, al, bl, ep, 32, 256, B * 400, 1, pick_splits(2, B * 400, 32, kWgFp32Splits),
                                                     c->wg_partial + kWgOff1, kWgMaxSplits * 32 * 256, pr.begin, pr.end, &wg_splits[0])));
        }
        const ProfPair pr = prof_pair(c, K_BIAS_GRAD);
        launch_timed(bias_grad_kernel<T>, dim3(small_blocks), dim3(256), kSmallGradsSmem, st, pr.begin, pr.end, bg);
        DQN_LAUNCH_CHECK();
    }
    {
        const ProfPair pr = prof_pair(c, K_RMSPROP);
        for (int l = 0; l < 3; ++l) ra.wg_splits[l] = wg_splits[l];
        for (int l = 0; l < 4; ++l) { ra.bias_chunks[l] = bias_chunks[l]; ra.bias_first[l] = bias_first[l]; }
        launch_timed(rmsprop_kernel<T, SHADOW>, dim3(kRmsConvBlocks + ra.flat_blocks + ra.fc1_tiles + kRmsBiasBlocks), dim3(256), 0, st, pr.begin, pr.end, ra.theta,
                     ra.grad, ra.v, ra.m, ra.flat_blocks, ra.fc1_tiles, ra.off.wf1, ra);
        DQN_LAUNCH_CHECK();
    }
    return DQN_OK;
}

// Public blob (OIHW, fc1 input index c*49 + h*7 + w)  <->  device layout (see layers.h).
static void permute_blob(const Offsets& o, const float* src, float* dst, bool to_device)
{
    memcpy(dst, src, o.total * sizeof(float));
    auto conv = [&](size_t off, int O, int C, int K) {
        for (int oc = 0; oc < O; ++oc)
            for (int c = 0; c < C; ++c)
                for (int p = 0; p < K; ++p)
                    for (int q = 0; q < K; ++q) {
                        const size_t pub = off + ((static_cast<size_t>(oc) * C + c) * K + p) * K + q;
                        const size_t dev = off + ((static_cast<size_t>(oc) * K + p) * K + q) * C + c;
                        if (to_device) dst[dev] = src[pub]; else dst[pub] = src[dev];
                    }
    };
    conv(o.w2, 64, 32, 4);
    conv(o.w3, 64, 64, 3);
    for (int oc = 0; oc < 512; ++oc)
        for (int c = 0; c < 64; ++c)
            for (int hw = 0; hw < 49; ++hw) {
                const size_t pub = o.wf1 + static_cast<size_t>(oc) * 3136 + c * 49 + hw;
                const size_t dev = o.wf1 + static_cast<size_t>(oc) * 3136 + hw * 64 + c;
                if (to_device) dst[dev] = src[pub]; else dst[pub] = src[dev];
            }
}

static float* blob_of(dqn_ctx* c, int which)
{
    switch (which) {
        case DQN_PARAMS_ONLINE: return c->theta;
        case DQN_PARAMS_TARGET: return c->theta_t;
        case DQN_PARAMS_RMS_V: return c->v;
        case DQN_PARAMS_RMS_M: return c->m;
        case DQN_PARAMS_GRAD: return c->grad;
        default: return nullptr;
    }
}

static int sync_both(dqn_ctx* c)
{
    DQN_HIP(hipStreamSynchronize(c->act_stream));
    DQN_HIP(hipStreamSynchronize(c->train_stream));
    return DQN_OK;
}

hipStream_t dqn_ctx_act_stream(dqn_ctx* c) { return c->act_stream; }
int dqn_ctx_num_actions(const dqn_ctx* c) { return c->A; }
int dqn_ctx_max_envs(const dqn_ctx* c) { return c->cfg.max_envs; }
int dqn_ctx_max_batch(const dqn_ctx* c) { return c->cfg.max_batch; }

}  // namespace dqn

extern "C" {

int dqn_create(const dqn_config* cfg, void* act_stream, void* train_stream, dqn_ctx** host_out)
{
    if (!host_out) return fail(DQN_EINVAL, "dqn_create: host_out is null");
    *host_out = nullptr;
    if (!cfg) return fail(DQN_EINVAL, "dqn_create: config is null");
    if (cfg->num_actions < 1 || cfg->num_actions > kMaxActions)
        return fail(DQN_EINVAL, "dqn_create: num_actions %d outside 1..%d", cfg->num_actions, kMaxActions);
    if (cfg->max_batch < 1 || cfg->max_batch > kMaxBatch)
        return fail(DQN_EINVAL, "dqn_create: max_batch %d outside 1..%d", cfg->max_batch, kMaxBatch);
    if (cfg->max_envs < 1 || cfg->max_envs > kMaxBatch)
        return fail(DQN_EINVAL, "dqn_create: max_envs %d outside 1..%d", cfg->max_envs, kMaxBatch);
    if (cfg->precision != DQN_PRECISION_FP32 && cfg->precision != DQN_PRECISION_BF16)
        return fail(DQN_EINVAL, "dqn_create: precision %d", cfg->precision);
    if (!(cfg->gamma >= 0.f && cfg->gamma <= 1.f) || !(cfg->huber_delta > 0.f) || !(cfg->lr >= 0.f) ||
        !(cfg->rms_alpha >= 0.f && cfg->rms_alpha <= 1.f) || !(cfg->rms_eps > 0.f))
        return fail(DQN_EINVAL, "dqn_create: hyperparameter out of range");
    dqn_ctx* c = new (std::nothrow) dqn_ctx();
    if (!c) return fail(DQN_ENOMEM, "dqn_create: host allocation failed");
    c->cfg = *cfg;
    c->A = cfg->num_actions;
    c->off = make_offsets(c->A);
    c->esize = cfg->precision == DQN_PRECISION_BF16 ? 2 : 4;
    c->act_stream = static_cast<hipStream_t>(act_stream);
    c->train_stream = static_cast<hipStream_t>(train_stream);
    const size_t n = c->off.total, B = cfg->max_batch;
    auto body = [&]() -> int {
        int dev = 0;
        DQN_HIP(hipGetDevice(&dev));
        c->device = dev;
        void* static_scratch = nullptr;
        DQN_HIP(static_scratch_of(dev, &static_scratch));   // dqn_act_static's array on this device
        DQN_HIP(hipDeviceGetAttribute(&c->num_cus, hipDeviceAttributeMultiprocessorCount, dev));
        if (c->num_cus < 1) c->num_cus = 1;
        float** blobs[5] = {&c->theta, &c->theta_t, &c->v, &c->m, &c->grad};
        for (auto p : blobs) {
            DQN_HIP(hipMalloc((void**)p, (n + 8) * sizeof(float)));
            DQN_HIP(hipMemset(*p, 0, (n + 8) * sizeof(float)));
        }
        if (cfg->precision == DQN_PRECISION_BF16) {
            DQN_HIP(hipMalloc(&c->sh, (n + 8) * 2));
            DQN_HIP(hipMalloc(&c->sh_t, (n + 8) * 2));
            DQN_HIP(hipMemset(c->sh, 0, (n + 8) * 2));
            DQN_HIP(hipMemset(c->sh_t, 0, (n + 8) * 2));
        } else {
            c->sh = c->theta;
            c->sh_t = c->theta_t;
        }
        int rc = alloc_ws(c->train_ws, cfg->max_batch, 3, c->A, c->esize, true);
        if (rc != DQN_OK) return rc;
        rc = alloc_ws(c->act_ws, cfg->max_envs, 1, c->A, c->esize, false);
        if (rc != DQN_OK) return rc;
        DQN_HIP(hipMalloc(&c->bsh, kBshTotal * c->esize));
        DQN_HIP(hipMemset(c->bsh, 0, kBshTotal * c->esize));
        DQN_HIP(hipMalloc((void**)&c->bias_partial, 65536 * sizeof(float)));
        DQN_HIP(hipMalloc((void**)&c->wg_partial, kWgTotal * sizeof(float)));
        DQN_HIP(hipMalloc(&c->dzh, B * 512 * c->esize));
        DQN_HIP(hipMalloc(&c->dz3, B * 3136 * c->esize));
        DQN_HIP(hipMalloc(&c->dz2, B * 5184 * c->esize));
        DQN_HIP(hipMalloc(&c->dz1, B * 12800 * c->esize));
        DQN_HIP(hipMalloc((void**)&c->dqv, B * sizeof(float)));
        DQN_HIP(hipMalloc((void**)&c->lossv, B * sizeof(float)));
        DQN_HIP(hipMalloc((void**)&c->loss_keep, sizeof(float)));
        for (int i = 0; i < 2; ++i) {
            DQN_HIP(hipMalloc((void**)&c->mb_s[i], B * kStateBytes));
            DQN_HIP(hipMalloc((void**)&c->mb_s2[i], B * kStateBytes));
            DQN_HIP(hipMalloc((void**)&c->mb_a[i], B * sizeof(int32_t)));
            DQN_HIP(hipMalloc((void**)&c->mb_r[i], B * sizeof(float)));
            DQN_HIP(hipMalloc((void**)&c->mb_d[i], B * sizeof(float)));
            DQN_HIP(hipMalloc((void**)&c->mb_desc[i], B * kDescInts * sizeof(int32_t)));
        }
        DQN_HIP(hipEventCreateWithFlags(&c->ev_train, hipEventDisableTiming));
        DQN_HIP(hipEventCreateWithFlags(&c->ev_act, hipEventDisableTiming));
        DQN_HIP(hipEventCreateWithFlags(&c->ev_sync, hipEventDisableTiming));
        DQN_HIP(hipDeviceSynchronize());
        return DQN_OK;
    };
    const int rc = body();
    if (rc != DQN_OK) {
        char saved[512];
        strncpy(saved, error_buffer(), sizeof(saved) - 1);
        saved[sizeof(saved) - 1] = 0;
        dqn_destroy(c);
        return fail(rc, "dqn_create: %s", saved);
    }
    *host_out = c;
    return DQN_OK;
}

int dqn_destroy(dqn_ctx* c)
{
    if (!c) return DQN_OK;
    (void)hipStreamSynchronize(c->act_stream);
    (void)hipStreamSynchronize(c->train_stream);
    if (c->sh != c->theta) (void)hipFree(c->sh);
    if (c->sh_t != c->theta_t) (void)hipFree(c->sh_t);
    (void)hipFree(c->theta); (void)hipFree(c->theta_t); (void)hipFree(c->v); (void)hipFree(c->m); (void)hipFree(c->grad);
    free_ws(c->train_ws); free_ws(c->act_ws);
    (void)hipFree(c->dzh); (void)hipFree(c->dz3); (void)hipFree(c->dz2); (void)hipFree(c->dz1);
    (void)hipFree(c->dqv); (void)hipFree(c->lossv); (void)hipFree(c->loss_keep);
    (void)hipFree(c->bsh); (void)hipFree(c->bias_partial); (void)hipFree(c->wg_partial);
    for (int i = 0; i < 2; ++i) {
        (void)hipFree(c->mb_s[i]); (void)hipFree(c->mb_s2[i]); (void)hipFree(c->mb_a[i]); (void)hipFree(c->mb_r[i]); (void)hipFree(c->mb_d[i]);
        (void)hipFree(c->mb_desc[i]);
    }
    if (c->ev_train) (void)hipEventDestroy(c->ev_train);
    if (c->ev_act) (void)hipEventDestroy(c->ev_act);
    if (c->ev_sync) (void)hipEventDestroy(c->ev_sync);
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    delete c;
    return DQN_OK;
}

size_t dqn_num_params(const dqn_ctx* c) { return c ? c->off.total : 0; }

int dqn_set_params(dqn_ctx* c, int which, const float* host_src, size_t n)
{
    if (!c || !host_src) return fail(DQN_EINVAL, "dqn_set_params: null pointer");
    if (n != c->off.total) return fail(DQN_EINVAL, "dqn_set_params: n = %zu, expected %zu", n, c->off.total);
    if (which < DQN_PARAMS_ONLINE || which > DQN_PARAMS_RMS_M) return fail(DQN_EINVAL, "dqn_set_params: which = %d", which);
    int rc = sync_both(c);
    if (rc != DQN_OK) return rc;
    std::vector<float> dev(n);
    permute_blob(c->off, host_src, dev.data(), true);
    float* dst = blob_of(c, which);
    DQN_HIP(hipMemcpy(dst, dev.data(), n * sizeof(float), hipMemcpyHostToDevice));
    const unsigned blocks = static_cast<unsigned>((n + 255) / 256);
    if (which == DQN_PARAMS_ONLINE) {
        if (c->cfg.precision == DQN_PRECISION_BF16)
            hipLaunchKernelGGL((build_copies_kernel<bf16_t, true>), dim3(blocks), dim3(256), 0, c->train_stream, dst,
                               static_cast<bf16_t*>(c->sh), static_cast<bf16_t*>(c->bsh), c->off);
        else
            hipLaunchKernelGGL((build_copies_kernel<float, false>), dim3(blocks), dim3(256), 0, c->train_stream, dst,
                               static_cast<float*>(nullptr), static_cast<float*>(c->bsh), c->off);
        DQN_LAUNCH_CHECK();
        DQN_HIP(hipStreamSynchronize(c->train_stream));
    } else if (which == DQN_PARAMS_TARGET && c->cfg.precision == DQN_PRECISION_BF16) {
        hipLaunchKernelGGL((build_copies_kernel<bf16_t, true>), dim3(blocks), dim3(256), 0, c->train_stream, dst,
                           static_cast<bf16_t*>(c->sh_t), static_cast<bf16_t*>(nullptr), c->off);
        DQN_LAUNCH_CHECK();
        DQN_HIP(hipStreamSynchronize(c->train_stream));
    }
    return DQN_OK;
}

int dqn_get_params(dqn_ctx* c, int which, float* host_dst, size_t n)
{
    if (!c || !host_dst) return fail(DQN_EINVAL, "dqn_get_params: null pointer");
    if (n != c->off.total) return fail(DQN_EINVAL, "dqn_get_params: n = %zu, expected %zu", n, c->off.total);
    const float* src = blob_of(c, which);
    if (!src) return fail(DQN_EINVAL, "dqn_get_params: which = %d", which);
    int rc = sync_both(c);
    if (rc != DQN_OK) return rc;
    std::vector<float> dev(n);
    DQN_HIP(hipMemcpy(dev.data(), src, n * sizeof(float), hipMemcpyDeviceToHost));
    permute_blob(c->off, dev.data(), host_dst, false);
    return DQN_OK;
}

// dqn_act on the given workspace (the context's own, or the fixed array of dqn_act_static); W has been checked.
static int act_call(dqn_ctx* c, Workspace& ws, const char* who, const uint8_t* states, int32_t W, float epsilon,
                    uint64_t act_step, int32_t use_target, int32_t* actions, float* q_out)
{
    if (!states || !actions) return fail(DQN_EINVAL, "%s: null pointer", who);
    if (!aligned16(states)) return fail(DQN_EINVAL, "%s: states not 16-byte aligned", who);
    if (!(epsilon >= 0.f && epsilon <= 1.f)) return fail(DQN_EINVAL, "%s: epsilon outside [0,1]", who);
    std::unique_lock<std::mutex> online_lock(c->online_mu, std::defer_lock);
    if (!use_target) {
        online_lock.lock();
        // standard DQN: the policy needs the parameters the last update produced (Section 3)
        DQN_HIP(wait_for_train(c));
    }
    const int rc = c->cfg.precision == DQN_PRECISION_BF16
                       ? act_impl<bf16_t>(c, ws, states, W, epsilon, act_step, use_target, actions, q_out)
                       : act_impl<float>(c, ws, states, W, epsilon, act_step, use_target, actions, q_out);
    if (rc != DQN_OK) return rc;
    if (!use_target) {
        DQN_HIP(hipEventRecord(c->ev_act, c->act_stream));
        c->act_reads_online.store(true, std::memory_order_release);
    }
    return DQN_OK;
}

int dqn_act(dqn_ctx* c, const uint8_t* states, int32_t W, float epsilon, uint64_t act_step, int32_t use_target,
            int32_t* actions, float* q_out)
{
    if (!c) return fail(DQN_EINVAL, "dqn_act: ctx is null");
    if (W < 1 || W > c->cfg.max_envs) return fail(DQN_EINVAL, "dqn_act: W = %d outside 1..%d", W, c->cfg.max_envs);
    return act_call(c, c->act_ws, "dqn_act", states, W, epsilon, act_step, use_target, actions, q_out);
}

int dqn_act_static(dqn_ctx* c, const uint8_t* states, int32_t W, float epsilon, uint64_t act_step, int32_t use_target,
                   int32_t* actions, float* q_out)
{
    if (!c) return fail(DQN_EINVAL, "dqn_act_static: ctx is null");
    if (W < 1 || W > c->cfg.max_envs || W > kActStaticMaxEnvs)
        return fail(DQN_EINVAL, "dqn_act_static: W = %d outside 1..%d (the fixed array holds at most %d states)", W,
                    c->cfg.max_envs < kActStaticMaxEnvs ? c->cfg.max_envs : kActStaticMaxEnvs, kActStaticMaxEnvs);
    void* base = nullptr;
    DQN_HIP(static_scratch_of(c->device, &base));   // looked up by dqn_create; here only a table read
    unsigned char* p = static_cast<unsigned char*>(base);
    Workspace ws;
    ws.act1 = p + kActStaticAct1; ws.act2 = p + kActStaticAct2; ws.act3 = p + kActStaticAct3;
    ws.partial = reinterpret_cast<float*>(p + kActStaticPartial);
    ws.partial_cap = static_cast<size_t>(7) * kActStaticMaxEnvs * 512;
    return act_call(c, ws, "dqn_act_static", states, W, epsilon, act_step, use_target, actions, q_out);
}

int dqn_act_push_step(dqn_ctx* c, replay* rb, const uint8_t* push_frames, const int32_t* push_actions,
                      const float* push_rewards, const uint8_t* push_terminals, const uint8_t* states, int32_t W,
                      float epsilon, uint64_t act_step, int32_t use_target, int32_t* actions, float* q_out)
{
    if (!c || !rb) return fail(DQN_EINVAL, "dqn_act_push_step: ctx or rb is null");
    if (replay_push_stream(rb) != c->act_stream)
        return fail(DQN_EINVAL, "dqn_act_push_step: the replay memory's push stream is not the context's act stream");
    if (c->cfg.precision != DQN_PRECISION_BF16) {
        // fp32 mode has no fused launch to ride in: the two calls, in order
        const int rc = replay_push_step(rb, push_frames, push_actions, push_rewards, push_terminals);
        return rc != DQN_OK ? rc : dqn_act(c, states, W, epsilon, act_step, use_target, actions, q_out);
    }
    if (W < 1 || W > c->cfg.max_envs) return fail(DQN_EINVAL, "dqn_act_push_step: W = %d outside 1..%d", W, c->cfg.max_envs);
    if (!states || !actions) return fail(DQN_EINVAL, "dqn_act_push_step: null pointer");
    if (!aligned16(states)) return fail(DQN_EINVAL, "dqn_act_push_step: states not 16-byte aligned");
    if (!(epsilon >= 0.f && epsilon <= 1.f)) return fail(DQN_EINVAL, "dqn_act_push_step: epsilon outside [0,1]");
    PushStepPlan plan;
    int rc = replay_plan_push_step(rb, push_frames, push_actions, push_rewards, push_terminals, &plan);
    if (rc != DQN_OK) return rc;
    std::unique_lock<std::mutex> online_lock(c->online_mu, std::defer_lock);
    if (!use_target) {
        online_lock.lock();
        DQN_HIP(wait_for_train(c));
    }
    rc = act_impl<bf16_t>(c, c->act_ws, states, W, epsilon, act_step, use_target, actions, q_out, &plan);
    if (rc != DQN_OK) return rc;
    replay_commit_push_step(rb);
    if (!use_target) {
        DQN_HIP(hipEventRecord(c->ev_act, c->act_stream));
        c->act_reads_online.store(true, std::memory_order_release);
    }
    return DQN_OK;
}

int dqn_train_step(dqn_ctx* c, const uint8_t* s, const int32_t* a, const float* r, const uint8_t* s2,
                   const float* done, int32_t B, float* loss_out)
{
    if (!c) return fail(DQN_EINVAL, "dqn_train_step: ctx is null");
    if (B < 1 || B > c->cfg.max_batch) return fail(DQN_EINVAL, "dqn_train_step: B = %d outside 1..%d", B, c->cfg.max_batch);
    if (!s || !a || !r || !s2 || !done) return fail(DQN_EINVAL, "dqn_train_step: null pointer");
    if (!aligned16(s) || !aligned16(s2)) return fail(DQN_EINVAL, "dqn_train_step: s/s2 not 16-byte aligned");
    std::lock_guard<std::mutex> online_lock(c->online_mu);
    DQN_HIP(wait_for_online_act(c));
    int rc;
    if (c->cfg.precision == DQN_PRECISION_BF16) rc = train_impl<bf16_t, true>(c, s, a, r, s2, done, B, loss_out);
    else rc = train_impl<float, false>(c, s, a, r, s2, done, B, loss_out);
    if (rc != DQN_OK) return rc;
    c->train_unrecorded.store(true, std::memory_order_release);   // the event is recorded by the first reader, if any
    c->last_B = B;
    return DQN_OK;
}

int dqn_train_step_sampled(dqn_ctx* c, replay* rb, int32_t B, uint64_t sample_step, int32_t prefetch_next, float* loss_out)
{
    if (!c || !rb) return fail(DQN_EINVAL, "dqn_train_step_sampled: null handle");
    if (B < 1 || B > c->cfg.max_batch) return fail(DQN_EINVAL, "dqn_train_step_sampled: B = %d outside 1..%d", B, c->cfg.max_batch);
    if (replay_sample_stream(rb) != c->train_stream)
        return fail(DQN_EINVAL, "dqn_train_step_sampled: the replay's sample stream must be the train stream");
    std::lock_guard<std::mutex> online_lock(c->online_mu);
    // Reduced precision, large minibatch: the minibatch is only DESCRIBED (replay slots per frame, a, r, done); the fused
    // conv kernel and conv1's weight gradient read the frames from the replay memory themselves.  Otherwise the states are
    // assembled (replay_sample_gather's kernel, riding in the previous step's head kernel where it can).
    const bool by_desc = c->cfg.precision == DQN_PRECISION_BF16 && B >= kDescMinBatch;
    int buf = 0;
    if (c->pre_valid && c->pre_rb == rb && c->pre_B == B && c->pre_step == sample_step && c->pre_epoch == replay_epoch(rb)) {
        buf = c->pre_buf;   // prepared inside the previous call's launches, and no flush since
    } else if (by_desc) {
        GatherPlan now;
        const int rc = replay_plan_sample_gather(rb, B, sample_step, nullptr, c->mb_s[0], c->mb_s2[0], c->mb_a[0], c->mb_r[0], c->mb_d[0], nullptr, &now);
        if (rc != DQN_OK) return rc;
        hipLaunchKernelGGL(sample_desc_kernel, dim3((B + 255) / 256), dim3(256), 0, c->train_stream, now, c->mb_desc[0]);
        DQN_LAUNCH_CHECK();
    } else {
        const int rc = replay_sample_gather(rb, B, sample_step, nullptr, c->mb_s[0], c->mb_s2[0], c->mb_a[0], c->mb_r[0], c->mb_d[0], nullptr);
        if (rc != DQN_OK) return rc;
    }
    c->pre_valid = false;
    GatherPlan plan;
    const GatherPlan* ride = nullptr;
    // full precision has only the head kernel to ride in, and beyond a few hundred samples the byte gather outlasts it
    if (prefetch_next && (by_desc || B <= 256)) {
        const int nb = buf ^ 1;
        const int rc = replay_plan_sample_gather(rb, B, sample_step + 1, nullptr, c->mb_s[nb], c->mb_s2[nb], c->mb_a[nb], c->mb_r[nb],
                                                 c->mb_d[nb], nullptr, &plan);
        if (rc != DQN_OK) return rc;
        ride = &plan;
    }
    DQN_HIP(wait_for_online_act(c));
    int rc;
    if (by_desc) {
        const StateSource src{c->mb_desc[buf], replay_ring_frames(rb), nullptr};   // nobody needs the assembled state
        rc = train_impl<bf16_t, true>(c, c->mb_s[buf], c->mb_a[buf], c->mb_r[buf], c->mb_s2[buf], c->mb_d[buf], B, loss_out, ride,
                                      ride ? c->mb_desc[buf ^ 1] : nullptr, &src);
    } else if (c->cfg.precision == DQN_PRECISION_BF16)
        rc = train_impl<bf16_t, true>(c, c->mb_s[buf], c->mb_a[buf], c->mb_r[buf], c->mb_s2[buf], c->mb_d[buf], B, loss_out, ride);
    else
        rc = train_impl<float, false>(c, c->mb_s[buf], c->mb_a[buf], c->mb_r[buf], c->mb_s2[buf], c->mb_d[buf], B, loss_out, ride);
    if (rc != DQN_OK) return rc;
    c->train_unrecorded.store(true, std::memory_order_release);
    c->last_B = B;
    if (ride) {
        c->pre_valid = true; c->pre_rb = rb; c->pre_B = B; c->pre_step = sample_step + 1; c->pre_epoch = replay_epoch(rb);
        c->pre_buf = buf ^ 1;
    }
    return DQN_OK;
}

int dqn_get_train_q(dqn_ctx* c, float* host_q_online, float* host_q_next_target, float* host_q_next_online)
{
    if (!c) return fail(DQN_EINVAL, "dqn_get_train_q: ctx is null");
    if (c->last_B == 0) return fail(DQN_ESTATE, "dqn_get_train_q: no train step has run");
    DQN_HIP(hipStreamSynchronize(c->train_stream));
    const size_t row = static_cast<size_t>(c->last_B) * c->A;
    if (host_q_online) DQN_HIP(hipMemcpy(host_q_online, c->train_ws.q, row * 4, hipMemcpyDeviceToHost));
    if (host_q_next_target) DQN_HIP(hipMemcpy(host_q_next_target, c->train_ws.q + row, row * 4, hipMemcpyDeviceToHost));
    if (host_q_next_online && c->cfg.double_dqn)
        DQN_HIP(hipMemcpy(host_q_next_online, c->train_ws.q + 2 * row, row * 4, hipMemcpyDeviceToHost));
    return DQN_OK;
}

int dqn_profile_kernel_count(void) { return K_COUNT - 1; }

const char* dqn_profile_kernel_name(int kernel_id)
{
    return kernel_id >= 1 && kernel_id < K_COUNT ? kKernelNames[kernel_id] : nullptr;
}

int dqn_profile_select(dqn_ctx* c, int kernel_id) { return dqn_profile_select_every(c, kernel_id, 1); }

int dqn_profile_select_every(dqn_ctx* c, int kernel_id, int32_t every)
{
    if (!c) return fail(DQN_EINVAL, "dqn_profile_select: ctx is null");
    if (kernel_id < 0 || kernel_id >= K_COUNT) return fail(DQN_EINVAL, "dqn_profile_select: kernel id %d", kernel_id);
    if (every < 1) return fail(DQN_EINVAL, "dqn_profile_select_every: every = %d", every);
    DQN_HIP(hipStreamSynchronize(c->train_stream));
    if (kernel_id != 0 && c->prof_events.empty()) {
        c->prof_events.reserve(2 * kProfPairs);
        for (size_t i = 0; i < 2 * kProfPairs; ++i) {
            hipEvent_t e;
            DQN_HIP(hipEventCreate(&e));
            c->prof_events.push_back(e);
        }
    }
    c->prof_id = kernel_id;
    c->prof_used = 0;
    c->prof_every = every;
    c->prof_seen = 0;
    return DQN_OK;
}

int dqn_profile_read(dqn_ctx* c, double* host_total_ms, int64_t* host_launches)
{
    if (!c || !host_total_ms || !host_launches) return fail(DQN_EINVAL, "dqn_profile_read: null pointer");
    DQN_HIP(hipStreamSynchronize(c->train_stream));
    double total = 0.0;
    for (size_t i = 0; i < c->prof_used; ++i) {
        float ms = 0.f;
        DQN_HIP(hipEventElapsedTime(&ms, c->prof_events[2 * i], c->prof_events[2 * i + 1]));
        total += ms;
    }
    *host_total_ms = total;
    *host_launches = static_cast<int64_t>(c->prof_used);
    return DQN_OK;
}

int dqn_sync_target(dqn_ctx* c, replay* rb, int32_t blocking)
{
    if (!c) return fail(DQN_EINVAL, "dqn_sync_target: ctx is null");
    if (rb && replay_sample_stream(rb) != c->train_stream)
        return fail(DQN_EINVAL, "dqn_sync_target: the replay's sample stream must be the train stream");
    // wait: train_stream <- act_stream
    DQN_HIP(hipEventRecord(c->ev_act, c->act_stream));
    DQN_HIP(hipStreamWaitEvent(c->train_stream, c->ev_act, 0));
    c->act_reads_online.store(false, std::memory_order_release);
    if (rb) {
        const int rc = replay_flush_ordered(rb);   // also orders the replay's push stream around the flush
        if (rc != DQN_OK) return rc;
    }
    const size_t n = c->off.total;
    if (c->cfg.precision == DQN_PRECISION_BF16)
        hipLaunchKernelGGL((target_copy_kernel<bf16_t, true>), dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                           c->train_stream, c->theta, c->theta_t, static_cast<const bf16_t*>(c->sh),
                           static_cast<bf16_t*>(c->sh_t), n);
    else
        hipLaunchKernelGGL((target_copy_kernel<float, false>), dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                           c->train_stream, c->theta, c->theta_t, static_cast<const float*>(nullptr),
                           static_cast<float*>(nullptr), n);
    DQN_LAUNCH_CHECK();
    DQN_HIP(hipEventRecord(c->ev_sync, c->train_stream));
    DQN_HIP(hipStreamWaitEvent(c->act_stream, c->ev_sync, 0));
    if (blocking) DQN_HIP(hipStreamSynchronize(c->train_stream));
    return DQN_OK;
}

}  // extern "C"
