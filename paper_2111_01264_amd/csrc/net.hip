// The Q-network side of the hot path: batched act step (Sections 3, 4), minibatch train step
// (Section 2.1, Eq. 1; Appendix B) and the synchronisation point (Algorithm 1), as sequences of
// hand-written gfx950 kernels on two HIP streams.
#include <math.h>
#include <string.h>

#include <new>
#include <vector>

#include "common.h"
#include "layers.h"
#include "philox.h"

namespace dqn {

// Offsets of the tensors inside a parameter blob (identical for the public and the device layout).
struct Offsets {
    size_t w1, b1, w2, b2, w3, b3, wf1, bf1, wf2, bf2, total;
};
static Offsets make_offsets(int A)
{
    Offsets o;
    o.w1 = 0;            o.b1 = o.w1 + 32 * 256;
    o.w2 = o.b1 + 32;    o.b2 = o.w2 + 64 * 512;
    o.w3 = o.b2 + 64;    o.b3 = o.w3 + 64 * 576;
    o.wf1 = o.b3 + 64;   o.bf1 = o.wf1 + 512 * 3136;
    o.wf2 = o.bf1 + 512; o.bf2 = o.wf2 + static_cast<size_t>(A) * 512;
    o.total = o.bf2 + A;
    return o;
}

enum KernelId {
    K_NONE = 0, K_CONV1_FWD, K_CONV2_FWD, K_CONV3_FWD, K_FC1_FWD, K_FC2_TD, K_TD_HEAD_BWD, K_FC1_WGRAD,
    K_FC1_DGRAD, K_CONV3_WGRAD, K_CONV3_DGRAD, K_CONV2_WGRAD, K_CONV2_DGRAD, K_CONV1_WGRAD, K_BIAS_GRAD,
    K_RMSPROP, K_COUNT
};
static const char* const kKernelNames[K_COUNT] = {
    "none", "conv1_fwd", "conv2_fwd", "conv3_fwd", "fc1_fwd", "fc2_td", "td_head_bwd", "fc1_wgrad",
    "fc1_dgrad", "conv3_wgrad", "conv3_dgrad", "conv2_wgrad", "conv2_dgrad", "conv1_wgrad", "bias_grad",
    "rmsprop"};
constexpr size_t kProfPairs = 4096;

constexpr int kMaxBatch = 1024;
constexpr int kMaxActions = 64;

// ---- small kernels ------------------------------------------------------------------------------

// Dot products of one 512-vector with the A rows of fc2, one wavefront per call: lane l owns
// k = 8l .. 8l+7; butterfly reduction (fixed order, so the result does not depend on the launch).
// Returns Q[a] in lane a (a < A) and -inf in the other lanes.
template <typename T>
__device__ inline float fc2_row(const T* __restrict__ h, const T* __restrict__ w2, const float* __restrict__ b2,
                                int A, int lane)
{
    typedef typename Vec8<T>::type V8;
    const V8 hv = *reinterpret_cast<const V8*>(h + lane * 8);
    float mine = -INFINITY;
    for (int a = 0; a < A; ++a) {
        const V8 wv = *reinterpret_cast<const V8*>(w2 + static_cast<size_t>(a) * 512 + lane * 8);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += to_float(hv[e]) * to_float(wv[e]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == a) mine = acc + b2[a];
    }
    return mine;
}

// argmax over the lanes of a wavefront, lowest lane on ties; result uniform across the wavefront.
__device__ inline int wave_argmax_lowest(float v, int lane)
{
    int idx = lane;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(v, off, 64);
        const int oi = __shfl_xor(idx, off, 64);
        if (ov > v || (ov == v && oi < idx)) { v = ov; idx = oi; }
    }
    return idx;
}

// Act step tail: fc2 + epsilon-greedy, one wavefront per environment.
template <typename T>
__global__ __launch_bounds__(256) void fc2_act_kernel(const T* __restrict__ h, const T* __restrict__ w2,
                                                      const float* __restrict__ b2, int W, int A, float epsilon,
                                                      uint64_t seed, uint64_t act_step,
                                                      int32_t* __restrict__ actions, float* __restrict__ q_out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = blockIdx.x * 4 + wave;
    if (j >= W) return;
    const float q = fc2_row<T>(h + static_cast<size_t>(j) * 512, w2, b2, A, lane);
    if (q_out && lane < A) q_out[static_cast<size_t>(j) * A + lane] = q;
    const int greedy = wave_argmax_lowest(q, lane);
    if (lane == 0) {
        const Philox4 d = philox_draw(seed, kTagAct, act_step, static_cast<uint32_t>(j));
        const float u = static_cast<float>(d.x[0] >> 8) * 0x1p-24f;
        int act = greedy;
        if (u < epsilon) act = static_cast<int>((static_cast<uint64_t>(d.x[1]) * static_cast<uint32_t>(A)) >> 32);
        actions[j] = act;
    }
}

// Train step head, forward half: fc2 for Q(s,.;theta), Q(s',.;theta^-) [and Q(s',.;theta)], then
// per sample the TD target, the error, its clipped gradient and its loss term (Eq. 1).
template <typename T>
__global__ __launch_bounds__(256) void fc2_td_kernel(
    const T* __restrict__ h, const T* __restrict__ w2_online, const T* __restrict__ w2_target,
    const float* __restrict__ b2_online, const float* __restrict__ b2_target, int B, int A, int double_dqn,
    const int32_t* __restrict__ act, const float* __restrict__ rew, const float* __restrict__ done,
    float gamma, float huber, float* __restrict__ q_all, float* __restrict__ dqv, float* __restrict__ lossv)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.x * 4 + wave;
    if (b >= B) return;
    const float q_on = fc2_row<T>(h + static_cast<size_t>(b) * 512, w2_online, b2_online, A, lane);
    const float q_nt = fc2_row<T>(h + static_cast<size_t>(B + b) * 512, w2_target, b2_target, A, lane);
    int astar;
    if (double_dqn) {
        const float q_no = fc2_row<T>(h + static_cast<size_t>(2 * B + b) * 512, w2_online, b2_online, A, lane);
        if (lane < A) q_all[(static_cast<size_t>(2) * B + b) * A + lane] = q_no;
        astar = wave_argmax_lowest(q_no, lane);
    } else {
        astar = wave_argmax_lowest(q_nt, lane);
    }
    if (lane < A) {
        q_all[static_cast<size_t>(b) * A + lane] = q_on;
        q_all[(static_cast<size_t>(B) + b) * A + lane] = q_nt;
    }
    const float boot = __shfl(q_nt, astar, 64);
    const float q_sa = __shfl(q_on, act[b], 64);
    if (lane == 0) {
        const float y = rew[b] + gamma * (1.f - done[b]) * boot;
        const float delta = q_sa - y;
        const float ad = fabsf(delta);
        lossv[b] = ad <= huber ? 0.5f * delta * delta : huber * (ad - 0.5f * huber);
        const float clipped = fminf(fmaxf(delta, -huber), huber);
        dqv[b] = clipped / static_cast<float>(B);
    }
}

// Train step head, backward half.  dQ has one non-zero per row (the taken action), so fc2's
// backward is a gather: dZ_fc1[b][o] = dq_b * W2[a_b][o] * [h[b][o] > 0];
// dW2[a][o] = sum_{b: a_b = a} dq_b h[b][o];  db2[a] = sum_{b: a_b = a} dq_b;  loss = mean_b loss_b.
// Each block owns 64 columns o; all sums run over b in increasing order.
template <typename T>
__global__ __launch_bounds__(256) void td_head_bwd_kernel(
    const T* __restrict__ h, const T* __restrict__ w2, const int32_t* __restrict__ act,
    const float* __restrict__ dqv, const float* __restrict__ lossv, int B, int A, T* __restrict__ dzh,
    float* __restrict__ g_w2, float* __restrict__ g_b2, float* __restrict__ loss_out, float* __restrict__ loss_keep)
{
    __shared__ float s_dq[kMaxBatch];
    __shared__ int s_a[kMaxBatch];
    for (int b = threadIdx.x; b < B; b += blockDim.x) { s_dq[b] = dqv[b]; s_a[b] = act[b]; }
    __syncthreads();
    const int o = blockIdx.x * 64 + (threadIdx.x & 63);
    const int part = threadIdx.x >> 6;
    for (int b = part; b < B; b += 4) {
        const size_t idx = static_cast<size_t>(b) * 512 + o;
        const float hv = to_float(h[idx]);
        const float g = s_dq[b] * to_float(w2[static_cast<size_t>(s_a[b]) * 512 + o]);
        dzh[idx] = hv > 0.f ? from_float<T>(g) : from_float<T>(0.f);
    }
    for (int a = part; a < A; a += 4) {
        float acc = 0.f;
        for (int b = 0; b < B; ++b)
            if (s_a[b] == a) acc += s_dq[b] * to_float(h[static_cast<size_t>(b) * 512 + o]);
        g_w2[static_cast<size_t>(a) * 512 + o] = acc;
    }
    if (blockIdx.x == 0) {
        for (int a = threadIdx.x; a < A; a += blockDim.x) {
            float acc = 0.f;
            for (int b = 0; b < B; ++b)
                if (s_a[b] == a) acc += s_dq[b];
            g_b2[a] = acc;
        }
        if (threadIdx.x == 0) {
            float acc = 0.f;
            for (int b = 0; b < B; ++b) acc += lossv[b];
            acc /= static_cast<float>(B);
            *loss_keep = acc;
            if (loss_out) *loss_out = acc;
        }
    }
}

// Bias gradients = column sums of the four dZ matrices ([rows][C], T).  One block per
// (layer, group of eight channels); rows are strided over the threads and combined by a fixed tree.
struct BiasGradArgs {
    const void* dz[4];
    float* out[4];
    int rows[4];
    int chans[4];
    int first_block[5];
};
template <typename T>
__global__ __launch_bounds__(256) void bias_grad_kernel(BiasGradArgs args)
{
    typedef typename Vec8<T>::type V8;
    __shared__ float red[256][9];
    int layer = 0;
    while (layer < 3 && static_cast<int>(blockIdx.x) >= args.first_block[layer + 1]) ++layer;
    const int cg = blockIdx.x - args.first_block[layer];
    const T* dz = static_cast<const T*>(args.dz[layer]) + cg * 8;
    const int C = args.chans[layer], rows = args.rows[layer];
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int r = threadIdx.x; r < rows; r += 256) {
        const V8 v = *reinterpret_cast<const V8*>(dz + static_cast<size_t>(r) * C);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += to_float(v[e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[threadIdx.x][e] = acc[e];
    __syncthreads();
    for (int stride = 128; stride >= 1; stride >>= 1) {
        if (static_cast<int>(threadIdx.x) < stride)
#pragma unroll
            for (int e = 0; e < 8; ++e) red[threadIdx.x][e] += red[threadIdx.x + stride][e];
        __syncthreads();
    }
    if (threadIdx.x < 8) args.out[layer][cg * 8 + threadIdx.x] = red[0][threadIdx.x];
}

// Centered RMSProp (Appendix B) fused with the refresh of the low-precision operand copy.
template <typename T, bool SHADOW>
__global__ __launch_bounds__(256) void rmsprop_kernel(float* __restrict__ theta, const float* __restrict__ grad,
                                                      float* __restrict__ v, float* __restrict__ m,
                                                      T* __restrict__ shadow, size_t n, float lr, float alpha,
                                                      float eps, int centered)
{
    const size_t n4 = n / 4;
    const size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    auto update = [&](float& th, float g, float& vv, float& mm) {
        vv = alpha * vv + (1.f - alpha) * g * g;
        float var = vv;
        if (centered) {
            mm = alpha * mm + (1.f - alpha) * g;
            var = fmaxf(vv - mm * mm, 0.f);
        }
        th -= lr * g / (sqrtf(var) + eps);
    };
    if (i < n4) {
        float4 th = reinterpret_cast<float4*>(theta)[i];
        const float4 g = reinterpret_cast<const float4*>(grad)[i];
        float4 vv = reinterpret_cast<float4*>(v)[i];
        float4 mm = reinterpret_cast<float4*>(m)[i];
        update(th.x, g.x, vv.x, mm.x);
        update(th.y, g.y, vv.y, mm.y);
        update(th.z, g.z, vv.z, mm.z);
        update(th.w, g.w, vv.w, mm.w);
        reinterpret_cast<float4*>(theta)[i] = th;
        reinterpret_cast<float4*>(v)[i] = vv;
        if (centered) reinterpret_cast<float4*>(m)[i] = mm;
        if (SHADOW) {
            shadow[4 * i + 0] = from_float<T>(th.x);
            shadow[4 * i + 1] = from_float<T>(th.y);
            shadow[4 * i + 2] = from_float<T>(th.z);
            shadow[4 * i + 3] = from_float<T>(th.w);
        }
    } else if (i < n4 + (n - 4 * n4)) {
        const size_t e = 4 * n4 + (i - n4);
        float th = theta[e], vv = v[e], mm = m[e];
        update(th, grad[e], vv, mm);
        theta[e] = th; v[e] = vv;
        if (centered) m[e] = mm;
        if (SHADOW) shadow[e] = from_float<T>(th);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void shadow_cast_kernel(const float* __restrict__ src, T* __restrict__ dst, size_t n)
{
    const size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    if (i < n) dst[i] = from_float<T>(src[i]);
}

// theta^- <- theta: fp32 master (bitwise) and, if present, the operand copy.
template <typename T, bool SHADOW>
__global__ __launch_bounds__(256) void target_copy_kernel(const float* __restrict__ theta, float* __restrict__ theta_t,
                                                          const T* __restrict__ sh, T* __restrict__ sh_t, size_t n)
{
    const size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    if (i < n) {
        theta_t[i] = theta[i];
        if (SHADOW) sh_t[i] = sh[i];
    }
}

}  // namespace dqn

using namespace dqn;

// Activations / gradients of one forward+backward workspace, sized for `cap` samples per group.
struct Workspace {
    void* act1 = nullptr;   // [G*cap][20][20][32]
    void* act2 = nullptr;   // [G*cap][9][9][64]
    void* act3 = nullptr;   // [G*cap][7][7][64]
    void* h = nullptr;      // [G*cap][512]
    float* q = nullptr;     // [G*cap][A]
    float* partial = nullptr;
    size_t partial_cap = 0;
};

struct dqn_ctx {
    dqn_config cfg;
    int A;
    Offsets off;
    size_t esize;           // bytes per operand element
    hipStream_t act_stream, train_stream;
    float *theta = nullptr, *theta_t = nullptr, *v = nullptr, *m = nullptr, *grad = nullptr;
    void *sh = nullptr, *sh_t = nullptr;   // operand copies; alias theta / theta_t in fp32 mode
    Workspace train_ws, act_ws;
    void *dzh = nullptr, *dz3 = nullptr, *dz2 = nullptr, *dz1 = nullptr;
    float *dqv = nullptr, *lossv = nullptr, *loss_keep = nullptr;
    hipEvent_t ev_train = nullptr, ev_act = nullptr, ev_sync = nullptr;
    bool act_reads_online = false;   // an act step with use_target = 0 is in flight
    int last_B = 0;
    // per-kernel timing (dqn_profile_*)
    int prof_id = 0;
    std::vector<hipEvent_t> prof_events;   // pairs
    size_t prof_used = 0;                  // pairs recorded since the last select
};

namespace dqn {

static size_t partial_floats(int n, int groups)
{
    // generous bound: the largest split-K product used below (see pick_splits)
    const size_t fwd = static_cast<size_t>(groups) * 64 * n * 512;          // fc1 forward, <= 64 splits
    const size_t wg = static_cast<size_t>(512) * 64 * 576;                  // conv weight grads, <= 512 splits
    const size_t dg = static_cast<size_t>(16) * n * 3136;                   // fc1 dgrad
    const size_t cv = static_cast<size_t>(groups) * 8 * n * 81 * 64;        // conv2/3 forward
    size_t best = fwd;
    if (wg > best) best = wg;
    if (dg > best) best = dg;
    if (cv > best) best = cv;
    return best;
}

static int alloc_ws(Workspace& ws, int cap, int groups, int A, size_t esize, bool with_partial_bwd)
{
    (void)with_partial_bwd;
    const size_t n = static_cast<size_t>(cap) * groups;
    DQN_HIP(hipMalloc(&ws.act1, n * 12800 * esize));
    DQN_HIP(hipMalloc(&ws.act2, n * 5184 * esize));
    DQN_HIP(hipMalloc(&ws.act3, n * 3136 * esize));
    DQN_HIP(hipMalloc(&ws.h, n * 512 * esize));
    DQN_HIP(hipMalloc((void**)&ws.q, n * A * sizeof(float)));
    ws.partial_cap = partial_floats(cap, groups);
    DQN_HIP(hipMalloc((void**)&ws.partial, ws.partial_cap * sizeof(float)));
    return DQN_OK;
}

static void free_ws(Workspace& ws)
{
    (void)hipFree(ws.act1); (void)hipFree(ws.act2); (void)hipFree(ws.act3); (void)hipFree(ws.h);
    (void)hipFree(ws.q); (void)hipFree(ws.partial);
}

// Event pair for a launch of kernel `id`, or nulls if that kernel is not the selected one.
struct ProfPair { hipEvent_t begin = nullptr, end = nullptr; };
static ProfPair prof_pair(dqn_ctx* c, int id)
{
    ProfPair p;
    if (c->prof_id == id && c->prof_used < c->prof_events.size() / 2) {
        p.begin = c->prof_events[2 * c->prof_used];
        p.end = c->prof_events[2 * c->prof_used + 1];
        ++c->prof_used;
    }
    return p;
}

static int pick_splits(int tiles, int groups, int K, int BK, int max_splits)
{
    const int target = 512;   // about two workgroups per compute unit
    int s = target / (tiles * groups > 0 ? tiles * groups : 1);
    const int by_k = K / (2 * BK) > 0 ? K / (2 * BK) : 1;
    if (s > by_k) s = by_k;
    if (s > max_splits) s = max_splits;
    return s < 1 ? 1 : s;
}

// Forward pass of `groups` independent (input, parameter set) pairs with n samples each, up to h.
template <typename T>
static int forward_to_h(dqn_ctx* c, hipStream_t st, Workspace& ws, int groups, const uint8_t* const* x,
                        const void* const* shadow, const float* const* master, int n, bool timed)
{
    auto pp = [&](int id) { return timed ? prof_pair(c, id) : ProfPair(); };
    const Offsets& o = c->off;
    const size_t e_act1 = static_cast<size_t>(n) * 12800, e_act2 = static_cast<size_t>(n) * 5184;
    const size_t e_act3 = static_cast<size_t>(n) * 3136, e_h = static_cast<size_t>(n) * 512;
    T* act1 = static_cast<T*>(ws.act1); T* act2 = static_cast<T*>(ws.act2);
    T* act3 = static_cast<T*>(ws.act3); T* h = static_cast<T*>(ws.h);
    {   // conv1: [n*400, 32] = im2col(u8)[n*400, 256] x W1^T, (1/255) scale + bias + ReLU
        Conv1A<T> al{}; DenseK<T> bl{}; EpiBiasAct<T, true> ep{};
        for (int g = 0; g < groups; ++g) {
            al.x[g] = x[g];
            bl.p[g] = static_cast<const T*>(shadow[g]) + o.w1;
            ep.out[g] = act1 + g * e_act1; ep.bias[g] = master[g] + o.b1;
        }
        bl.ld = 256; ep.ld = 32; ep.scale = 1.f / 255.f;
        const ProfPair pr = pp(K_CONV1_FWD);
        DQN_HIP((launch_gemm<T, 128, 32, 32, 4>(st, al, bl, ep, n * 400, 32, 256, groups, 1, ws.partial, ws.partial_cap,
                                                 pr.begin, pr.end)));
    }
    {   // conv2
        ConvA<T, 32, 20, 20, 9, 9, 4, 2> al{}; DenseK<T> bl{}; EpiBiasAct<T, true> ep{};
        for (int g = 0; g < groups; ++g) {
            al.x[g] = act1 + g * e_act1;
            bl.p[g] = static_cast<const T*>(shadow[g]) + o.w2;
            ep.out[g] = act2 + g * e_act2; ep.bias[g] = master[g] + o.b2;
        }
        bl.ld = 512; ep.ld = 64; ep.scale = 1.f;
        const int M = n * 81, tiles = (M + 63) / 64;
        const ProfPair pr = pp(K_CONV2_FWD);
        DQN_HIP((launch_gemm<T, 64, 64, 32, 2>(st, al, bl, ep, M, 64, 512, groups, pick_splits(tiles, groups, 512, 32, 8),
                                                ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {   // conv3
        ConvA<T, 64, 9, 9, 7, 7, 3, 1> al{}; DenseK<T> bl{}; EpiBiasAct<T, true> ep{};
        for (int g = 0; g < groups; ++g) {
            al.x[g] = act2 + g * e_act2;
            bl.p[g] = static_cast<const T*>(shadow[g]) + o.w3;
            ep.out[g] = act3 + g * e_act3; ep.bias[g] = master[g] + o.b3;
        }
        bl.ld = 576; ep.ld = 64; ep.scale = 1.f;
        const int M = n * 49, tiles = (M + 63) / 64;
        const ProfPair pr = pp(K_CONV3_FWD);
        DQN_HIP((launch_gemm<T, 64, 64, 32, 2>(st, al, bl, ep, M, 64, 576, groups, pick_splits(tiles, groups, 576, 32, 8),
                                                ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {   // fc1
        DenseK<T> al{}; DenseK<T> bl{}; EpiBiasAct<T, true> ep{};
        for (int g = 0; g < groups; ++g) {
            al.p[g] = act3 + g * e_act3;
            bl.p[g] = static_cast<const T*>(shadow[g]) + o.wf1;
            ep.out[g] = h + g * e_h; ep.bias[g] = master[g] + o.bf1;
        }
        al.ld = 3136; bl.ld = 3136; ep.ld = 512; ep.scale = 1.f;
        const int tiles = ((n + 31) / 32) * 4;
        const ProfPair pr = pp(K_FC1_FWD);
        DQN_HIP((launch_gemm<T, 32, 128, 32, 1>(st, al, bl, ep, n, 512, 3136, groups, pick_splits(tiles, groups, 3136, 32, 64),
                                                 ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    return DQN_OK;
}

template <typename T>
static int act_impl(dqn_ctx* c, const uint8_t* states, int W, float epsilon, uint64_t act_step, int use_target,
                    int32_t* actions, float* q_out)
{
    const uint8_t* x[1] = {states};
    const void* shadow[1] = {use_target ? c->sh_t : c->sh};
    const float* master[1] = {use_target ? c->theta_t : c->theta};
    const int rc = forward_to_h<T>(c, c->act_stream, c->act_ws, 1, x, shadow, master, W, false);
    if (rc != DQN_OK) return rc;
    hipLaunchKernelGGL((fc2_act_kernel<T>), dim3((W + 3) / 4), dim3(256), 0, c->act_stream,
                       static_cast<const T*>(c->act_ws.h), static_cast<const T*>(shadow[0]) + c->off.wf2,
                       master[0] + c->off.bf2, W, c->A, epsilon, c->cfg.seed, act_step, actions, q_out);
    DQN_LAUNCH_CHECK();
    return DQN_OK;
}

template <typename T, bool SHADOW>
static int train_impl(dqn_ctx* c, const uint8_t* s, const int32_t* a, const float* r, const uint8_t* s2,
                      const float* done, int B, float* loss_out)
{
    const Offsets& o = c->off;
    hipStream_t st = c->train_stream;
    Workspace& ws = c->train_ws;
    const int groups = c->cfg.double_dqn ? 3 : 2;
    const uint8_t* x[3] = {s, s2, s2};
    const void* shadow[3] = {c->sh, c->sh_t, c->sh};
    const float* master[3] = {c->theta, c->theta_t, c->theta};
    int rc = forward_to_h<T>(c, st, ws, groups, x, shadow, master, B, true);
    if (rc != DQN_OK) return rc;

    const T* sh = static_cast<const T*>(c->sh);
    const T* sh_t = static_cast<const T*>(c->sh_t);
    const T* act1 = static_cast<const T*>(ws.act1); const T* act2 = static_cast<const T*>(ws.act2);
    const T* act3 = static_cast<const T*>(ws.act3); const T* h = static_cast<const T*>(ws.h);
    T* dzh = static_cast<T*>(c->dzh); T* dz3 = static_cast<T*>(c->dz3);
    T* dz2 = static_cast<T*>(c->dz2); T* dz1 = static_cast<T*>(c->dz1);

    {
        const ProfPair pr = prof_pair(c, K_FC2_TD);
        if (pr.begin) (void)hipEventRecord(pr.begin, st);
        hipLaunchKernelGGL((fc2_td_kernel<T>), dim3((B + 3) / 4), dim3(256), 0, st, h, sh + o.wf2, sh_t + o.wf2,
                       c->theta + o.bf2, c->theta_t + o.bf2, B, c->A, c->cfg.double_dqn, a, r, done, c->cfg.gamma,
                       c->cfg.huber_delta, ws.q, c->dqv, c->lossv);
    if (pr.end) (void)hipEventRecord(pr.end, st);
        DQN_LAUNCH_CHECK();
    }
    {
        const ProfPair pr = prof_pair(c, K_TD_HEAD_BWD);
        if (pr.begin) (void)hipEventRecord(pr.begin, st);
        hipLaunchKernelGGL((td_head_bwd_kernel<T>), dim3(8), dim3(256), 0, st, h, sh + o.wf2, a, c->dqv, c->lossv, B, c->A,
                       dzh, c->grad + o.wf2, c->grad + o.bf2, loss_out, c->loss_keep);
    if (pr.end) (void)hipEventRecord(pr.end, st);
        DQN_LAUNCH_CHECK();
    }
    {   // fc1 weight gradient: dW[o][f] = sum_b dZ[b][o] act3[b][f]
        DenseM<T> al{}; DenseM<T> bl{}; EpiGrad ep{c->grad + o.wf1, 3136, 1.f};
        al.p[0] = dzh; al.ld = 512; bl.p[0] = act3; bl.ld = 3136;
        const ProfPair pr = prof_pair(c, K_FC1_WGRAD);
        DQN_HIP((launch_gemm<T, 64, 128, 32, 2>(st, al, bl, ep, 512, 3136, B, 1, 1, ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {   // fc1 data gradient through conv3's ReLU
        DenseK<T> al{}; DenseM<T> bl{}; EpiMaskDense<T> ep{dz3, act3, 3136};
        al.p[0] = dzh; al.ld = 512; bl.p[0] = sh + o.wf1; bl.ld = 3136;
        const int tiles = ((B + 31) / 32) * 25;
        const ProfPair pr = prof_pair(c, K_FC1_DGRAD);
        DQN_HIP((launch_gemm<T, 32, 128, 32, 1>(st, al, bl, ep, B, 3136, 512, 1, pick_splits(tiles, 1, 512, 32, 16),
                                                 ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {   // conv3 weight gradient
        DenseM<T> al{}; WgradB<T, 64, 9, 9, 7, 7, 3, 1> bl{act2}; EpiGrad ep{c->grad + o.w3, 576, 1.f};
        al.p[0] = dz3; al.ld = 64;
        const ProfPair pr = prof_pair(c, K_CONV3_WGRAD);
        DQN_HIP((launch_gemm<T, 64, 64, 32, 2>(st, al, bl, ep, 64, 576, B * 49, 1, pick_splits(9, 1, B * 49, 32, 512),
                                                ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {   // conv3 data gradient through conv2's ReLU
        DgradA<T, 64, 7, 7, 9, 9, 3, 1> al{dz3}; DgradB<T, 64, 64, 3, 1> bl{sh + o.w3};
        EpiDgradMask<T, 9, 9, 64, 1> ep{dz2, act2};
        const int M = B * 81, tiles = (M + 63) / 64;
        const ProfPair pr = prof_pair(c, K_CONV3_DGRAD);
        DQN_HIP((launch_gemm<T, 64, 64, 32, 2>(st, al, bl, ep, M, 64, 576, 1, pick_splits(tiles, 1, 576, 32, 8),
                                                ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {   // conv2 weight gradient
        DenseM<T> al{}; WgradB<T, 32, 20, 20, 9, 9, 4, 2> bl{act1}; EpiGrad ep{c->grad + o.w2, 512, 1.f};
        al.p[0] = dz2; al.ld = 64;
        const ProfPair pr = prof_pair(c, K_CONV2_WGRAD);
        DQN_HIP((launch_gemm<T, 64, 64, 32, 2>(st, al, bl, ep, 64, 512, B * 81, 1, pick_splits(8, 1, B * 81, 32, 512),
                                                ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {   // conv2 data gradient through conv1's ReLU: four stride-parity classes
        DgradA<T, 64, 9, 9, 20, 20, 4, 2> al{dz2}; DgradB<T, 32, 64, 4, 2> bl{sh + o.w2};
        EpiDgradMask<T, 20, 20, 32, 2> ep{dz1, act1};
        const ProfPair pr = prof_pair(c, K_CONV2_DGRAD);
        DQN_HIP((launch_gemm<T, 128, 32, 32, 4>(st, al, bl, ep, B * 100, 32, 256, 4, 1, ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {   // conv1 weight gradient (input scale 1/255 folded into the epilogue)
        DenseM<T> al{}; Conv1WgradB<T> bl{s}; EpiGrad ep{c->grad + o.w1, 256, 1.f / 255.f};
        al.p[0] = dz1; al.ld = 32;
        const ProfPair pr = prof_pair(c, K_CONV1_WGRAD);
        DQN_HIP((launch_gemm<T, 32, 128, 32, 1>(st, al, bl, ep, 32, 256, B * 400, 1, pick_splits(2, 1, B * 400, 32, 512),
                                                 ws.partial, ws.partial_cap, pr.begin, pr.end)));
    }
    {
        BiasGradArgs args;
        args.dz[0] = dz1; args.out[0] = c->grad + o.b1; args.rows[0] = B * 400; args.chans[0] = 32;
        args.dz[1] = dz2; args.out[1] = c->grad + o.b2; args.rows[1] = B * 81;  args.chans[1] = 64;
        args.dz[2] = dz3; args.out[2] = c->grad + o.b3; args.rows[2] = B * 49;  args.chans[2] = 64;
        args.dz[3] = dzh; args.out[3] = c->grad + o.bf1; args.rows[3] = B;      args.chans[3] = 512;
        args.first_block[0] = 0;
        for (int l = 0; l < 4; ++l) args.first_block[l + 1] = args.first_block[l] + args.chans[l] / 8;
        {
        const ProfPair pr = prof_pair(c, K_BIAS_GRAD);
        if (pr.begin) (void)hipEventRecord(pr.begin, st);
        hipLaunchKernelGGL((bias_grad_kernel<T>), dim3(args.first_block[4]), dim3(256), 0, st, args);
        if (pr.end) (void)hipEventRecord(pr.end, st);
        DQN_LAUNCH_CHECK();
    }
    }
    {
        const size_t n = o.total, threads = n / 4 + 4;
        {
        const ProfPair pr = prof_pair(c, K_RMSPROP);
        if (pr.begin) (void)hipEventRecord(pr.begin, st);
        hipLaunchKernelGGL((rmsprop_kernel<T, SHADOW>), dim3(static_cast<unsigned>((threads + 255) / 256)), dim3(256), 0,
                           st, c->theta, c->grad, c->v, c->m, static_cast<T*>(c->sh), n, c->cfg.lr, c->cfg.rms_alpha,
                           c->cfg.rms_eps, c->cfg.centered);
        if (pr.end) (void)hipEventRecord(pr.end, st);
        DQN_LAUNCH_CHECK();
    }
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
        DQN_HIP(hipMalloc(&c->dzh, B * 512 * c->esize));
        DQN_HIP(hipMalloc(&c->dz3, B * 3136 * c->esize));
        DQN_HIP(hipMalloc(&c->dz2, B * 5184 * c->esize));
        DQN_HIP(hipMalloc(&c->dz1, B * 12800 * c->esize));
        DQN_HIP(hipMalloc((void**)&c->dqv, B * sizeof(float)));
        DQN_HIP(hipMalloc((void**)&c->lossv, B * sizeof(float)));
        DQN_HIP(hipMalloc((void**)&c->loss_keep, sizeof(float)));
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
    if (c->cfg.precision == DQN_PRECISION_BF16 && (which == DQN_PARAMS_ONLINE || which == DQN_PARAMS_TARGET)) {
        bf16_t* sh = static_cast<bf16_t*>(which == DQN_PARAMS_ONLINE ? c->sh : c->sh_t);
        hipLaunchKernelGGL((shadow_cast_kernel<bf16_t>), dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                           c->train_stream, dst, sh, n);
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

int dqn_act(dqn_ctx* c, const uint8_t* states, int32_t W, float epsilon, uint64_t act_step, int32_t use_target,
            int32_t* actions, float* q_out)
{
    if (!c) return fail(DQN_EINVAL, "dqn_act: ctx is null");
    if (W < 1 || W > c->cfg.max_envs) return fail(DQN_EINVAL, "dqn_act: W = %d outside 1..%d", W, c->cfg.max_envs);
    if (!states || !actions) return fail(DQN_EINVAL, "dqn_act: null pointer");
    if (!aligned16(states)) return fail(DQN_EINVAL, "dqn_act: states not 16-byte aligned");
    if (!(epsilon >= 0.f && epsilon <= 1.f)) return fail(DQN_EINVAL, "dqn_act: epsilon outside [0,1]");
    if (!use_target) {
        // standard DQN: the policy needs the parameters the last update produced (Section 3)
        DQN_HIP(hipStreamWaitEvent(c->act_stream, c->ev_train, 0));
    }
    const int rc = c->cfg.precision == DQN_PRECISION_BF16
                       ? act_impl<bf16_t>(c, states, W, epsilon, act_step, use_target, actions, q_out)
                       : act_impl<float>(c, states, W, epsilon, act_step, use_target, actions, q_out);
    if (rc != DQN_OK) return rc;
    if (!use_target) {
        DQN_HIP(hipEventRecord(c->ev_act, c->act_stream));
        c->act_reads_online = true;
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
    if (c->act_reads_online) {
        // an act step that reads theta must finish before theta is overwritten
        DQN_HIP(hipStreamWaitEvent(c->train_stream, c->ev_act, 0));
        c->act_reads_online = false;
    }
    int rc;
    if (c->cfg.precision == DQN_PRECISION_BF16) rc = train_impl<bf16_t, true>(c, s, a, r, s2, done, B, loss_out);
    else rc = train_impl<float, false>(c, s, a, r, s2, done, B, loss_out);
    if (rc != DQN_OK) return rc;
    DQN_HIP(hipEventRecord(c->ev_train, c->train_stream));
    c->last_B = B;
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

int dqn_profile_select(dqn_ctx* c, int kernel_id)
{
    if (!c) return fail(DQN_EINVAL, "dqn_profile_select: ctx is null");
    if (kernel_id < 0 || kernel_id >= K_COUNT) return fail(DQN_EINVAL, "dqn_profile_select: kernel id %d", kernel_id);
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
    c->act_reads_online = false;
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
