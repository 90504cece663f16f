// The non-GEMM kernels of the act and train steps: fc2 + epsilon-greedy, fc2 + TD target / loss
// (Eq. 1), fc2 backward, bias gradients, centered RMSProp (Appendix B) with the refresh of the
// operand copies, and the target copy (theta^- <- theta).
#pragma once
#include "conv_ws.h"
#include "philox.h"

namespace dqn {

constexpr int kMaxBatch = 1024;
constexpr int kMaxActions = 32;

// Offsets of the tensors inside a parameter blob (identical for the public and the device layout).
struct Offsets {
    size_t w1, b1, w2, b2, w3, b3, wf1, bf1, wf2, bf2, total;
};
inline Offsets make_offsets(int A)
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

// Backward operand copies ("transposed shadows"), one buffer of T:
//   conv2: [4 parity classes][32 c][(p2, q2, o) = 256]   conv3: [64 c][(p, q, o) = 576]
//   fc1:   [3136 f][512 o]
constexpr size_t kBshW2 = 0, kBshW3 = 4 * 32 * 256, kBshWf1 = kBshW3 + 64 * 576;
constexpr size_t kBshTotal = kBshWf1 + static_cast<size_t>(3136) * 512;

// Where element r of conv2.w ([o][p][q][c]) / conv3.w lives in the backward copy.
__host__ __device__ inline size_t bsh_index_w2(int r)
{
    const int c = r % 32, q = (r / 32) % 4, p = (r / 128) % 4, oc = r / 512;
    const int cls = (p % 2) * 2 + (q % 2);
    return kBshW2 + ((static_cast<size_t>(cls) * 32 + c) * 4 + (p / 2) * 2 + (q / 2)) * 64 + oc;
}
__host__ __device__ inline size_t bsh_index_w3(int r)
{
    const int c = r % 64, q = (r / 64) % 3, p = (r / 192) % 3, oc = r / 576;
    return kBshW3 + (static_cast<size_t>(c) * 9 + p * 3 + q) * 64 + oc;
}

// h[b][8l .. 8l+7] for lane l: sum of the fc1 partial slices in slice order, + bias, ReLU, rounded
// to the operand type (so that forward and backward see the same h).
template <typename T>
__device__ inline typename Vec8<T>::type fc1_finish(const float* __restrict__ partial, int slices, size_t slice_stride,
                                                    const float* __restrict__ bias, int lane)
{
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const float* p = partial + lane * 8;
    for (int s = 0; s < slices; ++s) {
        const float4 lo = *reinterpret_cast<const float4*>(p + s * slice_stride);
        const float4 hi = *reinterpret_cast<const float4*>(p + s * slice_stride + 4);
        acc[0] += lo.x; acc[1] += lo.y; acc[2] += lo.z; acc[3] += lo.w;
        acc[4] += hi.x; acc[5] += hi.y; acc[6] += hi.z; acc[7] += hi.w;
    }
    const float4 blo = *reinterpret_cast<const float4*>(bias + lane * 8);
    const float4 bhi = *reinterpret_cast<const float4*>(bias + lane * 8 + 4);
    const float bv[8] = {blo.x, blo.y, blo.z, blo.w, bhi.x, bhi.y, bhi.z, bhi.w};
    typename Vec8<T>::type h;
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = from_float<T>(fmaxf(acc[e] + bv[e], 0.f));
    return h;
}

// Q[a] = b2[a] + <h, W2[a]> for all a, one wavefront: lane l owns k = 8l .. 8l+7; butterfly sums
// (fixed order).  Returns Q[a] in lane a (a < A) and -inf elsewhere.
template <typename T>
__device__ inline float fc2_row(const typename Vec8<T>::type& hv, const T* __restrict__ w2, const float* __restrict__ b2,
                                int A, int lane)
{
    typedef typename Vec8<T>::type V8;
    float mine = -INFINITY;
    for (int a0 = 0; a0 < A; a0 += 6) {
        V8 wv[6];
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            const int a = a0 + u < A ? a0 + u : A - 1;
            wv[u] = *reinterpret_cast<const V8*>(w2 + static_cast<size_t>(a) * 512 + lane * 8);
        }
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += to_float(hv[e]) * to_float(wv[u][e]);
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
            if (a0 + u < A && lane == a0 + u) mine = acc + b2[a0 + u];
        }
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

// Act step tail: finish fc1, fc2, epsilon-greedy; one wavefront per environment.
template <typename T>
__global__ __launch_bounds__(256) void fc2_act_kernel(const float* __restrict__ partial, int slices, const float* __restrict__ b1,
                                                      const T* __restrict__ w2, const float* __restrict__ b2, int W, int A,
                                                      float epsilon, uint64_t seed, uint64_t act_step,
                                                      int32_t* __restrict__ actions, float* __restrict__ q_out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = blockIdx.x * 4 + wave;
    if (j >= W) return;
    const typename Vec8<T>::type hv =
        fc1_finish<T>(partial + static_cast<size_t>(j) * 512, slices, static_cast<size_t>(W) * 512, b1, lane);
    const float q = fc2_row<T>(hv, w2, b2, A, lane);
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

// Train step head, forward half: finish fc1 and run fc2 for Q(s,.;theta), Q(s',.;theta^-) [and
// Q(s',.;theta)], then per sample the TD target, the error, its clipped gradient and its loss term.
// partial: [groups][slices][B][512].  Stores h of the online pass on s for the backward half.
template <typename T>
__global__ __launch_bounds__(256) void fc2_td_kernel(
    const float* __restrict__ partial, int slices, const float* __restrict__ b1_online, const float* __restrict__ b1_target,
    const T* __restrict__ w2_online, const T* __restrict__ w2_target, const float* __restrict__ b2_online,
    const float* __restrict__ b2_target, int B, int A, int double_dqn, const int32_t* __restrict__ act,
    const float* __restrict__ rew, const float* __restrict__ done, float gamma, float huber, T* __restrict__ h_online,
    float* __restrict__ q_all, float* __restrict__ dqv, float* __restrict__ lossv)
{
    typedef typename Vec8<T>::type V8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.x * 4 + wave;
    if (b >= B) return;
    const size_t sstride = static_cast<size_t>(B) * 512, gstride = sstride * slices;
    const V8 h0 = fc1_finish<T>(partial + static_cast<size_t>(b) * 512, slices, sstride, b1_online, lane);
    *reinterpret_cast<V8*>(h_online + static_cast<size_t>(b) * 512 + lane * 8) = h0;
    const V8 h1 = fc1_finish<T>(partial + gstride + static_cast<size_t>(b) * 512, slices, sstride, b1_target, lane);
    const float q_on = fc2_row<T>(h0, w2_online, b2_online, A, lane);
    const float q_nt = fc2_row<T>(h1, w2_target, b2_target, A, lane);
    int astar;
    if (double_dqn) {
        const V8 h2 = fc1_finish<T>(partial + 2 * gstride + static_cast<size_t>(b) * 512, slices, sstride, b1_online, lane);
        const float q_no = fc2_row<T>(h2, w2_online, b2_online, A, lane);
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
// Each block owns 64 columns o; thread (o, part) accumulates the samples b = part (mod 4) in
// increasing order into its own LDS column, the four parts are then added in order.
template <typename T>
__global__ __launch_bounds__(256) void td_head_bwd_kernel(
    const T* __restrict__ h, const T* __restrict__ w2, const int32_t* __restrict__ act,
    const float* __restrict__ dqv, const float* __restrict__ lossv, int B, int A, T* __restrict__ dzh,
    float* __restrict__ g_w2, float* __restrict__ g_b2, float* __restrict__ loss_out, float* __restrict__ loss_keep)
{
    __shared__ float s_dq[kMaxBatch];
    __shared__ int s_a[kMaxBatch];
    __shared__ float s_acc[kMaxActions][256];
    const int tid = threadIdx.x;
    for (int b = tid; b < B; b += 256) { s_dq[b] = dqv[b]; s_a[b] = act[b]; }
    for (int a = 0; a < A; ++a) s_acc[a][tid] = 0.f;
    __syncthreads();
    const int o = blockIdx.x * 64 + (tid & 63);
    const int part = tid >> 6;
    for (int b0 = part; b0 < B; b0 += 16) {
        float hv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int b = b0 + 4 * u;
            hv[u] = b < B ? to_float(h[static_cast<size_t>(b) * 512 + o]) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int b = b0 + 4 * u;
            if (b < B) {
                const int a = s_a[b];
                const float g = s_dq[b] * to_float(w2[static_cast<size_t>(a) * 512 + o]);
                dzh[static_cast<size_t>(b) * 512 + o] = hv[u] > 0.f ? from_float<T>(g) : from_float<T>(0.f);
                s_acc[a][tid] += s_dq[b] * hv[u];
            }
        }
    }
    __syncthreads();
    for (int a = part; a < A; a += 4) {
        const int oo = tid & 63;
        g_w2[static_cast<size_t>(a) * 512 + o] = ((s_acc[a][oo] + s_acc[a][64 + oo]) + s_acc[a][128 + oo]) + s_acc[a][192 + oo];
    }
    if (blockIdx.x == 0) {
        for (int a = tid; a < A; a += 256) {
            float acc = 0.f;
            for (int b = 0; b < B; ++b)
                if (s_a[b] == a) acc += s_dq[b];
            g_b2[a] = acc;
        }
        if (tid == 0) {
            float acc = 0.f;
            for (int b = 0; b < B; ++b) acc += lossv[b];
            acc /= static_cast<float>(B);
            *loss_keep = acc;
            if (loss_out) *loss_out = acc;
        }
    }
}

// Bias gradients = column sums of the four dZ matrices ([rows][C], T).  A block sums up to
// kBiasRows rows of eight channels; the block that finishes a layer last adds the per-block sums in
// block order, so the result does not depend on scheduling.
constexpr int kBiasRows = 1024;
struct BiasGradArgs {
    const void* dz[4];
    float* out[4];
    int rows[4];
    int chans[4];
    int chunks[4];
    int first_block[5];
    int first_partial[4];   // offsets into `partial` (floats)
    float* partial;
    unsigned int* tickets;  // [4], zero between launches
};
template <typename T>
__global__ __launch_bounds__(256) void bias_grad_kernel(BiasGradArgs args)
{
    typedef typename Vec8<T>::type V8;
    __shared__ float red[256][9];
    __shared__ bool is_last;
    int layer = 0;
    while (layer < 3 && static_cast<int>(blockIdx.x) >= args.first_block[layer + 1]) ++layer;
    const int local = blockIdx.x - args.first_block[layer];
    const int C = args.chans[layer], rows = args.rows[layer], cgs = C / 8, chunks = args.chunks[layer];
    const int cg = local % cgs, chunk = local / cgs;
    const T* dz = static_cast<const T*>(args.dz[layer]) + cg * 8;
    const int r_end = min(rows, (chunk + 1) * kBiasRows);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int r = chunk * kBiasRows + threadIdx.x; r < r_end; r += 256) {
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
    float* part = args.partial + args.first_partial[layer];
    if (threadIdx.x < 8) part[chunk * C + cg * 8 + threadIdx.x] = red[0][threadIdx.x];
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int t = atomicAdd(&args.tickets[layer], 1u);
        is_last = (t == static_cast<unsigned int>(cgs * chunks - 1));
    }
    __syncthreads();
    if (is_last) {
        __threadfence();
        for (int c = threadIdx.x; c < C; c += 256) {
            float sum = 0.f;
            for (int k = 0; k < chunks; ++k) sum += __hip_atomic_load(&part[k * C + c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            args.out[layer][c] = sum;
        }
        if (threadIdx.x == 0) args.tickets[layer] = 0u;
    }
}

// ---- optimiser --------------------------------------------------------------------------------

struct RmsArgs {
    float* theta;
    const float* grad;
    float* v;
    float* m;
    void* sh;        // forward operand copy (bf16 mode) or null
    void* bsh;       // backward operand copies
    Offsets off;
    float lr, alpha, eps;
    int centered;
    int flat_blocks; // blocks [0, flat_blocks) are elementwise, the rest are fc1.w tiles
};

__device__ inline void rms_update(const RmsArgs& a, float& th, float g, float& vv, float& mm)
{
    vv = a.alpha * vv + (1.f - a.alpha) * g * g;
    float var = vv;
    if (a.centered) {
        mm = a.alpha * mm + (1.f - a.alpha) * g;
        var = fmaxf(vv - mm * mm, 0.f);
    }
    th -= a.lr * g / (sqrtf(var) + a.eps);
}

template <typename T, bool SHADOW>
__device__ inline void publish(const RmsArgs& a, size_t e, float th)
{
    if (SHADOW) static_cast<T*>(a.sh)[e] = from_float<T>(th);
    if (e >= a.off.w2 && e < a.off.b2) static_cast<T*>(a.bsh)[bsh_index_w2(static_cast<int>(e - a.off.w2))] = from_float<T>(th);
    else if (e >= a.off.w3 && e < a.off.b3) static_cast<T*>(a.bsh)[bsh_index_w3(static_cast<int>(e - a.off.w3))] = from_float<T>(th);
}

// Centered RMSProp (Appendix B) fused with the refresh of the operand copies.  Elementwise blocks
// cover everything but fc1.w; fc1.w is walked in 32 x 64 tiles so that its transposed copy
// ([f][o], the operand of fc1's data gradient) is written in full 64/128-byte rows via LDS.
template <typename T, bool SHADOW>
__global__ __launch_bounds__(256) void rmsprop_kernel(RmsArgs a)
{
    __shared__ T tile[64][32 + 8];
    const int tid = threadIdx.x;
    if (static_cast<int>(blockIdx.x) < a.flat_blocks) {
        const size_t n_flat = a.off.total - static_cast<size_t>(512) * 3136;
        const size_t n4 = n_flat / 4;
        const size_t i = blockIdx.x * static_cast<size_t>(256) + tid;
        auto to_blob = [&](size_t f) { return f < a.off.wf1 ? f : f + static_cast<size_t>(512) * 3136; };
        if (i < n4) {
            const size_t e = to_blob(4 * i);
            float4 th = *reinterpret_cast<float4*>(a.theta + e);
            const float4 g = *reinterpret_cast<const float4*>(a.grad + e);
            float4 vv = *reinterpret_cast<float4*>(a.v + e);
            float4 mm = *reinterpret_cast<float4*>(a.m + e);
            rms_update(a, th.x, g.x, vv.x, mm.x);
            rms_update(a, th.y, g.y, vv.y, mm.y);
            rms_update(a, th.z, g.z, vv.z, mm.z);
            rms_update(a, th.w, g.w, vv.w, mm.w);
            *reinterpret_cast<float4*>(a.theta + e) = th;
            *reinterpret_cast<float4*>(a.v + e) = vv;
            if (a.centered) *reinterpret_cast<float4*>(a.m + e) = mm;
            publish<T, SHADOW>(a, e, th.x);
            publish<T, SHADOW>(a, e + 1, th.y);
            publish<T, SHADOW>(a, e + 2, th.z);
            publish<T, SHADOW>(a, e + 3, th.w);
        } else if (i < n4 + (n_flat - 4 * n4)) {
            const size_t e = to_blob(4 * n4 + (i - n4));
            float th = a.theta[e], vv = a.v[e], mm = a.m[e];
            rms_update(a, th, a.grad[e], vv, mm);
            a.theta[e] = th;
            a.v[e] = vv;
            if (a.centered) a.m[e] = mm;
            publish<T, SHADOW>(a, e, th);
        }
        return;
    }
    // fc1.w tile: rows o0 .. o0+31, columns f0 .. f0+63
    const int t = blockIdx.x - a.flat_blocks;
    const int o0 = (t / 49) * 32, f0 = (t % 49) * 64;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int v4 = tid + u * 256;            // 512 float4 per tile
        const int r = v4 / 16, c4 = (v4 % 16) * 4;
        const size_t e = a.off.wf1 + static_cast<size_t>(o0 + r) * 3136 + f0 + c4;
        float4 th = *reinterpret_cast<float4*>(a.theta + e);
        const float4 g = *reinterpret_cast<const float4*>(a.grad + e);
        float4 vv = *reinterpret_cast<float4*>(a.v + e);
        float4 mm = *reinterpret_cast<float4*>(a.m + e);
        rms_update(a, th.x, g.x, vv.x, mm.x);
        rms_update(a, th.y, g.y, vv.y, mm.y);
        rms_update(a, th.z, g.z, vv.z, mm.z);
        rms_update(a, th.w, g.w, vv.w, mm.w);
        *reinterpret_cast<float4*>(a.theta + e) = th;
        *reinterpret_cast<float4*>(a.v + e) = vv;
        if (a.centered) *reinterpret_cast<float4*>(a.m + e) = mm;
        if (SHADOW) store4<T>(static_cast<T*>(a.sh) + e, th.x, th.y, th.z, th.w);
        tile[c4 + 0][r] = from_float<T>(th.x);
        tile[c4 + 1][r] = from_float<T>(th.y);
        tile[c4 + 2][r] = from_float<T>(th.z);
        tile[c4 + 3][r] = from_float<T>(th.w);
    }
    __syncthreads();
    {
        typedef typename Vec8<T>::type V8;
        const int f = tid / 4, part = (tid % 4) * 8;
        const V8 val = *reinterpret_cast<const V8*>(&tile[f][part]);
        *reinterpret_cast<V8*>(static_cast<T*>(a.bsh) + kBshWf1 + static_cast<size_t>(f0 + f) * 512 + o0 + part) = val;
    }
}

// Builds every operand copy of theta from the fp32 master (after dqn_set_params).
template <typename T, bool SHADOW>
__global__ __launch_bounds__(256) void build_copies_kernel(const float* __restrict__ theta, T* __restrict__ sh,
                                                           T* __restrict__ bsh, Offsets off)
{
    const size_t e = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    if (e >= off.total) return;
    const T val = from_float<T>(theta[e]);
    if (SHADOW) sh[e] = val;
    if (bsh) {
        if (e >= off.w2 && e < off.b2) bsh[bsh_index_w2(static_cast<int>(e - off.w2))] = val;
        else if (e >= off.w3 && e < off.b3) bsh[bsh_index_w3(static_cast<int>(e - off.w3))] = val;
        else if (e >= off.wf1 && e < off.bf1) {
            const size_t r = e - off.wf1;
            bsh[kBshWf1 + (r % 3136) * 512 + r / 3136] = val;
        }
    }
}

// theta^- <- theta: fp32 master (bitwise) and, if present, the forward operand copy.
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
