// The non-GEMM kernels of the act and train steps: fc2 + epsilon-greedy, fc2 + TD target / loss
// (Eq. 1), fc2 backward, bias gradients, centered RMSProp (Appendix B) with the refresh of the
// operand copies, and the target copy (theta^- <- theta).
#pragma once
#include "common.h"
#include "conv_tower.h"
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
// In reduced precision all three are kept in MFMA fragment order (tower_frag_index over [row][k]: conv per
// (class,) [c][k], fc1 over [f][o]), the order their consumers load them in: one operand of a 32x32x16 MFMA is then
// one contiguous 1 KB row instead of 32 separate cache lines; fp32 keeps them row-major.
constexpr size_t kBshW2 = 0, kBshW3 = 4 * 32 * 256, kBshWf1 = kBshW3 + 64 * 576;
constexpr size_t kBshTotal = kBshWf1 + static_cast<size_t>(3136) * 512;

// Where element r of conv2.w ([o][p][q][c]) / conv3.w lives in the backward copy.
template <typename T> __host__ __device__ inline size_t bsh_index_w2(int r)
{
    const int c = r % 32, q = (r / 32) % 4, p = (r / 128) % 4, oc = r / 512;
    const int cls = (p % 2) * 2 + (q % 2), k = ((p / 2) * 2 + (q / 2)) * 64 + oc;
    return kBshW2 + static_cast<size_t>(cls) * 32 * 256 + (sizeof(T) == 2 ? tower_frag_index(c, k, 256) : static_cast<size_t>(c) * 256 + k);
}
template <typename T> __host__ __device__ inline size_t bsh_index_w3(int r)
{
    const int c = r % 64, q = (r / 64) % 3, p = (r / 192) % 3, oc = r / 576;
    const int k = (p * 3 + q) * 64 + oc;
    return kBshW3 + (sizeof(T) == 2 ? tower_frag_index(c, k, 576) : static_cast<size_t>(c) * 576 + k);
}

template <typename T> __host__ __device__ inline size_t bsh_index_wf1(int o, int f)
{
    return kBshWf1 + (sizeof(T) == 2 ? tower_frag_index(f, o, 512) : static_cast<size_t>(f) * 512 + o);
}

// Where blob element e lives in the 16-bit forward copy: identical, except that the conv weights and fc1's are
// kept in MFMA fragment order (of the fused conv kernel / the fc kernels).  conv1's weights are stored there as fp16 (that
// kernel runs conv1 on the f16 matrix instruction), everything else as bf16: shadow_store converts.
__host__ __device__ inline size_t shadow_index(const Offsets& off, size_t e)
{
    if (e >= off.w1 && e < off.b1) { const int r = static_cast<int>(e - off.w1); return off.w1 + tower_frag_index(r / 256, r % 256, 256); }
    if (e >= off.w2 && e < off.b2) { const int r = static_cast<int>(e - off.w2); return off.w2 + tower_frag_index(r / 512, r % 512, 512); }
    if (e >= off.w3 && e < off.b3) { const int r = static_cast<int>(e - off.w3); return off.w3 + tower_frag_index(r / 576, r % 576, 576); }
    if (e >= off.wf1 && e < off.bf1) { const int r = static_cast<int>(e - off.wf1); return off.wf1 + tower_frag_index(r / 3136, r % 3136, 3136); }
    return e;
}

template <typename T> __device__ inline void shadow_store(T* sh, const Offsets& off, size_t e, float v)
{
    if (e >= off.w1 && e < off.b1) reinterpret_cast<_Float16*>(sh)[shadow_index(off, e)] = static_cast<_Float16>(v);
    else sh[shadow_index(off, e)] = from_float<T>(v);
}

// ---- network head, forward: finish fc1, fc2 on the matrix cores, then action selection (act step)
// or TD target / error / loss (train step, Eq. 1) -------------------------------------------------
//
// fc1 arrives as k-slices of fp32 partial sums [groups][slices][rows][512].  A workgroup owns
// kHeadRows samples (few rows per workgroup: the slice sums are plain loads, and what bounds them is
// how many compute units pull at once).  (1) Thread t finishes four features of one row for every
// group -- slices added in slice order, bias, ReLU, rounded to the operand type so that forward and
// backward see the same h -- into an LDS tile; the fc2 weight fragments are requested before that,
// so both latencies overlap.  (2) Per group the four wavefronts each take a quarter of K = 512 of
// the fc2 product as 32x32 MFMAs (A = W2 rows, B = the h tile); the partial accumulators meet in LDS
// and are added in wavefront order.  (3) One thread per sample runs the tail.
constexpr int kHeadRows = 2;

struct HeadArgs {
    const float* partial;        // [groups][slices][rows][512]
    int slices, rows, A, groups;
    int head_blocks;             // workgroups of the head proper (the first ones of the grid)
    const float* b1[3];
    const void* w2[3];           // T [A][512]
    const float* b2[3];
    // act step
    float epsilon;
    uint64_t seed, act_step;
    int32_t* actions;
    float* q_out;                // [rows][A] or null
    // train step
    int double_dqn;
    const int32_t* act;
    const float* rew;
    const float* done;
    float gamma, huber;
    void* h_online;              // T [rows][512]: h of group 0, kept for the backward pass
    void* dzh;                   // T [rows][512]: dLoss/d(fc1 pre-activation) = dq_b W2[a_b][.] [h > 0]
    float* q_all;                // [groups][rows][A]
    float* dqv;
    float* lossv;
    // Train step: workgroups [head_blocks, head_blocks + 5 * gather.B) gather the NEXT minibatch from the replay memory
    // (D is constant between synchronisation points, Section 3): independent byte copies that would otherwise cost a
    // dependent launch of their own in front of every train step.  With desc_out set, the minibatch is only DESCRIBED
    // (sample_desc: replay slots per frame, a, r, done), by ceil(gather.B / 256) workgroups instead: the kernel that
    // consumes the states then reads the frames from the replay memory itself.  (Last in the struct: the act step
    // never reads it.)
    int32_t* desc_out;           // [gather.B][kDescInts] or null
    GatherPlan gather;
};

constexpr int kHeadAct = 0, kHeadTrain = 1;

// The leading scalar parameters repeat HeadArgs::partial, slices, rows, A, groups, head_blocks, w2[0], b1[0], b2[0] and
// epsilon: the kernel arguments' first 14 dwords are preloaded into scalar registers when a wavefront starts (see
// conv_tower_kernel); everything else is read from the struct.
template <typename T, int MODE>
__global__ __launch_bounds__(256) void head_fwd_kernel(const float* partial_, int slices_, int rows_, int A_, int groups_, int head_blocks_,
                                                       const void* w2_0_, const float* b1_0_, const float* b2_0_, float epsilon_, HeadArgs a)
{
    typedef typename Vec8<T>::type V8;
    constexpr int G = MODE == kHeadAct ? 1 : 3;
    constexpr int LDH = 512 + 8;
    __shared__ __attribute__((aligned(32))) T s_h[G][kHeadRows][LDH];
    __shared__ float s_red[G][4][16][64];   // fc2 partial accumulators: [group][k-quarter wavefront][slot][lane]
    __shared__ float s_dq[kHeadRows];
    if constexpr (MODE == kHeadTrain) {
        if (static_cast<int>(blockIdx.x) >= head_blocks_) {
            const int i = static_cast<int>(blockIdx.x) - head_blocks_;
            if (a.desc_out) {
                const int b = i * 256 + static_cast<int>(threadIdx.x);
                if (b < a.gather.B) sample_desc(a.gather, b, a.desc_out + static_cast<size_t>(b) * kDescInts);
            } else gather_block(a.gather, i % 5, i / 5);
            return;
        }
    }
    float h0[4] = {0.f, 0.f, 0.f, 0.f};   // this thread's four features of h (online pass on s)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row0 = blockIdx.x * kHeadRows;
    const int lr = lane & 31, kg = lane >> 5;
    const int arow = lr < A_ ? lr : A_ - 1;

    // Every global operand is requested here, before anything waits: a cold round trip to memory costs
    // over a microsecond, and the stages below would otherwise pay one each (fc2's bias, the transition's
    // reward / terminal flag / action, the taken action's row of W2).
    const int hr = tid >> 7, hf0 = (tid & 127) * 4;                 // stage (1) and the dzh epilogue: row, features
    const int hrow = row0 + hr < rows_ ? row0 + hr : rows_ - 1;
    const int trow_ = lane >> 5;                                      // tail: row of this lane
    const int trow_c = row0 + trow_ < rows_ ? row0 + trow_ : rows_ - 1;
    int act_taken = 0, act_tail = 0;
    float rew_tail = 0.f, done_tail = 0.f;
    bool act_ok = true;   // tail: the stored action of this lane's row lies in [0, A)
    if constexpr (MODE == kHeadTrain) {
        // A stored action outside [0, A) (replay_sample_gather marks a row it could not assemble with -1) must not
        // address anything: such a row gets loss 0 and gradient 0, and every index derived from it is clamped.
        act_taken = a.act[hrow];
        act_taken = static_cast<unsigned>(act_taken) < static_cast<unsigned>(A_) ? act_taken : 0;
        act_tail = a.act[trow_c];
        act_ok = static_cast<unsigned>(act_tail) < static_cast<unsigned>(A_);
        act_tail = act_ok ? act_tail : 0;
        rew_tail = a.rew[trow_c];
        done_tail = a.done[trow_c];
    }
    Philox4 draw{};   // act step: the exploration draw of this lane's row
    float b2_tail[G];   // fc2 bias of this lane's action in the tail (which reads its Q values straight from the partials)
#pragma unroll
    for (int g = 0; g < G; ++g) b2_tail[g] = (g == 0 || g >= groups_ ? b2_0_ : a.b2[g])[(lane & 31) < A_ ? (lane & 31) : A_ - 1];   // never skipped
    __builtin_amdgcn_sched_barrier(0);
    // fc2 weight fragments of every group: consumed last
    V8 wf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
        if (g < groups_) {
            const T* wp = static_cast<const T*>(g == 0 ? w2_0_ : a.w2[g]) + static_cast<size_t>(arow) * 512 + wave * 128 + kg * 8;
#pragma unroll
            for (int s = 0; s < 8; ++s) wf[g][s] = *reinterpret_cast<const V8*>(wp + s * 16);
        }

    float4 b1v[G];
#pragma unroll
    for (int g = 0; g < G; ++g)
        if (g < groups_) b1v[g] = *reinterpret_cast<const float4*>((g == 0 ? b1_0_ : a.b1[g]) + hf0);
    float4 w2row = make_float4(0.f, 0.f, 0.f, 0.f);   // train step: the taken action's row of W2 at this thread's features
    __builtin_amdgcn_sched_barrier(0);

    // (1) finish fc1: thread -> (row r = tid / 128, features 4 * (tid % 128) .. + 3).  The slices of ALL groups are
    // requested before any is added (group by group, each group's sum waited for its own round trip), from a clamped
    // row (no load is ever skipped); what depends on an earlier load (the taken action's row of W2) or on nothing
    // (the exploration draw) follows the requests and is covered by their latency.
    {
        const int r = hr, f0 = hf0;
        const int row = row0 + r;
        const size_t sstride = static_cast<size_t>(rows_) * 512, gstride = sstride * slices_;
        const float* p0 = partial_ + static_cast<size_t>(hrow) * 512 + f0;
        float4 acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s0 = 0; s0 < slices_; s0 += 7) {
            float4 v[G][7];
#pragma unroll
            for (int g = 0; g < G; ++g)
                if (g < groups_) {
#pragma unroll
                    for (int u = 0; u < 7; ++u) {
                        const int sl = s0 + u < slices_ ? s0 + u : slices_ - 1;
                        v[g][u] = *reinterpret_cast<const float4*>(p0 + g * gstride + sl * sstride);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
            if (s0 == 0) {
                if constexpr (MODE == kHeadTrain) {
                    float w[4];
                    load4<T>(static_cast<const T*>(w2_0_) + static_cast<size_t>(act_taken) * 512 + hf0, w);
                    w2row = make_float4(w[0], w[1], w[2], w[3]);
                } else {
                    draw = philox_draw(a.seed, kTagAct, a.act_step, static_cast<uint32_t>(row0 + trow_));
                    // computed HERE, under the slices' latency (left alone, the compiler moves the ten rounds into the
                    // tail, where only lane 0 of a row uses them and nothing hides them)
                    asm volatile("" :: "v"(draw.x[0]), "v"(draw.x[1]));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < G; ++g)
                if (g < groups_) {
#pragma unroll
                    for (int u = 0; u < 7; ++u)
                        if (s0 + u < slices_) { acc[g].x += v[g][u].x; acc[g].y += v[g][u].y; acc[g].z += v[g][u].z; acc[g].w += v[g][u].w; }
                }
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
            if (g < groups_) {
                const float4 bv = b1v[g];
                const float4 hv = make_float4(fmaxf(acc[g].x + bv.x, 0.f), fmaxf(acc[g].y + bv.y, 0.f), fmaxf(acc[g].z + bv.z, 0.f),
                                              fmaxf(acc[g].w + bv.w, 0.f));
                store4<T>(&s_h[g][r][f0], hv.x, hv.y, hv.z, hv.w);   // a row past the batch repeats the last one; nobody reads its Q
                if (MODE == kHeadTrain && g == 0) {
                    h0[0] = hv.x; h0[1] = hv.y; h0[2] = hv.z; h0[3] = hv.w;
                    if (row < rows_)
                        store4<T>(static_cast<T*>(a.h_online) + static_cast<size_t>(row) * 512 + f0, hv.x, hv.y, hv.z, hv.w);
                }
            }
    }
    __syncthreads();
    // (2) fc2 per group: every wavefront's k-quarter of the accumulator goes to LDS, one barrier for all groups
#pragma unroll
    for (int g = 0; g < G; ++g)
        if (g < groups_) {
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                V8 hf = vec8_zero<T>();
                if (lr < kHeadRows) hf = *reinterpret_cast<const V8*>(&s_h[g][lr][wave * 128 + s * 16 + kg * 8]);
                mma_32x32x16(acc, wf[g][s], hf);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) s_red[g][wave][v][lane] = acc[v];
        }
    __syncthreads();

    // Tail: wavefront 0, 32 lanes per row (kHeadRows = 2), lane k owns action k.  argmax with the lowest index
    // among equal values (the tie rule of the greedy policy, Section 2.1), as a butterfly over the 32 lanes.
    static_assert(kHeadRows == 2 && kMaxActions <= 32, "tail layout: one wavefront, 32 lanes per row");
    // "Better" is a total order on (value, index), so the pairs may meet in any tree: inside a row of sixteen lanes through
    // the lane-permuting moves of the vector unit (neighbours, pairs, mirrored halves of eight, mirrored sixteen -- a few
    // cycles each), across the two sixteens through one cross-lane exchange (ten of those in a row were 0.6 us of a 3 us kernel).
    auto argmax_lowest = [&](float v, int k) {   // lanes 0 .. 15 of the row return the winner
        int best = k;
        auto meet = [&](float ov, int ob) {
            if (ov > v || (ov == v && ob < best)) { v = ov; best = ob; }
        };
#define DQN_ARGMAX_DPP(ctrl)                                                                                              \
        meet(__builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xF, 0xF, false)), \
             __builtin_amdgcn_update_dpp(0, best, ctrl, 0xF, 0xF, false))
        DQN_ARGMAX_DPP(0xB1);    // quad_perm [1, 0, 3, 2]: lane ^ 1
        DQN_ARGMAX_DPP(0x4E);    // quad_perm [2, 3, 0, 1]: lane ^ 2
        DQN_ARGMAX_DPP(0x141);   // row_half_mirror: lane i of eight <-> 7 - i (the other quad)
        DQN_ARGMAX_DPP(0x140);   // row_mirror: lane i of sixteen <-> 15 - i (the other eight)
#undef DQN_ARGMAX_DPP
        // the other sixteen of the row: its result is read from its first lane (16, or 48 for the second row) -- a scalar
        // broadcast, where a cross-lane exchange costs ten times as much.  Only the FIRST sixteen lanes of a row end up with
        // the row's winner; the callers use lane 0 of the row.
        const int hv = lane < 32 ? __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16) : __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48);
        const int hb = lane < 32 ? __builtin_amdgcn_readlane(best, 16) : __builtin_amdgcn_readlane(best, 48);
        meet(__builtin_bit_cast(float, hv), hb);
        return best;
    };
    const int trow = lane >> 5, tk = lane & 31;    // tail row / action of this lane (wavefront 0 only)
    const float kNegInf = -__builtin_huge_valf();
    // Q_g(row trow, action tk): accumulator layout is sample lane % 32, action 8*(v/4) + 4*(lane/32) + (v%4); the four
    // k-quarter partials of that slot are added in wavefront order, then the bias
    const int tkc = tk < A_ ? tk : A_ - 1;
    const int qslot = 4 * (tkc >> 3) + (tkc & 3), qsrc = ((tkc >> 2) & 1) * 32 + trow;
    auto q_of = [&](int g) {
        return (((s_red[g][0][qslot][qsrc] + s_red[g][1][qslot][qsrc]) + s_red[g][2][qslot][qsrc]) + s_red[g][3][qslot][qsrc]) + b2_tail[g];
    };
    if constexpr (MODE == kHeadAct) {
        if (wave != 0) return;
        const int row = row0 + trow;
        const float qv = tk < A_ ? q_of(0) : kNegInf;
        int act = argmax_lowest(qv, tk);
        if (row >= rows_) return;
        if (a.q_out && tk < A_) a.q_out[static_cast<size_t>(row) * A_ + tk] = qv;
        if (tk == 0) {
            const Philox4 d = draw;
            const float u = static_cast<float>(d.x[0] >> 8) * 0x1p-24f;
            if (u < epsilon_) act = static_cast<int>((static_cast<uint64_t>(d.x[1]) * static_cast<uint32_t>(A_)) >> 32);
            a.actions[row] = act;
        }
    } else {
        if (wave == 0) {
            const int row = row0 + trow;
            const bool live = row < rows_;
            const float q0 = q_of(0), q1 = q_of(1);
            const float q2 = groups_ > 2 ? q_of(G - 1) : 0.f;   // Double DQN: Q(s', .; theta) selects the action
            const float qt = tk < A_ ? q1 : kNegInf;
            const float qsel = a.double_dqn ? (tk < A_ ? q2 : kNegInf) : qt;
            const int astar = argmax_lowest(qsel, tk);
            if (live && tk < A_) {
                a.q_all[(static_cast<size_t>(0) * rows_ + row) * A_ + tk] = q0;
                a.q_all[(static_cast<size_t>(1) * rows_ + row) * A_ + tk] = q1;
                if (groups_ > 2) a.q_all[(static_cast<size_t>(2) * rows_ + row) * A_ + tk] = q2;
            }
            // the two values the TD error needs sit in other lanes of this row: Q(s', a*; theta^-) and Q(s, a_b; theta)
            const float q1_star = __shfl(q1, astar, 32), q0_taken = __shfl(q0, act_tail, 32);
            if (tk == 0) {
                float dq = 0.f;
                int act_b = 0;
                if (live && !act_ok) { a.lossv[row] = 0.f; a.dqv[row] = 0.f; }
                if (live && act_ok) {
                    const float y = rew_tail + a.gamma * (1.f - done_tail) * q1_star;
                    act_b = act_tail;
                    const float delta = q0_taken - y;
                    const float ad = fabsf(delta);
                    a.lossv[row] = ad <= a.huber ? 0.5f * delta * delta : a.huber * (ad - 0.5f * a.huber);
                    dq = fminf(fmaxf(delta, -a.huber), a.huber) / static_cast<float>(rows_);
                    a.dqv[row] = dq;
                }
                s_dq[trow] = dq;
            }
        }
        __syncthreads();
        // fc2's data gradient through fc1's ReLU for this workgroup's rows: dQ has one non-zero per row
        const int r = tid >> 7, f0 = (tid & 127) * 4;
        const int row = row0 + r;
        if (row < rows_) {
            const float w[4] = {w2row.x, w2row.y, w2row.z, w2row.w};
            const float dq = s_dq[r];
            store4<T>(static_cast<T*>(a.dzh) + static_cast<size_t>(row) * 512 + f0, h0[0] > 0.f ? dq * w[0] : 0.f,
                      h0[1] > 0.f ? dq * w[1] : 0.f, h0[2] > 0.f ? dq * w[2] : 0.f, h0[3] > 0.f ? dq * w[3] : 0.f);
        }
    }
}

// Small reductions of the backward pass, one launch:
//  * blocks [0, first_block[4]): bias gradients = column sums of the four dZ matrices ([rows][C], T),
//    first stage: a block sums up to kBiasRows rows (all channels) into partial[layer][chunk][C];
//    the optimiser kernel adds the chunks in order, so no atomics and no extra launch are needed;
//  * the last 33 blocks: fc2's weight gradient (32 blocks of 16 columns) and its bias gradient + loss.  dQ has one non-zero per row (the taken action):
//    dW2[a][o] = sum_{b: a_b = a} dq_b h[b][o];  db2[a] = sum_{b: a_b = a} dq_b;  loss = mean_b loss_b.
//    Each block owns 16 columns o; thread (o, part) accumulates the samples b = part (mod 16) in
//    increasing order into its own LDS column, the sixteen parts are then added in order.
constexpr int kBiasRows = 1024;
constexpr int kRmsConvLanes = 8;                                    // lanes per float4 of a conv weight in the optimiser's conv blocks
constexpr int kRmsConvQuads = (32 * 256 + 64 * 512 + 64 * 576) / 4;
constexpr int kRmsConvBlocks = (kRmsConvQuads * kRmsConvLanes + 255) / 256;
constexpr int kRmsBiasLanes = 8;                                    // lanes per channel in the optimiser's bias blocks
constexpr int kRmsBiasBlocks = (672 * kRmsBiasLanes + 255) / 256;  // 32 + 64 + 64 + 512 hidden-layer bias channels
struct BiasGradArgs {
    const void* dz[4];
    int rows[4];
    int chans[4];
    int chunks[4];
    int chunk_rows[4];      // rows per chunk (a workgroup sums one chunk of one layer)
    int first_block[5];
    int first_partial[4];   // offsets into `partial` (floats)
    float* partial;
    // fc2 weight gradient
    const void* h;          // T [B][512]
    const int32_t* act;
    const float* dqv;
    const float* lossv;
    int B, A;
    float* g_w2;
    float* g_b2;
    float* loss_out;
    float* loss_keep;
};
constexpr size_t kSmallGradsSmem = (256 * 9 + kMaxBatch) * sizeof(float) + kMaxBatch * sizeof(int) + kMaxActions * 256 * sizeof(float);
constexpr int kSmallGradsExtraBlocks = 33;   // fc2 weight gradient (32) + fc2 bias gradient / loss (1)

// One workgroup of the small reductions; `block` counts from the first bias block, smem holds
// kSmallGradsSmem bytes.
template <typename T>
__device__ inline void small_grads_block(const BiasGradArgs& args, int block, unsigned char* smem)
{
    typedef typename Vec8<T>::type V8;
    float (*red)[9] = reinterpret_cast<float (*)[9]>(smem);
    float* s_dq = reinterpret_cast<float*>(smem) + 256 * 9;
    int* s_a = reinterpret_cast<int*>(s_dq + kMaxBatch);
    float (*s_acc)[256] = reinterpret_cast<float (*)[256]>(s_a + kMaxBatch);
    const int tid = threadIdx.x;
    if (block >= args.first_block[4]) {
        const int B = args.B, A = args.A;
        const T* h = static_cast<const T*>(args.h);
        float* s_loss = &red[0][0];   // 256 * 9 floats: room for kMaxBatch loss terms
        for (int b = tid; b < B; b += 256) {
            // a row whose stored action lies outside [0, A) has dq = 0 (head kernel); its index must still not leave s_acc
            const int ab = args.act[b];
            const bool ok = static_cast<unsigned>(ab) < static_cast<unsigned>(A);
            s_dq[b] = ok ? args.dqv[b] : 0.f; s_a[b] = ok ? ab : 0; s_loss[b] = args.lossv[b];
        }
        for (int a = 0; a < A; ++a) s_acc[a][tid] = 0.f;
        __syncthreads();
        // 16 columns per block; thread (o, part): samples b = part (mod 16) in increasing order.
        // Block 32 is the bias "column" (h = 1) and also owns the batch-mean loss.
        const int ob = block - args.first_block[4];
        const int oo = tid & 15, part = tid >> 4;
        const bool bias_block = ob == 32;
        const int o = ob * 16 + oo;
        // sixteen samples in flight per thread (clamped address: no load is ever skipped)
        const size_t oc = bias_block ? 0 : o;
        for (int b0 = part; b0 < B; b0 += 256) {
            T hv[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int b = b0 + 16 * u;
                hv[u] = h[static_cast<size_t>(b < B ? b : B - 1) * 512 + oc];
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int b = b0 + 16 * u;
                if (b < B) s_acc[s_a[b]][tid] += s_dq[b] * (bias_block ? 1.f : to_float(hv[u]));
            }
        }
        __syncthreads();
        for (int a = part; a < A; a += 16) {
            float sum = 0.f;
#pragma unroll
            for (int p = 0; p < 16; ++p) sum += s_acc[a][p * 16 + oo];
            if (!bias_block) args.g_w2[static_cast<size_t>(a) * 512 + o] = sum;
            else if (oo == 0) args.g_b2[a] = sum;
        }
        if (bias_block) {
            // loss = (1/B) sum_b loss_b: thread t adds b = t, t+256, .. then a fixed binary tree
            __syncthreads();
            float acc = 0.f;
            for (int b = tid; b < B; b += 256) acc += s_loss[b];
            __syncthreads();
            s_loss[tid] = acc;
            __syncthreads();
            for (int stride = 128; stride >= 1; stride >>= 1) {
                if (tid < stride) s_loss[tid] += s_loss[tid + stride];
                __syncthreads();
            }
            if (tid == 0) {
                const float mean = s_loss[0] / static_cast<float>(B);
                *args.loss_keep = mean;
                if (args.loss_out) *args.loss_out = mean;
            }
        }
        return;
    }
    // column sums of one chunk of rows, all channels: thread -> (16-byte vector of the row, row mod RP), so a
    // pass of the workgroup reads RP whole rows, fully coalesced; the RP partial rows meet in LDS in row order
    int layer = 0;
    while (layer < 3 && block >= args.first_block[layer + 1]) ++layer;
    const int chunk = block - args.first_block[layer];
    const int C = args.chans[layer], rows = args.rows[layer], VR = C / 8, RP = 256 / VR;
    const int vec = tid % VR, rsub = tid / VR;
    const T* dz = static_cast<const T*>(args.dz[layer]) + vec * 8;
    const int crows = args.chunk_rows[layer];
    const int r_end = min(rows, (chunk + 1) * crows);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    // sixteen rows in flight per thread (clamped address, masked value: no load is ever skipped)
    for (int r = chunk * crows + rsub; r < r_end; r += 16 * RP) {
        V8 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int rr = r + u * RP;
            v[u] = vec8_keep<T>(*reinterpret_cast<const V8*>(dz + static_cast<size_t>(rr < r_end ? rr : r_end - 1) * C), rr < r_end);
        }
#pragma unroll
        for (int u = 0; u < 16; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += to_float(v[u][e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[tid][e] = acc[e];
    __syncthreads();
    // RP partial rows per channel, added in row order; four lanes per channel take every fourth partial
    // and meet in a fixed tree (RP is 64, 32 or 4)
    for (int i = tid; i < 4 * C; i += 256) {
        const int c = i >> 2, j = i & 3;
        float sum = 0.f;
        for (int q = j; q < RP; q += 4) sum += red[q * VR + (c >> 3)][c & 7];
        sum += __shfl_down(sum, 2, 4);
        sum += __shfl_down(sum, 1, 4);
        if (j == 0) args.partial[args.first_partial[layer] + chunk * C + c] = sum;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void bias_grad_kernel(BiasGradArgs args)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char sg_smem[];
    small_grads_block<T>(args, static_cast<int>(blockIdx.x), sg_smem);
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
    int flat_blocks; // after the kRmsConvBlocks conv-weight blocks: [0, flat_blocks) elementwise, then fc1_tiles fc1.w tiles, then the bias blocks
    int fc1_tiles;   // 16 * 49 (32 x 64 tiles of fc1.w)
    // second stage of the bias gradients (conv1..3, fc1): chunk sums written by bias_grad_kernel
    const float* bias_partial;
    int bias_chunks[4];
    int bias_first[4];
    // deferred split-K sums of the conv weight gradients: [splits][tensor] fp32 each
    const float* wg_partial[3];
    int wg_splits[3];
    float wg_scale[3];
};

// Index of the hidden-layer bias vector that blob element e belongs to, or -1.
__device__ inline int hidden_bias_layer(const Offsets& o, size_t e)
{
    if (e >= o.b1 && e < o.w2) return 0;
    if (e >= o.b2 && e < o.w3) return 1;
    if (e >= o.b3 && e < o.wf1) return 2;
    if (e >= o.bf1 && e < o.wf2) return 3;
    return -1;
}

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
    if (SHADOW) shadow_store<T>(static_cast<T*>(a.sh), a.off, e, th);
    if (e >= a.off.w2 && e < a.off.b2) static_cast<T*>(a.bsh)[bsh_index_w2<T>(static_cast<int>(e - a.off.w2))] = from_float<T>(th);
    else if (e >= a.off.w3 && e < a.off.b3) static_cast<T*>(a.bsh)[bsh_index_w3<T>(static_cast<int>(e - a.off.w3))] = from_float<T>(th);
}

// Centered RMSProp (Appendix B) fused with the refresh of the operand copies.  The conv weights come first
// (their gradient is finished here from split-K slices), elementwise blocks cover the rest except fc1.w and the
// hidden-layer biases; fc1.w is walked in 32 x 64 tiles whose two 16-bit copies (forward [o][f] and backward
// [f][o], both in fragment order; fp32: the row-major [f][o] copy) are written in whole 512-byte pieces via LDS.
// The leading scalar parameters repeat RmsArgs::theta, grad, v, m, flat_blocks, fc1_tiles and off.wf1 (what the fc1.w
// tiles, 95 % of the parameters, need before their first load): the kernel arguments' first 14 dwords are preloaded into
// scalar registers when a wavefront starts (see conv_tower_kernel).
template <typename T, bool SHADOW>
__global__ __launch_bounds__(256) void rmsprop_kernel(float* theta_, const float* grad_, float* v_, float* m_, int flat_blocks_,
                                                      int fc1_tiles_, size_t wf1_, RmsArgs a)
{
    __shared__ T tile[64][32 + 8];
    const int tid = threadIdx.x;
    if (static_cast<int>(blockIdx.x) < kRmsConvBlocks) {
        // Conv weights: their gradient arrives as split-K slices (up to 128 of them at small batches).  Eight adjacent
        // lanes share four weights: lane j requests slices j, j + 8, ... (eight per round trip) and adds them in that order, the
        // eight sums meet in a fixed tree, lane 0 updates.  (One lane walking all slices, eight loads at a time, was a
        // chain of dependent round trips that outlasted the streaming of every other parameter.)
        const int idx = blockIdx.x * 256 + tid;
        const int q = idx / kRmsConvLanes, j = idx % kRmsConvLanes;
        if (q >= kRmsConvQuads) return;   // whole lane groups leave together
        int conv = 2;
        size_t r = static_cast<size_t>(q - (32 * 256 + 64 * 512) / 4) * 4, tsize = 64 * 576, e = a.off.w3 + r;
        if (q < 32 * 256 / 4) { conv = 0; r = static_cast<size_t>(q) * 4; tsize = 32 * 256; e = a.off.w1 + r; }
        else if (q < (32 * 256 + 64 * 512) / 4) { conv = 1; r = static_cast<size_t>(q - 32 * 256 / 4) * 4; tsize = 64 * 512; e = a.off.w2 + r; }
        const float* p = a.wg_partial[conv] + r;
        const int ns = a.wg_splits[conv];
        float4 th = make_float4(0.f, 0.f, 0.f, 0.f), vv = th, mm = th;
        if (j == 0) {
            th = *reinterpret_cast<float4*>(theta_ + e);
            vv = *reinterpret_cast<float4*>(v_ + e);
            mm = *reinterpret_cast<float4*>(m_ + e);
        }
        constexpr int kPerLane = 8;       // slices per lane and round trip: one trip up to 64 slices, two up to 128
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s0 = j; s0 < ns; s0 += kPerLane * kRmsConvLanes) {
            float4 v4[kPerLane];
#pragma unroll
            for (int u = 0; u < kPerLane; ++u) {
                const int sl = s0 + u * kRmsConvLanes;
                v4[u] = *reinterpret_cast<const float4*>(p + static_cast<size_t>(sl < ns ? sl : ns - 1) * tsize);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < kPerLane; ++u)
                if (s0 + u * kRmsConvLanes < ns) { sum.x += v4[u].x; sum.y += v4[u].y; sum.z += v4[u].z; sum.w += v4[u].w; }
        }
#pragma unroll
        for (int d = kRmsConvLanes / 2; d >= 1; d >>= 1) {
            sum.x += __shfl_down(sum.x, d, kRmsConvLanes); sum.y += __shfl_down(sum.y, d, kRmsConvLanes);
            sum.z += __shfl_down(sum.z, d, kRmsConvLanes); sum.w += __shfl_down(sum.w, d, kRmsConvLanes);
        }
        if (j != 0) return;
        const float sc = a.wg_scale[conv];
        const float4 g = make_float4(sum.x * sc, sum.y * sc, sum.z * sc, sum.w * sc);
        *reinterpret_cast<float4*>(const_cast<float*>(grad_) + e) = g;   // kept for readers of the gradient
        rms_update(a, th.x, g.x, vv.x, mm.x);
        rms_update(a, th.y, g.y, vv.y, mm.y);
        rms_update(a, th.z, g.z, vv.z, mm.z);
        rms_update(a, th.w, g.w, vv.w, mm.w);
        *reinterpret_cast<float4*>(theta_ + e) = th;
        *reinterpret_cast<float4*>(v_ + e) = vv;
        if (a.centered) *reinterpret_cast<float4*>(m_ + e) = mm;
        publish<T, SHADOW>(a, e, th.x);
        publish<T, SHADOW>(a, e + 1, th.y);
        publish<T, SHADOW>(a, e + 2, th.z);
        publish<T, SHADOW>(a, e + 3, th.w);
        return;
    }
    const int block = static_cast<int>(blockIdx.x) - kRmsConvBlocks;
    if (block < flat_blocks_) {
        const size_t n_flat = a.off.total - static_cast<size_t>(512) * 3136;
        const size_t n4 = n_flat / 4;
        const size_t i = block * static_cast<size_t>(256) + tid;
        auto to_blob = [&](size_t f) { return f < wf1_ ? f : f + static_cast<size_t>(512) * 3136; };
        if (i < n4) {
            const size_t e = to_blob(4 * i);
            if (hidden_bias_layer(a.off, e) >= 0) return;   // bias vectors are 4-aligned: handled by the bias blocks
            if (e < a.off.b1 || (e >= a.off.w2 && e < a.off.b2) || (e >= a.off.w3 && e < a.off.b3)) return;   // conv weights: the blocks above
            float4 th = *reinterpret_cast<float4*>(theta_ + e);
            const float4 g = *reinterpret_cast<const float4*>(grad_ + e);
            float4 vv = *reinterpret_cast<float4*>(v_ + e);
            float4 mm = *reinterpret_cast<float4*>(m_ + e);
            rms_update(a, th.x, g.x, vv.x, mm.x);
            rms_update(a, th.y, g.y, vv.y, mm.y);
            rms_update(a, th.z, g.z, vv.z, mm.z);
            rms_update(a, th.w, g.w, vv.w, mm.w);
            *reinterpret_cast<float4*>(theta_ + e) = th;
            *reinterpret_cast<float4*>(v_ + e) = vv;
            if (a.centered) *reinterpret_cast<float4*>(m_ + e) = mm;
            publish<T, SHADOW>(a, e, th.x);
            publish<T, SHADOW>(a, e + 1, th.y);
            publish<T, SHADOW>(a, e + 2, th.z);
            publish<T, SHADOW>(a, e + 3, th.w);
        } else if (i < n4 + (n_flat - 4 * n4)) {
            const size_t e = to_blob(4 * n4 + (i - n4));
            float th = theta_[e], vv = v_[e], mm = m_[e];
            rms_update(a, th, grad_[e], vv, mm);
            theta_[e] = th;
            v_[e] = vv;
            if (a.centered) m_[e] = mm;
            publish<T, SHADOW>(a, e, th);
        }
        return;
    }
    if (block >= flat_blocks_ + fc1_tiles_) {
        // hidden-layer biases: finish the gradient, then update.  Eight adjacent lanes share a channel: lane j
        // adds chunks j, j + 8, ... in order, then the eight sums meet in a fixed tree -- a large batch has
        // hundreds of chunks and one lane walking them alone was the tail of this kernel.
        const int idx = (block - flat_blocks_ - fc1_tiles_) * 256 + tid;
        const int ch = idx / kRmsBiasLanes, j = idx % kRmsBiasLanes;
        const bool live = ch < 32 + 64 + 64 + 512;
        int layer = 3, c = 0;
        size_t e = 0;
        if (ch < 32) { layer = 0; c = ch; e = a.off.b1 + c; }
        else if (ch < 96) { layer = 1; c = ch - 32; e = a.off.b2 + c; }
        else if (ch < 160) { layer = 2; c = ch - 96; e = a.off.b3 + c; }
        else if (live) { layer = 3; c = ch - 160; e = a.off.bf1 + c; }
        const int C = layer == 0 ? 32 : (layer == 3 ? 512 : 64);
        const float* part = a.bias_partial + a.bias_first[layer] + c;
        float g = 0.f;
        if (live)
            for (int k = j; k < a.bias_chunks[layer]; k += kRmsBiasLanes) g += part[k * C];
        g += __shfl_down(g, 4, kRmsBiasLanes);
        g += __shfl_down(g, 2, kRmsBiasLanes);
        g += __shfl_down(g, 1, kRmsBiasLanes);
        if (!live || j != 0) return;
        const_cast<float*>(grad_)[e] = g;
        float th = theta_[e], vv = v_[e], mm = m_[e];
        rms_update(a, th, g, vv, mm);
        theta_[e] = th;
        v_[e] = vv;
        if (a.centered) m_[e] = mm;
        if (SHADOW) static_cast<T*>(a.sh)[e] = from_float<T>(th);
        return;
    }
    // fc1.w tile: rows o0 .. o0+31, columns f0 .. f0+63
    const int t = block - flat_blocks_;
    const int o0 = (t / 49) * 32, f0 = (t % 49) * 64;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int v4 = tid + u * 256;            // 512 float4 per tile
        const int r = v4 / 16, c4 = (v4 % 16) * 4;
        const size_t e = wf1_ + static_cast<size_t>(o0 + r) * 3136 + f0 + c4;
        float4 th = *reinterpret_cast<float4*>(theta_ + e);
        const float4 g = *reinterpret_cast<const float4*>(grad_ + e);
        float4 vv = *reinterpret_cast<float4*>(v_ + e);
        float4 mm = *reinterpret_cast<float4*>(m_ + e);
        rms_update(a, th.x, g.x, vv.x, mm.x);
        rms_update(a, th.y, g.y, vv.y, mm.y);
        rms_update(a, th.z, g.z, vv.z, mm.z);
        rms_update(a, th.w, g.w, vv.w, mm.w);
        *reinterpret_cast<float4*>(theta_ + e) = th;
        *reinterpret_cast<float4*>(v_ + e) = vv;
        if (a.centered) *reinterpret_cast<float4*>(m_ + e) = mm;
        tile[c4 + 0][r] = from_float<T>(th.x);
        tile[c4 + 1][r] = from_float<T>(th.y);
        tile[c4 + 2][r] = from_float<T>(th.z);
        tile[c4 + 3][r] = from_float<T>(th.w);
    }
    __syncthreads();
    typedef typename Vec8<T>::type V8;
    if constexpr (sizeof(T) == 2) {
        // Both 16-bit copies of the tile in fragment order: a copy's eight (32 rows x 8 k) pieces are 512 contiguous
        // bytes each, one piece per 32 threads.
        const int piece = tid >> 5, rr = tid & 31;
        {   // backward copy, rows = f (two 32-row tiles), k = o
            const int ft = piece >> 2, k8 = (piece & 3) * 8;
            const V8 val = *reinterpret_cast<const V8*>(&tile[ft * 32 + rr][k8]);
            *reinterpret_cast<V8*>(static_cast<T*>(a.bsh) + bsh_index_wf1<T>(o0 + k8, f0 + ft * 32 + rr)) = val;
        }
        if (SHADOW) {   // forward copy, rows = o, k = f
            const int k8 = piece * 8;
            V8 val;
#pragma unroll
            for (int j = 0; j < 8; ++j) val[j] = tile[k8 + j][rr];
            *reinterpret_cast<V8*>(static_cast<T*>(a.sh) + wf1_ + tower_frag_index(o0 + rr, f0 + k8, 3136)) = val;
        }
    } else {
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
    if (SHADOW) shadow_store<T>(sh, off, e, theta[e]);
    if (bsh) {
        if (e >= off.w2 && e < off.b2) bsh[bsh_index_w2<T>(static_cast<int>(e - off.w2))] = val;
        else if (e >= off.w3 && e < off.b3) bsh[bsh_index_w3<T>(static_cast<int>(e - off.w3))] = val;
        else if (e >= off.wf1 && e < off.bf1) {
            const size_t r = e - off.wf1;
            bsh[bsh_index_wf1<T>(static_cast<int>(r / 3136), static_cast<int>(r % 3136))] = val;
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
