// Fused conv1 -> conv2 -> conv3 of the Q-network (Section 5: the Nature-DQN layers), reduced-precision
// mode: a persistent workgroup of 8 wavefronts (two per SIMD) walks a contiguous range of (group, sample)
// items; the activations of conv1 and conv2 never leave LDS, and every weight is fetched once per
// workgroup and group.
//
// Why it looks like this (all of it measured on the device):
//   * one sample is far too little work to hide memory latency, and MFMA operand fragments gathered
//     straight from [o][k] weight rows or from the strided uint8 state are one cache line per lane -- the
//     address unit, not the matrix core, sets the time.  So the weight copies this kernel reads are stored
//     in *fragment order*: the 64 x 16-byte operand of one 32x32x16 MFMA is one contiguous 1 KB row,
//     fetched with one fully coalesced load (tower_frag_index below; the optimizer kernel writes it), and
//     the 28 KB uint8 state is fetched with 16-byte loads, one item ahead, and staged in LDS.
//   * a single wavefront issues one 32x32x16 MFMA per 32 cycles at best (the matrix core could take one
//     every 16), pays about 13 issue cycles per MFMA plus 4 per other instruction, and is served at most
//     one LDS fragment per ~40 cycles: two wavefronts per SIMD are needed to keep either unit busy.  That
//     leaves 256 registers per wavefront, so the wavefronts hold *disjoint* parts of conv2's and conv3's
//     weights -- wavefront (nt, kq) owns channel tile nt and k-quarter kq, 32 + 36 VGPRs -- and conv1's
//     16 KB, which every wavefront needs in full, stay in LDS.
//   * within a phase every wavefront runs a hand-pipelined stream of k-steps: the LDS reads of step s + D
//     are issued before the MFMA of step s, pinned in program order.
//
// conv1 runs on the f16 MFMA: a pixel byte x, zero-extended to 16 bits, *is* the fp16 subnormal x * 2^-24,
// which the matrix core takes without flushing; no integer-to-float conversion is needed (the VALU would
// otherwise be the bottleneck of conv1), the products are exact, and the factor 2^24 / 255 is applied to
// the fp32 accumulator.  conv1's weight copy is therefore fp16, the other two are bf16.
//
// Work split per sample (wavefront w = (nt, kq), 32-pixel tiles, 32-channel tiles):
//   conv1: 13 pixel tiles x K = 256; w takes tiles w and w + 8, sharing each weight fragment between them.
//   conv2: 81 pixels = 3 tiles; w accumulates channel tile nt over k-quarter kq (= filter row kq) for all three.
//   conv3: 49 pixels = 2 tiles; same scheme (k-quarter = 9 of the 36 k-steps).
//   The four k-quarters of a channel tile meet through LDS: wavefront (nt, q) finishes accumulator rows
//   4q .. 4q + 3 of each 16 and receives them from the other three, added in k order.
// act1 / act2 also go to global memory when the backward pass will need them.
// With few items (an act step, a small minibatch) an item is one band of a sample's output rows instead of a whole
// sample, and one workgroup runs one item: see PARTS at the kernel.
#pragma once
#include <type_traits>

#include "conv_ws.h"

namespace dqn {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Position of element (o, k) of an [O][K] weight matrix in fragment order: 1 KB rows indexed
// (channel tile o / 32, k-step k / 16), lane = 32 * ((k % 16) / 8) + o % 32, eight consecutive k per lane.
__host__ __device__ inline size_t tower_frag_index(int o, int k, int K)
{
    return ((static_cast<size_t>(o >> 5) * (K >> 4) + (k >> 4)) * 64 + (((k >> 3) & 1) << 5) + (o & 31)) * 8 + (k & 7);
}

// Eight bytes -> eight fp16 subnormals (value = byte * 2^-24).  v_perm_b32 picks result bytes out of
// {src0, src1}: selector 0..3 = byte of src1, 0x0c = constant zero.
__device__ inline f16x8 bytes_as_f16_subnormals(uint32_t lo, uint32_t hi)
{
    u32x4 d;
    d[0] = __builtin_amdgcn_perm(0u, lo, 0x0c010c00u);   // [0, byte1, 0, byte0]
    d[1] = __builtin_amdgcn_perm(0u, lo, 0x0c030c02u);   // [0, byte3, 0, byte2]
    d[2] = __builtin_amdgcn_perm(0u, hi, 0x0c010c00u);
    d[3] = __builtin_amdgcn_perm(0u, hi, 0x0c030c02u);
    return __builtin_bit_cast(f16x8, d);
}

// Exchange of accumulator rows between the four k-quarters of a channel tile.  `x` points at the
// [4 finisher][3 sender slot][64 lane] float4 block of one (channel tile, pixel tile); the sender slot of
// quarter s at finisher f is s for s < f and s - 1 for s > f.  The callers branch on the (wavefront-uniform)
// quarter; the markers keep the compiler from folding the branches into run-time register indexing.
template <int KQ> __device__ inline void tower_send(float4* x, const f32x16& acc, int lane)
{
    asm volatile("; send, k-quarter %0" ::"n"(KQ));
#pragma unroll
    for (int f = 0; f < 4; ++f)
        if (f != KQ) x[(f * 3 + (KQ < f ? KQ : KQ - 1)) * 64 + lane] = make_float4(acc[4 * f], acc[4 * f + 1], acc[4 * f + 2], acc[4 * f + 3]);
    asm volatile("; sent, k-quarter %0" ::"n"(KQ) : "memory");
}
// Rows 4 * KQ .. + 3: the four partial sums in k order, + bias, ReLU.
template <int KQ> __device__ inline float4 tower_finish(const float4* x, const f32x16& acc, int lane, const float4& bias)
{
    asm volatile("; finish, k-quarter %0" ::"n"(KQ));
    float4 p[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        p[s] = s == KQ ? make_float4(acc[4 * KQ], acc[4 * KQ + 1], acc[4 * KQ + 2], acc[4 * KQ + 3])
                       : x[(KQ * 3 + (s < KQ ? s : s - 1)) * 64 + lane];
    float4 r;
    r.x = fmaxf(((p[0].x + p[1].x) + p[2].x) + p[3].x + bias.x, 0.f);
    r.y = fmaxf(((p[0].y + p[1].y) + p[2].y) + p[3].y + bias.y, 0.f);
    r.z = fmaxf(((p[0].z + p[1].z) + p[2].z) + p[3].z + bias.z, 0.f);
    r.w = fmaxf(((p[0].w + p[1].w) + p[2].w) + p[3].w + bias.w, 0.f);
    asm volatile("; finished, k-quarter %0" ::"n"(KQ) : "memory");
    return r;
}

constexpr int kTowerP2_ = 72;

struct TowerArgs {
    // what a workgroup needs first sits in the first 64 bytes: kernel arguments are fetched by cache line, and every
    // further line touched on the way to the first load of the state is a dependent miss of its own
    int n, groups;
    int per;                    // items per workgroup = ceil(n * groups / grid size), computed by the host
    int tower_blocks;           // workgroups [0, tower_blocks) run the tower, the next push.L ones the append below
    const uint8_t* x[kMaxGroups];      // [n][4][84][84], 16-byte aligned (unused with a descriptor table)
    // Minibatch given as per-sample descriptors (sample_desc in common.h: replay slots of the frames of s and s', -1 =
    // zero frame) instead of assembled states: group 0 reads the four frames of s, every other group those of s',
    // straight from the replay memory's frame array.  Null: states come from x.
    const int32_t* desc;               // [n][8]
    const uint8_t* ring;               // [capacity][84][84]
    const _Float16* w1[kMaxGroups];    // fragment order, fp16
    const float* b1[kMaxGroups];
    const float* b2[kMaxGroups];
    const float* b3[kMaxGroups];
    const bf16_t* w2[kMaxGroups];      // fragment order, bf16
    const bf16_t* w3[kMaxGroups];
    bf16_t* act1[kMaxGroups];   // [n][400][32] or null
    bf16_t* act2[kMaxGroups];   // [n][81][64] or null
    bf16_t* act3[kMaxGroups];   // [n][49][64]
    uint8_t* s_out;             // with desc: group 0 also stores the state it assembled, [n][4][84][84] (the weight gradient of conv1 reads it)
    PushStepPlan push;          // optional (L = 0: none): one experience per lane into the temporary buffers
};

constexpr int kTowerP1 = 40, kTowerP2 = kTowerP2_;   // LDS pixel pitch (elements) of conv1 / conv2 outputs
constexpr int kTowerXBytes = 4 * 84 * 84;             // 28,224 = 1764 x 16
constexpr int kTowerThreads = 512;                    // the index arithmetic below assumes exactly this block size
constexpr int kTowerXchgBytes = 2 * 3 * 4 * 3 * 64 * 16;   // row exchange, [nt][tile][finisher][slot][lane] float4
// LDS: exchange block (its head doubles as the state buffer), conv1 weights, act1, act2, biases
constexpr size_t kTowerSmem = kTowerXchgBytes + 32 * 256 * 2 + 400 * kTowerP1 * 2 + 81 * kTowerP2 * 2 + kTowerThreads * 4;   // biases: 160 floats used, one slot per thread
static_assert(kTowerXBytes <= kTowerXchgBytes, "the state buffer overlays the exchange block");

// DESC: the minibatch comes as a descriptor table (a.desc, a.ring) instead of assembled states (a.x); a separate
// instantiation, so that the act step and small minibatches run the kernel without any of the descriptor logic.
//
// The leading scalar parameters repeat what a workgroup needs before its first load (TowerArgs::n, groups, per,
// tower_blocks, x[0], x[1], desc, ring, w1[0]): the first 14 dwords of the kernel arguments are preloaded into scalar
// registers when a wavefront starts (build option amdgpu-kernarg-preload-count), while a field of the struct is a load
// from cold memory in front of everything that depends on it.
//
// PARTS = 3: one item is a THIRD of a sample's work -- output rows 0-2 / 3-4 / 5-6 of conv3, with the rows of conv2 (0-4 /
// 3-6 / 5-8) and conv1 (0-11 / 6-15 / 10-19) they depend on -- and every workgroup runs exactly one item.  A round of a few
// synchronized samplers (Section 4) or a minibatch of 32 leaves most of the chip idle while each sample's chain of layers
// takes its seven microseconds on one compute unit; in thirds the chain is conv1 in one pass instead of two (at most eight
// pixel tiles for eight wavefronts), two pixel tiles of conv2 instead of three and one of conv3 instead of two.  Every
// output element is computed by the same instructions in the same order as with PARTS = 1 (rows that two parts both need
// are computed twice), so the results are equal bit for bit.  PARTS = 7, for a single round of samplers: one output row of
// conv3 per workgroup (three rows of conv2: one pixel tile, eight rows of conv1: five tiles).
template <bool DESC, int PARTS>
__global__ __launch_bounds__(kTowerThreads) void conv_tower_kernel(int n_, int groups_, int per_, int tower_blocks_, const uint8_t* x0_,
                                                                   const uint8_t* x1_, const int32_t* desc_, const uint8_t* ring_,
                                                                   const _Float16* w1_0_, TowerArgs a)
{
    typedef bf16_t T;
    typedef bf16x8 V8;
    extern __shared__ __attribute__((aligned(16))) unsigned char tw_smem[];
    uint8_t* sX = tw_smem;                                   // live from an item's opening barrier to the end of its conv1
    float4* sXchg = reinterpret_cast<float4*>(tw_smem);      // live from conv2's MFMAs to the end of the item
    _Float16* sW1 = reinterpret_cast<_Float16*>(tw_smem + kTowerXchgBytes);
    T* sA1 = reinterpret_cast<T*>(sW1 + 32 * 256);
    T* sA2 = sA1 + 400 * kTowerP1;
    float* sB1 = reinterpret_cast<float*>(sA2 + 81 * kTowerP2);   // biases: conv1 [32], conv2 [64], conv3 [64]
    float* sB2 = sB1 + 32;
    float* sB3 = sB2 + 64;

    if (static_cast<int>(blockIdx.x) >= tower_blocks_) {
        // An act step's launch sequence also carries the append of the previous step's experiences (Section 3:
        // temporary buffers): independent byte copies that would otherwise cost a dependent launch of their own.
        push_step_block(a.push, static_cast<int>(blockIdx.x) - tower_blocks_);
        return;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lp = lane & 31, kg = lane >> 5;
    const int nt = wave >> 2, kq = wave & 3;
    static_assert(PARTS == 1 || PARTS == 3 || PARTS == 7, "whole samples, thirds, or sevenths");
    const int total = n_ * groups_;
    // PARTS = 3: workgroup j runs part j % 3 of item j / 3 (the host launches 3 * total workgroups, per_ = 1)
    const int part = PARTS == 1 ? 0 : static_cast<int>(blockIdx.x % PARTS);
    const int first = PARTS == 1 ? blockIdx.x * per_ : static_cast<int>(blockIdx.x / PARTS), last = PARTS == 1 ? min(total, first + per_) : min(total, first + 1);
    if (first >= last) return;
    // first row and pixel count of this part in each layer's output (whole sample: all of it)
    // (conv3 rows [r, r') need conv2 rows [r, r' + 2), and those need conv1 rows [2 r, 2 r' + 6))
    const int r3_lo = PARTS == 1 ? 0 : PARTS == 7 ? part : (part == 0 ? 0 : part == 1 ? 3 : 5);
    const int r2_lo = r3_lo, r1_lo = 2 * r3_lo;
    const int n3 = PARTS == 1 ? 49 : PARTS == 7 ? 7 : (part == 0 ? 21 : 14);
    const int n2 = PARTS == 1 ? 81 : PARTS == 7 ? 27 : (part == 0 ? 45 : 36);
    const int n1 = PARTS == 1 ? 400 : PARTS == 7 ? 160 : (part == 0 ? 240 : 200);
    constexpr int T2 = PARTS == 1 ? 3 : PARTS == 3 ? 2 : 1, T3 = PARTS == 1 ? 2 : 1;   // pixel tiles of conv2 / conv3 per wavefront

    // The state of item (g_, b_), 16 bytes per lane and load (the last load is clamped, not predicated);
    // named registers rather than an array, which the compiler would keep in scratch memory.  With a descriptor table
    // the four frames of the state sit anywhere in the replay memory: vector v of the state belongs to frame v / 441
    // (a frame is 441 vectors), so each of a thread's four loads chooses between two neighbouring frames; a zero frame
    // (slot -1) is loaded from slot 0 and ANDed away.  The descriptor of an item is requested a whole item before its
    // frames are (dn*: the item after next), so that the frames never wait for it.
    constexpr int kXVecs = kTowerXBytes / 16;   // 1764
    const int last_vec = tid + 1536 < kXVecs ? tid + 1536 : kXVecs - 1;
    constexpr bool use_desc = DESC;
    const bool hi0 = tid >= 441, hi1 = tid + 512 >= 882, hi2 = tid + 1024 >= 1323;         // second of the two candidate frames
    const int w0 = tid - (hi0 ? 441 : 0), w1 = tid + 512 - (hi1 ? 882 : 441), w2 = tid + 1024 - (hi2 ? 1323 : 882), w3 = last_vec - 1323;
    V8 wf2[8], wf3[9];
    uint4 xv0, xv1, xv2, xv3;
    int dn0 = 0, dn1 = 0, dn2 = 0, dn3 = 0;   // descriptor (four slots) of the item whose frames are requested next
#define DQN_TOWER_FETCH_DESC(g_, b_)                                                                          \
    {                                                                                                        \
        const int32_t* dp_ = desc_ + static_cast<size_t>(b_) * kDescInts + ((g_) > 0 ? 4 : 0);                \
        dn0 = dp_[0]; dn1 = dp_[1]; dn2 = dp_[2]; dn3 = dp_[3];                                                \
    }
#define DQN_TOWER_FETCH_STATE(g_, b_)                                                                        \
    if constexpr (use_desc) {                                                                                \
        const int s0_ = hi0 ? dn1 : dn0, s1_ = hi1 ? dn2 : dn1, s2_ = hi2 ? dn3 : dn2, s3_ = dn3;              \
        const uint4* r_ = reinterpret_cast<const uint4*>(ring_);                                             \
        xv0 = r_[static_cast<size_t>(s0_ < 0 ? 0 : s0_) * kFrameVec16 + w0];                                  \
        xv1 = r_[static_cast<size_t>(s1_ < 0 ? 0 : s1_) * kFrameVec16 + w1];                                  \
        xv2 = r_[static_cast<size_t>(s2_ < 0 ? 0 : s2_) * kFrameVec16 + w2];                                  \
        xv3 = r_[static_cast<size_t>(s3_ < 0 ? 0 : s3_) * kFrameVec16 + w3];                                  \
        const uint32_t m0_ = s0_ < 0 ? 0u : ~0u, m1_ = s1_ < 0 ? 0u : ~0u, m2_ = s2_ < 0 ? 0u : ~0u, m3_ = s3_ < 0 ? 0u : ~0u; \
        xv0.x &= m0_; xv0.y &= m0_; xv0.z &= m0_; xv0.w &= m0_;                                              \
        xv1.x &= m1_; xv1.y &= m1_; xv1.z &= m1_; xv1.w &= m1_;                                              \
        xv2.x &= m2_; xv2.y &= m2_; xv2.z &= m2_; xv2.w &= m2_;                                              \
        xv3.x &= m3_; xv3.y &= m3_; xv3.z &= m3_; xv3.w &= m3_;                                              \
    } else {                                                                                                 \
        const uint8_t* xg_ = (g_) == 0 ? x0_ : (g_) == 1 ? x1_ : a.x[g_];                                     \
        const uint4* xs_ = reinterpret_cast<const uint4*>(xg_ + static_cast<size_t>(b_) * kTowerXBytes);      \
        xv0 = xs_[tid]; xv1 = xs_[tid + 512]; xv2 = xs_[tid + 1024]; xv3 = xs_[last_vec];                      \
    }

    int g = 0, b = first;   // item = (group, sample); no run-time division (groups <= 4)
    while (b >= n_) { b -= n_; ++g; }
    if constexpr (use_desc) {
        DQN_TOWER_FETCH_DESC(g, b)
    }
    DQN_TOWER_FETCH_STATE(g, b)   // first thing on the way: everything below it is address arithmetic
    if (use_desc && first + 1 < last) {
        if (b + 1 < n_) DQN_TOWER_FETCH_DESC(g, b + 1) else DQN_TOWER_FETCH_DESC(g + 1, 0)
    }

    // conv3 k-steps of this wavefront's quarter: offsets inside a pixel's window (wavefront-uniform, plain scalar
    // arithmetic -- written as a choice between per-quarter constants it compiled to a chain of ~30 branches in
    // front of the first load)
    int off3[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) {
        const int ks = 9 * kq + k, tap = ks >> 2, p = (tap * 11) >> 5 /* tap / 3 for tap <= 8 */, q = tap - 3 * p;
        off3[k] = (p * 9 + q) * kTowerP2_ + (ks & 3) * 16;
    }

    int cur_g = -1;
    for (int it = first; it < last; ++it, ++b) {
        if (b == n_) { b = 0; ++g; }
        // First item, or the range crosses into the next group: (re)load the weights (every wavefront has passed the
        // barrier that ends the previous item).  What conv1 needs -- its own 16 KB of weights and the state -- is requested
        // and parked in LDS first; the 139 KB of conv2/conv3 fragments are requested after that and arrive while conv1 runs
        // (requested first, they stood in front of conv1's operands in the memory pipeline: a CU draws ~64 B/clk).
        const bool new_group = g != cur_g;
        if (new_group) {
            cur_g = g;
            const _Float16* w1g = g == 0 ? w1_0_ : a.w1[g];
            const f16x8 w1a = *reinterpret_cast<const f16x8*>(w1g + tid * 8);
            const f16x8 w1b = *reinterpret_cast<const f16x8*>(w1g + (tid + 512) * 8);
            // biases: every thread loads one (address chosen without a branch, clamped) and stores it to a slot of its own --
            // behind a condition the compiler sinks the load to the store, a dependent round trip of its own
            const int bt = tid < 160 ? tid : 159;
            const float* bp = bt < 32 ? a.b1[g] + bt : (bt < 96 ? a.b2[g] + (bt - 32) : a.b3[g] + (bt - 96));
            const float bias = *bp;
            *reinterpret_cast<f16x8*>(sW1 + tid * 8) = w1a;
            *reinterpret_cast<f16x8*>(sW1 + (tid + 512) * 8) = w1b;
            sB1[tid] = bias;
        }
        {
            uint4* d = reinterpret_cast<uint4*>(sX);
            d[tid] = xv0; d[tid + 512] = xv1; d[tid + 1024] = xv2; d[last_vec] = xv3;   // clamped lanes rewrite the last vector with itself
            if (use_desc && g == 0 && a.s_out) {   // the assembled state, kept for the weight gradient of conv1
                uint4* so = reinterpret_cast<uint4*>(a.s_out + static_cast<size_t>(b) * kTowerXBytes);
                so[tid] = xv0; so[tid + 512] = xv1; so[tid + 1024] = xv2; so[last_vec] = xv3;
            }
        }
        // conv2/conv3 fragments of a new group: requested a few k-steps apart inside conv1's (conv2's weights) and conv2's
        // (conv3's weights) MFMA streams (17 KB per wavefront -- requested in one go they hold every wavefront ~0.5 us in
        // front of the barrier below, just being issued)
        const T* p2 = a.w2[g] + (static_cast<size_t>(nt * 32 + kq * 8) * 64 + lane) * 8;
        const T* p3 = a.w3[g] + (static_cast<size_t>(nt * 36 + kq * 9) * 64 + lane) * 8;
        if (it + 1 < last) {   // the next item's state: in flight while this item computes
            if (b + 1 < n_) DQN_TOWER_FETCH_STATE(g, b + 1) else DQN_TOWER_FETCH_STATE(g + 1, 0)
            if (use_desc && it + 2 < last) {   // and the descriptor of the item after it
                int g2 = g, b2 = b + 2;
                while (b2 >= n_) { b2 -= n_; ++g2; }
                DQN_TOWER_FETCH_DESC(g2, b2)
            }
        }
        __syncthreads();

        // ---- conv1: k = (c, p, q); k-step k covers c = k / 4, p = 2 * (k % 4) + kg, q = 0..7 -------------
        {
            T* g1 = a.act1[g];
            constexpr int D = 5;   // k-steps of LDS reads in flight
            auto run = [&](auto nt_) {
                constexpr int NT = decltype(nt_)::value;   // pixel tiles of this wavefront: w (and w + 8)
                const uint8_t* base[NT];
                f32x16 acc[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int lpx = (wave + 8 * t) * 32 + lp;
                    const int pc = r1_lo * 20 + (lpx < n1 ? lpx : n1 - 1);
                    base[t] = sX + (4 * (pc / 20) + kg) * 84 + 4 * (pc % 20);
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
                }
                auto fetch_px = [&](int t, int k) {
                    const uint32_t* wp = reinterpret_cast<const uint32_t*>(base[t] + (k / 4) * 7056 + ((k % 4) * 2) * 84);
                    return make_uint2(wp[0], wp[1]);
                };
                auto fetch_w = [&](int k) { return *reinterpret_cast<const f16x8*>(sW1 + (k * 64 + lane) * 8); };
                uint2 ring_px[NT][D];
                f16x8 ring_w[D];
#pragma unroll
                for (int u = 0; u < D; ++u) {
                    ring_w[u] = fetch_w(u);
#pragma unroll
                    for (int t = 0; t < NT; ++t) ring_px[t][u] = fetch_px(t, u);
                }
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const f16x8 w = ring_w[k % D];
                    uint2 cur[NT];
#pragma unroll
                    for (int t = 0; t < NT; ++t) cur[t] = ring_px[t][k % D];
                    if (k + D < 16) {
                        ring_w[k % D] = fetch_w(k + D);
#pragma unroll
                        for (int t = 0; t < NT; ++t) ring_px[t][k % D] = fetch_px(t, k + D);
                    }
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(w, bytes_as_f16_subnormals(cur[t].x, cur[t].y), acc[t], 0, 0, 0);
                    if (new_group && (k & 1)) wf2[k >> 1] = *reinterpret_cast<const V8*>(p2 + (k >> 1) * 512);   // conv2's: every other k-step
                    __builtin_amdgcn_sched_barrier(0);
                }
                // output stage: scale, bias, ReLU -> LDS (+ global); rows 8q + 4kg .. + 3 are channels of this lane's pixel
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int lpx = (wave + 8 * t) * 32 + lp, px = r1_lo * 20 + lpx;
                    if (lpx < n1) {
                        constexpr float kScale = 16777216.f / 255.f;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int ch = 8 * q + 4 * kg;
                            const float4 bv = *reinterpret_cast<const float4*>(sB1 + ch);
                            const float v0 = fmaxf(acc[t][4 * q] * kScale + bv.x, 0.f), v1 = fmaxf(acc[t][4 * q + 1] * kScale + bv.y, 0.f);
                            const float v2 = fmaxf(acc[t][4 * q + 2] * kScale + bv.z, 0.f), v3 = fmaxf(acc[t][4 * q + 3] * kScale + bv.w, 0.f);
                            store4<T>(sA1 + px * kTowerP1 + ch, v0, v1, v2, v3);
                            if (g1) store4<T>(g1 + (static_cast<size_t>(b) * 400 + px) * 32 + ch, v0, v1, v2, v3);
                        }
                    }
                }
            };
            if (PARTS == 1 && wave < 5) run(std::integral_constant<int, 2>{}); else run(std::integral_constant<int, 1>{});   // 13 tiles (a third: at most 8)
        }
        __syncthreads();

        // ---- conv2: k = (p, q, c); this quarter is filter row p = kq; k-step k covers q = k / 2, channels 16 * (k % 2) + 8 * kg .. + 7
        {
            f32x16 acc[T2];
            const T* base[T2];
#pragma unroll
            for (int t = 0; t < T2; ++t) {
                const int lpx = t * 32 + lp;
                const int pc = r2_lo * 9 + (lpx < n2 ? lpx : n2 - 1);
                base[t] = sA1 + ((2 * (pc / 9) + kq) * 20 + 2 * (pc % 9)) * kTowerP1 + kg * 8;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
            }
            {
                constexpr int D = 6;
                auto fetch = [&](int step) {
                    const int t = step / 8, k = step % 8;
                    return *reinterpret_cast<const V8*>(base[t] + (k >> 1) * kTowerP1 + (k & 1) * 16);
                };
                V8 ring[D];
#pragma unroll
                for (int u = 0; u < D; ++u) ring[u] = fetch(u);
#pragma unroll
                for (int step = 0; step < 8 * T2; ++step) {
                    const V8 cur = ring[step % D];
                    if (step + D < 8 * T2) ring[step % D] = fetch(step + D);
                    mma_32x32x16(acc[step / 8], wf2[step % 8], cur);
                    // conv3's fragments: nine requests spread over the stream (every other step of 24, every step of 16 or 8)
                    constexpr int W3_FIRST = T2 == 3 ? 4 : T2 == 2 ? 3 : 0, W3_EVERY = T2 == 3 ? 2 : 1;
                    if (new_group && step >= W3_FIRST && (step - W3_FIRST) % W3_EVERY == 0 && (step - W3_FIRST) / W3_EVERY < 9)
                        wf3[(step - W3_FIRST) / W3_EVERY] = *reinterpret_cast<const V8*>(p3 + ((step - W3_FIRST) / W3_EVERY) * 512);
                    if (T2 == 1 && new_group && step == 7) wf3[8] = *reinterpret_cast<const V8*>(p3 + 8 * 512);   // eight steps, nine fragments
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            float4* xc = sXchg + static_cast<size_t>(nt * 3) * (4 * 3 * 64);
#pragma unroll
            for (int t = 0; t < T2; ++t) {
                float4* x = xc + t * (4 * 3 * 64);
                if (kq == 0) tower_send<0>(x, acc[t], lane); else if (kq == 1) tower_send<1>(x, acc[t], lane);
                else if (kq == 2) tower_send<2>(x, acc[t], lane); else tower_send<3>(x, acc[t], lane);
            }
            __syncthreads();
            T* g2 = a.act2[g];
            const int ch = nt * 32 + 8 * kq + 4 * kg;
            const float4 bv = *reinterpret_cast<const float4*>(sB2 + ch);
#pragma unroll
            for (int t = 0; t < T2; ++t) {
                const float4* x = xc + t * (4 * 3 * 64);
                float4 v;
                if (kq == 0) v = tower_finish<0>(x, acc[t], lane, bv); else if (kq == 1) v = tower_finish<1>(x, acc[t], lane, bv);
                else if (kq == 2) v = tower_finish<2>(x, acc[t], lane, bv); else v = tower_finish<3>(x, acc[t], lane, bv);
                const int lpx = t * 32 + lp, px = r2_lo * 9 + lpx;
                if (lpx < n2) {
                    store4<T>(sA2 + px * kTowerP2 + ch, v.x, v.y, v.z, v.w);
                    if (g2) store4<T>(g2 + (static_cast<size_t>(b) * 81 + px) * 64 + ch, v.x, v.y, v.z, v.w);
                }
            }
        }
        __syncthreads();

        // ---- conv3: k = (p, q, c); k-step ks = 9 * kq + k covers tap ks / 4, channels 16 * (ks % 4) + 8 * kg .. + 7
        {
            f32x16 acc[T3];
            const T* base[T3];
#pragma unroll
            for (int t = 0; t < T3; ++t) {
                const int lpx = t * 32 + lp;
                const int pc = r3_lo * 7 + (lpx < n3 ? lpx : n3 - 1);
                base[t] = sA2 + ((pc / 7) * 9 + pc % 7) * kTowerP2 + kg * 8;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
            }
            {
                constexpr int D = 6;
                auto fetch = [&](int step) { return *reinterpret_cast<const V8*>(base[step / 9] + off3[step % 9]); };
                V8 ring[D];
#pragma unroll
                for (int u = 0; u < D; ++u) ring[u] = fetch(u);
#pragma unroll
                for (int step = 0; step < 9 * T3; ++step) {
                    const V8 cur = ring[step % D];
                    if (step + D < 9 * T3) ring[step % D] = fetch(step + D);
                    mma_32x32x16(acc[step / 9], wf3[step % 9], cur);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            float4* xc = sXchg + static_cast<size_t>(nt * 3) * (4 * 3 * 64);
#pragma unroll
            for (int t = 0; t < T3; ++t) {
                float4* x = xc + t * (4 * 3 * 64);
                if (kq == 0) tower_send<0>(x, acc[t], lane); else if (kq == 1) tower_send<1>(x, acc[t], lane);
                else if (kq == 2) tower_send<2>(x, acc[t], lane); else tower_send<3>(x, acc[t], lane);
            }
            __syncthreads();
            const int ch = nt * 32 + 8 * kq + 4 * kg;
            const float4 bv = *reinterpret_cast<const float4*>(sB3 + ch);
#pragma unroll
            for (int t = 0; t < T3; ++t) {
                const float4* x = xc + t * (4 * 3 * 64);
                float4 v;
                if (kq == 0) v = tower_finish<0>(x, acc[t], lane, bv); else if (kq == 1) v = tower_finish<1>(x, acc[t], lane, bv);
                else if (kq == 2) v = tower_finish<2>(x, acc[t], lane, bv); else v = tower_finish<3>(x, acc[t], lane, bv);
                const int lpx = t * 32 + lp, px = r3_lo * 7 + lpx;
                if (lpx < n3) store4<T>(a.act3[g] + (static_cast<size_t>(b) * 49 + px) * 64 + ch, v.x, v.y, v.z, v.w);
            }
        }
        __syncthreads();   // the exchange block is read until here; its head is the next item's state buffer
    }
#undef DQN_TOWER_FETCH_STATE
#undef DQN_TOWER_FETCH_DESC
}

}  // namespace dqn
