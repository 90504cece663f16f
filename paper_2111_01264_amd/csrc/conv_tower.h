// Fused conv1 -> conv2 -> conv3 of the Q-network (Section 5: the Nature-DQN layers), reduced-precision
// mode: a persistent workgroup of 4 wavefronts -- one per SIMD, so that each may use the whole 512-entry
// register file -- walks a contiguous range of (group, sample) items; the activations of conv1 and conv2
// never leave LDS and every weight is fetched once per workgroup and group, then lives in registers.
//
// Why it looks like this: one sample is far too little work to hide memory latency, and MFMA operand
// fragments gathered straight from [o][k] weight rows or from the strided uint8 state are one cache line
// per lane -- the address unit, not the matrix core, sets the time.  So
//   * the weight copies this kernel reads are stored in *fragment order*: the 64 x 16-byte operand of one
//     32x32x16 MFMA is one contiguous 1 KB row, fetched with one fully coalesced load
//     (tower_frag_index below is the layout; the optimizer kernel writes it);
//   * the 28 KB uint8 state is fetched with 16-byte loads into registers one item ahead (the loads are
//     issued as soon as this item's state has been written to LDS) and conv1's pixel fragments come from LDS.
//     (Loads that write LDS directly would save the registers, but the compiler then orders every later LDS
//     access behind all outstanding vector-memory operations, which serialises the prefetch.);
//   * the wavefronts hold disjoint (channel tile, k-half) parts of conv2's and conv3's weights, and all of
//     conv1's (64 + 64 + 72 VGPRs per lane);
//   * with one wavefront per SIMD there is no second wavefront to fill the gaps, so every phase is a
//     hand-pipelined stream of k-steps: the LDS read of step s + D, the operand preparation and the MFMA
//     of step s, and a slice of the previous tile's output stage share one slot, pinned in program order
//     (a 32x32x16 MFMA occupies the wavefront for 32 cycles, during which about six other instructions
//     issue for free).
//
// conv1 runs on the f16 MFMA: a pixel byte x, zero-extended to 16 bits, *is* the fp16 subnormal x * 2^-24,
// which the matrix core takes without flushing; no integer-to-float conversion is needed (the VALU would
// otherwise be the bottleneck of conv1), the products are exact, and the factor 2^24 / 255 is applied to
// the fp32 accumulator.  conv1's weight copy is therefore fp16, the other two are bf16.
//
// Work split per sample (wavefront w = (nt, kh), 32-pixel tiles, 32-channel tiles):
//   conv1: 13 pixel tiles x K = 256; w takes tiles w, w + 4, w + 8, w + 12.
//   conv2: 81 pixels = 3 tiles; w accumulates channel tile nt over k-half kh for all three.
//   conv3: 49 pixels = 2 tiles; same scheme.
//   The two k-halves of a channel tile meet through LDS: each wavefront hands over the accumulator rows
//   the other one finishes (rows 0..7 of each 16 stay with kh = 0, rows 8..15 with kh = 1).
// act1 / act2 also go to global memory when the backward pass will need them.
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

// Hand-over of accumulator rows between the two k-halves of a channel tile (KH = this wavefront's half):
// rows 8 * (1 - KH) .. + 7 of each 16 go to the partner through LDS, rows 8 * KH .. + 7 are finished here.
// The callers branch on the (wavefront-uniform) half; the marker keeps the compiler from folding the two
// branches into one with run-time register indexing.
template <int KH> __device__ inline void tower_hand_over(float4 (*mine)[2], const f32x16& acc, int lane)
{
    asm volatile("; hand over, k-half %0" ::"n"(KH));
    constexpr int r = 8 * (1 - KH);
#pragma unroll
    for (int h = 0; h < 2; ++h)
        mine[lane][h] = make_float4(acc[r + 4 * h], acc[r + 4 * h + 1], acc[r + 4 * h + 2], acc[r + 4 * h + 3]);
    asm volatile("; handed over, k-half %0" ::"n"(KH) : "memory");
}
// Sum of both halves + bias, ReLU, for the four rows 8 * KH + 4 * h .. + 3 of a tile.
template <int KH> __device__ inline float4 tower_finish(const f32x16& acc, int h, const float4& other, const float4& bias)
{
    asm volatile("; finish, k-half %0" ::"n"(KH));
    const int r = 8 * KH + 4 * h;
    return make_float4(fmaxf(acc[r] + other.x + bias.x, 0.f), fmaxf(acc[r + 1] + other.y + bias.y, 0.f),
                       fmaxf(acc[r + 2] + other.z + bias.z, 0.f), fmaxf(acc[r + 3] + other.w + bias.w, 0.f));
}

// Offset (elements) of conv3's k-step ks inside a pixel's 3x3x64 window of the LDS copy of conv2's output.
constexpr int kTowerP2_ = 72;
constexpr int tower_conv3_offset(int ks) { return (((ks >> 2) / 3) * 9 + (ks >> 2) % 3) * kTowerP2_ + (ks & 3) * 16; }

struct TowerArgs {
    const uint8_t* x[kMaxGroups];      // [n][4][84][84], 16-byte aligned
    const _Float16* w1[kMaxGroups];    // fragment order, fp16
    const bf16_t* w2[kMaxGroups];      // fragment order, bf16
    const bf16_t* w3[kMaxGroups];
    const float* b1[kMaxGroups];
    const float* b2[kMaxGroups];
    const float* b3[kMaxGroups];
    bf16_t* act1[kMaxGroups];   // [n][400][32] or null
    bf16_t* act2[kMaxGroups];   // [n][81][64] or null
    bf16_t* act3[kMaxGroups];   // [n][49][64]
    int n, groups;
    int per;                    // items per workgroup = ceil(n * groups / grid size), computed by the host
};

constexpr int kTowerP1 = 40, kTowerP2 = kTowerP2_;   // LDS pixel pitch (elements) of conv1 / conv2 outputs
constexpr int kTowerXBytes = 4 * 84 * 84;     // 28,224 = 27 x 1024 + 576
constexpr int kTowerThreads = 256;            // the index arithmetic below assumes exactly this block size
constexpr size_t kTowerSmem = kTowerXBytes + 400 * kTowerP1 * 2 + 81 * kTowerP2 * 2 + 4 * 3 * 64 * 8 * 4 + 160 * 4;

__global__ __launch_bounds__(kTowerThreads) void conv_tower_kernel(TowerArgs a)
{
    typedef bf16_t T;
    typedef bf16x8 V8;
    extern __shared__ __attribute__((aligned(16))) unsigned char tw_smem[];
    uint8_t* sX = tw_smem;
    T* sA1 = reinterpret_cast<T*>(tw_smem + kTowerXBytes);
    T* sA2 = sA1 + 400 * kTowerP1;
    float4 (*red)[3][64][2] = reinterpret_cast<float4 (*)[3][64][2]>(sA2 + 81 * kTowerP2);   // [wavefront][tile][lane][8 rows]
    float* sB1 = reinterpret_cast<float*>(red + 4);   // biases: conv1 [32], conv2 [64], conv3 [64]
    float* sB2 = sB1 + 32;
    float* sB3 = sB2 + 64;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lp = lane & 31, kg = lane >> 5;
    const int nt = wave >> 1, kh = wave & 1;
    const int total = a.n * a.groups;
    const int first = blockIdx.x * a.per, last = min(total, first + a.per);
    if (first >= last) return;

    // The state of item (g_, b_), 16 bytes per lane and load (the last load is clamped, not predicated);
    // seven named registers rather than an array, which the compiler would keep in scratch memory.
    constexpr int kXVecs = kTowerXBytes / 16;   // 1764
    const int last_vec = tid + 1536 < kXVecs ? tid + 1536 : kXVecs - 1;
#define DQN_TOWER_FETCH_STATE(g_, b_)                                                                        \
    {                                                                                                        \
        const uint4* xs_ = reinterpret_cast<const uint4*>(a.x[g_] + static_cast<size_t>(b_) * kTowerXBytes);  \
        xv0 = xs_[tid]; xv1 = xs_[tid + 256]; xv2 = xs_[tid + 512]; xv3 = xs_[tid + 768];                      \
        xv4 = xs_[tid + 1024]; xv5 = xs_[tid + 1280]; xv6 = xs_[last_vec];                                     \
    }

    // conv1 output: rows 8q + 4kg .. + 3 (channels) of this lane's pixel: scale, bias, ReLU -> LDS (+ global).
    // The bias values sit in registers (bq): an LDS read here would make the k-step pipeline drain.
    float4 bq[4];
    auto conv1_store_quad = [&](int tile, const f32x16& acc, int q, T* g1, int b) {
        const int px = tile * 32 + lp;
        if (px < 400) {
            constexpr float kScale = 16777216.f / 255.f;
            const int ch = 8 * q + 4 * kg;
            const float v0 = fmaxf(acc[4 * q] * kScale + bq[q].x, 0.f), v1 = fmaxf(acc[4 * q + 1] * kScale + bq[q].y, 0.f);
            const float v2 = fmaxf(acc[4 * q + 2] * kScale + bq[q].z, 0.f), v3 = fmaxf(acc[4 * q + 3] * kScale + bq[q].w, 0.f);
            store4<T>(sA1 + px * kTowerP1 + ch, v0, v1, v2, v3);
            if (g1) store4<T>(g1 + (static_cast<size_t>(b) * 400 + px) * 32 + ch, v0, v1, v2, v3);
        }
    };

    f16x8 wf1[16];
    V8 wf2[16], wf3[18];
    int g = 0, b = first;   // item = (group, sample); no run-time division (groups <= 4)
    while (b >= a.n) { b -= a.n; ++g; }
    uint4 xv0, xv1, xv2, xv3, xv4, xv5, xv6;
    DQN_TOWER_FETCH_STATE(g, b)
    int cur_g = -1;
    for (int it = first; it < last; ++it, ++b) {
        if (b == a.n) { b = 0; ++g; }
        if (g != cur_g) {   // first item, or the range crosses into the next group: (re)load the weights
            if (cur_g >= 0) __syncthreads();   // the previous item may still be reading its biases
            cur_g = g;
            const _Float16* p1 = a.w1[g] + lane * 8;
#pragma unroll
            for (int s = 0; s < 16; ++s) wf1[s] = *reinterpret_cast<const f16x8*>(p1 + s * 512);
            const T* p2 = a.w2[g] + (static_cast<size_t>(nt * 32 + kh * 16) * 64 + lane) * 8;
#pragma unroll
            for (int s = 0; s < 16; ++s) wf2[s] = *reinterpret_cast<const V8*>(p2 + s * 512);
            const T* p3 = a.w3[g] + (static_cast<size_t>(nt * 36 + kh * 18) * 64 + lane) * 8;
#pragma unroll
            for (int s = 0; s < 18; ++s) wf3[s] = *reinterpret_cast<const V8*>(p3 + s * 512);
            if (tid < 160) sB1[tid] = tid < 32 ? a.b1[g][tid] : (tid < 96 ? a.b2[g][tid - 32] : a.b3[g][tid - 96]);
#pragma unroll
            for (int q = 0; q < 4; ++q) bq[q] = *reinterpret_cast<const float4*>(a.b1[g] + 8 * q + 4 * kg);
        }
        {   // sX was last read by conv1 of the previous item, which every wavefront has left
            uint4* d = reinterpret_cast<uint4*>(sX);
            d[tid] = xv0; d[tid + 256] = xv1; d[tid + 512] = xv2; d[tid + 768] = xv3;
            d[tid + 1024] = xv4; d[tid + 1280] = xv5; d[last_vec] = xv6;   // clamped lanes rewrite the last vector with itself
        }
        if (it + 1 < last) {   // the next item's state: in flight while this item computes
            if (b + 1 < a.n) DQN_TOWER_FETCH_STATE(g, b + 1) else DQN_TOWER_FETCH_STATE(g + 1, 0)
        }
        __syncthreads();

        // ---- conv1: k = (c, p, q); k-step s covers c = s / 4, p = 2 * (s % 4) + kg, q = 0..7 -------------
        {
            T* g1 = a.act1[g];
            const uint8_t* xb = sX;
            constexpr int D = 6;   // k-steps of LDS reads in flight
            auto run = [&](auto nt_) {
                constexpr int NT = decltype(nt_)::value;   // pixel tiles of this wavefront: w, w + 4, ...
                const uint8_t* base[NT];
                f32x16 acc[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int px = (wave + 4 * t) * 32 + lp;
                    const int pc = px < 400 ? px : 399;
                    base[t] = xb + (4 * (pc / 20) + kg) * 84 + 4 * (pc % 20);
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
                }
                auto fetch = [&](int step) {
                    const int t = step / 16, k = step % 16;
                    const uint32_t* wp = reinterpret_cast<const uint32_t*>(base[t] + (k / 4) * 7056 + ((k % 4) * 2) * 84);
                    return make_uint2(wp[0], wp[1]);
                };
                uint2 ring[D];
#pragma unroll
                for (int u = 0; u < D; ++u) ring[u] = fetch(u);
#pragma unroll
                for (int step = 0; step < NT * 16; ++step) {
                    const int t = step / 16, k = step % 16;
                    const uint2 cur = ring[step % D];
                    if (step + D < NT * 16) ring[step % D] = fetch(step + D);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf1[k], bytes_as_f16_subnormals(cur.x, cur.y), acc[t], 0, 0, 0);
                    if (t > 0 && k % 4 == 1) conv1_store_quad(wave + 4 * (t - 1), acc[t - 1], k / 4, g1, b);   // previous tile's output
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) conv1_store_quad(wave + 4 * (NT - 1), acc[NT - 1], q, g1, b);
            };
            if (wave == 0) run(std::integral_constant<int, 4>{}); else run(std::integral_constant<int, 3>{});   // tile 12 is w = 0's
        }
        __syncthreads();

        // ---- conv2: k = (p, q, c); k-step ks covers tap ks / 2, channels 16 * (ks % 2) + 8 * kg .. + 7 ------
        {
            f32x16 acc[3];
            const T* base[3];
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                const int px = t * 32 + lp;
                const int pc = px < 81 ? px : 80;
                const int i = pc / 9, j = pc % 9;
                base[t] = sA1 + ((2 * i) * 20 + 2 * j) * kTowerP1 + kg * 8 + kh * (2 * 20 * kTowerP1);
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
            }
            // k-step ks = 16 * kh + k: tap (p, q) = (2 * kh + k / 8, (k / 2) % 4), channels 16 * (k % 2) + 8 * kg .. + 7
            {
                constexpr int D = 6;
                auto fetch = [&](int step) {
                    const int t = step / 16, k = step % 16;
                    return *reinterpret_cast<const V8*>(base[t] + ((k >> 3) * 20 + ((k >> 1) & 3)) * kTowerP1 + (k & 1) * 16);
                };
                V8 ring[D];
#pragma unroll
                for (int u = 0; u < D; ++u) ring[u] = fetch(u);
#pragma unroll
                for (int step = 0; step < 48; ++step) {
                    const int t = step / 16, k = step % 16;
                    const V8 cur = ring[step % D];
                    if (step + D < 48) ring[step % D] = fetch(step + D);
                    mma_32x32x16(acc[t], wf2[k], cur);
                    if (t > 0 && k == 2) {   // the previous tile's rows for the other k-half
                        if (kh) tower_hand_over<1>(red[wave][t - 1], acc[t - 1], lane); else tower_hand_over<0>(red[wave][t - 1], acc[t - 1], lane);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (kh) tower_hand_over<1>(red[wave][2], acc[2], lane); else tower_hand_over<0>(red[wave][2], acc[2], lane);
            }
            __syncthreads();
            float4 other[3][2], bv[2];
#pragma unroll
            for (int t = 0; t < 3; ++t)
#pragma unroll
                for (int h = 0; h < 2; ++h) other[t][h] = red[wave ^ 1][t][lane][h];
#pragma unroll
            for (int h = 0; h < 2; ++h) bv[h] = *reinterpret_cast<const float4*>(sB2 + nt * 32 + 8 * (2 * kh + h) + 4 * kg);
            __builtin_amdgcn_sched_barrier(0);
            T* g2 = a.act2[g];
            float4 v[3][2];
            if (kh) {
#pragma unroll
                for (int t = 0; t < 3; ++t)
#pragma unroll
                    for (int h = 0; h < 2; ++h) v[t][h] = tower_finish<1>(acc[t], h, other[t][h], bv[h]);
            } else {
#pragma unroll
                for (int t = 0; t < 3; ++t)
#pragma unroll
                    for (int h = 0; h < 2; ++h) v[t][h] = tower_finish<0>(acc[t], h, other[t][h], bv[h]);
            }
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                const int px = t * 32 + lp;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int ch = nt * 32 + 8 * (2 * kh + h) + 4 * kg;
                    if (px < 81) {
                        store4<T>(sA2 + px * kTowerP2 + ch, v[t][h].x, v[t][h].y, v[t][h].z, v[t][h].w);
                        if (g2) store4<T>(g2 + (static_cast<size_t>(b) * 81 + px) * 64 + ch, v[t][h].x, v[t][h].y, v[t][h].z, v[t][h].w);
                    }
                }
            }
        }
        __syncthreads();

        // ---- conv3: k = (p, q, c); k-step ks covers tap ks / 4, channels 16 * (ks % 4) + 8 * kg .. + 7 -----
        {
            f32x16 acc[2];
            const T* base[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int px = t * 32 + lp;
                const int pc = px < 49 ? px : 48;
                base[t] = sA2 + ((pc / 7) * 9 + pc % 7) * kTowerP2 + kg * 8;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
            }
            {
                constexpr int D = 6;
                auto fetch = [&](int step) {   // k-step 18 * kh + k; both candidate offsets are compile-time constants
                    const int t = step / 18, k = step % 18;
                    return *reinterpret_cast<const V8*>(base[t] + (kh ? tower_conv3_offset(18 + k) : tower_conv3_offset(k)));
                };
                V8 ring[D];
#pragma unroll
                for (int u = 0; u < D; ++u) ring[u] = fetch(u);
#pragma unroll
                for (int step = 0; step < 36; ++step) {
                    const int t = step / 18, k = step % 18;
                    const V8 cur = ring[step % D];
                    if (step + D < 36) ring[step % D] = fetch(step + D);
                    mma_32x32x16(acc[t], wf3[k], cur);
                    if (t > 0 && k == 2) {
                        if (kh) tower_hand_over<1>(red[wave][0], acc[0], lane); else tower_hand_over<0>(red[wave][0], acc[0], lane);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (kh) tower_hand_over<1>(red[wave][1], acc[1], lane); else tower_hand_over<0>(red[wave][1], acc[1], lane);
            }
            __syncthreads();
            float4 other[2][2], bv[2];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int h = 0; h < 2; ++h) other[t][h] = red[wave ^ 1][t][lane][h];
#pragma unroll
            for (int h = 0; h < 2; ++h) bv[h] = *reinterpret_cast<const float4*>(sB3 + nt * 32 + 8 * (2 * kh + h) + 4 * kg);
            __builtin_amdgcn_sched_barrier(0);
            float4 v[2][2];
            if (kh) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int h = 0; h < 2; ++h) v[t][h] = tower_finish<1>(acc[t], h, other[t][h], bv[h]);
            } else {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int h = 0; h < 2; ++h) v[t][h] = tower_finish<0>(acc[t], h, other[t][h], bv[h]);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int px = t * 32 + lp;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int ch = nt * 32 + 8 * (2 * kh + h) + 4 * kg;
                    if (px < 49) store4<T>(a.act3[g] + (static_cast<size_t>(b) * 49 + px) * 64 + ch, v[t][h].x, v[t][h].y, v[t][h].z, v[t][h].w);
                }
            }
        }
        // no barrier here: what the next item writes first (conv1's output, after its opening barrier) was last
        // read before barriers that every wavefront has passed by then
    }
#undef DQN_TOWER_FETCH_STATE
}

}  // namespace dqn
