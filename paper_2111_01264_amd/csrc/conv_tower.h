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
//   * the 28 KB uint8 state goes from global memory straight into LDS (16 bytes per lane, no registers in
//     between), double-buffered: the next item's state is requested as soon as this item's has landed;
//     conv1's pixel fragments come from LDS;
//   * the wavefronts hold disjoint (channel tile, k-half) parts of conv2's and conv3's weights, and all of
//     conv1's (64 + 64 + 72 VGPRs per lane);
//   * with one wavefront per SIMD nothing else hides LDS latency, so every phase first issues all of its
//     LDS reads and only then starts on the matrix core, two or three independent accumulators at a time.
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
template <int KH, int TILES> __device__ inline void tower_hand_over(float4 (*mine)[64][2], const f32x16* acc, int lane)
{
    asm volatile("; hand over, k-half %0" ::"n"(KH));
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            constexpr int r = 8 * (1 - KH);
            mine[t][lane][h] = make_float4(acc[t][r + 4 * h], acc[t][r + 4 * h + 1], acc[t][r + 4 * h + 2], acc[t][r + 4 * h + 3]);
        }
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
};

constexpr int kTowerP1 = 40, kTowerP2 = 72;   // LDS pixel pitch (elements) of conv1 / conv2 outputs
constexpr int kTowerXBytes = 4 * 84 * 84;     // 28,224 = 27 x 1024 + 576
constexpr int kTowerThreads = 256;            // the index arithmetic below assumes exactly this block size
constexpr size_t kTowerSmem = 2 * kTowerXBytes + 400 * kTowerP1 * 2 + 81 * kTowerP2 * 2 + 4 * 3 * 64 * 8 * 4 + 160 * 4;

__global__ __launch_bounds__(kTowerThreads) void conv_tower_kernel(TowerArgs a)
{
    typedef bf16_t T;
    typedef bf16x8 V8;
    extern __shared__ __attribute__((aligned(16))) unsigned char tw_smem[];
    uint8_t* sX = tw_smem;                                   // two state buffers
    T* sA1 = reinterpret_cast<T*>(tw_smem + 2 * kTowerXBytes);
    T* sA2 = sA1 + 400 * kTowerP1;
    float4 (*red)[3][64][2] = reinterpret_cast<float4 (*)[3][64][2]>(sA2 + 81 * kTowerP2);   // [wavefront][tile][lane][8 rows]
    float* sB1 = reinterpret_cast<float*>(red + 4);   // biases: conv1 [32], conv2 [64], conv3 [64]
    float* sB2 = sB1 + 32;
    float* sB3 = sB2 + 64;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lp = lane & 31, kg = lane >> 5;
    const int nt = wave >> 1, kh = wave & 1;
    const int total = a.n * a.groups;
    const int per = (total + gridDim.x - 1) / gridDim.x;
    const int first = blockIdx.x * per, last = min(total, first + per);
    if (first >= last) return;

    // Requests the state of item `it` into buffer `buf`: 1 KB per wavefront and instruction, lane l's 16 bytes
    // land at (LDS base of the instruction) + 16 * l.  Completion is waited for with vmcnt(0) before the
    // barrier that opens the item.
    auto request_state = [&](int it, int buf) {
        const int g = it / a.n, b = it - g * a.n;
        const uint8_t* src = a.x[g] + static_cast<size_t>(b) * kTowerXBytes;
        uint8_t* dst = sX + buf * kTowerXBytes;
#pragma unroll
        for (int c = 0; c < 7; ++c) {
            const int chunk = wave + 4 * c;          // 28 chunks, the last one 576 bytes
            const int off = chunk * 1024 + lane * 16;
            if (off < kTowerXBytes)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + off),
                                                 (__attribute__((address_space(3))) void*)(dst + chunk * 1024), 16, 0, 0);
        }
    };

    // conv1 output tile: scale, bias, ReLU -> LDS (+ global)
    auto conv1_store = [&](int tile, const f32x16& acc, T* g1, int b) {
        const int px = tile * 32 + lp;
        if (px < 400) {
            constexpr float kScale = 16777216.f / 255.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ch = 8 * q + 4 * kg;
                const float4 bv = *reinterpret_cast<const float4*>(sB1 + ch);
                const float v0 = fmaxf(acc[4 * q] * kScale + bv.x, 0.f), v1 = fmaxf(acc[4 * q + 1] * kScale + bv.y, 0.f);
                const float v2 = fmaxf(acc[4 * q + 2] * kScale + bv.z, 0.f), v3 = fmaxf(acc[4 * q + 3] * kScale + bv.w, 0.f);
                store4<T>(sA1 + px * kTowerP1 + ch, v0, v1, v2, v3);
                if (g1) store4<T>(g1 + (static_cast<size_t>(b) * 400 + px) * 32 + ch, v0, v1, v2, v3);
            }
        }
    };

    f16x8 wf1[16];
    V8 wf2[16], wf3[18];
    request_state(first, 0);
    int cur_g = -1;
    for (int it = first; it < last; ++it) {
        const int g = it / a.n, b = it - g * a.n;
        const int buf = (it - first) & 1;
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
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's part of the state is in LDS
        __syncthreads();                                     // ... and everybody else's
        // the other buffer was last read by conv1 of the previous item, which every wavefront has left
        if (it + 1 < last) request_state(it + 1, buf ^ 1);

        // ---- conv1: k = (c, p, q); k-step s covers c = s / 4, p = 2 * (s % 4) + kg, q = 0..7 -------------
        {
            T* g1 = a.act1[g];
            const uint8_t* xb = sX + buf * kTowerXBytes;
            auto load_tile = [&](int tile, uint2 (&raw)[16]) {
                const int px = tile * 32 + lp;
                const int pc = px < 400 ? px : 399;
                const uint8_t* base = xb + (4 * (pc / 20) + kg) * 84 + 4 * (pc % 20);
#pragma unroll
                for (int s = 0; s < 16; ++s) {
                    const uint32_t* wp = reinterpret_cast<const uint32_t*>(base + (s / 4) * 7056 + ((s % 4) * 2) * 84);
                    raw[s] = make_uint2(wp[0], wp[1]);
                }
            };
            {   // tiles w and w + 4
                uint2 r0[16], r1[16];
                load_tile(wave, r0);
                load_tile(wave + 4, r1);
                __builtin_amdgcn_sched_barrier(0);
                f32x16 acc0, acc1;
#pragma unroll
                for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
#pragma unroll
                for (int s = 0; s < 16; ++s) {
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf1[s], bytes_as_f16_subnormals(r0[s].x, r0[s].y), acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf1[s], bytes_as_f16_subnormals(r1[s].x, r1[s].y), acc1, 0, 0, 0);
                }
                conv1_store(wave, acc0, g1, b);
                conv1_store(wave + 4, acc1, g1, b);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (wave == 0) {   // tiles 8 and 12 (tile w + 12 exists for w = 0 only)
                uint2 r0[16], r1[16];
                load_tile(8, r0);
                load_tile(12, r1);
                __builtin_amdgcn_sched_barrier(0);
                f32x16 acc0, acc1;
#pragma unroll
                for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
#pragma unroll
                for (int s = 0; s < 16; ++s) {
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf1[s], bytes_as_f16_subnormals(r0[s].x, r0[s].y), acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf1[s], bytes_as_f16_subnormals(r1[s].x, r1[s].y), acc1, 0, 0, 0);
                }
                conv1_store(8, acc0, g1, b);
                conv1_store(12, acc1, g1, b);
            } else {           // tile w + 8
                uint2 r0[16];
                load_tile(wave + 8, r0);
                __builtin_amdgcn_sched_barrier(0);
                f32x16 acc0;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc0[v] = 0.f;
#pragma unroll
                for (int s = 0; s < 16; ++s)
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf1[s], bytes_as_f16_subnormals(r0[s].x, r0[s].y), acc0, 0, 0, 0);
                conv1_store(wave + 8, acc0, g1, b);
            }
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
            // ks = 16 * kh + s: tap (p, q) = (2 * kh + s / 8, (s / 2) % 4); tiles 0 and 1 first, then tile 2
            // (all three at once would not leave the register allocator enough room)
            {
                V8 f[2][16];
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int s = 0; s < 16; ++s)
                        f[t][s] = *reinterpret_cast<const V8*>(base[t] + ((s >> 3) * 20 + ((s >> 1) & 3)) * kTowerP1 + (s & 1) * 16);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < 16; ++s) {
                    mma_32x32x16(acc[0], wf2[s], f[0][s]);
                    mma_32x32x16(acc[1], wf2[s], f[1][s]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            {
                V8 f[16];
#pragma unroll
                for (int s = 0; s < 16; ++s)
                    f[s] = *reinterpret_cast<const V8*>(base[2] + ((s >> 3) * 20 + ((s >> 1) & 3)) * kTowerP1 + (s & 1) * 16);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < 16; ++s) mma_32x32x16(acc[2], wf2[s], f[s]);
            }
            if (kh) tower_hand_over<1, 3>(red[wave], acc, lane); else tower_hand_over<0, 3>(red[wave], acc, lane);
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
            V8 f[2][18];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int px = t * 32 + lp;
                const int pc = px < 49 ? px : 48;
                const int i = pc / 7, j = pc % 7;
                const T* base = sA2 + (i * 9 + j) * kTowerP2 + kg * 8;
#pragma unroll
                for (int s = 0; s < 18; ++s) {
                    const int ks = kh * 18 + s;   // wave-uniform
                    const int pq = ks >> 2;
                    f[t][s] = *reinterpret_cast<const V8*>(base + ((pq / 3) * 9 + pq % 3) * kTowerP2 + (ks & 3) * 16);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
#pragma unroll
            for (int s = 0; s < 18; ++s)
#pragma unroll
                for (int t = 0; t < 2; ++t) mma_32x32x16(acc[t], wf3[s], f[t][s]);
            if (kh) tower_hand_over<1, 2>(red[wave], acc, lane); else tower_hand_over<0, 2>(red[wave], acc, lane);
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
}

}  // namespace dqn
