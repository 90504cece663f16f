// Fused conv1 -> conv2 -> conv3 for small batches: one workgroup (8 wavefronts) per sample, the
// activations of conv1 and conv2 never leave LDS (25.6 KB + 10.4 KB in bf16 out of the 160 KB of a
// compute unit).  At batch 32 / W = 8 a layer-by-layer pass is three dependent launches of ~5 us each,
// most of it launch and cross-die memory latency; fused, the three layers cost about one of them.
//
// conv1: 13 tiles of 32 pixels, wavefront w takes tiles w and w + 8; pixels come straight from the
//        uint8 state in global memory, the 16 KB of weights live in each wavefront's registers.
// conv2: 3 pixel tiles; wavefront (kq, nt) owns k-quarter kq and 32-channel tile nt, keeps its weight
//        fragments in registers (requested before conv1 starts), reads pixel fragments from the LDS copy
//        of conv1's output; the four k-partials of a tile meet in LDS and are added in kq order.
// conv3: same scheme over 2 pixel tiles, output to global memory (the input of fc1).
// act1 / act2 are also written to global memory when the backward pass will need them.
#pragma once
#include "conv_ws.h"

namespace dqn {

template <typename T> struct TowerArgs {
    const uint8_t* x[kMaxGroups];
    const T* w1[kMaxGroups];
    const T* w2[kMaxGroups];
    const T* w3[kMaxGroups];
    const float* b1[kMaxGroups];
    const float* b2[kMaxGroups];
    const float* b3[kMaxGroups];
    T* act1[kMaxGroups];   // [n][400][32] or null
    T* act2[kMaxGroups];   // [n][81][64] or null
    T* act3[kMaxGroups];   // [n][49][64]
};

constexpr int kTowerP1 = 40, kTowerP2 = 72;   // LDS pixel pitch (elements) of conv1 / conv2 outputs
template <typename T> constexpr size_t conv_tower_smem()
{
    return (static_cast<size_t>(400) * kTowerP1 + 81 * kTowerP2) * sizeof(T) + 4 * 2 * 16 * 64 * sizeof(float);
}

template <typename T>
__global__ __launch_bounds__(512) void conv_tower_kernel(TowerArgs<T> a)
{
    typedef typename Vec8<T>::type V8;
    extern __shared__ __attribute__((aligned(32))) unsigned char tw_smem[];
    T* sA1 = reinterpret_cast<T*>(tw_smem);
    T* sA2 = sA1 + 400 * kTowerP1;
    float (*red)[2][16][64] = reinterpret_cast<float (*)[2][16][64]>(sA2 + 81 * kTowerP2);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = blockIdx.x, g = blockIdx.y;
    const int lp = lane & 31, kg = lane >> 5;
    const int kq = wave & 3, nt = wave >> 2;

    // weight fragments: conv1 (all of K), conv2 and conv3 (this wavefront's k-quarter and channel tile)
    V8 wf1[16], wf2[8], wf3[9];
    {
        const T* p1 = a.w1[g] + static_cast<size_t>(lp) * 256 + kg * 8;
#pragma unroll
        for (int s = 0; s < 16; ++s) wf1[s] = *reinterpret_cast<const V8*>(p1 + s * 16);
    }
    // conv1 pixel fragments of both tiles, straight from the uint8 state
    const uint8_t* xs = a.x[g] + static_cast<size_t>(b) * 28224;
    uint2 pf[2][16];   // raw bytes; converted to the operand type right before use
    int px1[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int tile = wave + 8 * t;
        px1[t] = tile * 32 + lp;
        const int pc = px1[t] < 400 ? px1[t] : 0;
        const int i = pc / 20, j = pc % 20;
        const uint8_t* base = xs + (4 * i + kg) * 84 + 4 * j;
#pragma unroll
        for (int s = 0; s < 16; ++s)
            if (tile < 13) {
                const uint32_t* wp = reinterpret_cast<const uint32_t*>(base + (s / 4) * 7056 + ((s % 4) * 2) * 84);
                pf[t][s] = make_uint2(wp[0], wp[1]);
            }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- conv1 ------------------------------------------------------------------------------------
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int tile = wave + 8 * t;
        if (tile < 13) {
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int s = 0; s < 16; ++s) mma_32x32x16(acc, wf1[s], vec8_from_u8<T>(pf[t][s].x, pf[t][s].y));
            if (t == 1 || wave + 8 >= 13) {
                // last conv1 tile of this wavefront: request the conv2 / conv3 weight fragments now, so that
                // their latency hides behind the epilogue and the barrier
                const T* p2 = a.w2[g] + static_cast<size_t>(nt * 32 + lp) * 512 + kq * 128 + kg * 8;
#pragma unroll
                for (int s = 0; s < 8; ++s) wf2[s] = *reinterpret_cast<const V8*>(p2 + s * 16);
                const T* p3 = a.w3[g] + static_cast<size_t>(nt * 32 + lp) * 576 + kq * 144 + kg * 8;
#pragma unroll
                for (int s = 0; s < 9; ++s) wf3[s] = *reinterpret_cast<const V8*>(p3 + s * 16);
            }
            if (px1[t] < 400) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int ch = 8 * q + 4 * kg;
                    const float4 bv = *reinterpret_cast<const float4*>(a.b1[g] + ch);
                    const float v0 = fmaxf(acc[4 * q] * (1.f / 255.f) + bv.x, 0.f), v1 = fmaxf(acc[4 * q + 1] * (1.f / 255.f) + bv.y, 0.f);
                    const float v2 = fmaxf(acc[4 * q + 2] * (1.f / 255.f) + bv.z, 0.f), v3 = fmaxf(acc[4 * q + 3] * (1.f / 255.f) + bv.w, 0.f);
                    store4<T>(sA1 + px1[t] * kTowerP1 + ch, v0, v1, v2, v3);
                    if (a.act1[g]) store4<T>(a.act1[g] + (static_cast<size_t>(b) * 400 + px1[t]) * 32 + ch, v0, v1, v2, v3);
                }
            }
        }
    }
    __syncthreads();

    // ---- conv2: 81 pixels = 3 tiles, k-quarter kq (8 k-steps), channel tile nt ---------------------------
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        const int px = t * 32 + lp;
        const int pc = px < 81 ? px : 0;
        const int i = pc / 9, j = pc % 9;
        const T* base = sA1 + ((2 * i) * 20 + 2 * j) * kTowerP1 + kg * 8;
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int pq = kq * 4 + s / 2;           // filter tap (p, q) = (pq / 4, pq % 4); channels (s % 2) * 16 + kg * 8
            const V8 f = *reinterpret_cast<const V8*>(base + ((pq >> 2) * 20 + (pq & 3)) * kTowerP1 + (s & 1) * 16);
            mma_32x32x16(acc, wf2[s], f);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) red[kq][nt][v][lane] = acc[v];
        __syncthreads();
        {   // wavefront (kq, nt) finishes quad kq of channel tile nt
            const int q = kq, ch = nt * 32 + 8 * q + 4 * kg;
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                v[e] = ((red[0][nt][4 * q + e][lane] + red[1][nt][4 * q + e][lane]) + red[2][nt][4 * q + e][lane]) + red[3][nt][4 * q + e][lane];
            if (px < 81) {
                const float4 bv = *reinterpret_cast<const float4*>(a.b2[g] + ch);
                v[0] = fmaxf(v[0] + bv.x, 0.f); v[1] = fmaxf(v[1] + bv.y, 0.f);
                v[2] = fmaxf(v[2] + bv.z, 0.f); v[3] = fmaxf(v[3] + bv.w, 0.f);
                store4<T>(sA2 + px * kTowerP2 + ch, v[0], v[1], v[2], v[3]);
                if (a.act2[g]) store4<T>(a.act2[g] + (static_cast<size_t>(b) * 81 + px) * 64 + ch, v[0], v[1], v[2], v[3]);
            }
        }
        __syncthreads();
    }

    // ---- conv3: 49 pixels = 2 tiles, k-quarter kq (9 k-steps), channel tile nt ---------------------------
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int px = t * 32 + lp;
        const int pc = px < 49 ? px : 0;
        const int i = pc / 7, j = pc % 7;
        const T* base = sA2 + (i * 9 + j) * kTowerP2 + kg * 8;
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < 9; ++s) {
            const int ks = kq * 9 + s;               // runtime k-step: tap ks / 4, channels (ks % 4) * 16 + kg * 8
            const int pq = ks >> 2;
            const V8 f = *reinterpret_cast<const V8*>(base + ((pq / 3) * 9 + pq % 3) * kTowerP2 + (ks & 3) * 16);
            mma_32x32x16(acc, wf3[s], f);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) red[kq][nt][v][lane] = acc[v];
        __syncthreads();
        {
            const int q = kq, ch = nt * 32 + 8 * q + 4 * kg;
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                v[e] = ((red[0][nt][4 * q + e][lane] + red[1][nt][4 * q + e][lane]) + red[2][nt][4 * q + e][lane]) + red[3][nt][4 * q + e][lane];
            if (px < 49) {
                const float4 bv = *reinterpret_cast<const float4*>(a.b3[g] + ch);
                store4<T>(a.act3[g] + (static_cast<size_t>(b) * 49 + px) * 64 + ch, fmaxf(v[0] + bv.x, 0.f), fmaxf(v[1] + bv.y, 0.f),
                          fmaxf(v[2] + bv.z, 0.f), fmaxf(v[3] + bv.w, 0.f));
            }
        }
        __syncthreads();
    }
}

}  // namespace dqn
