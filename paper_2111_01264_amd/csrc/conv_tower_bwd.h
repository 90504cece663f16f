// Fused data-gradient chain conv3 -> conv2 of the Q-network's backward pass (Section 2.1, Eq. 1: the gradient of
// the TD loss with respect to theta needs dLoss/d(activation) of every layer), reduced-precision mode: the mirror
// image of conv_tower.h.  A persistent workgroup of 8 wavefronts walks a contiguous range of samples; per sample
//
//   dz2[y][x][c] = [act2 > 0] * sum_{p,q,o} dz3[y-p][x-q][o]   * W3[o][p][q][c]          (9x9x64 from 7x7x64, 3x3 taps)
//   dz1[y][x][c] = [act1 > 0] * sum_{p,q,o} dz2[(y-p)/2][(x-q)/2][o] * W2[o][p][q][c]    (20x20x32 from 9x9x64, stride 2)
//
// dz3 and dz2 live in LDS as zero-bordered 11x11 images, so "outside the image" needs no test; the stride-2
// layer is four stride-1 problems, one per parity class (py, px) of the output pixel, each with the 2x2 taps of
// that parity.  Weights come from the backward operand copies, stored in MFMA fragment order (see
// tower_frag_index) and held in registers: wavefront (nt, kq) owns channel tile nt and k-quarter kq of conv3's
// 64 x 576 matrix (36 VGPRs), wavefront (class, kh) owns k-half kh of that class's 32 x 256 matrix (32 VGPRs).
// k-quarters / k-halves meet through the LDS exchange block, added in k order.  dz2 also goes to global memory
// (the weight gradient of conv2 reads it), dz1 only there.
#pragma once
#include "conv_tower.h"

namespace dqn {

struct TowerBwdArgs {
    const bf16_t* dz3;    // [n][49][64], already through conv3's ReLU mask
    const bf16_t* act2;   // [n][81][64]
    const bf16_t* act1;   // [n][400][32]
    const bf16_t* w3d;    // fragment order of [c 64][k = (p, q, o) 576]
    const bf16_t* w2d;    // four classes, each fragment order of [c 32][k = (p2, q2, o) 256]
    bf16_t* dz2;          // [n][81][64]
    bf16_t* dz1;          // [n][400][32]
    int n, per;           // samples, samples per workgroup
};

constexpr int kTbPitch = 72;                          // elements per pixel of the padded LDS images
constexpr int kTbImg = 11 * 11 * kTbPitch;            // one padded image
constexpr size_t kTowerBwdSmem = kTowerXchgBytes + 2 * kTbImg * 2;

// Sum of the four k-quarters' rows 4 * KQ .. + 3 (no bias, no activation); layout as tower_send.
template <int KQ> __device__ inline float4 tower_sum(const float4* x, const f32x16& acc, int lane)
{
    asm volatile("; sum, k-quarter %0" ::"n"(KQ));
    float4 p[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        p[s] = s == KQ ? make_float4(acc[4 * KQ], acc[4 * KQ + 1], acc[4 * KQ + 2], acc[4 * KQ + 3])
                       : x[(KQ * 3 + (s < KQ ? s : s - 1)) * 64 + lane];
    float4 r;
    r.x = ((p[0].x + p[1].x) + p[2].x) + p[3].x;
    r.y = ((p[0].y + p[1].y) + p[2].y) + p[3].y;
    r.z = ((p[0].z + p[1].z) + p[2].z) + p[3].z;
    r.w = ((p[0].w + p[1].w) + p[2].w) + p[3].w;
    asm volatile("; summed, k-quarter %0" ::"n"(KQ) : "memory");
    return r;
}

// Two k-halves: half KH keeps accumulator rows 8 * KH .. + 7 and hands the other eight to its partner.
template <int KH> __device__ inline void tower_send_half(float4* mine /* [64 lanes][2] */, const f32x16& acc, int lane)
{
    asm volatile("; send, k-half %0" ::"n"(KH));
    constexpr int r = 8 * (1 - KH);
#pragma unroll
    for (int h = 0; h < 2; ++h)
        mine[lane * 2 + h] = make_float4(acc[r + 4 * h], acc[r + 4 * h + 1], acc[r + 4 * h + 2], acc[r + 4 * h + 3]);
    asm volatile("; sent, k-half %0" ::"n"(KH) : "memory");
}
template <int KH> __device__ inline float4 tower_sum_half(const float4* theirs, const f32x16& acc, int lane, int h)
{
    asm volatile("; sum, k-half %0" ::"n"(KH));
    const int r = 8 * KH + 4 * h;
    const float4 o = theirs[lane * 2 + h];
    // (k-half 0) + (k-half 1): addition commutes exactly, so both halves produce the same bits either way
    const float4 v = make_float4(acc[r] + o.x, acc[r + 1] + o.y, acc[r + 2] + o.z, acc[r + 3] + o.w);
    asm volatile("; summed, k-half %0" ::"n"(KH) : "memory");
    return v;
}

// The arguments are TowerBwdArgs' fields one by one, in the order a workgroup needs them: the first 14 dwords of the
// kernel arguments are preloaded into scalar registers when a wavefront starts (see conv_tower_kernel).
//
// PARTS = 5: an item is a FIFTH of a sample -- rows 2 j, 2 j + 1 of every parity class of dz1 (four rows of dz1) with the
// two or three rows of dz2 they depend on -- and every workgroup runs exactly one item: one pixel tile per stage instead of
// three and four.  For minibatches that leave most of the chip idle (see conv_tower_kernel's PARTS); every element is
// computed by the same instructions in the same order as with PARTS = 1, rows of dz2 that two parts need are computed and
// stored by both.
template <int PARTS>
__global__ __launch_bounds__(kTowerThreads) void conv_tower_bwd_kernel(int n_, int per_, const bf16_t* dz3_, const bf16_t* w3d_, const bf16_t* w2d_,
                                                                       const bf16_t* act2_, const bf16_t* act1_, bf16_t* dz2_, bf16_t* dz1_)
{
    typedef bf16_t T;
    typedef bf16x8 V8;
    extern __shared__ __attribute__((aligned(16))) unsigned char tb_smem[];
    float4* sXchg = reinterpret_cast<float4*>(tb_smem);
    T* sP3 = reinterpret_cast<T*>(tb_smem + kTowerXchgBytes);   // dz3, 7x7 at offset (2, 2) of an 11x11 image
    T* sP2 = sP3 + kTbImg;                                      // dz2, 9x9 at offset (1, 1)

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lp = lane & 31, kg = lane >> 5;
    const int nt = wave >> 2, kq = wave & 3;     // conv3 stage
    const int cls = wave >> 1, kh = wave & 1;    // conv2 stage: class (py, px) = (cls >> 1, cls & 1)
    static_assert(PARTS == 1 || PARTS == 5, "whole samples, or fifths");
    const int part = PARTS == 1 ? 0 : static_cast<int>(blockIdx.x % PARTS);
    const int first = PARTS == 1 ? blockIdx.x * per_ : static_cast<int>(blockIdx.x / PARTS), last = PARTS == 1 ? min(n_, first + per_) : min(n_, first + 1);
    if (first >= last) return;
    // this part's rows: [y_lo, y_lo + 2) of each parity class of dz1 (20 pixels), rows [r2_lo, y_lo + 2) of dz2
    const int y_lo = PARTS == 1 ? 0 : 2 * part, nc = PARTS == 1 ? 100 : 20;
    const int r2_lo = PARTS == 1 ? 0 : (part == 0 ? 0 : 2 * part - 1), n2 = PARTS == 1 ? 81 : (part == 0 || part == 4 ? 18 : 27);   // rows 2 part - 1 .. 2 part + 1 of dz2's nine
    constexpr int T3 = PARTS == 1 ? 3 : 1, T2 = PARTS == 1 ? 4 : 1;   // pixel tiles per wavefront: conv3 stage, conv2 stage

    // a sample's dz3: 49 pixels x 128 bytes = 392 vectors, one per thread, fetched one sample ahead.  The first sample's is
    // requested before the weights: loads return in order, and behind 139 KB of fragments the staging below waited ~1 us
    uint4 xv = make_uint4(0, 0, 0, 0);
    if (tid < 392) xv = reinterpret_cast<const uint4*>(dz3_ + static_cast<size_t>(first) * 3136)[tid];
    __builtin_amdgcn_sched_barrier(0);

    // zero both images once: the borders are never written again
    for (int v = tid; v < 2 * kTbImg / 8; v += kTowerThreads) reinterpret_cast<uint4*>(sP3)[v] = make_uint4(0, 0, 0, 0);

    V8 wf3[9], wf2[8];
    {
        const T* p3 = w3d_ + (static_cast<size_t>(nt * 36 + kq * 9) * 64 + lane) * 8;
#pragma unroll
        for (int k = 0; k < 9; ++k) wf3[k] = *reinterpret_cast<const V8*>(p3 + k * 512);
        const T* p2 = w2d_ + static_cast<size_t>(cls) * 32 * 256 + (static_cast<size_t>(kh * 8) * 64 + lane) * 8;
#pragma unroll
        for (int k = 0; k < 8; ++k) wf2[k] = *reinterpret_cast<const V8*>(p2 + k * 512);
    }
    // conv3 stage, k-step 9 * kq + k: tap (p, q) = (ks / 4 / 3, ks / 4 % 3), channels 16 * (ks % 4) + 8 * kg .. + 7 of
    // dz3 at (y - p, x - q): element offset relative to the pixel's own position in the padded image
    int off3[9];   // plain scalar arithmetic: a choice between per-quarter constants compiles to a chain of branches
#pragma unroll
    for (int k = 0; k < 9; ++k) {
        const int ks = 9 * kq + k, tap = ks >> 2, p = (tap * 11) >> 5 /* tap / 3 for tap <= 8 */, q = tap - 3 * p;
        off3[k] = -((p * 11 + q) * kTbPitch) + (ks & 3) * 16;
    }

    const int my_px = tid >> 3, my_part = tid & 7;
    const int my_dst = (((my_px / 7) + 2) * 11 + (my_px % 7) + 2) * kTbPitch + my_part * 8;
    __syncthreads();   // the zero fill is complete

    for (int b = first; b < last; ++b) {
        if (tid < 392) *reinterpret_cast<uint4*>(sP3 + my_dst) = xv;
        if (b + 1 < last && tid < 392) xv = reinterpret_cast<const uint4*>(dz3_ + static_cast<size_t>(b + 1) * 3136)[tid];
        // ReLU masks of both stages: requested now, used after the exchanges
        uint2 m2[T3], m1[T2][2];
        {
            const int ch = nt * 32 + 8 * kq + 4 * kg;
#pragma unroll
            for (int t = 0; t < T3; ++t) {
                const int lpx = t * 32 + lp;
                m2[t] = *reinterpret_cast<const uint2*>(act2_ + (static_cast<size_t>(b) * 81 + r2_lo * 9 + (lpx < n2 ? lpx : n2 - 1)) * 64 + ch);
            }
#pragma unroll
            for (int t = 0; t < T2; ++t) {
                const int lpx = t * 32 + lp, pc = y_lo * 10 + (lpx < nc ? lpx : nc - 1);
                const int pix = (2 * (pc / 10) + (cls >> 1)) * 20 + 2 * (pc % 10) + (cls & 1);
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    m1[t][h] = *reinterpret_cast<const uint2*>(act1_ + (static_cast<size_t>(b) * 400 + pix) * 32 + 8 * (2 * kh + h) + 4 * kg);
            }
        }
        __syncthreads();

        // ---- conv3 data gradient: 81 pixels = 3 tiles, channel tile nt, k-quarter kq (9 k-steps) ------------
        {
            f32x16 acc[T3];
            const T* base[T3];
#pragma unroll
            for (int t = 0; t < T3; ++t) {
                const int lpx = t * 32 + lp, pc = r2_lo * 9 + (lpx < n2 ? lpx : n2 - 1);
                base[t] = sP3 + ((pc / 9 + 2) * 11 + pc % 9 + 2) * kTbPitch + kg * 8;
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
#pragma unroll
            for (int t = 0; t < T3; ++t) {
                const float4* x = xc + t * (4 * 3 * 64);
                float4 v;
                if (kq == 0) v = tower_sum<0>(x, acc[t], lane); else if (kq == 1) v = tower_sum<1>(x, acc[t], lane);
                else if (kq == 2) v = tower_sum<2>(x, acc[t], lane); else v = tower_sum<3>(x, acc[t], lane);
                const int lpx = t * 32 + lp, px = r2_lo * 9 + lpx;
                if (lpx < n2) {
                    // ReLU mask: a bf16 activation is positive iff its bit pattern is in 0x0001 .. 0x7FFF (no NaNs here)
                    const uint32_t lo = m2[t].x, hi = m2[t].y;
                    const float v0 = static_cast<int16_t>(lo & 0xFFFF) > 0 ? v.x : 0.f, v1 = static_cast<int16_t>(lo >> 16) > 0 ? v.y : 0.f;
                    const float v2 = static_cast<int16_t>(hi & 0xFFFF) > 0 ? v.z : 0.f, v3 = static_cast<int16_t>(hi >> 16) > 0 ? v.w : 0.f;
                    store4<T>(sP2 + ((px / 9 + 1) * 11 + px % 9 + 1) * kTbPitch + ch, v0, v1, v2, v3);
                    store4<T>(dz2_ + (static_cast<size_t>(b) * 81 + px) * 64 + ch, v0, v1, v2, v3);
                }
            }
        }
        __syncthreads();

        // ---- conv2 data gradient: class (py, px), 100 pixels = 4 tiles, k-half kh (8 k-steps) --------------------
        {
            f32x16 acc[T2];
            const T* base[T2];
#pragma unroll
            for (int t = 0; t < T2; ++t) {
                const int lpx = t * 32 + lp, pc = y_lo * 10 + (lpx < nc ? lpx : nc - 1);
                // k-step 8 * kh + k: tap (p2, q2) = (kh, k / 4), channels 16 * (k % 4) + 8 * kg .. + 7 of dz2 at (y2 - p2, x2 - q2)
                base[t] = sP2 + ((pc / 10 + 1 - kh) * 11 + pc % 10 + 1) * kTbPitch + kg * 8;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
            }
            {
                constexpr int D = 6;
                auto fetch = [&](int step) {
                    const int t = step / 8, k = step % 8;
                    return *reinterpret_cast<const V8*>(base[t] - (k >> 2) * kTbPitch + (k & 3) * 16);
                };
                V8 ring[D];
#pragma unroll
                for (int u = 0; u < D; ++u) ring[u] = fetch(u);
#pragma unroll
                for (int step = 0; step < 8 * T2; ++step) {
                    const V8 cur = ring[step % D];
                    if (step + D < 8 * T2) ring[step % D] = fetch(step + D);
                    mma_32x32x16(acc[step / 8], wf2[step % 8], cur);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // exchange block reused as [wavefront][tile][lane][2] float4 (64 KB); conv3's readers are behind the barrier above
            float4* mine = sXchg + static_cast<size_t>(wave) * (4 * 64 * 2);
            const float4* theirs = sXchg + static_cast<size_t>(wave ^ 1) * (4 * 64 * 2);
#pragma unroll
            for (int t = 0; t < T2; ++t) {
                if (kh) tower_send_half<1>(mine + t * 128, acc[t], lane); else tower_send_half<0>(mine + t * 128, acc[t], lane);
            }
            __syncthreads();
#pragma unroll
            for (int t = 0; t < T2; ++t) {
                const int lpx = t * 32 + lp, px = y_lo * 10 + lpx;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float4 v;
                    if (kh) v = tower_sum_half<1>(theirs + t * 128, acc[t], lane, h); else v = tower_sum_half<0>(theirs + t * 128, acc[t], lane, h);
                    if (lpx < nc) {
                        const int pix = (2 * (px / 10) + (cls >> 1)) * 20 + 2 * (px % 10) + (cls & 1);
                        const uint32_t lo = m1[t][h].x, hi = m1[t][h].y;
                        store4<T>(dz1_ + (static_cast<size_t>(b) * 400 + pix) * 32 + 8 * (2 * kh + h) + 4 * kg,
                                  static_cast<int16_t>(lo & 0xFFFF) > 0 ? v.x : 0.f, static_cast<int16_t>(lo >> 16) > 0 ? v.y : 0.f,
                                  static_cast<int16_t>(hi & 0xFFFF) > 0 ? v.z : 0.f, static_cast<int16_t>(hi >> 16) > 0 ? v.w : 0.f);
                    }
                }
            }
        }
        // no barrier here: the next sample's first writes to the images and the exchange block sit behind its own barriers
    }
}

}  // namespace dqn
