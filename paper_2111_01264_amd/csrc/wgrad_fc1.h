// Weight gradient of fc1 (reduced precision):
//
//     dW[o][f] = sum_b dZ[b][o] * act3[b][f]            (Section 2.1: first-order minimisation with respect to theta)
//
// The contraction runs over the minibatch only, so a workgroup that owns a [64 x 128] tile of dW needs no split: both
// operands are stored k-major (dZ is [b][512], act3 is [b][3136]), staged as stored in chunks of 128 minibatch rows
// (lanes walk along a row: fully coalesced; a whole chunk's loads are in flight at once, the next chunk is requested
// before the current one is multiplied) and read with the transposing LDS read (gemm_tn_tr.h).  One barrier pair per
// 128 rows instead of one per 32: at batch 256 the tile costs two round trips to memory instead of eight.
// The accumulators (one column, sixteen rows per lane) go through LDS once more so that the gradient is written as
// 16-byte vectors, 512 contiguous bytes per row.
//
// Tried and dropped: applying the optimiser step to the tile right here (the workgroup has the final gradient, so theta,
// v, m could be read and written once and the gradient never read back).  Correct, but slower in sum: the optimiser
// kernel that remains (conv weights from their split-K slices, biases, fc2) takes about as long as before -- its time
// is the slice sums' chain of round trips, not the streaming of fc1.w -- while this kernel grows by the 60 MB it then
// moves (batch 32: 15.5 + 9.6 us against 12.1 + 12.7 us; batch 256: 28.3 + 13.8 against 19.8 + 17.3).
#pragma once
#include "gemm_tn_tr.h"
#include "head_kernels.h"
#include "wgrad_conv.h"

namespace dqn {

struct WgFc1Args {
    const bf16_t* dz;     // [B][512]
    const bf16_t* x;      // [B][3136] (act3; feature index (h*7+w)*64 + c)
    int B;
    float* grad;          // [512][3136] fp32, the device layout of fc1.w
};

constexpr int kWgF1BM = 64, kWgF1BN = 128, kWgF1KC = 128;
constexpr int kWgF1LDA = kWgF1BM + 16, kWgF1LDB = kWgF1BN + 16;
constexpr size_t kWgF1Smem = static_cast<size_t>(kWgF1KC) * (kWgF1LDA + kWgF1LDB) * 2;
constexpr int kWgF1Cols = (3136 + kWgF1BN - 1) / kWgF1BN, kWgF1Rows = 512 / kWgF1BM;   // 25 x 8 workgroups

// Workgroup (column block bx, row block bz); 256 threads; smem: kWgF1Smem bytes, 16-byte aligned.
__device__ inline void wgrad_fc1_block(const WgFc1Args& a, int bx, int bz, unsigned char* smem)
{
    constexpr int BM = kWgF1BM, BN = kWgF1BN, KC = kWgF1KC, LDA = kWgF1LDA, LDB = kWgF1LDB;
    constexpr int CVA = BM / 8, CVB = BN / 8;                      // 16-byte vectors per minibatch row
    constexpr int NA = KC * CVA / 256, NB = KC * CVB / 256;        // 4 + 8 vectors per thread and chunk
    constexpr int N = 3136;
    bf16_t* sA = reinterpret_cast<bf16_t*>(smem);
    bf16_t* sB = sA + KC * LDA;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m0 = bz * BM, n0 = bx * BN;
    const int B = a.B;

    // per-thread constants of its vectors: row inside the chunk, column part of the address, LDS slot
    const int ka = tid / CVA, ca = (tid % CVA) * 8;                // + 32 rows per further vector (256 / CVA)
    const int kb = tid / CVB, cbv = (tid % CVB) * 8;               // + 16 rows per further vector
    const bool okb = n0 + cbv < N;                                 // the last column block is half empty
    const bf16_t* pa = a.dz + m0 + ca;
    const bf16_t* pb = a.x + (okb ? n0 + cbv : 0);

    wg_u32x4 ra[NA], rb[NB];
    // rows past the minibatch repeat its last row (no load is skipped) and are zeroed when they are stored
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = *reinterpret_cast<const wg_u32x4*>(pa + static_cast<size_t>(min(k0 + ka + i * (256 / CVA), B - 1)) * 512);
#pragma unroll
        for (int i = 0; i < NB; ++i) rb[i] = *reinterpret_cast<const wg_u32x4*>(pb + static_cast<size_t>(min(k0 + kb + i * (256 / CVB), B - 1)) * N);
    };
    auto stash = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int k = ka + i * (256 / CVA);
            *reinterpret_cast<wg_u32x4*>(sA + k * LDA + ca) = ra[i] & (k0 + k < B ? ~0u : 0u);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int k = kb + i * (256 / CVB);
            *reinterpret_cast<wg_u32x4*>(sB + k * LDB + cbv) = rb[i] & (okb && k0 + k < B ? ~0u : 0u);
        }
    };

    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const int G4 = lane >> 4, s16 = lane & 15;
    const int krow = 8 * (G4 >> 1) + (s16 >> 2);
    const int col4 = 16 * (G4 & 1) + 4 * (s16 & 3);

    // the chunk staged in LDS: 16 minibatch rows per step; the fragments of step ks + 1 are requested before the matrix work of step ks
    auto contract = [&]() {
        bf16x8 fa[2][2], fb[2];
        auto frags = [&](auto buf_, auto ks_) {
            constexpr int buf = decltype(buf_)::value, ks = decltype(ks_)::value;
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[buf][i] = tr_fragment(sA + (ks * 16 + krow) * LDA + i * 32 + col4, 4 * LDA);
            fb[buf] = tr_fragment(sB + (ks * 16 + krow) * LDB + wave * 32 + col4, 4 * LDB);
        };
        frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        auto step = [&](auto ks_) {
            constexpr int ks = decltype(ks_)::value, buf = ks & 1;
            if constexpr (ks + 1 < KC / 16) frags(std::integral_constant<int, (ks + 1) & 1>{}, std::integral_constant<int, ks + 1>{});
#pragma unroll
            for (int i = 0; i < 2; ++i) mma_32x32x16(acc[i], fa[buf][i], fb[buf]);
            __builtin_amdgcn_sched_barrier(0);
        };
        static_for<0, KC / 16>(step);
    };

    fetch(0);
    int k0 = 0;
    for (; k0 + KC < B; k0 += KC) {     // every chunk but the last
        if (k0 != 0) __syncthreads();   // every wavefront has finished reading the previous chunk
        stash(k0);
        fetch(k0 + KC);
        __syncthreads();
        contract();
    }
    if (k0 != 0) __syncthreads();
    stash(k0);
    __syncthreads();
    contract();

    // ---- the gradient tile, through LDS: a thread then holds four consecutive columns of one row
    __syncthreads();   // the operand buffers are free
    constexpr int LDG = BN + 4;
    float* sG = reinterpret_cast<float*>(smem);
    static_assert(static_cast<size_t>(BM) * LDG * 4 <= kWgF1Smem, "the fp32 tile fits the operand buffers");
    {
        const int fl = wave * 32 + (lane & 31);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) sG[(i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * LDG + fl] = acc[i][v];
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < BM * BN / 4 / 256; ++u) {
        const int q = tid + u * 256, row = q / (BN / 4), c4 = (q % (BN / 4)) * 4;
        if (n0 + c4 < N)   // N is a multiple of 4: a quad is valid or not as a whole
            *reinterpret_cast<float4*>(a.grad + static_cast<size_t>(m0 + row) * N + n0 + c4) = *reinterpret_cast<const float4*>(sG + row * LDG + c4);
    }
}

}  // namespace dqn
