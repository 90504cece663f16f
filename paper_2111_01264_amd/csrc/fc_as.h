// Activation-stationary GEMM for the fully connected layer fc1 (512 x 3136) and its data gradient.
//
//   out[b][n] = sum_k X[b][k] * W[n][k]        X: [M][ldx] activations (few rows), W: [N][ldw] weights
//
// With at most a few hundred rows of X the layer is bound by streaming W once, so the roles are
// the reverse of the convolution kernel: a workgroup parks a [32*TB][KC] slab of X in LDS and every
// wavefront streams 32 rows of W straight from global memory in MFMA operand layout (eight
// consecutive k per lane).  MFMA A = weights (row i = output feature), B = samples (column j = b),
// so lane l ends up with sample (l % 32) and four consecutive features per register quad.
//
// 16-bit weights arrive in MFMA fragment order (tower_frag_index over [feature][k]): the operand of k-step ks of
// feature tile nt is the contiguous 1 KB row (nt * K/16 + ks); row-major weights (fp32 mode) are read as 32 separate
// 32-byte pieces per wavefront load, which is bound by the address unit (a full pass per cache line).
//
// K may be split over blockIdx.z: each slice then writes fp32 partial sums [slice][b][n], which the
// consumer kernel adds in slice order while it loads them (no separate reduction pass).
#pragma once
#include <atomic>

#include "conv_ws.h"

namespace dqn {

template <typename T> struct FcAsArgs {
    const T* x[kMaxGroups];      // [M][ldx]
    const T* w[kMaxGroups];      // [N][ldw]
    float* partial;              // kFcPartial: [group][slice][M][N] fp32
    T* dz;                       // kFcReluMask: [M][N]
    const T* mask;               // kFcReluMask: activation indexed like dz
    int M, N, K, ldx, ldw;      // K is a multiple of 64
    int kc;                      // k per slice, multiple of 64 (the last slice may be shorter)
    int slices;
};

constexpr int kFcPartial = 0, kFcReluMask = 1;

// Pointer to this lane's 8 weights of k-step ks (16 k each) of the 32-feature tile nt; w is [N][K].
template <typename T> __device__ inline const T* fc_weight_fragment(const T* w, int nt, int ks, int K, int lane)
{
    if constexpr (sizeof(T) == 2) return w + (static_cast<size_t>(nt * (K >> 4) + ks) * 64 + lane) * 8;
    else return w + static_cast<size_t>(nt * 32 + (lane & 31)) * K + ks * 16 + (lane >> 5) * 8;
}

template <typename T, int EPI, int TB, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void fc_as_kernel(FcAsArgs<T> a)
{
    typedef typename Vec8<T>::type V8;
    extern __shared__ __attribute__((aligned(32))) unsigned char as_smem[];
    T* sX = reinterpret_cast<T*>(as_smem);
    const int ldk = a.kc + 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.z / a.slices, slice = blockIdx.z % a.slices;
    const int m0 = blockIdx.y * (TB * 32);
    const int k0 = slice * a.kc;
    const int klen = min(a.kc, a.K - k0);
    const int lane_r = lane & 31, kg = lane >> 5;
    const int n = (blockIdx.x * WAVES + wave) * 32 + lane_r;
    const bool n_ok = n < a.N;
    const int ntile = n_ok ? blockIdx.x * WAVES + wave : 0, ks0 = k0 >> 4;   // N is a multiple of 32: tiles are whole

    // The weight stream: a ring of D k-steps of fragments in flight per wavefront, requested before the slab of X
    // is staged so that both latencies overlap.  Loads are never skipped (the k-step is clamped): the count of
    // loads in flight stays known to the compiler, which then waits for one slot only.
    constexpr int D = sizeof(T) == 2 ? 16 : 8;   // 16 KB per wavefront in flight: a step waits for the fragment requested D steps earlier, so the stream runs at D fragments per memory round trip
    const int steps = klen >> 4;
    auto wload = [&](int st) {
        return *reinterpret_cast<const V8*>(fc_weight_fragment<T>(a.w[g], ntile, ks0 + (st < steps ? st : steps - 1), a.ldw, lane));
    };
    V8 ring[D];
#pragma unroll
    for (int u = 0; u < D; ++u) ring[u] = wload(u);
    // kFcReluMask: the activations that mask this lane's outputs are requested now, not in the epilogue (there they were one
    // more dependent round trip to memory at the end of every workgroup); clamped addresses, no load is skipped
    [[maybe_unused]] float mask[TB][4][4];
    if constexpr (EPI == kFcReluMask) {
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            const int b = min(m0 + t * 32 + lane_r, a.M - 1);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                load4<T>(a.mask + static_cast<size_t>(b) * a.N + min(static_cast<int>(blockIdx.x * WAVES + wave) * 32 + 8 * q + 4 * kg, a.N - 4), mask[t][q]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    {
        // the slab of X: eight 16-byte vectors in flight per thread (clamped address, masked value), then their LDS stores --
        // one vector per trip of a plain loop would be a chain of dependent memory round trips
        const T* xg = a.x[g];
        const int vec_per_row = klen / 8, total = TB * 32 * vec_per_row;
        for (int v0 = tid; v0 < total; v0 += 8 * WAVES * 64) {
            V8 val[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int v = v0 + u * WAVES * 64 < total ? v0 + u * WAVES * 64 : total - 1;
                const int r = v / vec_per_row, kc8 = v % vec_per_row;
                const int row = m0 + r < a.M ? m0 + r : a.M - 1;
                val[u] = vec8_keep<T>(*reinterpret_cast<const V8*>(xg + static_cast<size_t>(row) * a.ldx + k0 + kc8 * 8), m0 + r < a.M);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int v = v0 + u * WAVES * 64;
                if (v < total) *reinterpret_cast<V8*>(&sX[(v / vec_per_row) * ldk + (v % vec_per_row) * 8]) = val[u];
            }
        }
    }
    __syncthreads();

    f32x16 acc[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    // steps is a multiple of 4 (k per slice is a multiple of 64): whole chunks of D steps, then the rest
    const T* xrow[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) xrow[t] = &sX[(t * 32 + lane_r) * ldk + kg * 8];
    int base = 0;
    for (; base + D <= steps; base += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const V8 w = ring[u];
            ring[u] = wload(base + u + D);
#pragma unroll
            for (int t = 0; t < TB; ++t) mma_32x32x16(acc[t], w, *reinterpret_cast<const V8*>(xrow[t] + (base + u) * 16));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // what is left (fewer than D steps, a multiple of four) sits in the ring already
#pragma unroll
    for (int u = 0; u < D; u += 4)
        if (base + u < steps) {
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
                for (int t = 0; t < TB; ++t) mma_32x32x16(acc[t], ring[u + w], *reinterpret_cast<const V8*>(xrow[t] + (base + u + w) * 16));
        }

    // lane: sample b = m0 + t*32 + lane_r; values: features 8*q + 4*kg + e of this wavefront's 32
    const int n_base = (blockIdx.x * WAVES + wave) * 32;
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const int b = m0 + t * 32 + lane_r;
        if (b >= a.M) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int nn = n_base + 8 * q + 4 * kg;
            if (nn >= a.N) continue;   // N is a multiple of 4
            if constexpr (EPI == kFcPartial) {
                float* dst = a.partial + ((static_cast<size_t>(g) * a.slices + slice) * a.M + b) * a.N + nn;
                *reinterpret_cast<float4*>(dst) = make_float4(acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]);
            } else {
                const size_t idx = static_cast<size_t>(b) * a.N + nn;
                const float* m = mask[t][q];
                store4<T>(a.dz + idx, m[0] > 0.f ? acc[t][4 * q] : 0.f, m[1] > 0.f ? acc[t][4 * q + 1] : 0.f,
                          m[2] > 0.f ? acc[t][4 * q + 2] : 0.f, m[3] > 0.f ? acc[t][4 * q + 3] : 0.f);
            }
        }
    }
}

// Small-batch variant (at most 32 rows of X): one workgroup per (32 output features, K slice), its
// four wavefronts split the slice between them, both operands go straight from global memory into
// MFMA registers and the partial accumulators meet in LDS, added in wavefront order.  Streaming the
// 3.2 MB of fc1 weights within a few microseconds takes ~100 compute units pulling at once, hence
// the K slices across workgroups; like the large-batch kernel it then writes fp32 slices
// [group][slice][M][N] that the consumer adds in slice order.  (Finishing inside this kernel through
// a last-workgroup ticket was tried and is several times slower: the device-scope fence it needs
// writes back the L2 of the issuing XCD.)
template <typename T> struct FcSkArgs {
    const T* x[kMaxGroups];      // [M][ldx], M <= 32
    const T* w[kMaxGroups];      // [N][ldw]
    float* partial;              // kFcPartial: [group][slice][M][N] fp32
    T* dz;                       // kFcReluMask: [M][N]
    const T* mask;               // kFcReluMask: activation indexed like dz
    int M, N, ldx, ldw;
};

// The leading scalar parameters repeat FcSkArgs::x[0], x[1], w[0], w[1], M, N, ldx, ldw, partial: the kernel arguments'
// first 14 dwords are preloaded into scalar registers when a wavefront starts (see conv_tower_kernel).
template <typename T, int EPI, int KPW, int KSLICES>
__global__ __launch_bounds__(256) void fc_sk_kernel(const T* x0_, const T* x1_, const T* w0_, const T* w1_, int M_, int N_, int ldx_, int ldw_,
                                                    float* partial_, FcSkArgs<T> a)
{
    typedef typename Vec8<T>::type V8;
    static_assert(EPI == kFcPartial || KSLICES == 1, "only partial sums can be split over workgroups");
    __shared__ float red[4][16][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.y, n0 = blockIdx.x * 32, slice = blockIdx.z;
    const int lr = lane & 31, kg = lane >> 5;
    const int n = n0 + lr;
    const int k0 = (slice * 4 + wave) * (KPW * 16) + kg * 8;
    const int ntile = n < N_ ? blockIdx.x : 0, ks0 = (slice * 4 + wave) * KPW;   // N is a multiple of 32
    const bool x_ok = lr < M_;
    const T* xg = g == 0 ? x0_ : g == 1 ? x1_ : a.x[g];
    const T* wg = g == 0 ? w0_ : g == 1 ? w1_ : a.w[g];
    const T* xp = xg + static_cast<size_t>(x_ok ? lr : 0) * ldx_ + k0;
    V8 wf[KPW], xf[KPW];
#pragma unroll
    for (int s = 0; s < KPW; ++s) {
        wf[s] = *reinterpret_cast<const V8*>(fc_weight_fragment<T>(wg, ntile, ks0 + s, ldw_, lane));
        xf[s] = *reinterpret_cast<const V8*>(xp + s * 16);
    }
    // thread t finishes accumulator slots (v, l) = (4*(t/64) + e, t%64), e = 0..3: one quad of features of one sample.
    // kFcReluMask: the activations that mask them are requested now (clamped address), behind the operands -- in the
    // epilogue they were one more dependent round trip to memory at the end of a two-microsecond kernel
    const int q = tid >> 6, l = tid & 63;
    const int sample = l & 31;
    const int nn = n0 + 8 * q + 4 * (l >> 5);
    [[maybe_unused]] float m[4];
    if constexpr (EPI == kFcReluMask) load4<T>(a.mask + static_cast<size_t>(min(sample, M_ - 1)) * N_ + min(nn, N_ - 4), m);
    __builtin_amdgcn_sched_barrier(0);
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int s = 0; s < KPW; ++s) mma_32x32x16(acc, wf[s], x_ok ? xf[s] : vec8_zero<T>());
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[v];
    __syncthreads();
    float v4[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        v4[e] = ((red[0][4 * q + e][l] + red[1][4 * q + e][l]) + red[2][4 * q + e][l]) + red[3][4 * q + e][l];
    if (sample >= M_ || nn >= N_) return;
    if constexpr (EPI == kFcPartial) {
        float* dst = partial_ + ((static_cast<size_t>(g) * KSLICES + slice) * M_ + sample) * N_ + nn;
        *reinterpret_cast<float4*>(dst) = make_float4(v4[0], v4[1], v4[2], v4[3]);
    } else {
        const size_t idx = static_cast<size_t>(sample) * N_ + nn;
        store4<T>(a.dz + idx, m[0] > 0.f ? v4[0] : 0.f, m[1] > 0.f ? v4[1] : 0.f, m[2] > 0.f ? v4[2] : 0.f,
                  m[3] > 0.f ? v4[3] : 0.f);
    }
}

template <typename T, int EPI>
inline hipError_t launch_fc_as(hipStream_t st, FcAsArgs<T> a, int K, int groups, int want_slices, int* slices_used,
                               hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr)
{
    constexpr int WAVES = 4;
    int slices = want_slices < 1 ? 1 : want_slices;
    int kc = ((K + slices - 1) / slices + 63) / 64 * 64;
    slices = (K + kc - 1) / kc;
    if (slices_used) *slices_used = slices;
    a.K = K;
    a.kc = kc;
    a.slices = slices;
    const int n_blocks = (a.N + WAVES * 32 - 1) / (WAVES * 32);
    hipError_t e = hipSuccess;
    {
        // One 32-row tile of X per workgroup: with two, the grid of a batch-256 step was 100-224 workgroups on 256 CUs,
        // one per CU, and nothing overlapped a workgroup's staging, streaming and storing phases.
        constexpr int TB = 1;
        const size_t smem = static_cast<size_t>(TB) * 32 * (kc + 8) * sizeof(T);
        auto kern = fc_as_kernel<T, EPI, TB, WAVES>;
        static std::atomic<size_t> attr_smem{0};   // launches come from the act thread and the train thread; setting the attribute twice is harmless
        if (smem > attr_smem.load(std::memory_order_relaxed)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return e;
            attr_smem.store(smem, std::memory_order_relaxed);
        }
        launch_timed(kern, dim3(n_blocks, (a.M + TB * 32 - 1) / (TB * 32), groups * slices), dim3(WAVES * 64), smem, st, ev_begin, ev_end, a);
    }
    e = hipGetLastError();
    return e;
}

}  // namespace dqn
