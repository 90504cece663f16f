// Weight-stationary implicit-GEMM convolution for the Q-network's skinny layers (32 or 64 output
// channels, K = 256 .. 576) on CDNA4 matrix cores.
//
// The whole [N][K] weight matrix of a layer fits in the 160 KB LDS of a compute unit, and the
// im2col operand has no reuse across output channels beyond one wavefront.  So a workgroup loads
// the weights into LDS once and then streams tiles of 32 pixels per wavefront: each lane fetches
// the eight consecutive k-elements of its own pixel straight from global memory into registers --
// already in MFMA operand layout, no LDS staging and no workgroup barrier in the main loop -- with
// every k-offset a compile-time constant of the fully unrolled loop.
//
// MFMA roles: A = weights (row i = output channel, from LDS), B = pixels (column j = pixel, from
// global).  Lane l then holds pixel (l % 32) of its tile and, per 32x32 block, channels
// 8*(v/4) + 4*(l/32) + (v%4): four consecutive channels per register quad, stored as one 8-byte
// (bf16) or 16-byte (fp32) vector into the channels-last output.
//
// The same kernel computes the data gradient of a strided convolution: "pixels" are then the input
// pixels of one stride-parity class, k runs over (tap, output channel) of dY with out-of-range taps
// predicated to zero, the LDS-resident matrix is the transposed filter of that class, and the
// epilogue applies the ReLU mask of the layer below.
#pragma once
#include <atomic>

#include "gemm_mfma.h"

namespace dqn {

struct RowInfo {
    int in_off;        // element offset of the row's patch origin in the input
    int out_off;       // element offset of the row's first channel in the output
    uint32_t tapmask;  // bit t set: tap t of this row lies inside the input (dgrad only)
};

// Forward convolution on a channels-last activation; k = (p, q, c).
template <typename T, int CIN, int HIN, int WIN, int COUT, int HOUT, int WOUT, int KS, int S> struct FwdGeo {
    typedef T In;
    static constexpr int N = COUT, K = KS * KS * CIN, KSTEPS = K / 16;
    static constexpr int kLaneStep = 8;   // element distance between the two k-halves of a k-step
    static constexpr bool kPredicated = false;
    static constexpr int kInPerSample = HIN * WIN * CIN;
    __device__ static RowInfo row(int, int r)
    {
        const int b = r / (HOUT * WOUT), ij = r % (HOUT * WOUT), i = ij / WOUT, j = ij % WOUT;
        RowInfo ri;
        ri.in_off = ((b * HIN + i * S) * WIN + j * S) * CIN;
        ri.out_off = r * COUT;
        ri.tapmask = 0xFFFFFFFFu;
        return ri;
    }
    __host__ __device__ static constexpr int koff(int ks)
    {
        return (((ks * 16) / CIN / KS) * WIN + ((ks * 16) / CIN) % KS) * CIN + (ks * 16) % CIN;
    }
    __host__ __device__ static constexpr int tap(int) { return 0; }
};

// conv1 on the raw uint8 state [n][4][84][84]; k = (c, p, q), one k-half = the 8 bytes of one (c, p).
template <typename T> struct Conv1Geo {
    typedef uint8_t In;
    static constexpr int N = 32, K = 256, KSTEPS = 16;
    static constexpr int kLaneStep = 84;  // the second k-half is the next filter row p
    static constexpr bool kPredicated = false;
    static constexpr int kInPerSample = 4 * 84 * 84;
    __device__ static RowInfo row(int, int r)
    {
        const int b = r / 400, ij = r % 400, i = ij / 20, j = ij % 20;
        RowInfo ri;
        ri.in_off = (b * 4 * 84 + 4 * i) * 84 + 4 * j;
        ri.out_off = r * 32;
        ri.tapmask = 0xFFFFFFFFu;
        return ri;
    }
    __host__ __device__ static constexpr int koff(int ks) { return (ks / 4) * 7056 + ((ks % 4) * 2) * 84; }
    __host__ __device__ static constexpr int tap(int) { return 0; }
};

// Data gradient of a stride-S convolution for parity class g = (py, px): rows = input pixels
// (b, y2, x2) with y = S*y2 + py, x = S*x2 + px; k = (p2, q2, o) reads dY[b][y2 - p2][x2 - q2][o].
template <typename T, int CIN, int HIN, int WIN, int COUT, int HOUT, int WOUT, int KS, int S> struct DgradGeo {
    typedef T In;
    static constexpr int K2 = KS / S, H2 = HIN / S, W2 = WIN / S;
    static constexpr int N = CIN, K = K2 * K2 * COUT, KSTEPS = K / 16;
    static constexpr int kLaneStep = 8;
    static constexpr bool kPredicated = true;
    __device__ static RowInfo row(int g, int r)
    {
        const int b = r / (H2 * W2), yx = r % (H2 * W2), y2 = yx / W2, x2 = yx % W2;
        RowInfo ri;
        ri.in_off = ((b * HOUT + y2) * WOUT + x2) * COUT;
        ri.out_off = ((b * HIN + S * y2 + g / S) * WIN + S * x2 + g % S) * CIN;
        uint32_t m = 0;
#pragma unroll
        for (int p2 = 0; p2 < K2; ++p2)
#pragma unroll
            for (int q2 = 0; q2 < K2; ++q2) {
                const int i = y2 - p2, j = x2 - q2;
                if (i >= 0 && i < HOUT && j >= 0 && j < WOUT) m |= 1u << (p2 * K2 + q2);
            }
        ri.tapmask = m;
        return ri;
    }
    __host__ __device__ static constexpr int koff(int ks)
    {
        return -((((ks * 16) / COUT) / K2) * WOUT + ((ks * 16) / COUT) % K2) * COUT + (ks * 16) % COUT;
    }
    __host__ __device__ static constexpr int tap(int ks) { return (ks * 16) / COUT; }
};

template <typename T, typename In> struct FragLoad;
template <typename T> struct FragLoad<T, T> {
    __device__ static typename Vec8<T>::type get(const T* p) { return *reinterpret_cast<const typename Vec8<T>::type*>(p); }
};
template <typename T> struct FragLoad<T, uint8_t> {
    __device__ static typename Vec8<T>::type get(const uint8_t* p)
    {
        const uint32_t* w = reinterpret_cast<const uint32_t*>(p);
        return vec8_from_u8<T>(w[0], w[1]);
    }
};

template <typename T, class Geo> struct ConvWsArgs {
    const typename Geo::In* x[kMaxGroups];
    const T* w[kMaxGroups];          // [N][K], k contiguous
    const float* bias[kMaxGroups];   // forward only
    T* out[kMaxGroups];
    const T* mask;                   // dgrad only: activation of the layer below, indexed like out
    int M;                           // rows (pixels) per group
    float scale;
};

constexpr int kEpiBiasRelu = 0, kEpiReluMask = 1;

template <typename T> __device__ inline void store4(T* dst, float a, float b, float c, float d);
template <> __device__ inline void store4<float>(float* dst, float a, float b, float c, float d)
{
    *reinterpret_cast<float4*>(dst) = make_float4(a, b, c, d);
}
template <> __device__ inline void store4<bf16_t>(bf16_t* dst, float a, float b, float c, float d)
{
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    bf16x4 v;
    v[0] = static_cast<bf16_t>(a); v[1] = static_cast<bf16_t>(b);
    v[2] = static_cast<bf16_t>(c); v[3] = static_cast<bf16_t>(d);
    *reinterpret_cast<bf16x4*>(dst) = v;
}
template <typename T> __device__ inline void load4(const T* src, float* o);
template <> __device__ inline void load4<float>(const float* src, float* o)
{
    const float4 v = *reinterpret_cast<const float4*>(src);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
template <> __device__ inline void load4<bf16_t>(const bf16_t* src, float* o)
{
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    const bf16x4 v = *reinterpret_cast<const bf16x4*>(src);
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = static_cast<float>(v[i]);
}

// TP = 32-pixel tiles per wavefront, WAVES wavefronts per workgroup; a wavefront covers all N channels.
template <typename T, class Geo, int EPI, int TP, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void conv_ws_kernel(ConvWsArgs<T, Geo> a)
{
    typedef typename Vec8<T>::type V8;
    typedef typename Geo::In In;
    constexpr int N = Geo::N, K = Geo::K, KSTEPS = Geo::KSTEPS, TN = N / 32;
    constexpr int LDW = K + 8;
    constexpr int PD = KSTEPS < 4 ? KSTEPS : 4;   // k-steps of pixel fragments in flight
    constexpr int TILE_ROWS = WAVES * TP * 32;
    extern __shared__ __attribute__((aligned(32))) unsigned char ws_smem[];
    T* sW = reinterpret_cast<T*>(ws_smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.y;
    {
        const T* wg = a.w[g];
        for (int v = tid; v < N * K / 8; v += WAVES * 64) {
            const int n = v / (K / 8), kc = v % (K / 8);
            *reinterpret_cast<V8*>(&sW[n * LDW + kc * 8]) = *reinterpret_cast<const V8*>(wg + n * K + kc * 8);
        }
    }
    __syncthreads();

    const int lane_px = lane & 31, kg = lane >> 5;
    const In* xg = a.x[g];
    T* og = a.out[g];

    for (int tile = blockIdx.x; tile * TILE_ROWS < a.M; tile += gridDim.x) {
        // The LDS-resident weights are loop-invariant; without this fence the compiler hoists every
        // weight fragment of the unrolled k-loop out of the tile loop and runs out of registers.
        asm volatile("" ::: "memory");
        RowInfo ri[TP];
        const In* px[TP];
        bool live[TP];
#pragma unroll
        for (int t = 0; t < TP; ++t) {
            const int r = tile * TILE_ROWS + (wave * TP + t) * 32 + lane_px;
            live[t] = r < a.M;
            ri[t] = Geo::row(g, live[t] ? r : 0);
            if (!live[t]) ri[t].tapmask = Geo::kPredicated ? 0u : ri[t].tapmask;
            px[t] = xg + ri[t].in_off + kg * Geo::kLaneStep;
        }
        auto fetch = [&](int ks, int t) -> V8 {
            if constexpr (Geo::kPredicated) {
                const bool ok = (ri[t].tapmask >> Geo::tap(ks)) & 1u;
                const In* p = ok ? px[t] + Geo::koff(ks) : xg;     // always a readable address
                V8 v = FragLoad<T, In>::get(p);
                return ok ? v : vec8_zero<T>();
            } else {
                return FragLoad<T, In>::get(px[t] + Geo::koff(ks));
            }
        };

        f32x16 acc[TN][TP];
#pragma unroll
        for (int n = 0; n < TN; ++n)
#pragma unroll
            for (int t = 0; t < TP; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[n][t][v] = 0.f;

        V8 ring[PD][TP];
#pragma unroll
        for (int s = 0; s < PD; ++s)
#pragma unroll
            for (int t = 0; t < TP; ++t) ring[s][t] = fetch(s, t);
        __builtin_amdgcn_sched_barrier(0);   // keep the whole ring in flight
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            V8 cur[TP];
#pragma unroll
            for (int t = 0; t < TP; ++t) cur[t] = ring[ks % PD][t];
            if (ks + PD < KSTEPS) {
#pragma unroll
                for (int t = 0; t < TP; ++t) ring[ks % PD][t] = fetch(ks + PD, t);
                __builtin_amdgcn_sched_barrier(0);   // refill issued before this k-step's MFMAs
            }
#pragma unroll
            for (int n = 0; n < TN; ++n) {
                const V8 wf = *reinterpret_cast<const V8*>(&sW[(n * 32 + lane_px) * LDW + ks * 16 + kg * 8]);
#pragma unroll
                for (int t = 0; t < TP; ++t) mma_32x32x16(acc[n][t], wf, cur[t]);
            }
        }

#pragma unroll
        for (int t = 0; t < TP; ++t) {
            if (!live[t]) continue;
#pragma unroll
            for (int n = 0; n < TN; ++n)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int ch = n * 32 + 8 * q + 4 * kg;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[n][t][4 * q + e];
                    if constexpr (EPI == kEpiBiasRelu) {
                        const float4 bv = *reinterpret_cast<const float4*>(a.bias[g] + ch);
                        v[0] = fmaxf(v[0] * a.scale + bv.x, 0.f);
                        v[1] = fmaxf(v[1] * a.scale + bv.y, 0.f);
                        v[2] = fmaxf(v[2] * a.scale + bv.z, 0.f);
                        v[3] = fmaxf(v[3] * a.scale + bv.w, 0.f);
                    } else {
                        float m[4];
                        load4<T>(a.mask + ri[t].out_off + ch, m);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = m[e] > 0.f ? v[e] : 0.f;
                    }
                    store4<T>(og + ri[t].out_off + ch, v[0], v[1], v[2], v[3]);
                }
        }
    }
}

// Small-problem variant (an act step over W environments, a batch-32 train step): one workgroup per
// 32-pixel tile, the four wavefronts split K between them, both operands go straight from global
// memory (L2) into MFMA operand registers -- with one tile per workgroup there is no weight reuse
// that LDS staging could serve -- and the four partial accumulators meet in LDS, added in wavefront
// order.  Short dependent chains instead of one wavefront walking all of K.
template <typename T, class Geo, int EPI>
__global__ __launch_bounds__(256) void conv_sk_kernel(ConvWsArgs<T, Geo> a)
{
    typedef typename Vec8<T>::type V8;
    typedef typename Geo::In In;
    constexpr int N = Geo::N, K = Geo::K, KSTEPS = Geo::KSTEPS, TN = N / 32;
    constexpr int KQ = KSTEPS / 4;
    static_assert(KSTEPS % 4 == 0, "k-steps must split over four wavefronts");
    __shared__ float red[4][TN * 16][64];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.y, tile = blockIdx.x;
    const int lane_px = lane & 31, kg = lane >> 5;
    const int r = tile * 32 + lane_px;
    const bool live = r < a.M;
    RowInfo ri = Geo::row(g, live ? r : 0);
    if (!live && Geo::kPredicated) ri.tapmask = 0u;
    const In* xg = a.x[g];
    const In* px = xg + ri.in_off + kg * Geo::kLaneStep;
    const T* wl = a.w[g] + static_cast<size_t>(lane_px) * K + kg * 8;

    V8 pf[KQ], wf[KQ][TN];
#pragma unroll
    for (int s = 0; s < KQ; ++s) {
        const int ks = wave * KQ + s;          // runtime k-step: offsets via the constexpr tables below
        int koff = 0, tap = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            if (w == wave) { koff = Geo::koff(w * KQ + s); tap = Geo::tap(w * KQ + s); }
        if constexpr (Geo::kPredicated) {
            const bool ok = (ri.tapmask >> tap) & 1u;
            const V8 v = FragLoad<T, In>::get(ok ? px + koff : xg);
            pf[s] = ok ? v : vec8_zero<T>();
        } else {
            pf[s] = FragLoad<T, In>::get(px + koff);
        }
#pragma unroll
        for (int n = 0; n < TN; ++n) wf[s][n] = *reinterpret_cast<const V8*>(wl + static_cast<size_t>(n) * 32 * K + ks * 16);
    }
    __builtin_amdgcn_sched_barrier(0);   // every operand load is issued before the first MFMA waits
    f32x16 acc[TN];
#pragma unroll
    for (int n = 0; n < TN; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
#pragma unroll
    for (int s = 0; s < KQ; ++s)
#pragma unroll
        for (int n = 0; n < TN; ++n) mma_32x32x16(acc[n], wf[s][n], pf[s]);

#pragma unroll
    for (int n = 0; n < TN; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][n * 16 + v][lane] = acc[n][v];
    __syncthreads();
    if (!live) return;
    // quad (n, q) = four consecutive channels; the TN*4 quads are dealt round-robin to the wavefronts
    T* og = a.out[g];
    for (int quad = wave; quad < TN * 4; quad += 4) {
        const int n = quad / 4, q = quad % 4;
        const int ch = n * 32 + 8 * q + 4 * kg;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = n * 16 + 4 * q + e;
            v[e] = ((red[0][idx][lane] + red[1][idx][lane]) + red[2][idx][lane]) + red[3][idx][lane];
        }
        if constexpr (EPI == kEpiBiasRelu) {
            const float4 bv = *reinterpret_cast<const float4*>(a.bias[g] + ch);
            v[0] = fmaxf(v[0] * a.scale + bv.x, 0.f);
            v[1] = fmaxf(v[1] * a.scale + bv.y, 0.f);
            v[2] = fmaxf(v[2] * a.scale + bv.z, 0.f);
            v[3] = fmaxf(v[3] * a.scale + bv.w, 0.f);
        } else {
            float m[4];
            load4<T>(a.mask + ri.out_off + ch, m);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = m[e] > 0.f ? v[e] : 0.f;
        }
        store4<T>(og + ri.out_off + ch, v[0], v[1], v[2], v[3]);
    }
}

template <typename T, class Geo> constexpr size_t conv_ws_smem() { return static_cast<size_t>(Geo::N) * (Geo::K + 8) * sizeof(T); }

// Launches the kernel over `groups` independent problems of M rows each.
template <typename T, class Geo, int EPI>
inline hipError_t launch_conv_ws(hipStream_t st, const ConvWsArgs<T, Geo>& a, int groups, hipEvent_t ev_begin = nullptr,
                                 hipEvent_t ev_end = nullptr)
{
    constexpr size_t smem = conv_ws_smem<T, Geo>();
    // Large problems: the wavefronts of a workgroup share one LDS copy of the weights (two
    // workgroups fit a compute unit).  More wavefronts per workgroup keep more operand loads in
    // flight, but the grid must still cover the chip about twice.
    const int max_blocks = 512 / (groups > 0 ? groups : 1);
    hipError_t e = hipSuccess;
    const int tiles32 = (a.M + 31) / 32;
    auto launch_ws = [&](auto kern, int waves) {
        // one flag per kernel instantiation (generic lambda); the act thread and the train thread both come here, and
        // setting the attribute twice is harmless
        static std::atomic<bool> attr_set{false};
        if (!attr_set.load(std::memory_order_acquire)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return;
            attr_set.store(true, std::memory_order_release);
        }
        int tiles = (a.M + waves * 32 - 1) / (waves * 32);
        if (tiles > max_blocks) tiles = max_blocks;
        launch_timed(kern, dim3(tiles, groups), dim3(waves * 64), smem, st, ev_begin, ev_end, a);
    };
    if (tiles32 * groups <= 1024) launch_timed(conv_sk_kernel<T, Geo, EPI>, dim3(tiles32, groups), dim3(256), 0, st, ev_begin, ev_end, a);
    else if (tiles32 * groups >= 16 * 512) launch_ws(conv_ws_kernel<T, Geo, EPI, 1, 16>, 16);
    else if (tiles32 * groups >= 8 * 512) launch_ws(conv_ws_kernel<T, Geo, EPI, 1, 8>, 8);
    else launch_ws(conv_ws_kernel<T, Geo, EPI, 1, 4>, 4);
    if (e != hipSuccess) return e;
    e = hipGetLastError();
    return e;
}

}  // namespace dqn
