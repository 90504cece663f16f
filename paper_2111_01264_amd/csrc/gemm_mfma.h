// Implicit-GEMM core for the Q-network's conv / fc layers on CDNA4 matrix cores.
//
//   C[m, n] = sum_k A(m, k) * B(n, k)            (both operands indexed "row, k")
//
// A and B are *loader functors*: they map a (row, k) position to eight consecutive elements in
// global memory (the im2col of a convolution is never materialised).  A loader is either
//   k-contiguous  (kAlongK = true):  load(g, row, k)  -> elements (row, k .. k+7)
//   row-contiguous (kAlongK = false): load(g, row, k)  -> elements (row .. row+7, k)
// and returns zeros outside [0, rows) x [0, k_end).  Tiles are staged through LDS in a
// [row][k] layout (row-contiguous sources are transposed on the way in), each wavefront then
// reads 8-element k-vectors per lane -- exactly the operand shape of the 32x32 MFMA: lane l feeds
// row (l % 32) with k-slice 8 * (l / 32) .. + 7, and receives column (l % 32) of the 32x32 result
// with rows 8 * (v / 4) + 4 * (l / 32) + (v % 4), v = 0 .. 15.
//
// One source serves both precisions: T = __bf16 issues v_mfma_f32_32x32x16_bf16 (fp32 accumulate),
// T = float issues eight v_mfma_f32_32x32x2_f32 over the same 16-wide k-slice.
//
// Grid: x = m-tiles * n-tiles, y = split-K slices, z = groups (independent problems that share
// shapes: online/target networks in the forward pass, stride-parity classes in a strided dgrad).
// With split-K the block writes fp32 partial sums [g][split][m][n]; splitk_finalize_kernel adds
// them in split order (bitwise reproducible) and applies the epilogue.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dqn {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <typename T> struct Vec8;
template <> struct Vec8<float> { typedef f32x8 type; };
template <> struct Vec8<bf16_t> { typedef bf16x8 type; };

template <typename T> __device__ inline typename Vec8<T>::type vec8_zero()
{
    typename Vec8<T>::type z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = static_cast<T>(0.f);
    return z;
}

// v if keep, else all-zero bits -- as a bitwise AND, not a select: the compiler turns "select(cond, loaded
// value, 0)" back into a branch around the load, and a load that may be skipped spoils its count of loads in flight.
template <typename T> __device__ inline typename Vec8<T>::type vec8_keep(const typename Vec8<T>::type& v, bool keep)
{
    typedef uint32_t words_t __attribute__((ext_vector_type(sizeof(typename Vec8<T>::type) / 4)));
    words_t w = __builtin_bit_cast(words_t, v);
    const uint32_t m = keep ? 0xFFFFFFFFu : 0u;
#pragma unroll
    for (int i = 0; i < static_cast<int>(sizeof(w) / 4); ++i) w[i] &= m;
    return __builtin_bit_cast(typename Vec8<T>::type, w);
}

template <typename T> __device__ inline T from_float(float x) { return static_cast<T>(x); }
template <typename T> __device__ inline float to_float(T x) { return static_cast<float>(x); }

// Eight uint8 pixels (already in two 32-bit words) -> eight operand elements; exact in bf16.
template <typename T> __device__ inline typename Vec8<T>::type vec8_from_u8(uint32_t lo, uint32_t hi)
{
    typename Vec8<T>::type v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[i] = static_cast<T>(static_cast<float>((lo >> (8 * i)) & 0xFFu));
        v[4 + i] = static_cast<T>(static_cast<float>((hi >> (8 * i)) & 0xFFu));
    }
    return v;
}

__device__ inline void mma_32x32x16(f32x16& acc, const bf16x8& a, const bf16x8& b)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}
__device__ inline void mma_32x32x16(f32x16& acc, const f32x8& a, const f32x8& b)
{
#pragma unroll
    for (int t = 0; t < 8; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], acc, 0, 0, 0);
}

// Launch with an optional pair of timing events bound to the kernel's OWN dispatch: the time between them is the
// kernel's begin-to-end time on the GPU, which is what a kernel trace reports.  (A pair of event records around a launch
// also spans the records themselves and the dispatch gap: about 5 us on this machine, more than many of these kernels.)
template <typename F, typename... Args>
inline void launch_timed(F kernel, dim3 grid, dim3 block, size_t smem, hipStream_t st, hipEvent_t begin, hipEvent_t end,
                         Args... args)
{
    if (begin || end) hipExtLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(smem), st, begin, end, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, smem, st, args...);
}

constexpr int kMaxGroups = 4;   // independent problems per launch (online/target nets, parity classes)
constexpr int kGemmThreads = 256;
constexpr int kLdsPad = 8;  // elements of padding per LDS row

template <typename T, class AL, class BL, class EP, int BM, int BN, int BK, int WGM>
__global__ __launch_bounds__(kGemmThreads) void gemm_nt_kernel(AL al, BL bl, EP ep, int M, int N, int K,
                                                               int k_per_split, int n_tiles,
                                                               float* __restrict__ partial, int always_partial)
{
    typedef typename Vec8<T>::type V8;
    constexpr int WGN = 4 / WGM;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int LDK = BK + kLdsPad;
    constexpr int VA = BM * BK / 8, VB = BN * BK / 8;           // 8-element vectors per tile
    constexpr int NA = (VA + kGemmThreads - 1) / kGemmThreads;  // per-thread vector counts
    constexpr int NB = (VB + kGemmThreads - 1) / kGemmThreads;
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "tile shape");

    __shared__ __attribute__((aligned(32))) T sA[BM * LDK];
    __shared__ __attribute__((aligned(32))) T sB[BN * LDK];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / WGN, wave_n = wave % WGN;
    const int tile_m = blockIdx.x / n_tiles, tile_n = blockIdx.x % n_tiles;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int split = blockIdx.y, g = blockIdx.z;
    const int k_begin = split * k_per_split;
    const int k_end = min(K, k_begin + k_per_split);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    V8 ra[NA], rb[NB];

    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int v = tid + i * kGemmThreads;
            if (VA % kGemmThreads == 0 || v < VA) {
                if constexpr (AL::kAlongK) ra[i] = al.load(g, m0 + v / (BK / 8), k0 + (v % (BK / 8)) * 8, M, k_end);
                else ra[i] = al.load(g, m0 + (v % (BM / 8)) * 8, k0 + v / (BM / 8), M, k_end);
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int v = tid + i * kGemmThreads;
            if (VB % kGemmThreads == 0 || v < VB) {
                if constexpr (BL::kAlongK) rb[i] = bl.load(g, n0 + v / (BK / 8), k0 + (v % (BK / 8)) * 8, N, k_end);
                else rb[i] = bl.load(g, n0 + (v % (BN / 8)) * 8, k0 + v / (BN / 8), N, k_end);
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int v = tid + i * kGemmThreads;
            if (VA % kGemmThreads == 0 || v < VA) {
                if constexpr (AL::kAlongK) {
                    *reinterpret_cast<V8*>(&sA[(v / (BK / 8)) * LDK + (v % (BK / 8)) * 8]) = ra[i];
                } else {
                    const int r0 = (v % (BM / 8)) * 8, kk = v / (BM / 8);
#pragma unroll
                    for (int e = 0; e < 8; ++e) sA[(r0 + e) * LDK + kk] = ra[i][e];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int v = tid + i * kGemmThreads;
            if (VB % kGemmThreads == 0 || v < VB) {
                if constexpr (BL::kAlongK) {
                    *reinterpret_cast<V8*>(&sB[(v / (BK / 8)) * LDK + (v % (BK / 8)) * 8]) = rb[i];
                } else {
                    const int r0 = (v % (BN / 8)) * 8, kk = v / (BN / 8);
#pragma unroll
                    for (int e = 0; e < 8; ++e) sB[(r0 + e) * LDK + kk] = rb[i][e];
                }
            }
        }
    };

    if (k_begin < k_end) fetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
        __syncthreads();   // previous tile fully consumed
        stash();
        __syncthreads();
        if (k0 + BK < k_end) fetch(k0 + BK);   // global loads of the next tile overlap the MFMAs
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            V8 fa[TM], fb[TN];
            const int kk = ks * 16 + (lane >> 5) * 8;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const V8*>(&sA[(wave_m * WM + i * 32 + (lane & 31)) * LDK + kk]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const V8*>(&sB[(wave_n * WN + j * 32 + (lane & 31)) * LDK + kk]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma_32x32x16(acc[i][j], fa[i], fb[j]);
        }
    }

    const bool to_partial = gridDim.y > 1 || always_partial;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wave_m * WM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int n = n0 + wave_n * WN + j * 32 + (lane & 31);
                if (m < M && n < N) {
                    if (to_partial)
                        partial[((static_cast<size_t>(g) * gridDim.y + split) * M + m) * N + n] = acc[i][j][v];
                    else
                        ep.store(g, m, n, acc[i][j][v]);
                }
            }
}

template <class EP>
__global__ __launch_bounds__(256) void splitk_finalize_kernel(EP ep, const float* __restrict__ partial,
                                                              int splits, int M, int N)
{
    const int g = blockIdx.y;
    const size_t mn = static_cast<size_t>(M) * N;
    const size_t e = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    if (e >= mn) return;
    const float* p = partial + static_cast<size_t>(g) * splits * mn + e;
    float sum = 0.f;
    for (int s = 0; s < splits; ++s) sum += p[s * mn];
    ep.store(g, static_cast<int>(e / N), static_cast<int>(e % N), sum);
}

// Host-side launcher.  `target_blocks` steers the split-K factor; partial must hold
// groups * splits * M * N floats when splits > 1 (capacity given in floats).
template <typename T, int BM, int BN, int BK, int WGM, class AL, class BL, class EP>
inline hipError_t launch_gemm(hipStream_t st, const AL& al, const BL& bl, const EP& ep, int M, int N, int K,
                              int groups, int want_splits, float* partial, size_t partial_capacity,
                              hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr, int* splits_deferred = nullptr)
{
    // splits_deferred != nullptr: always write partial sums [split][M][N], skip the reduction pass and
    // report the number of splits; the caller's consumer kernel adds them in split order.
    const int m_tiles = (M + BM - 1) / BM, n_tiles = (N + BN - 1) / BN;
    int splits = want_splits < 1 ? 1 : want_splits;
    int kps = ((K + splits - 1) / splits + BK - 1) / BK * BK;
    splits = (K + kps - 1) / kps;
    while (splits > 1 && static_cast<size_t>(groups) * splits * M * N > partial_capacity) {
        kps += BK;
        splits = (K + kps - 1) / kps;
    }
    if (splits == 1) kps = (K + BK - 1) / BK * BK;
    if (splits_deferred) *splits_deferred = splits;
    // optional timing of the main kernel only
    launch_timed(gemm_nt_kernel<T, AL, BL, EP, BM, BN, BK, WGM>, dim3(m_tiles * n_tiles, splits, groups), dim3(kGemmThreads), 0, st,
                 ev_begin, ev_end, al, bl, ep, M, N, K, kps, n_tiles, partial, splits_deferred ? 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (splits > 1 && !splits_deferred) {
        const size_t mn = static_cast<size_t>(M) * N;
        hipLaunchKernelGGL((splitk_finalize_kernel<EP>), dim3(static_cast<unsigned>((mn + 255) / 256), groups),
                           dim3(256), 0, st, ep, partial, splits, M, N);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace dqn
