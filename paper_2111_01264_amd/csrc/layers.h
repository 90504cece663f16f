// Loader and epilogue functors that turn the Q-network's layers (Section 2.1; the Nature-DQN
// architecture the paper adopts in Section 5) into the implicit GEMMs of gemm_mfma.h.
//
// Device-side layouts (chosen so every contraction index is contiguous where it is streamed):
//   input states  uint8 [n][4][84][84]          (as handed over by the caller / the replay gather)
//   conv1 out     T     [n][20][20][32]          channels-last
//   conv2 out     T     [n][9][9][64]
//   conv3 out     T     [n][7][7][64]            = fc1 input, feature index (h*7 + w)*64 + c
//   conv1 weights [32][c][p][q]  (k = c*64 + p*8 + q, eight q's = eight adjacent input bytes)
//   conv2 weights [64][p][q][c]  conv3 weights [64][p][q][c]  fc1 weights [512][(h*7+w)*64 + c]
// The host converts to/from the public blob layout in dqn_set_params / dqn_get_params.
#pragma once
#include "gemm_mfma.h"

namespace dqn {

// ---- forward A-operands -------------------------------------------------------------------------

// conv1 im2col on the raw uint8 state: rows (b, i, j) over the 20x20 output, k = (c, p, q).
template <typename T> struct Conv1A {
    static constexpr bool kAlongK = true;
    const uint8_t* x[kMaxGroups];
    __device__ typename Vec8<T>::type load(int g, int row, int k, int rows, int k_end) const
    {
        if (row >= rows || k >= k_end) return vec8_zero<T>();
        const int b = row / 400, ij = row % 400, i = ij / 20, j = ij % 20;
        const int c = k >> 6, p = (k >> 3) & 7;
        const uint32_t* ptr = reinterpret_cast<const uint32_t*>(
            x[g] + (static_cast<size_t>(b * 4 + c) * 84 + 4 * i + p) * 84 + 4 * j);
        return vec8_from_u8<T>(ptr[0], ptr[1]);
    }
};

// conv im2col on a channels-last activation: rows (b, i, j), k = (p, q, c).
template <typename T, int CIN, int HIN, int WIN, int HOUT, int WOUT, int KS, int S> struct ConvA {
    static constexpr bool kAlongK = true;
    const T* x[kMaxGroups];
    __device__ typename Vec8<T>::type load(int g, int row, int k, int rows, int k_end) const
    {
        if (row >= rows || k >= k_end) return vec8_zero<T>();
        const int b = row / (HOUT * WOUT), ij = row % (HOUT * WOUT), i = ij / WOUT, j = ij % WOUT;
        const int c0 = k % CIN, pq = k / CIN, q = pq % KS, p = pq / KS;
        return *reinterpret_cast<const typename Vec8<T>::type*>(
            x[g] + (static_cast<size_t>(b * HIN + i * S + p) * WIN + j * S + q) * CIN + c0);
    }
};

// Dense row-major [rows][ld] operand read along k.
template <typename T> struct DenseK {
    static constexpr bool kAlongK = true;
    const T* p[kMaxGroups];
    int ld;
    __device__ typename Vec8<T>::type load(int g, int row, int k, int rows, int k_end) const
    {
        if (row >= rows || k >= k_end) return vec8_zero<T>();
        return *reinterpret_cast<const typename Vec8<T>::type*>(p[g] + static_cast<size_t>(row) * ld + k);
    }
};

// Dense [k][ld] operand whose *rows* are contiguous in memory (element (row, k) at p[k*ld + row]).
template <typename T> struct DenseM {
    static constexpr bool kAlongK = false;
    const T* p[kMaxGroups];
    int ld;
    // Branch-free (the address is clamped, the value selected): a load that may be skipped makes the
    // compiler wait for *all* outstanding loads wherever it needs one of them, which defeats a prefetch ring.
    __device__ typename Vec8<T>::type load(int g, int row0, int k, int rows, int k_end) const
    {
        const bool ok = row0 < rows && k < k_end;
        const int kc = k < k_end ? k : k_end - 1, rc = row0 < rows ? row0 : 0;
        const typename Vec8<T>::type v = *reinterpret_cast<const typename Vec8<T>::type*>(p[g] + static_cast<size_t>(kc) * ld + rc);
        return vec8_keep<T>(v, ok);
    }
    // The same load split into its contraction-row part (changes per k-tile) and its row part (fixed per thread):
    // element (row0 .. row0+7, k) sits at k_offset(k) + row_offset(row0).  kTableK: k_offset is worth caching.
    static constexpr bool kTableK = false;
    __device__ int k_offset(int k) const { return k * ld; }
    __device__ int row_offset(int row0) const { return row0; }
    __device__ typename Vec8<T>::type load_at(int g, int koff, int roff) const
    {
        return *reinterpret_cast<const typename Vec8<T>::type*>(p[g] + koff + roff);
    }
};

// ---- backward operands ----------------------------------------------------------------------------

// Data gradient of a stride-S convolution, one GEMM per stride-parity class g = (py, px):
// rows (b, y2, x2) with y = S*y2 + py, x = S*x2 + px;  k = (p2, q2, o) with p = S*p2 + py,
// q = S*q2 + px;  A(row, k) = dY[b][y2 - p2][x2 - q2][o] (zero outside the output).
template <typename T, int COUT, int HOUT, int WOUT, int HIN, int WIN, int KS, int S> struct DgradA {
    static constexpr bool kAlongK = true;
    const T* dy;
    __device__ typename Vec8<T>::type load(int, int row, int k, int rows, int k_end) const
    {
        if (row >= rows || k >= k_end) return vec8_zero<T>();
        constexpr int H2 = HIN / S, W2 = WIN / S, K2 = KS / S;
        const int b = row / (H2 * W2), yx = row % (H2 * W2), y2 = yx / W2, x2 = yx % W2;
        const int o = k % COUT, pq = k / COUT, q2 = pq % K2, p2 = pq / K2;
        const int i = y2 - p2, j = x2 - q2;
        if (i < 0 || i >= HOUT || j < 0 || j >= WOUT) return vec8_zero<T>();
        return *reinterpret_cast<const typename Vec8<T>::type*>(
            dy + (static_cast<size_t>(b * HOUT + i) * WOUT + j) * COUT + o);
    }
};

// Weights for the data gradient: rows n = input channel c, k = (p2, q2, o); [o][p][q][c] storage
// makes eight consecutive c's contiguous.
template <typename T, int CIN, int COUT, int KS, int S> struct DgradB {
    static constexpr bool kAlongK = false;
    const T* w;
    __device__ typename Vec8<T>::type load(int g, int row0, int k, int rows, int k_end) const
    {
        if (row0 >= rows || k >= k_end) return vec8_zero<T>();
        constexpr int K2 = KS / S;
        const int o = k % COUT, pq = k / COUT, q2 = pq % K2, p2 = pq / K2;
        const int p = S * p2 + g / S, q = S * q2 + g % S;
        return *reinterpret_cast<const typename Vec8<T>::type*>(
            w + (static_cast<size_t>(o) * KS * KS + p * KS + q) * CIN + row0);
    }
};

// Weight gradient, B-operand: rows n = (p, q, c) of the filter, k = output pixel (b, i, j).
template <typename T, int CIN, int HIN, int WIN, int HOUT, int WOUT, int KS, int S> struct WgradB {
    static constexpr bool kAlongK = false;
    const T* x;
    __device__ typename Vec8<T>::type load(int, int row0, int k, int rows, int k_end) const   // branch-free, see DenseM
    {
        const bool ok = row0 < rows && k < k_end;
        const int kc = k < k_end ? k : k_end - 1, rc = row0 < rows ? row0 : 0;
        const int c0 = rc % CIN, pq = rc / CIN, q = pq % KS, p = pq / KS;
        const int b = kc / (HOUT * WOUT), ij = kc % (HOUT * WOUT), i = ij / WOUT, j = ij % WOUT;
        const typename Vec8<T>::type v = *reinterpret_cast<const typename Vec8<T>::type*>(
            x + (static_cast<size_t>(b * HIN + i * S + p) * WIN + j * S + q) * CIN + c0);
        return vec8_keep<T>(v, ok);
    }
    static constexpr bool kTableK = true;   // k -> (sample, output row, output column): three divisions
    __device__ int k_offset(int k) const
    {
        const int b = k / (HOUT * WOUT), ij = k % (HOUT * WOUT), i = ij / WOUT, j = ij % WOUT;
        return ((b * HIN + i * S) * WIN + j * S) * CIN;
    }
    __device__ int row_offset(int row0) const
    {
        const int c0 = row0 % CIN, pq = row0 / CIN, q = pq % KS, p = pq / KS;
        return (p * WIN + q) * CIN + c0;
    }
    __device__ typename Vec8<T>::type load_at(int, int koff, int roff) const
    {
        return *reinterpret_cast<const typename Vec8<T>::type*>(x + koff + roff);
    }
};

// conv1 weight gradient, B-operand on the raw uint8 state: rows n = (c, p, q), k = (b, i, j).
template <typename T> struct Conv1WgradB {
    static constexpr bool kAlongK = false;
    const uint8_t* x;
    __device__ typename Vec8<T>::type load(int, int row0, int k, int rows, int k_end) const   // branch-free, see DenseM
    {
        const bool ok = row0 < rows && k < k_end;
        const int kc = k < k_end ? k : k_end - 1, rc = row0 < rows ? row0 : 0;
        const int c = rc >> 6, p = (rc >> 3) & 7;
        const int b = kc / 400, ij = kc % 400, i = ij / 20, j = ij % 20;
        const uint32_t* ptr = reinterpret_cast<const uint32_t*>(
            x + (static_cast<size_t>(b * 4 + c) * 84 + 4 * i + p) * 84 + 4 * j);
        const uint32_t lo = ptr[0], hi = ptr[1];
        const uint32_t m = ok ? 0xFFFFFFFFu : 0u;   // byte 0 converts to 0.0
        return vec8_from_u8<T>(lo & m, hi & m);
    }
    static constexpr bool kTableK = true;
    __device__ int k_offset(int k) const   // byte offsets
    {
        const int b = k / 400, ij = k % 400, i = ij / 20, j = ij % 20;
        return (b * 4 * 84 + 4 * i) * 84 + 4 * j;
    }
    __device__ int row_offset(int row0) const { return ((row0 >> 6) * 84 + ((row0 >> 3) & 7)) * 84; }
    __device__ typename Vec8<T>::type load_at(int, int koff, int roff) const
    {
        const uint32_t* ptr = reinterpret_cast<const uint32_t*>(x + koff + roff);
        return vec8_from_u8<T>(ptr[0], ptr[1]);
    }
};

// ---- epilogues ----------------------------------------------------------------------------------

// out[m][n] = act(scale * acc + bias[n]) stored as T.
template <typename T, bool RELU> struct EpiBiasAct {
    T* out[kMaxGroups];
    const float* bias[kMaxGroups];
    int ld;
    float scale;
    __device__ void store(int g, int m, int n, float v) const
    {
        v = v * scale + bias[g][n];
        if (RELU) v = fmaxf(v, 0.f);
        out[g][static_cast<size_t>(m) * ld + n] = from_float<T>(v);
    }
};

// Data gradient through the ReLU of the layer below: dz = acc * [act > 0], scattered back from the
// stride-parity row order to channels-last.
template <typename T, int HIN, int WIN, int CIN, int S> struct EpiDgradMask {
    T* dz;
    const T* act;
    __device__ void store(int g, int m, int n, float v) const
    {
        constexpr int H2 = HIN / S, W2 = WIN / S;
        const int b = m / (H2 * W2), yx = m % (H2 * W2);
        const int y = S * (yx / W2) + g / S, x = S * (yx % W2) + g % S;
        const size_t idx = (static_cast<size_t>(b * HIN + y) * WIN + x) * CIN + n;
        dz[idx] = to_float(act[idx]) > 0.f ? from_float<T>(v) : from_float<T>(0.f);
    }
};

template <typename T> struct EpiMaskDense {
    T* dz;
    const T* act;
    int ld;
    __device__ void store(int, int m, int n, float v) const
    {
        const size_t idx = static_cast<size_t>(m) * ld + n;
        dz[idx] = to_float(act[idx]) > 0.f ? from_float<T>(v) : from_float<T>(0.f);
    }
};

struct EpiGrad {
    float* grad;
    int ld;
    float scale;
    __device__ void store(int, int m, int n, float v) const { grad[static_cast<size_t>(m) * ld + n] = v * scale; }
};

}  // namespace dqn
