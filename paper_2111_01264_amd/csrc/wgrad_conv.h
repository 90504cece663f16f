// Weight gradient of a convolution layer, sample by sample (Section 2.1: first-order minimisation with respect to
// theta; the layers are those of the adopted Nature-DQN setup, Section 5):
//
//     dW[o][n] = sum over samples b and output pixels (i, j) of  dZ[b][i][j][o] * X_b(i, j; n)
//
// where n runs over the filter elements and X_b(i, j; n) is the input element under filter element n at output pixel
// (i, j) -- the im2col matrix, which is never materialised.  The contraction runs over pixels, the slow index of both
// operands, so the operand fragments of the matrix instruction are formed with the transposing LDS read
// (ds_read_b64_tr_b16, see gemm_tn_tr.h).
//
// Unit of work: one sample (conv1: half a sample, ten output rows).  A workgroup owns a contiguous range of items and
// the WHOLE gradient tile [C_out][n] in its accumulators (split-K over samples: it writes one fp32 slice, the
// optimiser kernel adds the slices in order).  Per item it stages the sample's dZ ([pixel][C_out], as stored) and the
// sample's INPUT (not its im2col: 36 KB instead of ~130 KB for conv2) in LDS with fully coalesced 16-byte loads --
// requested one item ahead into registers -- and then walks the pixels in steps of 16: the B fragment of filter-element
// tile nt is read straight out of the input image, each lane addressing the 8-byte chunk (pixel k, elements n..n+3) at
//     image[pixel_offset(k) + element_offset(n)]
// (the transposing read takes an arbitrary address per lane, so im2col costs nothing but this address).  Two barriers
// per item, instead of one per 32 contraction rows as a tiled GEMM over the im2col matrix needs, and every input
// byte crosses the memory system once per sample.
//
// conv1 reads the raw uint8 state (converted to bf16 on the way into LDS: 0..255 are exact), either from assembled
// states or, given a descriptor table (sample_desc), frame by frame from the replay memory.
#pragma once
#include <type_traits>
#include <utility>

#include "common.h"
#include "gemm_tn_tr.h"

namespace dqn {

typedef uint32_t wg_u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte vector the compiler keeps in registers (HIP's uint4 struct, in an array, went to scratch memory)

template <int CIN_, int HIN_, int WIN_, int COUT_, int HOUT_, int WOUT_, int KS_, int S_, int PITCH_, bool U8_, int CS_>
struct WgGeo {
    static constexpr int CIN = CIN_, HIN = HIN_, WIN = WIN_, COUT = COUT_, HOUT = HOUT_, WOUT = WOUT_, KS = KS_, S = S_;
    static constexpr int PITCH = PITCH_;                       // LDS elements per input pixel (channels-last layers)
    static constexpr bool U8 = U8_;                            // conv1: uint8 planes [c][row][col], filter element n = (c, p, q)
    static constexpr int ITEMS = U8_ ? 2 : 1;                  // items per sample
    static constexpr int ROWS = HOUT_ / ITEMS;                 // output rows per item
    static constexpr int KPIX = ROWS * WOUT_;                  // contraction rows per item: 200, 81, 49
    static constexpr int KPAD = (KPIX + 15) / 16 * 16;         // 208, 96, 64
    static constexpr int N = KS_ * KS_ * CIN_;                 // 256, 512, 576
    static constexpr int CS = CS_;                             // column blocks: a workgroup owns N / CS filter elements (its accumulators must fit the register file twice per SIMD)
    static constexpr int MT = COUT_ / 32, NT = N / 32 / CS_, NTW = (NT + 3) / 4;   // 32 x 32 tiles per workgroup, per wavefront
    static constexpr int LDA = COUT_ + 16;                     // LDS pitch of a dZ row
    static constexpr int IN_ROWS = U8_ ? S_ * (ROWS - 1) + KS_ : HIN_;           // conv1: 44 image rows per item
    static constexpr int IN_ELEMS = U8_ ? CIN_ * IN_ROWS * WIN_ : HIN_ * WIN_ * PITCH_;
    static constexpr int IN_VECS = U8_ ? CIN_ * (IN_ROWS * WIN_ / 16) : HIN_ * WIN_ * CIN_ / 8;   // 16-byte vectors per item
    static constexpr int DZ_VECS = KPIX * COUT_ / 8;
    static constexpr int NVI = (IN_VECS + 255) / 256, NVD = (DZ_VECS + 255) / 256;
    static constexpr size_t SMEM = static_cast<size_t>(IN_ELEMS) * 2 + static_cast<size_t>(KPAD) * LDA * 2;
    static_assert(!U8_ || (IN_ROWS * WIN_) % 16 == 0, "a channel's rows of one item are whole 16-byte vectors");
    static_assert(!U8_ || (S_ * ROWS * WIN_) % 16 == 0, "the second item of a sample starts on a 16-byte boundary");
    static_assert(IN_ELEMS % 8 == 0 && (KPAD * LDA) % 2 == 0, "LDS regions stay 16-byte / 4-byte aligned");
};
typedef WgGeo<4, 84, 84, 32, 20, 20, 8, 4, 0, true, 1> WgConv1;
typedef WgGeo<32, 20, 20, 64, 9, 9, 4, 2, 40, false, 2> WgConv2;
typedef WgGeo<64, 9, 9, 64, 7, 7, 3, 1, 72, false, 3> WgConv3;

struct WgConvArgs {
    const bf16_t* dz;        // [n][HOUT][WOUT][COUT]
    const void* in;          // conv2 / conv3: bf16 [n][HIN][WIN][CIN];  conv1: uint8 [n][4][84][84], unused with desc
    float* partial;          // [slices][COUT][N] fp32
    float* bias_partial;     // [slices][COUT] fp32: column sums of dZ over the slice's items (the bias gradient)
    int n;                   // samples
    int per;                 // items per workgroup (the host sizes the grid so that every workgroup has at least one)
    const int32_t* desc;     // conv1: [n][kDescInts] (entries 0..3: replay slots of the frames of s, -1 = zero frame) or null
    const uint8_t* ring;     // conv1 with desc: the replay memory's frame array
};

// Two transposing reads at arbitrary addresses -> one operand fragment (rows k..k+3 from p0, k+4..k+7 from p1).
__device__ inline bf16x8 tr_fragment2(const bf16_t* p0, const bf16_t* p1)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p1));
    const bf16x4 blo = __builtin_bit_cast(bf16x4, lo), bhi = __builtin_bit_cast(bf16x4, hi);
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) { r[e] = blo[e]; r[4 + e] = bhi[e]; }
    return r;
}

// f(integral_constant<int, I>) for I = I0 .. N-1: a loop whose index is a compile-time constant inside the body.
template <int I, int N, class F> __device__ inline void static_for(F& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Eight pixels (two 32-bit words) -> eight bf16: float(b) of a byte has at most eight significant bits, so its bf16 is the
// upper half of the float, bit for bit; v_perm_b32 packs two upper halves into one word.
__device__ inline bf16x8 bf16x8_from_bytes(uint32_t lo, uint32_t hi)
{
    wg_u32x4 d;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t w = h ? hi : lo;
        const uint32_t f0 = __builtin_bit_cast(uint32_t, static_cast<float>(w & 0xFFu));
        const uint32_t f1 = __builtin_bit_cast(uint32_t, static_cast<float>((w >> 8) & 0xFFu));
        const uint32_t f2 = __builtin_bit_cast(uint32_t, static_cast<float>((w >> 16) & 0xFFu));
        const uint32_t f3 = __builtin_bit_cast(uint32_t, static_cast<float>(w >> 24));
        d[2 * h] = __builtin_amdgcn_perm(f1, f0, 0x07060302u);       // [f1 >> 16 : f0 >> 16]
        d[2 * h + 1] = __builtin_amdgcn_perm(f3, f2, 0x07060302u);
    }
    return __builtin_bit_cast(bf16x8, d);
}

// Workgroup (slice `wg`, column block `cb`) of layer G's weight gradient (256 threads; smem: G::SMEM bytes, 16-byte aligned).
template <class G>
__device__ inline void wgrad_conv_block(const WgConvArgs& a, int wg, int cb, unsigned char* smem)
{
    constexpr int LDA = G::LDA, MT = G::MT, NT = G::NT, NTW = G::NTW, NVI = G::NVI, NVD = G::NVD, KSTEPS = G::KPAD / 16;
    bf16_t* sIn = reinterpret_cast<bf16_t*>(smem);
    bf16_t* sDz = sIn + G::IN_ELEMS;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int total = a.n * G::ITEMS;
    const int first = wg * a.per, last = min(total, first + a.per);
    if (first >= last) return;

    // once per workgroup: zero rows of dZ beyond the item's pixels (their products vanish whatever the B operand reads)
    for (int e = tid; e < (G::KPAD - G::KPIX) * LDA; e += 256) sDz[G::KPIX * LDA + e] = static_cast<bf16_t>(0.f);

    // this lane's share of an operand fragment (see gemm_tn_tr.h): contraction row inside a 16-step, first of its four columns
    const int G4 = lane >> 4, s16 = lane & 15;
    const int krow = 8 * (G4 >> 1) + (s16 >> 2);
    const int col4 = 16 * (G4 & 1) + 4 * (s16 & 3);
    // LDS element offsets of this lane's B chunks: pixel part (one per contraction row it addresses: pixel -> top-left corner
    // of its window in the input image; rows past the item's pixels point at pixel 0) + filter-element part (one per tile)
    int pixoff[KSTEPS][2];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int k = ks * 16 + krow + 4 * t;
            const int kc = k < G::KPIX ? k : 0, i = kc / G::WOUT, j = kc % G::WOUT;
            pixoff[ks][t] = G::U8 ? (G::S * i) * G::WIN + G::S * j : ((G::S * i) * G::WIN + G::S * j) * G::PITCH;
        }
    int coloff[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        const int nt = wave + 4 * j;
        const int n = (cb * NT + (nt < NT ? nt : 0)) * 32 + col4;
        if constexpr (G::U8) coloff[j] = (n >> 6) * (G::IN_ROWS * G::WIN) + ((n >> 3) & 7) * G::WIN + (n & 7);
        else coloff[j] = ((n / (G::KS * G::CIN)) * G::WIN + (n / G::CIN) % G::KS) * G::PITCH + n % G::CIN;
    }

    f32x16 acc[MT][NTW];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    // The bias gradient (column sums of dZ) is taken on the way: a thread's dZ vectors all belong to the same eight
    // channels (256 is a multiple of the vectors per row), so it adds them up in eight registers while it stores them to
    // LDS; the threads' sums meet in LDS once, at the end, in thread order.  (A reduction kernel of its own read every
    // dZ tensor from memory a second time.)
    float bsum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    static_assert(256 % (G::COUT / 8) == 0, "a thread's dZ vectors share their channel chunk");

    // Operands are requested TWO items ahead into registers (one dependent round trip to memory takes about as long as
    // two items' matrix work; with one item ahead every item waited for its loads).
    wg_u32x4 pin[2][NVI], pdz[2][NVD];
    uint32_t keep[2] = {15u, 15u};   // conv1 with descriptors: bit c = frame c of the requested item is a real frame (not all zeros)
    uint32_t live[2] = {~0u, ~0u};   // all ones if the requested item exists, zero for the padding item of an odd range (its dZ is stored as zeros)
    // conv1 with descriptors: replay slots of the four frames of an item, one set per register set.  The request of an item
    // starts by asking for the NEXT item's slots (into the other set): asked for after the item's own loads, that small load
    // would be the youngest one in flight, and waiting for it would wait for everything before it.
    int sl[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    auto fetch_slots = [&](auto ps_, int item) {
        constexpr int ps = decltype(ps_)::value;
        if constexpr (G::U8) {
            if (a.desc) {
                const int32_t* dp = a.desc + static_cast<size_t>(min(item, last - 1) / G::ITEMS) * kDescInts;
#pragma unroll
                for (int c = 0; c < 4; ++c) sl[ps][c] = dp[c];
            }
        }
    };
    // No request is ever skipped (an item past the range repeats the last one): with a load behind a condition the
    // compiler waits for everything outstanding wherever it needs one register set, and the prefetch is lost.
    auto fetch = [&](auto ps_, int item_) {
        constexpr int ps = decltype(ps_)::value;
        fetch_slots(std::integral_constant<int, ps ^ 1>{}, item_ + 1);
        live[ps] = item_ < last ? ~0u : 0u;
        const int item = min(item_, last - 1);
        const int b = item / G::ITEMS, h = item % G::ITEMS;
        const wg_u32x4* dzp = reinterpret_cast<const wg_u32x4*>(a.dz + (static_cast<size_t>(b) * G::HOUT * G::WOUT + h * G::KPIX) * G::COUT);
#pragma unroll
        for (int u = 0; u < NVD; ++u) pdz[ps][u] = dzp[min(tid + u * 256, G::DZ_VECS - 1)];
        if constexpr (G::U8) {
            constexpr int VPC = G::IN_ROWS * G::WIN / 16;   // vectors per channel: 231
#pragma unroll
            for (int u = 0; u < NVI; ++u) {
                const int v = min(tid + u * 256, G::IN_VECS - 1), c = v / VPC, w = v % VPC;
                const size_t within = static_cast<size_t>(h) * (G::S * G::ROWS * G::WIN) + static_cast<size_t>(w) * 16;
                if (a.desc) {   // a zero frame is loaded from slot 0 and masked when it is stored (masking here would wait for the load)
                    const int fs = c == 0 ? sl[ps][0] : c == 1 ? sl[ps][1] : c == 2 ? sl[ps][2] : sl[ps][3];
                    pin[ps][u] = *reinterpret_cast<const wg_u32x4*>(a.ring + static_cast<size_t>(fs < 0 ? 0 : fs) * kFrameBytes + within);
                } else {
                    pin[ps][u] = *reinterpret_cast<const wg_u32x4*>(static_cast<const uint8_t*>(a.in) + (static_cast<size_t>(b) * 4 + c) * kFrameBytes + within);
                }
            }
        } else {
            const wg_u32x4* inp = reinterpret_cast<const wg_u32x4*>(static_cast<const bf16_t*>(a.in) + static_cast<size_t>(b) * G::HIN * G::WIN * G::CIN);
#pragma unroll
            for (int u = 0; u < NVI; ++u) pin[ps][u] = inp[min(tid + u * 256, G::IN_VECS - 1)];
        }
        if constexpr (G::U8) {
            if (a.desc) keep[ps] = (sl[ps][0] < 0 ? 0u : 1u) | (sl[ps][1] < 0 ? 0u : 2u) | (sl[ps][2] < 0 ? 0u : 4u) | (sl[ps][3] < 0 ? 0u : 8u);
        }
    };
    // registers -> LDS.  Surplus threads hold a copy of the last vector and store it again (same bytes, same place): with a
    // predicate around a store the compiler no longer counts the loads in flight and waits for ALL of them, the next items' included.
    auto stash = [&](auto ps_) {
        constexpr int ps = decltype(ps_)::value;
#pragma unroll
        for (int u = 0; u < NVD; ++u) {
            const int v = min(tid + u * 256, G::DZ_VECS - 1);
            const wg_u32x4 d = pdz[ps][u] & live[ps];
            *reinterpret_cast<wg_u32x4*>(sDz + (v / (G::COUT / 8)) * LDA + (v % (G::COUT / 8)) * 8) = d;
            if (cb == 0) {
                const bf16x8 dv = __builtin_bit_cast(bf16x8, d);
                const float w = (G::DZ_VECS % 256 == 0 || tid + u * 256 < G::DZ_VECS) ? 1.f : 0.f;   // surplus threads hold a copy
#pragma unroll
                for (int e = 0; e < 8; ++e) bsum[e] += w * static_cast<float>(dv[e]);
            }
        }
#pragma unroll
        for (int u = 0; u < NVI; ++u) {
            const int v = min(tid + u * 256, G::IN_VECS - 1);
            if constexpr (G::U8) {
                // sixteen pixels -> sixteen bf16 (exact), contiguous in the plane: the LDS planes keep the image's row pitch
                bf16_t* d = sIn + static_cast<size_t>(v) * 16;
                const uint32_t m = (keep[ps] >> (v / (G::IN_ROWS * G::WIN / 16))) & 1u ? ~0u : 0u;
                *reinterpret_cast<bf16x8*>(d) = bf16x8_from_bytes(pin[ps][u][0] & m, pin[ps][u][1] & m);
                *reinterpret_cast<bf16x8*>(d + 8) = bf16x8_from_bytes(pin[ps][u][2] & m, pin[ps][u][3] & m);
            } else {
                *reinterpret_cast<wg_u32x4*>(sIn + (v / (G::CIN / 8)) * G::PITCH + (v % (G::CIN / 8)) * 8) = pin[ps][u];
            }
        }
    };
    // the item staged in LDS: sixteen pixels per step, the fragments of step ks + 1 requested before the matrix work of step ks
    auto contract = [&]() {
        bf16x8 fa[2][MT], fb[2][NTW];
        auto frags = [&](auto buf_, auto ks_) {
            constexpr int buf = decltype(buf_)::value, ks = decltype(ks_)::value;
#pragma unroll
            for (int i = 0; i < MT; ++i) fa[buf][i] = tr_fragment(sDz + (ks * 16 + krow) * LDA + i * 32 + col4, 4 * LDA);
#pragma unroll
            for (int j = 0; j < NTW; ++j)
                if (NT % 4 == 0 || wave + 4 * j < NT)
                    fb[buf][j] = tr_fragment2(sIn + pixoff[ks][0] + coloff[j], sIn + pixoff[ks][1] + coloff[j]);
        };
        frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        auto step = [&](auto ks_) {
            constexpr int ks = decltype(ks_)::value, buf = ks & 1;
            if constexpr (ks + 1 < KSTEPS) frags(std::integral_constant<int, (ks + 1) & 1>{}, std::integral_constant<int, ks + 1>{});
#pragma unroll
            for (int j = 0; j < NTW; ++j)
                if (NT % 4 == 0 || wave + 4 * j < NT)
#pragma unroll
                    for (int i = 0; i < MT; ++i) mma_32x32x16(acc[i][j], fa[buf][i], fb[buf][j]);
            __builtin_amdgcn_sched_barrier(0);
        };
        static_for<0, KSTEPS>(step);
    };

    typedef std::integral_constant<int, 0> P0;
    typedef std::integral_constant<int, 1> P1;
    if (last - first == 1) {
        // a single item (small minibatches: one workgroup per item keeps the chain of dependent steps shortest)
        fetch_slots(P0{}, first);
        fetch(P0{}, first);
        stash(P0{});
        __syncthreads();
        contract();
    } else {
        // items in pairs, one per register set; an odd range ends with a padding item whose dZ is zero
        fetch_slots(P0{}, first);
        fetch(P0{}, first);
        fetch(P1{}, first + 1);
        for (int it = first; it < last; it += 2) {
            if (it != first) __syncthreads();   // every wavefront has finished reading the previous item
            stash(P0{});
            fetch(P0{}, it + 2);
            __syncthreads();
            contract();
            __syncthreads();
            stash(P1{});
            fetch(P1{}, it + 3);
            __syncthreads();
            contract();
        }
    }

    if (cb == 0) {   // workgroup-uniform
        __syncthreads();   // the last item has been read; sIn is free
        constexpr int LDS_E = 256 + 8;                  // padded: the reads below stride through the threads in steps of CH
        float* sSum = reinterpret_cast<float*>(smem);   // [8][256 threads]
        static_assert(8 * LDS_E * 4 <= G::SMEM, "the partial sums fit the operand buffers");
#pragma unroll
        for (int e = 0; e < 8; ++e) sSum[e * LDS_E + tid] = bsum[e];
        __syncthreads();
        // channel ch is held by the threads t = ch / 8 + CH * k (k = 0 .. 256 / CH - 1).  P adjacent lanes share a channel:
        // lane p adds eight consecutive k (eight independent LDS reads), the P sums meet in a fixed shuffle tree.  (One lane
        // per channel walking all 256 / CH values was a chain of dependent LDS reads: 1.5 - 2.4 us at the end of every block.)
        {
            constexpr int CH = G::COUT / 8, P = 256 / G::COUT, PER = 256 / CH / P;
            static_assert(PER == 8 && (P == 4 || P == 8), "eight values per lane, a power-of-two group of lanes per channel");
            const int ch = tid / P, p = tid % P;
            float v[PER];
#pragma unroll
            for (int k = 0; k < PER; ++k) v[k] = sSum[(ch & 7) * LDS_E + (ch >> 3) + CH * (p * PER + k)];
            float sum = 0.f;
#pragma unroll
            for (int k = 0; k < PER; ++k) sum += v[k];
#pragma unroll
            for (int d = P / 2; d >= 1; d >>= 1) sum += __shfl_down(sum, d, P);
            if (p == 0) a.bias_partial[static_cast<size_t>(wg) * G::COUT + ch] = sum;
        }
    }
    float* out = a.partial + static_cast<size_t>(wg) * G::COUT * G::N;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
            const int nt = wave + 4 * j;
            if (NT % 4 != 0 && nt >= NT) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int n = (cb * NT + nt) * 32 + (lane & 31);
                out[static_cast<size_t>(m) * G::N + n] = acc[i][j][v];
            }
        }
}

}  // namespace dqn
