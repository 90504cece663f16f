// Weight-gradient GEMM for bf16 operands on gfx950:   C[m][n] = sum_k A(m, k) * B(n, k)   where both
// operands are stored k-major -- dY is [pixel][channel], the im2col of the layer input is
// [pixel][filter element] -- i.e. the contraction index is the *slow* one.  The MFMA wants eight
// consecutive k per lane, so earlier GPUs had to transpose on the way into LDS with 2-byte writes.
// CDNA4 has a transposing LDS read (ds_read_b64_tr_b16): the tiles are staged exactly as they come
// from memory ([k][row], 16-byte vector writes) and every lane receives four consecutive k of its
// own row per read.
//
// ds_read_b64_tr_b16 semantics used here (checked on the device): within each group of 16 lanes,
// lane i receives, for e = 0..3, element (i % 4) of the 8-byte chunk addressed by lane 4*e + i/4 of
// the group.  With lane 16*G + s addressing  tile[k0 + 8*(G/2) + 4*t + s/4][col0 + 16*(G%2) + 4*(s%4)]
// lane l ends up with tile[k0 + 8*(l/32) + 4*t + e][col0 + l%32], e = 0..3: two reads (t = 0, 1) are
// one 32x32x16 operand fragment.
//
// Loaders are the row-contiguous functors of layers.h (load(g, row0, k) -> rows row0..row0+7 at k).
// A workgroup covers BM rows (one or two 32-row tiles) and BN columns of one split-K slice;
// wavefront w owns the 32-column tiles w, w+4, ...  The caller (the fused weight-gradient kernel)
// maps its block index to (column block, slice, row block).
#pragma once
#include "gemm_mfma.h"

namespace dqn {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

// One operand fragment: rows k .. k+3 (first read) and k+4 .. k+7 (second read) of this lane's column.
__device__ inline bf16x8 tr_fragment(const bf16_t* p, int pitch4 /* elements between row k and row k+4 */)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + pitch4));
    const bf16x4 blo = __builtin_bit_cast(bf16x4, lo), bhi = __builtin_bit_cast(bf16x4, hi);
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) { r[e] = blo[e]; r[4 + e] = bhi[e]; }
    return r;
}

// Bytes of LDS one workgroup of gemm_tn_tr_block needs.
template <int BM, int BN> constexpr size_t gemm_tn_tr_smem() { return static_cast<size_t>(2) * 32 * ((BM + 16) + (BN + 16)) * 2; }

// One workgroup's share: column block bx, split-K slice `split`, row block bz.  D = k-tiles of operand
// vectors in flight per thread (registers); LDS (smem, gemm_tn_tr_smem bytes, 16-byte aligned) is
// double-buffered.  to_partial: write fp32 slices [split][M][N] instead of calling the epilogue.
template <class AL, class BL, class EP, int BM, int BN, int D>
__device__ inline void gemm_tn_tr_block(const AL& al, const BL& bl, const EP& ep, int M, int N, int K, int k_per_split,
                                        float* __restrict__ partial, bool to_partial, int bx, int split, int bz,
                                        unsigned char* smem)
{
    constexpr int KT = 32;
    constexpr int LDA = BM + 16, LDB = BN + 16;     // row pitch = 32 (mod 128) bytes: conflict-free transposing reads
    constexpr int MT = BM / 32, NT = BN / 32, NTW = (NT + 3) / 4;
    constexpr int VA = KT * BM / 8, VB = KT * BN / 8;
    constexpr int NA = (VA + 255) / 256, NB = (VB + 255) / 256;
    bf16_t (*sA)[KT * LDA] = reinterpret_cast<bf16_t (*)[KT * LDA]>(smem);
    bf16_t (*sB)[KT * LDB] = reinterpret_cast<bf16_t (*)[KT * LDB]>(smem + static_cast<size_t>(2) * KT * LDA * 2);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n0 = bx * BN, m0 = bz * BM;
    const int k_begin = split * k_per_split;
    const int k_end = min(K, k_begin + k_per_split);

    f32x16 acc[MT][NTW];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    static_assert(D % 2 == 0, "the LDS buffer index must be a compile-time function of the ring slot");
    bf16x8 ra[D][NA], rb[D][NB];
    // Vector v of a k-tile = (k row v % KT, eight columns v / KT): a thread's vectors share their k row, so the
    // loader's decomposition of k (sample, pixel row, pixel column -- divisions) is computed once per thread and
    // k-tile.  Every thread issues every load (surplus threads repeat the last vector; only `stash` is
    // predicated): the number of loads in flight is then the same for all wavefronts and known to the compiler,
    // which can wait for one ring slot instead of for everything outstanding.
    auto fetch = [&](int slot, int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int v = VA % 256 == 0 ? tid + i * 256 : min(tid + i * 256, VA - 1);
            ra[slot][i] = al.load(0, m0 + (v / KT) * 8, k0 + v % KT, M, k_end);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int v = VB % 256 == 0 ? tid + i * 256 : min(tid + i * 256, VB - 1);
            rb[slot][i] = bl.load(0, n0 + (v / KT) * 8, k0 + v % KT, N, k_end);
        }
    };
    auto stash = [&](int slot, int buf) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int v = tid + i * 256;
            if (VA % 256 == 0 || v < VA) *reinterpret_cast<bf16x8*>(&sA[buf][(v % KT) * LDA + (v / KT) * 8]) = ra[slot][i];
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int v = tid + i * 256;
            if (VB % 256 == 0 || v < VB) *reinterpret_cast<bf16x8*>(&sB[buf][(v % KT) * LDB + (v / KT) * 8]) = rb[slot][i];
        }
    };

    const int G = lane >> 4, s = lane & 15;
    const int frag_row = 8 * (G >> 1) + (s >> 2);      // + 16 * ks (+4 for the second read)
    const int frag_col = 16 * (G & 1) + 4 * (s & 3);   // + 32 * tile

    // tiles beyond k_end load zeros (the loaders bound-check k), so the ring needs no tail logic
#pragma unroll
    for (int u = 0; u < D - 1; ++u) fetch(u, k_begin + u * KT);
    for (int kb = k_begin; kb < k_end; kb += D * KT) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int k0 = kb + u * KT;
            fetch((u + D - 1) % D, k0 + (D - 1) * KT);   // unconditional: see fetch
            if (k0 < k_end) {                 // uniform across the workgroup
                const int buf = u & 1;
                stash(u, buf);
                __syncthreads();     // also: every wavefront is done reading the other buffer
#pragma unroll
                for (int ks = 0; ks < KT / 16; ++ks) {
                    bf16x8 fa[MT];
#pragma unroll
                    for (int i = 0; i < MT; ++i)
                        fa[i] = tr_fragment(&sA[buf][(ks * 16 + frag_row) * LDA + i * 32 + frag_col], 4 * LDA);
#pragma unroll
                    for (int j = 0; j < NTW; ++j) {
                        const int nt = wave + 4 * j;
                        if (NT % 4 == 0 || nt < NT) {
                            const bf16x8 fb = tr_fragment(&sB[buf][(ks * 16 + frag_row) * LDB + nt * 32 + frag_col], 4 * LDB);
#pragma unroll
                            for (int i = 0; i < MT; ++i) mma_32x32x16(acc[i][j], fa[i], fb);
                        }
                    }
                }
            }
        }
    }

#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
            const int nt = wave + 4 * j;
            if (NT % 4 != 0 && nt >= NT) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int n = n0 + nt * 32 + (lane & 31);
                if (m < M && n < N) {
                    if (to_partial) partial[(static_cast<size_t>(split) * M + m) * N + n] = acc[i][j][v];
                    else ep.store(0, m, n, acc[i][j][v]);
                }
            }
        }
}

// Split-K geometry: k rows per slice (a multiple of the 32-row k-tile) and the resulting slice count,
// clamped so that the slices fit `capacity` floats.
inline void tn_tr_splits(int K, int want_splits, size_t mn, size_t capacity, int* kps_out, int* splits_out)
{
    constexpr int KT = 32;
    int splits = want_splits < 1 ? 1 : want_splits;
    int kps = ((K + splits - 1) / splits + KT - 1) / KT * KT;
    splits = (K + kps - 1) / kps;
    while (splits > 1 && static_cast<size_t>(splits) * mn > capacity) {
        kps += KT;
        splits = (K + kps - 1) / kps;
    }
    *kps_out = kps;
    *splits_out = splits;
}

}  // namespace dqn
