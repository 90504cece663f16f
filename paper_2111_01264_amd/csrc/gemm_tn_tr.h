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

// Contraction rows covered by one fill of the k-offset table, and the table's slack for the prefetch ring.
constexpr int kTnTrKChunk = 1024, kTnTrKSlack = 6 * 32;

// Bytes of LDS one workgroup of gemm_tn_tr_block needs: two buffers of each operand tile, then the k-offset table.
template <int BM, int BN> constexpr size_t gemm_tn_tr_smem()
{
    return static_cast<size_t>(2) * 32 * ((BM + 16) + (BN + 16)) * 2 + static_cast<size_t>(kTnTrKChunk + kTnTrKSlack) * sizeof(int);
}

// One workgroup's share: column block bx, split-K slice `split`, row block bz.  D = k-tiles of operand
// vectors in flight per thread (registers); LDS (smem, gemm_tn_tr_smem bytes, 16-byte aligned) is
// double-buffered.  to_partial: write fp32 slices [split][M][N] instead of calling the epilogue.
//
// Global loads: vector v of a k-tile = (contraction row v / CV, eight operand rows starting at 8 * (v % CV)), CV =
// vectors per contraction row, so the lanes of a wavefront walk ALONG a contraction row: a row of dY is 64-128
// contiguous bytes, a row of an im2col matrix a few contiguous runs of 256-384 bytes, a row of act3 / dZ of fc1
// 256 bytes -- a wavefront's load touches 8-16 cache lines.  (Walking down the contraction index instead, one
// line per lane, kept the address unit busy for 64 passes per load and set the time of a k-tile.)  What an
// operand row contributes to the address is fixed per thread; what the contraction row contributes (sample, output
// row, output column of an implicit-GEMM operand: three divisions) is computed once per workgroup into an LDS table
// and read one k-tile ahead.  Every thread issues every load (surplus threads repeat the last vector, rows past the
// end are clamped and their value masked): the number of loads in flight is the same for all wavefronts and known
// to the compiler, which can then wait for one ring slot instead of for everything outstanding.
template <class AL, class BL, class EP, int BM, int BN, int D>
__device__ inline void gemm_tn_tr_block(const AL& al, const BL& bl, const EP& ep, int M, int N, int K, int k_per_split,
                                        float* __restrict__ partial, bool to_partial, int bx, int split, int bz,
                                        unsigned char* smem)
{
    constexpr int KT = 32;
    constexpr int LDA = BM + 16, LDB = BN + 16;     // row pitch = 32 (mod 128) bytes: conflict-free transposing reads
    constexpr int MT = BM / 32, NT = BN / 32, NTW = (NT + 3) / 4;
    constexpr int CVA = BM / 8, CVB = BN / 8;
    constexpr int VA = KT * CVA, VB = KT * CVB;
    constexpr int NA = (VA + 255) / 256, NB = (VB + 255) / 256;
    static_assert(D % 2 == 0 && D <= 4, "the LDS buffer index must be a compile-time function of the ring slot; table slack");
    static_assert(!AL::kTableK, "only the B operand goes through the k-offset table");
    bf16_t (*sA)[KT * LDA] = reinterpret_cast<bf16_t (*)[KT * LDA]>(smem);
    bf16_t (*sB)[KT * LDB] = reinterpret_cast<bf16_t (*)[KT * LDB]>(smem + static_cast<size_t>(2) * KT * LDA * 2);
    int* s_ktab = reinterpret_cast<int*>(smem + static_cast<size_t>(2) * KT * (LDA + LDB) * 2);

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

    // per-thread constants of its vectors: contraction row inside the tile, operand-row part of the address, LDS slot
    int ka[NA], roa[NA], sa[NA], kb[NB], rob[NB], sb[NB];
    bool oka[NA], okb[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int v = VA % 256 == 0 ? tid + i * 256 : min(tid + i * 256, VA - 1);
        const int row0 = m0 + (v % CVA) * 8;
        ka[i] = v / CVA; oka[i] = row0 < M; roa[i] = al.row_offset(oka[i] ? row0 : 0); sa[i] = (v / CVA) * LDA + (v % CVA) * 8;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int v = VB % 256 == 0 ? tid + i * 256 : min(tid + i * 256, VB - 1);
        const int row0 = n0 + (v % CVB) * 8;
        kb[i] = v / CVB; okb[i] = row0 < N; rob[i] = bl.row_offset(okb[i] ? row0 : 0); sb[i] = (v / CVB) * LDB + (v % CVB) * 8;
    }

    const int G = lane >> 4, s = lane & 15;
    const int frag_row = 8 * (G >> 1) + (s >> 2);      // + 16 * ks (+4 for the second read)
    const int frag_col = 16 * (G & 1) + 4 * (s & 3);   // + 32 * tile

    for (int kc0 = k_begin; kc0 < k_end; kc0 += kTnTrKChunk) {
        const int kc_end = min(k_end, kc0 + kTnTrKChunk);
        if (kc0 != k_begin) __syncthreads();   // the last tile of the previous chunk has been read; the table may change
        if constexpr (BL::kTableK) {
            for (int e = tid; e < kTnTrKChunk + kTnTrKSlack; e += 256) s_ktab[e] = bl.k_offset(min(kc0 + e, k_end - 1));
            __syncthreads();
        }
        bf16x8 ra[D][NA], rb[D][NB];
        int kofb[NB];   // B's contraction-row offsets of the NEXT tile to be requested
        auto ktab_read = [&](int k0) {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                if constexpr (BL::kTableK) kofb[i] = s_ktab[k0 - kc0 + kb[i]];
                else kofb[i] = bl.k_offset(min(k0 + kb[i], k_end - 1));
            }
        };
        // requests tile k0 into ring slot `slot`; calls come with k0 ascending by KT
        auto fetch = [&](int slot, int k0) {
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int k = k0 + ka[i];
                ra[slot][i] = vec8_keep<bf16_t>(al.load_at(0, al.k_offset(min(k, k_end - 1)), roa[i]), oka[i] && k < k_end);
            }
#pragma unroll
            for (int i = 0; i < NB; ++i) rb[slot][i] = vec8_keep<bf16_t>(bl.load_at(0, kofb[i], rob[i]), okb[i] && k0 + kb[i] < k_end);
            ktab_read(k0 + KT);
        };
        auto stash = [&](int slot, int buf) {
#pragma unroll
            for (int i = 0; i < NA; ++i)
                if (VA % 256 == 0 || tid + i * 256 < VA) *reinterpret_cast<bf16x8*>(&sA[buf][sa[i]]) = ra[slot][i];
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (VB % 256 == 0 || tid + i * 256 < VB) *reinterpret_cast<bf16x8*>(&sB[buf][sb[i]]) = rb[slot][i];
        };

        // tiles beyond k_end load zeros, so the ring needs no tail logic
        ktab_read(kc0);
#pragma unroll
        for (int u = 0; u < D - 1; ++u) fetch(u, kc0 + u * KT);
        for (int kb0 = kc0; kb0 < kc_end; kb0 += D * KT) {
#pragma unroll
            for (int u = 0; u < D; ++u) {
                const int k0 = kb0 + u * KT;
                fetch((u + D - 1) % D, k0 + (D - 1) * KT);   // unconditional: see above
                if (k0 < kc_end) {                 // uniform across the workgroup
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
