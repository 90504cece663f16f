// Every weight gradient of a bf16 train step in ONE launch.  After the data-gradient chain all dZ
// tensors exist, and the four weight-gradient GEMMs (conv1, conv2, conv3, fc1) and the small
// reductions (bias gradients, fc2 gradient, loss) are independent of each other; at batch 32 each is
// a few microseconds of work behind a launch that costs about as much on the host.  The grid is the
// concatenation of their workgroups.
#pragma once
#include "gemm_tn_tr.h"
#include "head_kernels.h"
#include "layers.h"

namespace dqn {

struct WgradAllArgs {
    // conv weight gradients: dW[o][n] = sum_pixels dZ[pixel][o] * im2col(X)[pixel][n], split-K slices
    DenseM<bf16_t> a1; Conv1WgradB<bf16_t> b1; int K1, kps1, splits1; float* p1;
    DenseM<bf16_t> a2; WgradB<bf16_t, 32, 20, 20, 9, 9, 4, 2> b2; int K2, kps2, splits2; float* p2;
    DenseM<bf16_t> a3; WgradB<bf16_t, 64, 9, 9, 7, 7, 3, 1> b3; int K3, kps3, splits3; float* p3;
    // fc1: dW[o][f] = sum_b dZ[b][o] * act3[b][f], written straight into the gradient blob
    DenseM<bf16_t> af, bf; EpiGrad epf; int Kf;
    BiasGradArgs small;
    int first[6];   // first block of: small reductions, conv3, conv2, fc1, conv1, end
    GatherPlan gather;   // workgroups from first[5] on gather the next minibatch (5 per sample; gather.B == 0: none)
};

constexpr int kWg1BN = 128, kWg2BN = 256, kWg3BN = 192, kWgfBN = 128;   // column blocks: 2, 2, 3, 25 per slice
constexpr size_t kWgradAllSmem =
    kSmallGradsSmem > gemm_tn_tr_smem<64, 256>() ? kSmallGradsSmem : gemm_tn_tr_smem<64, 256>();

__global__ __launch_bounds__(256) void wgrad_all_kernel(WgradAllArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char wg_smem[];
    // grid order: small reductions, conv3, conv2, fc1, conv1 -- longest workgroups first; the grid exceeds what is
    // resident at once, and the workgroups that start late should be the short ones (conv1's)
    const int blk = blockIdx.x;
    const EpiGrad none{nullptr, 0, 1.f};
    // the four boundaries in one scalar load (read one by one, each is a load-wait-branch step of its own)
    const int f1 = a.first[1], f2 = a.first[2], f3 = a.first[3], f4 = a.first[4], f5 = a.first[5];
    asm volatile("" :: "s"(f1), "s"(f2), "s"(f3), "s"(f4), "s"(f5));
    if (blk >= f5) {
        // byte copies that no part of this step depends on: they fill the memory pipes this kernel leaves idle
        const int i = blk - f5;
        gather_block(a.gather, i % 5, i / 5);
    } else if (blk < f1) {
        small_grads_block<bf16_t>(a.small, blk - a.first[0], wg_smem);
    } else if (blk < f2) {
        const int i = blk - a.first[1];
        gemm_tn_tr_block<DenseM<bf16_t>, WgradB<bf16_t, 64, 9, 9, 7, 7, 3, 1>, EpiGrad, 64, kWg3BN, 4>(
            a.a3, a.b3, none, 64, 576, a.K3, a.kps3, a.p3, true, i % 3, i / 3, 0, wg_smem);
    } else if (blk < f3) {
        const int i = blk - a.first[2];
        gemm_tn_tr_block<DenseM<bf16_t>, WgradB<bf16_t, 32, 20, 20, 9, 9, 4, 2>, EpiGrad, 64, kWg2BN, 4>(
            a.a2, a.b2, none, 64, 512, a.K2, a.kps2, a.p2, true, i % 2, i / 2, 0, wg_smem);
    } else if (blk < f4) {
        const int i = blk - a.first[3];
        gemm_tn_tr_block<DenseM<bf16_t>, DenseM<bf16_t>, EpiGrad, 64, kWgfBN, 2>(
            a.af, a.bf, a.epf, 512, 3136, a.Kf, (a.Kf + 31) / 32 * 32, nullptr, false, i % 25, 0, i / 25, wg_smem);
    } else {
        const int i = blk - a.first[4];
        gemm_tn_tr_block<DenseM<bf16_t>, Conv1WgradB<bf16_t>, EpiGrad, 32, kWg1BN, 4>(
            a.a1, a.b1, none, 32, 256, a.K1, a.kps1, a.p1, true, i % 2, i / 2, 0, wg_smem);
    }
}

}  // namespace dqn
