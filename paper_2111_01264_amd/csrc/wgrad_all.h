// Every weight gradient of a bf16 train step in ONE launch.  After the data-gradient chain all dZ
// tensors exist, and the four weight gradients (conv1, conv2, conv3, fc1) and the small
// reductions (bias gradients, fc2 gradient, loss) are independent of each other; at batch 32 each is
// a few microseconds of work behind a launch that costs about as much on the host.  The grid is the
// concatenation of their workgroups: conv layers sample by sample (wgrad_conv.h), fc1 as a tiled GEMM
// over the batch (gemm_tn_tr.h).
#pragma once
#include "gemm_tn_tr.h"
#include "head_kernels.h"
#include "layers.h"
#include "wgrad_conv.h"

namespace dqn {

struct WgradAllArgs {
    WgConvArgs c1, c2, c3;   // split-K over samples: workgroup j of a layer writes slice j
    // fc1: dW[o][f] = sum_b dZ[b][o] * act3[b][f], written straight into the gradient blob
    DenseM<bf16_t> af, bf; EpiGrad epf; int Kf;
    BiasGradArgs small;
    int first[6];   // first block of: small reductions, conv3, conv2, fc1, conv1, end
};

constexpr int kWgfBN = 128;
constexpr int kWgfCols = (3136 + kWgfBN - 1) / kWgfBN;   // column blocks of fc1's gradient: 25
constexpr size_t kWgradAllSmem = []() {
    size_t m = kSmallGradsSmem;
    if (gemm_tn_tr_smem<64, kWgfBN>() > m) m = gemm_tn_tr_smem<64, kWgfBN>();
    if (WgConv1::SMEM > m) m = WgConv1::SMEM;
    if (WgConv2::SMEM > m) m = WgConv2::SMEM;
    if (WgConv3::SMEM > m) m = WgConv3::SMEM;
    return (m + 15) / 16 * 16;
}();

__global__ __launch_bounds__(256) void wgrad_all_kernel(WgradAllArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char wg_smem[];
    // grid order: small reductions, conv3, conv2, fc1, conv1
    const int blk = blockIdx.x;
    // the four boundaries in one scalar load (read one by one, each is a load-wait-branch step of its own)
    const int f1 = a.first[1], f2 = a.first[2], f3 = a.first[3], f4 = a.first[4];
    asm volatile("" :: "s"(f1), "s"(f2), "s"(f3), "s"(f4));
    if (blk < f1) {
        small_grads_block<bf16_t>(a.small, blk - a.first[0], wg_smem);
    } else if (blk < f2) {
        wgrad_conv_block<WgConv3>(a.c3, (blk - f1) / WgConv3::CS, (blk - f1) % WgConv3::CS, wg_smem);
    } else if (blk < f3) {
        wgrad_conv_block<WgConv2>(a.c2, (blk - f2) / WgConv2::CS, (blk - f2) % WgConv2::CS, wg_smem);
    } else if (blk < f4) {
        const int i = blk - f3;
        gemm_tn_tr_block<DenseM<bf16_t>, DenseM<bf16_t>, EpiGrad, 64, kWgfBN, 2>(
            a.af, a.bf, a.epf, 512, 3136, a.Kf, (a.Kf + 31) / 32 * 32, nullptr, false, i % kWgfCols, 0, i / kWgfCols, wg_smem);
    } else {
        wgrad_conv_block<WgConv1>(a.c1, blk - f4, 0, wg_smem);
    }
}

}  // namespace dqn
