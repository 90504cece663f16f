// Every weight gradient of a bf16 train step in ONE launch.  After the data-gradient chain all dZ
// tensors exist, and the four weight gradients (conv1, conv2, conv3, fc1) and the small
// reductions (bias gradients, fc2 gradient, loss) are independent of each other; at batch 32 each is
// a few microseconds of work behind a launch that costs about as much on the host.  The grid is the
// concatenation of their workgroups: conv layers sample by sample (wgrad_conv.h), fc1 tile by tile over the
// minibatch (wgrad_fc1.h).
#pragma once
#include "gemm_tn_tr.h"
#include "head_kernels.h"
#include "layers.h"
#include "wgrad_conv.h"
#include "wgrad_fc1.h"

namespace dqn {

struct WgradAllArgs {
    WgConvArgs c1, c2, c3;   // split-K over samples: workgroup j of a layer writes slice j
    WgFc1Args f1;            // fc1 (wgrad_fc1.h), written straight into the gradient blob
    BiasGradArgs small;
    int first[6];   // first block of: conv1, conv2, conv3, fc1, small reductions, end
};

constexpr size_t kWgradAllSmem = []() {
    size_t m = kSmallGradsSmem;
    if (kWgF1Smem > m) m = kWgF1Smem;
    if (WgConv1::SMEM > m) m = WgConv1::SMEM;
    if (WgConv2::SMEM > m) m = WgConv2::SMEM;
    if (WgConv3::SMEM > m) m = WgConv3::SMEM;
    return (m + 15) / 16 * 16;
}();

__global__ __launch_bounds__(256, 2) void wgrad_all_kernel(WgradAllArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char wg_smem[];
    // grid order: conv1, conv2, conv3, fc1, small reductions -- the longest workgroups first (the grid can exceed what is
    // resident at once, and what starts late should be short)
    const int blk = blockIdx.x;
    // the four boundaries in one scalar load (read one by one, each is a load-wait-branch step of its own)
    const int f1 = a.first[1], f2 = a.first[2], f3 = a.first[3], f4 = a.first[4];
    asm volatile("" :: "s"(f1), "s"(f2), "s"(f3), "s"(f4));
    if (blk < f1) {
        wgrad_conv_block<WgConv1>(a.c1, blk, 0, wg_smem);
    } else if (blk < f2) {
        wgrad_conv_block<WgConv2>(a.c2, (blk - f1) / WgConv2::CS, (blk - f1) % WgConv2::CS, wg_smem);
    } else if (blk < f3) {
        wgrad_conv_block<WgConv3>(a.c3, (blk - f2) / WgConv3::CS, (blk - f2) % WgConv3::CS, wg_smem);
    } else if (blk < f4) {
        const int i = blk - f3;
        wgrad_fc1_block(a.f1, i % kWgF1Cols, i / kWgF1Cols, wg_smem);
    } else {
        small_grads_block<bf16_t>(a.small, blk - f4, wg_smem);
    }
}

}  // namespace dqn
