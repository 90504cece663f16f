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

// The leading scalar parameters repeat the four block boundaries (first[1..4]) and what conv1's workgroups -- the longest
// ones -- need before their first load (c1.dz, in, n, per, desc, ring): the kernel arguments' first 14 dwords are preloaded
// into scalar registers when a wavefront starts (see conv_tower_kernel); the other layers read their part of the struct.
__global__ __launch_bounds__(256, 2) void wgrad_all_kernel(int f1, int f2, int f3, int f4, const bf16_t* c1_dz, const void* c1_in, int c1_n, int c1_per,
                                                           const int32_t* c1_desc, const uint8_t* c1_ring, WgradAllArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char wg_smem[];
    // grid order: conv1, conv2, conv3, fc1, small reductions -- the longest workgroups first (the grid can exceed what is
    // resident at once, and what starts late should be short)
    const int blk = blockIdx.x;
    if (blk < f1) {
        WgConvArgs c1;
        c1.dz = c1_dz; c1.in = c1_in; c1.n = c1_n; c1.per = c1_per; c1.desc = c1_desc; c1.ring = c1_ring;
        c1.partial = a.c1.partial; c1.bias_partial = a.c1.bias_partial;
        wgrad_conv_block<WgConv1>(c1, blk, 0, wg_smem);
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
