// Philox4x32-10 (Salmon et al., SC'11), device + host inline, written from the published
// definition: ten rounds of two 32x32->64 multiplies with key bumps by the Weyl constants.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dqn {

struct Philox4 {
    uint32_t x[4];
};

__host__ __device__ inline Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1)
{
    const uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
    const uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t pa = static_cast<uint64_t>(kMulA) * c0;
        const uint64_t pb = static_cast<uint64_t>(kMulB) * c2;
        const uint32_t n0 = static_cast<uint32_t>(pb >> 32) ^ c1 ^ k0;
        const uint32_t n1 = static_cast<uint32_t>(pb);
        const uint32_t n2 = static_cast<uint32_t>(pa >> 32) ^ c3 ^ k1;
        const uint32_t n3 = static_cast<uint32_t>(pa);
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += kWeylA;
        k1 += kWeylB;
    }
    Philox4 out;
    out.x[0] = c0; out.x[1] = c1; out.x[2] = c2; out.x[3] = c3;
    return out;
}

// counter = (index, tag, step lo, step hi), key = (seed lo, seed hi)
__host__ __device__ inline Philox4 philox_draw(uint64_t seed, uint32_t tag, uint64_t step, uint32_t index)
{
    return philox4x32_10(index, tag, static_cast<uint32_t>(step), static_cast<uint32_t>(step >> 32),
                         static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
}

constexpr uint32_t kTagAct = 1;
constexpr uint32_t kTagSample = 2;

}  // namespace dqn
