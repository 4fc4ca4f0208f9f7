// Device-side index generator: Philox4x32-10 (Salmon et al., SC'11) and the
// map from a 32-bit word to a slot choice.
#pragma once

#include <hip/hip_runtime.h>

namespace rp {

struct Philox4 {
    unsigned int x, y, z, w;
};

// Ten Philox rounds on counter (c0..c3) under key (k0, k1).
__device__ __forceinline__ Philox4 philox4x32_10(unsigned int c0, unsigned int c1, unsigned int c2,
                                                 unsigned int c3, unsigned int k0,
                                                 unsigned int k1) {
    constexpr unsigned int kMul0 = 0xD2511F53u, kMul1 = 0xCD9E8D57u;
    constexpr unsigned int kWeyl0 = 0x9E3779B9u, kWeyl1 = 0xBB67AE85u;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const unsigned int hi0 = __umulhi(kMul0, c0), lo0 = kMul0 * c0;
        const unsigned int hi1 = __umulhi(kMul1, c2), lo1 = kMul1 * c2;
        const unsigned int t0 = hi1 ^ c1 ^ k0;
        const unsigned int t2 = hi0 ^ c3 ^ k1;
        c0 = t0;
        c1 = lo1;
        c2 = t2;
        c3 = lo0;
        k0 += kWeyl0;
        k1 += kWeyl1;
    }
    return {c0, c1, c2, c3};
}

// Draw i of sampling step `step`: word (i mod 4) of the block with counter
// (i div 4, stream 0, step) and key = seed, scaled to [0, choices) by a
// 32x32 -> high-32 multiply.  choices must be below 2^32.
__device__ __forceinline__ unsigned int uniform_draw(unsigned long long seed,
                                                     unsigned long long step, unsigned int i,
                                                     unsigned int choices) {
    const Philox4 b = philox4x32_10(i >> 2, 0u, (unsigned int)step, (unsigned int)(step >> 32),
                                    (unsigned int)seed, (unsigned int)(seed >> 32));
    const unsigned int lane = i & 3u;
    const unsigned int word = lane == 0 ? b.x : lane == 1 ? b.y : lane == 2 ? b.z : b.w;
    return __umulhi(word, choices);
}

}  // namespace rp
