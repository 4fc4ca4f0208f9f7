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

// Member i (i < choices) of a sample without duplicates: the image of i under a keyed
// permutation of [0, choices), a swap-or-not shuffle (Hoang, Morris, Rogaway, CRYPTO 2012) of
// 2 * bitlen(choices - 1) + 8 rounds.  Round r pairs x with K_r - x (mod choices), K_r = the
// scaled word r mod 4 of the block with counter (r div 4, stream 1, step), and swaps the pair
// when bit 0 of word 0 of the block with counter (larger of the pair, stream 2 + r, step) is set.
__device__ __forceinline__ unsigned int distinct_draw(unsigned long long seed,
                                                      unsigned long long step, unsigned int i,
                                                      unsigned int choices) {
    const unsigned int k0 = (unsigned int)seed, k1 = (unsigned int)(seed >> 32);
    const unsigned int s0 = (unsigned int)step, s1 = (unsigned int)(step >> 32);
    const unsigned int bitlen = choices > 1u ? 32u - (unsigned int)__clz((int)(choices - 1u)) : 0u;
    const unsigned int rounds = 2u * bitlen + 8u;
    unsigned int x = i;
    Philox4 kw = {0u, 0u, 0u, 0u};
    for (unsigned int r = 0; r < rounds; ++r) {
        if ((r & 3u) == 0u) kw = philox4x32_10(r >> 2, 1u, s0, s1, k0, k1);
        const unsigned int lane = r & 3u;
        const unsigned int word = lane == 0 ? kw.x : lane == 1 ? kw.y : lane == 2 ? kw.z : kw.w;
        const unsigned int K = __umulhi(word, choices);
        const unsigned int partner = K >= x ? K - x : K + (choices - x);
        const unsigned int larger = partner > x ? partner : x;
        const Philox4 b = philox4x32_10(larger, 2u + r, s0, s1, k0, k1);
        if (b.x & 1u) x = partner;
    }
    return x;
}

// Draw i of a batch in the replay's sampling mode (0 = with replacement).
__device__ __forceinline__ unsigned int batch_draw(unsigned int sampling, unsigned long long seed,
                                                   unsigned long long step, unsigned int i,
                                                   unsigned int choices) {
    return sampling ? distinct_draw(seed, step, i, choices) : uniform_draw(seed, step, i, choices);
}

}  // namespace rp
