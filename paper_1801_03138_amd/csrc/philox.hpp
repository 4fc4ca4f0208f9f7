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
        // (written as 64-bit products: one multiply instruction yields both halves)
        const unsigned long long p0 = (unsigned long long)kMul0 * c0, p1 = (unsigned long long)kMul1 * c2;
        const unsigned int hi0 = (unsigned int)(p0 >> 32), lo0 = (unsigned int)p0;
        const unsigned int hi1 = (unsigned int)(p1 >> 32), lo1 = (unsigned int)p1;
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

// ---- the same permutation, arranged for a kernel that does nothing but draw ----------------
// Rounds of the shuffle on a domain of `choices` elements.
__device__ __forceinline__ unsigned int distinct_rounds(unsigned int choices) {
    const unsigned int bitlen = choices > 1u ? 32u - (unsigned int)__clz((int)(choices - 1u)) : 0u;
    return 2u * bitlen + 8u;
}
constexpr unsigned int kMaxDistinctRounds = 72;   // 2 * 32 + 8
constexpr unsigned int kDistinctTableWords = 80;  // the table's size: readers fetch a few entries past `rounds`

// The round constants K_r of one sampling step, r = 0 .. rounds-1, into a table of
// kMaxDistinctRounds words: lane l (l < rounds / 4, rounded up) fills entries 4 l .. 4 l + 3.
__device__ __forceinline__ void distinct_round_keys(unsigned long long seed, unsigned long long step,
                                                    unsigned int choices, unsigned int rounds,
                                                    unsigned int lane, unsigned int* table) {
    if (4u * lane < rounds) {
        const Philox4 kw = philox4x32_10(lane, 1u, (unsigned int)step, (unsigned int)(step >> 32),
                                         (unsigned int)seed, (unsigned int)(seed >> 32));
        table[4u * lane + 0u] = __umulhi(kw.x, choices);
        table[4u * lane + 1u] = __umulhi(kw.y, choices);
        table[4u * lane + 2u] = __umulhi(kw.z, choices);
        table[4u * lane + 3u] = __umulhi(kw.w, choices);
    }
}

__device__ __forceinline__ unsigned int swap_partner(unsigned int K, unsigned int x, unsigned int choices) {
    return K >= x ? K - x : K + (choices - x);
}
// the swap bit of round r for the pair whose larger member is `larger`
__device__ __forceinline__ unsigned int swap_bit(unsigned long long seed, unsigned long long step,
                                                 unsigned int r, unsigned int larger) {
    return philox4x32_10(larger, 2u + r, (unsigned int)step, (unsigned int)(step >> 32),
                         (unsigned int)seed, (unsigned int)(seed >> 32)).x & 1u;
}

// distinct_draw with the round constants taken from a table (one lane, one draw).  The table
// holds kMaxDistinctRounds words (entries past `rounds` are never used for a decision), and the
// constants of four rounds are fetched at a time, ahead of the chain of dependent blocks.
__device__ __forceinline__ unsigned int distinct_draw_serial(unsigned long long seed, unsigned long long step,
                                                             unsigned int i, unsigned int choices,
                                                             unsigned int rounds, const unsigned int* table) {
    unsigned int x = i;
    for (unsigned int r0 = 0; r0 < rounds; r0 += 4u) {
        unsigned int k[4];
#pragma unroll
        for (unsigned int j = 0; j < 4u; ++j) k[j] = table[r0 + j];
#pragma unroll
        for (unsigned int j = 0; j < 4u; ++j) {
            if (r0 + j < rounds) {
                const unsigned int partner = swap_partner(k[j], x, choices);
                if (swap_bit(seed, step, r0 + j, partner > x ? partner : x)) x = partner;
            }
        }
    }
    return x;
}

// One draw by a team of 2^G adjacent lanes, G rounds at a time.  A draw is a chain of dependent
// rounds, each costing a ten-round Philox block, so a single lane needs `rounds` block
// latencies.  But after G rounds x can only be one of 2^G values, and the pair a round decides
// on is known before the earlier decisions are: member v (1 <= v < 2^G, heap numbering: root 1,
// children 2v = "not swapped" and 2v + 1 = "swapped") takes the round at its depth d for the
// position reached by the decisions its number spells, and computes that round's bit.  The
// 2^G - 1 bits of a group then resolve in G cheap steps.  All lanes of a team return the draw;
// i must be uniform over the team.  The group's round constants are fetched into registers
// first, so that the two short chains around the Philox block are arithmetic only.
template <int G>
__device__ __forceinline__ unsigned int distinct_draw_team(unsigned long long seed, unsigned long long step,
                                                           unsigned int i, unsigned int choices,
                                                           unsigned int rounds, const unsigned int* table,
                                                           unsigned int lane) {
    constexpr unsigned int T = 1u << G;
    const unsigned int v = lane & (T - 1u);                       // member number; 0 has no node
    const unsigned int d = v ? 31u - (unsigned int)__clz((int)v) : 0u;
    const unsigned int team_shift = lane & ~(T - 1u) & 63u;
    unsigned int x = i;
    for (unsigned int r0 = 0; r0 < rounds; r0 += G) {
        // (the table has room for every index read here: r0 + G - 1 < kMaxDistinctRounds + G)
        unsigned int k[G];
#pragma unroll
        for (unsigned int j = 0; j < (unsigned int)G; ++j) k[j] = r0 + j < rounds ? table[r0 + j] : 0u;
        // this member's position: x moved by the decisions its number spells (most significant
        // first), and the constant of the round at its depth
        unsigned int xc = x, kd = k[0];
#pragma unroll
        for (unsigned int j = 0; j + 1u < (unsigned int)G; ++j) {
            if (j < d) {
                if ((v >> (d - 1u - j)) & 1u) xc = swap_partner(k[j], xc, choices);
                kd = k[j + 1u];
            }
        }
        unsigned int bit = 0;
        const unsigned int r = r0 + d;
        if (v && r < rounds) {
            const unsigned int partner = swap_partner(kd, xc, choices);
            bit = swap_bit(seed, step, r, partner > xc ? partner : xc);
        }
        const unsigned long long bits = __ballot(bit) >> team_shift;
        unsigned int node = 1;
#pragma unroll
        for (unsigned int j = 0; j < (unsigned int)G; ++j) {
            if (r0 + j < rounds) {
                const unsigned int b = (unsigned int)(bits >> node) & 1u;
                if (b) x = swap_partner(k[j], x, choices);
                node = 2u * node + b;
            }
        }
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
