// One dense fp32 product per workgroup grid on 16x16x4 MFMA, operands straight from global memory
// into the registers the instruction reads: the device code of the fp32 train step's layered
// products, shared by the kernels that run one product per launch and by the launch that runs a
// product beside the weight-gradient tiles.
#pragma once
#include <hip/hip_runtime.h>

namespace rp {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) char* gbytes;   // global memory, byte-addressed

constexpr unsigned int kMmThreads = 256;

enum { MM_BIAS_RELU = 0, MM_BIAS = 1, MM_MASK = 2, MM_PARTIAL = 3 };

// C = A B (+ epilogue).  A is [M x K] with K contiguous.  NT: B is [N x K], K contiguous;
// otherwise B is [K x N], N contiguous.  The M rows come in `parts` equal parts (1, or 2: the
// rows of s and the rows of s'); a tile never straddles two parts, and the tiles of part 1 take
// B_hi and bias_hi (the frozen target network's layer) instead of B and bias.
struct MmArgs {
    const float* A;
    unsigned int lda;
    const float* B;
    const float* B_hi;
    unsigned int ldb;
    const float* bias;
    const float* bias_hi;
    const float* mask;       // MM_MASK: [M x N], the output is kept where mask > 0
    unsigned int ldmask;
    float* C;
    unsigned int ldc;
    unsigned int rows_per_part, parts, tiles_per_part;
    unsigned int N, K;       // K: what one workgroup contracts over
    // MM_PARTIAL: the contraction is split over gridDim.z workgroups per tile as well, K columns
    // each; workgroup z stores its partial product (no bias) c_stride elements after the one before.
    size_t c_stride;
};

// One wavefront's 16 x 16 tile of C over the K range [k_lo, k_lo + 16 * ngroups).
// Lane l = 16 q + c of a 16x16x4 MFMA supplies A[row c][k slot q] and B[k slot q][column c] and
// receives C[rows 4 q .. 4 q + 3][column c].  A group is 16 consecutive k: MFMA j of a group
// takes k = 16 g + 4 q + j in slot q, so that a lane's share of A (and of B when it is K
// contiguous) for a whole group is one 16-byte load.  P groups are in flight at a time: the
// loads of group g + P are requested as soon as group g has been multiplied.  Loads never
// branch: a group past the end re-reads the last one and is multiplied by zero.
template <bool NT, int P>
__device__ __forceinline__ f32x4 mm_tile(const float* __restrict__ A, unsigned int lda, unsigned int arow,
                                         const float* __restrict__ B, unsigned int ldb, unsigned int bcol,
                                         unsigned int k_lo, unsigned int ngroups, unsigned int lane) {
    const unsigned int q = lane >> 4;
    const gbytes ap = (gbytes)reinterpret_cast<const char*>(A) + ((size_t)arow * lda + k_lo + 4u * q) * 4u;
    const gbytes bp = NT ? (gbytes)reinterpret_cast<const char*>(B) + ((size_t)bcol * ldb + k_lo + 4u * q) * 4u
                         : (gbytes)reinterpret_cast<const char*>(B) + ((size_t)(k_lo + 4u * q) * ldb + bcol) * 4u;
    f32x4 a[P], b[P];
    auto load = [&](int s, unsigned int g) {
        const unsigned int gc = g < ngroups ? g : ngroups - 1u;
        a[s] = *(const __attribute__((address_space(1))) f32x4*)(ap + (size_t)gc * 64u);
        if (NT) {
            b[s] = *(const __attribute__((address_space(1))) f32x4*)(bp + (size_t)gc * 64u);
        } else {
            const gbytes rb = bp + (size_t)gc * 16u * ldb * 4u;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                b[s][j] = *(const __attribute__((address_space(1))) float*)(rb + (size_t)j * ldb * 4u);
        }
    };
#pragma unroll
    for (int s = 0; s < P; ++s) load(s, (unsigned int)s);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (unsigned int g0 = 0; g0 < ngroups; g0 += P) {
#pragma unroll
        for (int s = 0; s < P; ++s) {
            const bool live = g0 + s < ngroups;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(live ? a[s][j] : 0.f, b[s][j], acc, 0, 0, 0);
            load(s, g0 + s + P);
        }
    }
    return acc;
}

// Tiles of 32 x 32 per workgroup, a 16 x 16 quarter per wavefront over the whole K (KSPLIT
// false), or 16 x 16 per workgroup with K split over its four wavefronts, summed through LDS
// in a fixed order (KSPLIT true: long K, few tiles).
// (bx, by, bz: the workgroup's place in the product's grid; part: 3 KB of LDS, used when KSPLIT)
template <bool NT, int EPI, bool KSPLIT, int P>
__device__ __forceinline__ void mm_f32_block(const MmArgs& p, unsigned int bx, unsigned int by, unsigned int bz,
                                             float (*part)[64][4]) {
    const unsigned int lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const unsigned int c = lane & 15u, q = lane >> 4;
    constexpr unsigned int TM = KSPLIT ? 16u : 32u;
    const unsigned int part_id = by / p.tiles_per_part;
    const unsigned int m_begin = part_id * p.rows_per_part, m_end = m_begin + p.rows_per_part;
    const unsigned int m0 = m_begin + (by - part_id * p.tiles_per_part) * TM + (KSPLIT ? 0u : 16u * (wave >> 1));
    const unsigned int n0 = bx * TM + (KSPLIT ? 0u : 16u * (wave & 1u));
    const float* Bm = part_id ? p.B_hi : p.B;
    const float* bias = part_id ? p.bias_hi : p.bias;
    // rows past the part's end re-read its last row; they are not stored
    const unsigned int arow = min(m0 + c, m_end - 1u);
    const unsigned int groups = p.K >> 4;
    const unsigned int ng = KSPLIT ? groups >> 2 : groups;
    const unsigned int k_lo = (EPI == MM_PARTIAL ? bz * p.K : 0u) + (KSPLIT ? wave * ng * 16u : 0u);
    f32x4 acc = mm_tile<NT, P>(p.A, p.lda, arow, Bm, p.ldb, n0 + c, k_lo, ng, lane);
    if (KSPLIT) {
        if (wave) {
#pragma unroll
            for (int v = 0; v < 4; ++v) part[wave - 1u][lane][v] = acc[v];
        }
        __syncthreads();
        if (wave) return;
#pragma unroll
        for (unsigned int w = 0; w < 3; ++w)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] += part[w][lane][v];
    }
    const unsigned int n = n0 + c;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const unsigned int m = m0 + 4u * q + v;
        if (m >= m_end) continue;
        float x = acc[v];
        if (EPI == MM_BIAS_RELU) {
            x += bias[n];
            x = x > 0.f ? x : 0.f;
        } else if (EPI == MM_BIAS) {
            x += bias[n];
        } else if (EPI == MM_MASK) {
            if (!(p.mask[(size_t)m * p.ldmask + n] > 0.f)) x = 0.f;
        }
        p.C[(EPI == MM_PARTIAL ? bz * p.c_stride : 0) + (size_t)m * p.ldc + n] = x;
    }
}

// K is split over a workgroup's wavefronts when a product has few tiles and a long contraction.
inline bool want_ksplit(unsigned int M, unsigned int N, unsigned int K) {
    const unsigned int tiles32 = ((M + 31u) / 32u) * (N / 32u);
    return K >= 256u && K % 64u == 0 && tiles32 < 256u;
}

// Whether dZ1 = (dZ2 W2^T) masked, [B x H] over K = G, runs in the launch of the weight-gradient
// tiles rather than in one of its own: that launch holds one variant of the product (16 x 16 per
// workgroup, K over its wavefronts, eight groups of 16 in flight), the one a batch of the
// paper's sizes and a wide second layer take.
inline bool dz1_rides_with_tiles(unsigned int B, unsigned int H, unsigned int G) {
    return want_ksplit(B, H, G) && G >= 512u;
}

}  // namespace rp
