// fp32 train step on MFMA for networks the two-kernel step does not take: hidden layers wider
// than 256 units, two hidden layers of different widths (the paper's own network: a shared layer
// of 128 units, then a value and an advantage stream of 512 units each), wide states or action
// sets.  One dense product per kernel, fp32 16x16x4 MFMA, operands straight from global memory
// into the registers the instruction reads; the weight gradients and the optimizer are the
// second kernel of the two-kernel step, which takes any whole number of 32 x 32 tiles.
//
// At the batch sizes of the paper (16 .. 256) every one of these products is a fraction of a
// microsecond of arithmetic: what counts is that each kernel spreads over many compute units,
// requests all its operands before the first multiply, and that there are few kernels.
//
// Paper: Deep Q-Network Model (the network and the update equation), Integration with
// Reinforcement Learning Algorithm (train step with no host inputs).
#include "mm_f32.hpp"
#include "replay_kernels.hpp"
#include "trainer.hpp"

namespace rp {
namespace {

template <bool NT, int EPI, bool KSPLIT, int P>
__global__ __launch_bounds__(kMmThreads) void mm_f32_kernel(MmArgs p) {
    __shared__ float part[3][64][4];
    mm_f32_block<NT, EPI, KSPLIT, P>(p, blockIdx.x, blockIdx.y, blockIdx.z, part);
}

// The same launch with more rows of workgroups after the product's tiles_y, which copy n4
// 16-byte pieces from src to dst (up to four per thread, all requested before the first store).
struct CopyArgs {
    const f32x4* src;
    f32x4* dst;
    unsigned int n4;
};

__device__ __forceinline__ void copy_block(const CopyArgs& c, unsigned int block) {
    const unsigned int i0 = block * 4u * kMmThreads + threadIdx.x;
    f32x4 x[4];
#pragma unroll
    for (unsigned int u = 0; u < 4; ++u) {
        const unsigned int i = i0 + u * kMmThreads;
        x[u] = c.src[i < c.n4 ? i : c.n4 - 1u];
    }
#pragma unroll
    for (unsigned int u = 0; u < 4; ++u) {
        const unsigned int i = i0 + u * kMmThreads;
        if (i < c.n4) c.dst[i] = x[u];
    }
}

template <bool NT, int EPI, bool KSPLIT, int P>
__global__ __launch_bounds__(kMmThreads) void mm_f32_copy_kernel(MmArgs p, unsigned int tiles_y, CopyArgs c) {
    __shared__ float part[3][64][4];
    if (blockIdx.y >= tiles_y) {
        copy_block(c, (blockIdx.y - tiles_y) * gridDim.x + blockIdx.x);
        return;
    }
    mm_f32_block<NT, EPI, KSPLIT, P>(p, blockIdx.x, blockIdx.y, blockIdx.z, part);
}

// The first two layers in one launch, for a narrow first layer (H = 32 TPW <= 128 units over
// Dp = 16 NG1 <= 64 inputs): H2 = relu(relu(X W1 + b1) W2 + b2).  A workgroup owns a 32 x 32 tile
// of H2.  It first works out the 32 x H block of H1 its rows need (every workgroup of a tile row
// repeats that small product; the one in tile column 0 also stores the block, which the backward
// pass reads), leaves it in LDS, and contracts it with its 32 columns of W2, whose loads it
// requested before anything else: the launch takes about as long as the second layer's alone.
// Operand layout of the MFMA as in mm_tile: lane 16 q + c gives A[row c][k = 16 g + 4 q + j]
// and B[that k][column c] to MFMA j of group g and receives C[rows 4 q .. 4 q + 3][column c].
// l1, l2: the two products as a launch of their own would get them (l2.tiles_per_part for
// 32-row tiles); rows past a part's end repeat its last row and are not stored.
template <int TPW, int NG1>
__global__ __launch_bounds__(kMmThreads) void mm_f32_two_layers_kernel(MmArgs l1, MmArgs l2, unsigned int tiles_y,
                                                                       CopyArgs cp) {
    constexpr unsigned int H = 32u * TPW, NG2 = H / 16u, LD = H + 4u;
    __shared__ __attribute__((aligned(16))) float h1s[32][LD];
    if (blockIdx.y >= tiles_y) {
        copy_block(cp, (blockIdx.y - tiles_y) * gridDim.x + blockIdx.x);
        return;
    }
    const unsigned int lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const unsigned int c = lane & 15u, q = lane >> 4;
    const unsigned int part_id = blockIdx.y / l2.tiles_per_part;
    const unsigned int m_begin = part_id * l2.rows_per_part, m_end = m_begin + l2.rows_per_part;
    const unsigned int m_tile = m_begin + (blockIdx.y - part_id * l2.tiles_per_part) * 32u;
    const float* W1 = part_id ? l1.B_hi : l1.B;
    const float* W2 = part_id ? l2.B_hi : l2.B;
    const float* bias1 = part_id ? l1.bias_hi : l1.bias;
    const float* bias2 = part_id ? l2.bias_hi : l2.bias;
    // second product: this wavefront's quarter (wave >> 1, wave & 1) of the tile; its share of W2
    const unsigned int n2 = blockIdx.x * 32u + 16u * (wave & 1u) + c;
    f32x4 b2[NG2];
#pragma unroll
    for (unsigned int g = 0; g < NG2; ++g)
#pragma unroll
        for (unsigned int j = 0; j < 4; ++j) b2[g][j] = W2[(size_t)(16u * g + 4u * q + j) * l2.ldb + n2];
    const float bias2_n = bias2[n2];
    // first product: rows 16 (wave & 1) .., column blocks TPW (wave >> 1) .. + TPW of the H1 block
    const unsigned int rb = wave & 1u, cb0 = (wave >> 1) * TPW;
    const unsigned int arow = min(m_tile + 16u * rb + c, m_end - 1u);
    f32x4 a1[NG1];
#pragma unroll
    for (unsigned int g = 0; g < NG1; ++g)
        a1[g] = *reinterpret_cast<const f32x4*>(l1.A + (size_t)arow * l1.lda + 16u * g + 4u * q);
    f32x4 b1[TPW][NG1];
    float bias1_n[TPW];
#pragma unroll
    for (unsigned int i = 0; i < TPW; ++i) {
        const unsigned int n1 = (cb0 + i) * 16u + c;
#pragma unroll
        for (unsigned int g = 0; g < NG1; ++g)
#pragma unroll
            for (unsigned int j = 0; j < 4; ++j) b1[i][g][j] = W1[(size_t)(16u * g + 4u * q + j) * l1.ldb + n1];
        bias1_n[i] = bias1[n1];
    }
#pragma unroll
    for (unsigned int i = 0; i < TPW; ++i) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (unsigned int g = 0; g < NG1; ++g)
#pragma unroll
            for (unsigned int j = 0; j < 4; ++j)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[g][j], b1[i][g][j], acc, 0, 0, 0);
        const unsigned int n1 = (cb0 + i) * 16u + c;
#pragma unroll
        for (unsigned int v = 0; v < 4; ++v) {
            float x = acc[v] + bias1_n[i];
            x = x > 0.f ? x : 0.f;
            const unsigned int r = 16u * rb + 4u * q + v;
            h1s[r][n1] = x;
            if (blockIdx.x == 0 && m_tile + r < m_end) l1.C[(size_t)(m_tile + r) * l1.ldc + n1] = x;
        }
    }
    __syncthreads();
    const unsigned int r2 = 16u * (wave >> 1);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (unsigned int g = 0; g < NG2; ++g) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(&h1s[r2 + c][16u * g + 4u * q]);
#pragma unroll
        for (unsigned int j = 0; j < 4; ++j)
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j], b2[g][j], acc, 0, 0, 0);
    }
#pragma unroll
    for (unsigned int v = 0; v < 4; ++v) {
        const unsigned int m = m_tile + r2 + 4u * q + v;
        if (m >= m_end) continue;
        const float x = acc[v] + bias2_n;
        l2.C[(size_t)m * l2.ldc + n2] = x > 0.f ? x : 0.f;
    }
}

// Whether the first two layers run in one launch (mm_f32_two_layers_kernel's shapes).
bool two_layers_in_one_launch(unsigned int Dp, unsigned int H) { return (Dp == 32u || Dp == 64u) && (H == 64u || H == 128u); }

hipError_t launch_two_layers(hipStream_t st, const MmArgs& l1, const MmArgs& l2, const CopyArgs* copy) {
    MmArgs p1 = l1, p2 = l2;
    p2.tiles_per_part = (l2.rows_per_part + 31u) / 32u;
    p1.tiles_per_part = p2.tiles_per_part;
    const unsigned int tiles_y = p2.tiles_per_part * l2.parts, nx = l2.N / 32u;
    CopyArgs c{nullptr, nullptr, 0u};
    unsigned int cb = 0;
    if (copy) {
        c = *copy;
        cb = (c.n4 + 4u * kMmThreads - 1u) / (4u * kMmThreads);
    }
    const dim3 grid(nx, tiles_y + (cb + nx - 1u) / nx, 1), block(kMmThreads);
    const unsigned int H = l1.N, Dp = l1.K;
#define RP_TWO_LAYERS(TPW, NG1) \
    hipLaunchKernelGGL((mm_f32_two_layers_kernel<TPW, NG1>), grid, block, 0, st, p1, p2, tiles_y, c)
    if (H == 128u && Dp == 32u) RP_TWO_LAYERS(4, 2);
    else if (H == 128u && Dp == 64u) RP_TWO_LAYERS(4, 4);
    else if (H == 64u && Dp == 32u) RP_TWO_LAYERS(2, 2);
    else if (H == 64u && Dp == 64u) RP_TWO_LAYERS(2, 4);
    else return hipErrorInvalidValue;
#undef RP_TWO_LAYERS
    return hipGetLastError();
}

// Workgroups per tile that share a long contraction with few tiles (their partial products are
// added up by the kernel that reads the result): 1 = none.
unsigned int want_kgroups(unsigned int M, unsigned int N, unsigned int K) {
    const unsigned int tiles16 = ((M + 15u) / 16u) * (N / 16u);
    unsigned int z = 1;
    while (z < 8u && tiles16 * z < 256u && K % (2u * z * 64u) == 0 && K / (2u * z) >= 128u) z *= 2u;
    return z;
}

// kgroups > 1 (MM_PARTIAL only): a.K is the whole contraction, split over that many workgroups per tile.
// copy (kgroups 1 only): the launch also copies copy->n4 16-byte pieces, in workgroups of its own.
template <bool NT, int EPI>
hipError_t launch_mm(hipStream_t st, const MmArgs& a, unsigned int M_total, unsigned int kgroups = 1,
                     const CopyArgs* copy = nullptr) {
    MmArgs p = a;
    p.K = a.K / kgroups;
    const bool ks = kgroups > 1 || want_ksplit(M_total, a.N, p.K);
    const unsigned int TM = ks ? 16u : 32u;
    p.tiles_per_part = (a.rows_per_part + TM - 1u) / TM;
    const unsigned int tiles_y = p.tiles_per_part * a.parts;
    const dim3 block(kMmThreads);
    const unsigned int ng = (p.K >> 4) >> (ks ? 2 : 0);
    if constexpr (!NT && EPI == MM_BIAS_RELU) if (copy) {
        const unsigned int cb = (copy->n4 + 4u * kMmThreads - 1u) / (4u * kMmThreads), nx = a.N / TM;
        const dim3 grid(nx, tiles_y + (cb + nx - 1u) / nx, 1);
#define RP_MM_COPY(KS, P_) \
    hipLaunchKernelGGL((mm_f32_copy_kernel<NT, EPI, KS, P_>), grid, block, 0, st, p, tiles_y, *copy)
        if (ks) {
            if (ng >= 8) RP_MM_COPY(true, 8);
            else if (ng >= 4) RP_MM_COPY(true, 4);
            else RP_MM_COPY(true, 2);
        } else {
            if (ng >= 8) RP_MM_COPY(false, 8);
            else if (ng >= 4) RP_MM_COPY(false, 4);
            else RP_MM_COPY(false, 2);
        }
#undef RP_MM_COPY
        return hipGetLastError();
    }
    const dim3 grid(a.N / TM, tiles_y, kgroups);
    if (ks) {
        if (ng >= 8) hipLaunchKernelGGL((mm_f32_kernel<NT, EPI, true, 8>), grid, block, 0, st, p);
        else if (ng >= 4) hipLaunchKernelGGL((mm_f32_kernel<NT, EPI, true, 4>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((mm_f32_kernel<NT, EPI, true, 2>), grid, block, 0, st, p);
    } else {
        if (ng >= 8) hipLaunchKernelGGL((mm_f32_kernel<NT, EPI, false, 8>), grid, block, 0, st, p);
        else if (ng >= 4) hipLaunchKernelGGL((mm_f32_kernel<NT, EPI, false, 4>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((mm_f32_kernel<NT, EPI, false, 2>), grid, block, 0, st, p);
    }
    return hipGetLastError();
}

// ----------------------------------------------------------------------------------------
// TD target, loss and the gradient at the second hidden layer's pre-activation, one workgroup
// per experience i:  y_i = r_i + gamma (1 - term_i) max_a Q[B + i][a],  delta_i = y_i - Q[i][a_i],
// the loss term, the one non-zero of dL/dQ in row i (every wavefront works these out for
// itself: a few loads, no exchange), and
//   dZ2[i][k] = dL/dQ[i][a_i] * W3[k][a_i] * 1[H2[i][k] > 0],
// a few k per thread with all loads requested at once (a load that misses the local L2 takes
// microseconds here, so a loop of dependent iterations would pay that once per iteration).
// Thread 0 of block 0 also advances Adam's step count and its bias corrections 1 - beta^t, from
// running products beta^t kept in double precision (no power function on the device).
// ----------------------------------------------------------------------------------------
struct MidTdArgs {
    unsigned int B, G, A, Ap;
    // kz > 1: the output layer's product arrives as kz partial products [2B x Ap], part_stride
    // elements apart, without the bias; this kernel adds them up (in a fixed order), adds the
    // bias (b3 for the rows of s, b3_hi for the rows of s') and writes Q
    unsigned int kz;
    const float* part;
    size_t part_stride;
    const float *b3, *b3_hi;
    float* Q;
    const int* act;
    const float* rew;
    const unsigned char* term;
    float gamma;
    unsigned int loss_kind;
    float beta1, beta2;
    float *y, *delta, *lossi, *dQ;
    const float* W3;     // [G x Ap]
    const float* H2;     // [2B x G]
    float* dZ2;          // [B x G]
    TrainCounters* ctr;
};

__global__ __launch_bounds__(256) void mid_td_kernel(MidTdArgs p) {
    const unsigned int tid = threadIdx.x, lane = tid & 63u;
    const unsigned int i = blockIdx.x;
    // this thread's hidden units and their activations: requested before anything else
    constexpr unsigned int KU = 4;
    const float* h2 = p.H2 + (size_t)i * p.G;
    float hv[KU];
#pragma unroll
    for (unsigned int u = 0; u < KU; ++u) {
        const unsigned int k = tid + 256u * u;
        hv[u] = k < p.G ? h2[k] : 0.f;
    }
    if (i == 0 && tid == 0) {
        const unsigned long long t = p.ctr->adam_t + 1;
        const double pw1 = p.ctr->pw1 * (double)p.beta1, pw2 = p.ctr->pw2 * (double)p.beta2;
        p.ctr->adam_t = t;
        p.ctr->pw1 = pw1;
        p.ctr->pw2 = pw2;
        p.ctr->c1 = (float)(1.0 - pw1);
        p.ctr->c2 = (float)(1.0 - pw2);
    }
    unsigned int ai = (unsigned int)p.act[i];
    if (ai >= p.A) ai = p.A - 1;  // an out-of-range action must not turn into a wild address
    float best = -INFINITY, q;
    if (p.kz > 1) {
        // (every wavefront for itself; the first one stores the rows)
        // (all loads requested before the first sum: partial z beyond kz re-reads partial 0 and
        // counts as zero)
        constexpr unsigned int KZ = 8;
        const size_t row_s = (size_t)i * p.Ap, row_n = (size_t)(p.B + i) * p.Ap;
        float pa[KZ];
#pragma unroll
        for (unsigned int z = 0; z < KZ; ++z) pa[z] = p.part[(z < p.kz ? z : 0u) * p.part_stride + row_s + ai];
        for (unsigned int k = lane; k < p.Ap; k += 64) {
            float ps[KZ], pn[KZ];
#pragma unroll
            for (unsigned int z = 0; z < KZ; ++z) {
                const size_t at = (z < p.kz ? z : 0u) * p.part_stride;
                ps[z] = p.part[at + row_s + k];
                pn[z] = p.part[at + row_n + k];
            }
            float qs = 0.f, qn = 0.f;
#pragma unroll
            for (unsigned int z = 0; z < KZ; ++z) {
                qs += z < p.kz ? ps[z] : 0.f;
                qn += z < p.kz ? pn[z] : 0.f;
            }
            qs += p.b3[k];
            qn += p.b3_hi[k];
            if (k < p.A) best = fmaxf(best, qn);
            if (tid < 64) {
                p.Q[row_s + k] = qs;
                p.Q[row_n + k] = qn;
            }
        }
        q = 0.f;
#pragma unroll
        for (unsigned int z = 0; z < KZ; ++z) q += z < p.kz ? pa[z] : 0.f;
        q += p.b3[ai];
    } else {
        const float* qn = p.Q + (size_t)(p.B + i) * p.Ap;
        for (unsigned int k = lane; k < p.A; k += 64) best = fmaxf(best, qn[k]);
        q = p.Q[(size_t)i * p.Ap + ai];
    }
    best = wave_max(best);
    float w3[KU];
#pragma unroll
    for (unsigned int u = 0; u < KU; ++u) {
        const unsigned int k = tid + 256u * u;
        w3[u] = k < p.G ? p.W3[(size_t)k * p.Ap + ai] : 0.f;
    }
    const float y = p.rew[i] + (p.term[i] ? 0.f : p.gamma * best);
    const float d = y - q;
    float li, slope;
    if (p.loss_kind == RP_MSE || fabsf(d) <= 1.f) {
        li = 0.5f * d * d;
        slope = d;
    } else {
        li = fabsf(d) - 0.5f;
        slope = d > 0.f ? 1.f : -1.f;
    }
    const float g = -slope / (float)p.B;
    for (unsigned int k = tid; k < p.Ap; k += 256) p.dQ[(size_t)i * p.Ap + k] = (k == ai) ? g : 0.f;
    if (tid == 0) {
        p.y[i] = y;
        p.delta[i] = d;
        p.lossi[i] = li;
    }
    float* dz = p.dZ2 + (size_t)i * p.G;
#pragma unroll
    for (unsigned int u = 0; u < KU; ++u) {
        const unsigned int k = tid + 256u * u;
        if (k < p.G) dz[k] = hv[u] > 0.f ? g * w3[u] : 0.f;
    }
    // (layers wider than 256 * KU units: the rest, one unit at a time)
    for (unsigned int k = tid + 256u * KU; k < p.G; k += 256)
        dz[k] = h2[k] > 0.f ? g * p.W3[(size_t)k * p.Ap + ai] : 0.f;
}

}  // namespace

bool mid_step_supported(const train_config& cfg, const replay* rp_) {
    // fp32 states and parameters; every matrix a whole number of 32 x 32 tiles (hidden widths are
    // multiples of 64, states and action sets are padded to multiples of 32 in the workspace)
    return cfg.param_dtype == RP_F32 && rp_->cfg.state_dtype == RP_F32 && rp_->cfg.layout == RP_PAIR &&
           cfg.hidden % 64 == 0 && cfg.hidden2 % 64 == 0;
}

unsigned int mid_step_kernels(const trainer* t) { return two_layers_in_one_launch(t->Dp, t->H) ? 6u : 7u; }

// Enqueue the step's kernels from the gathered batch on (X = [S ; S'], the per-row fields).
hipError_t enqueue_mid_step(trainer* t, hipStream_t st, unsigned int* count) {
    const unsigned int B = t->B, H = t->H, G = t->Hb, Dp = t->Dp, Ap = t->Ap;
    const float* X = static_cast<const float*>(t->X);
    float* H1 = static_cast<float*>(t->H1);
    float* H2 = static_cast<float*>(t->H2);
    float* dZ2 = static_cast<float*>(t->dZ2);
    float* dZ1 = static_cast<float*>(t->dZ1);
    const float* w = t->w;
    const float* wt = t->wt ? t->wt : t->w;   // the network that evaluates s'
    unsigned int n = 0;
    // forward: the rows of s through the trained network, the rows of s' through the target's
    // (the same when there is none: then the 2B rows are one part)
    const unsigned int parts = t->wt ? 2u : 1u, rows = t->wt ? B : 2u * B;
    MmArgs a;
    a.mask = nullptr; a.ldmask = 0; a.rows_per_part = rows; a.parts = parts; a.tiles_per_part = 0; a.c_stride = 0;
    a.A = X; a.lda = Dp; a.B = w + t->oW1; a.B_hi = wt + t->oW1; a.ldb = H;
    a.bias = w + t->ob1; a.bias_hi = wt + t->ob1; a.C = H1; a.ldc = H; a.N = H; a.K = Dp;
    // (when dZ1's product will run beside the second layer's tiles, which update W2 in place, it
    // takes W2 from a copy: made here, by workgroups of the first layer's launch)
    const bool dz1_beside_tiles = dz1_rides_with_tiles(B, H, G);
    const CopyArgs w2_copy{reinterpret_cast<const f32x4*>(w + t->oW2), reinterpret_cast<f32x4*>(t->w2t),
                           H * G / 4u};
    hipError_t e;
    if (two_layers_in_one_launch(Dp, H)) {
        MmArgs a2 = a;
        a2.A = H1; a2.lda = H; a2.B = w + t->oW2; a2.B_hi = wt + t->oW2; a2.ldb = G;
        a2.bias = w + t->ob2; a2.bias_hi = wt + t->ob2; a2.C = H2; a2.ldc = G; a2.N = G; a2.K = H;
        e = launch_two_layers(st, a, a2, dz1_beside_tiles ? &w2_copy : nullptr);
        if (e != hipSuccess) return e;
        ++n;
    } else {
        e = launch_mm<false, MM_BIAS_RELU>(st, a, 2u * B, 1, dz1_beside_tiles ? &w2_copy : nullptr);
        if (e != hipSuccess) return e;
        ++n;
        a.A = H1; a.lda = H; a.B = w + t->oW2; a.B_hi = wt + t->oW2; a.ldb = G;
        a.bias = w + t->ob2; a.bias_hi = wt + t->ob2; a.C = H2; a.ldc = G; a.N = G; a.K = H;
        e = launch_mm<false, MM_BIAS_RELU>(st, a, 2u * B);
        if (e != hipSuccess) return e;
        ++n;
    }
    a.A = H2; a.lda = G; a.B = w + t->oW3; a.B_hi = wt + t->oW3; a.ldb = Ap;
    a.bias = w + t->ob3; a.bias_hi = wt + t->ob3; a.C = t->Q; a.ldc = Ap; a.N = Ap; a.K = G;
    // a long contraction with few tiles: several workgroups per tile, each a stretch of K; the TD
    // kernel adds their partial products up
    const unsigned int kz = want_kgroups(2u * B, Ap, G);
    if (kz > 1) {
        a.C = t->qpart;
        a.c_stride = (size_t)2u * B * Ap;
        e = launch_mm<false, MM_PARTIAL>(st, a, 2u * B, kz);
    } else {
        e = launch_mm<false, MM_BIAS>(st, a, 2u * B);
    }
    if (e != hipSuccess) return e;
    ++n;
    {
        MidTdArgs d;
        d.B = B; d.G = G; d.A = t->cfg.num_actions; d.Ap = Ap;
        d.kz = kz; d.part = t->qpart; d.part_stride = (size_t)2u * B * Ap;
        d.b3 = w + t->ob3; d.b3_hi = wt + t->ob3;
        d.Q = t->Q; d.act = t->act; d.rew = t->rew; d.term = t->term;
        d.gamma = t->cfg.gamma; d.loss_kind = t->cfg.loss; d.beta1 = t->cfg.beta1; d.beta2 = t->cfg.beta2;
        d.y = t->y; d.delta = t->delta; d.lossi = t->lossi; d.dQ = t->dQ;
        d.W3 = w + t->oW3; d.H2 = H2; d.dZ2 = dZ2; d.ctr = t->ctr;
        hipLaunchKernelGGL(mid_td_kernel, dim3(B), dim3(256), 0, st, d);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        ++n;
    }
    // dZ1 = (dZ2 W2^T) masked by the first ReLU: W2 is [H x G], i.e. K contiguous as it stands
    a.rows_per_part = B; a.parts = 1;
    a.A = dZ2; a.lda = G; a.B = w + t->oW2; a.B_hi = a.B; a.ldb = G; a.bias = nullptr; a.bias_hi = nullptr;
    a.mask = H1; a.ldmask = H; a.C = dZ1; a.ldc = H; a.N = H; a.K = G;
    bool folded = false;
    if (dz1_beside_tiles) {
        a.B = t->w2t; a.B_hi = a.B;
        a.tiles_per_part = (B + 15u) / 16u;
        unsigned int launches = 0;
        e = enqueue_weights_update(t, st, &folded, &a, &launches);
        if (e != hipSuccess) return e;
        n += launches;
    } else {
        e = launch_mm<true, MM_MASK>(st, a, B);
        if (e != hipSuccess) return e;
        ++n;
        e = enqueue_weights_update(t, st, &folded);
        if (e != hipSuccess) return e;
        ++n;
    }
    unsigned int nh = 0;
    if (!folded) e = enqueue_head_update(t, st, &nh);
    if (count) *count = n + nh;
    return e;
}

}  // namespace rp
