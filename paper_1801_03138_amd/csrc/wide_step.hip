// Mixed-precision train step for wide networks, where the step is bound by the dense products:
// bf16 operands, fp32 accumulation on 32x32x16 MFMA, fp32 master weights and Adam moments.
//
// Every product is brought to one form, C[m][n] = sum_k A[m][k] * Bt[n][k] with both operands
// stored K-contiguous, which is the form the MFMA lane layout reads with 16-byte loads.  The
// forward layers therefore read transposed bf16 copies of the weights, and the weight
// gradients, which contract over the batch, read transposed copies of the activations and of
// the pre-activation gradients; the kernels that produce those tensors write both orientations.
// A bias gradient is the product of the error with a vector of ones: the transposed activation
// buffers carry one extra row of ones, so the bias gradient falls out of the weight-gradient
// product as one more output row.  The weight-gradient products contract over the batch, which
// is long while their outputs are small: they are split along the batch over several workgroups
// per tile, and the optimizer kernels add the fp32 partial products up.
//
// Paper: Integration with Reinforcement Learning Algorithm (train step with no host inputs),
// Deep Q-Network Model (update equation).
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <type_traits>
#include <vector>

#include "gather_block.hpp"
#include "replay_kernels.hpp"
#include "trainer.hpp"

namespace rp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short bf16_bits;
// 16 bytes in flight between a load and its use.  A native vector type: arrays of HIP's uint4
// struct are not promoted to registers by the compiler and end up in scratch memory.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr unsigned int kGemmThreads = 256;

__device__ __forceinline__ float bits_to_float(bf16_bits b) {
    return __uint_as_float((unsigned int)b << 16);
}

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) {
    return __builtin_bit_cast(bf16x8, v);
}

// Row (0..31 within the 32x32 tile) of accumulator element v held by `lane`; its column is lane % 32.
__device__ __forceinline__ unsigned int acc_row(unsigned int v, unsigned int lane) {
    return 8u * (v >> 2) + 4u * (lane >> 5) + (v & 3u);
}

// ----------------------------------------------------------------------------------------
// Optimizer applied to one parameter from inside a product's epilogue.
// ----------------------------------------------------------------------------------------
struct OptState {
    float *w, *g, *m, *v;
    unsigned int opt;
    float lr, beta1, beta2, eps;
    const TrainCounters* ctr;
    float* wt;                  // frozen target network, or null
    unsigned int sync_every;    // the target takes the new weights when Adam's t is a multiple of this
};

// What every update of one step shares: Adam's bias corrections 1 - beta^t and whether the
// target network is due for a sync (t was advanced earlier in the step).
struct OptStep {
    float c1, c2;
    bool sync;
};
__device__ __forceinline__ OptStep opt_step(const OptState& o) {
    OptStep s;
    s.c1 = o.ctr->c1;
    s.c2 = o.ctr->c2;
    s.sync = o.wt && o.sync_every && o.ctr->adam_t % o.sync_every == 0;
    return s;
}

__device__ __forceinline__ float opt_update(const OptState& o, size_t k, float gk, const OptStep& st) {
    float wk = o.w[k];
    o.g[k] = gk;
    if (o.opt == RP_SGD) {
        wk -= o.lr * gk;
    } else {
        const float mk = o.beta1 * o.m[k] + (1.f - o.beta1) * gk;
        const float vk = o.beta2 * o.v[k] + (1.f - o.beta2) * gk * gk;
        o.m[k] = mk;
        o.v[k] = vk;
        wk -= o.lr * (mk / st.c1) / (sqrtf(vk / st.c2) + o.eps);
    }
    o.w[k] = wk;
    if (st.sync) o.wt[k] = wk;
    return wk;
}

// ----------------------------------------------------------------------------------------
// Epilogues of the tiled product.
// "Staged" epilogues (bf16 output in the product's own orientation; pre() also gets the first
// row of the workgroup's tile): the product is formed with
// the MFMA operands exchanged, so a lane holds four consecutive columns of one output row; it
// passes each value through pre(), rounds to bf16 and parks the wavefront's tile in LDS, from
// where it leaves in 16-byte pieces -- eight lanes write one 128-byte run of a row -- through
// store().  Other epilogues get the raw 32x32 accumulator tiles.
// ----------------------------------------------------------------------------------------
// out[m][n] = bf16(relu(acc + bias[n]))
struct EpiForward {
    static constexpr bool kStaged = true;
    const float* bias;
    const float* bias_hi;     // bias for rows from m_split on (the target network's)
    unsigned int m_split;
    bf16_bits* out;
    unsigned int ldo;
    unsigned int M, N;
    __device__ __forceinline__ float pre(unsigned int m0, unsigned int n, float x) const {
        x += (m0 >= m_split ? bias_hi : bias)[n < N ? n : 0u];
        return x > 0.f ? x : 0.f;
    }
    // eight consecutive columns n..n+7 of row m (N is a multiple of 8)
    __device__ __forceinline__ void store(unsigned int m, unsigned int n, const u32x4& v) const {
        if (m < M && n < N) *reinterpret_cast<u32x4*>(out + (size_t)m * ldo + n) = v;
    }
};

// out[m][n] = bf16(acc) where mask[m][n] > 0, else 0  (the ReLU derivative; both [M x ld]).
// Columns from N up to the next multiple of 8 are written as zeros.
struct EpiMask {
    static constexpr bool kStaged = true;
    const bf16_bits* mask;
    bf16_bits* out;
    unsigned int ld;
    unsigned int M, N;
    __device__ __forceinline__ float pre(unsigned int, unsigned int, float x) const { return x; }
    __device__ __forceinline__ void store(unsigned int m, unsigned int n, const u32x4& v) const {
        if (m >= M || n >= N) return;
        const size_t at = (size_t)m * ld + n;
        const u32x4 k = *reinterpret_cast<const u32x4*>(mask + at);
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // a bf16 is positive when it is non-zero with the sign bit clear (NaN counts as not)
            const unsigned int lo = k[e] & 0xFFFFu, hi = k[e] >> 16;
            const bool lo_on = lo != 0u && lo <= 0x7F80u && n + 2u * e < N;
            const bool hi_on = hi != 0u && hi <= 0x7F80u && n + 2u * e + 1u < N;
            o[e] = (lo_on ? v[e] & 0xFFFFu : 0u) | (hi_on ? v[e] & 0xFFFF0000u : 0u);
        }
        *reinterpret_cast<u32x4*>(out + at) = o;
    }
};

// part[split][m][n] = acc: the partial product of one K split, added up by a later kernel
struct EpiPartial {
    static constexpr bool kStaged = false;
    float* part;
    unsigned int M, N;
    __device__ __forceinline__ void tile(unsigned int mb, unsigned int nb, const f32x16& c,
                                         unsigned int lane, unsigned int split) const {
        const unsigned int n = nb + (lane & 31u);
        if (n >= N) return;
#pragma unroll
        for (unsigned int v = 0; v < 16; ++v) {
            const unsigned int m = mb + acc_row(v, lane);
            if (m < M) part[((size_t)split * M + m) * N + n] = c[v];
        }
    }
};

// ----------------------------------------------------------------------------------------
// Tiled product C = A Bt^T: a workgroup of four wavefronts owns a BM x BN tile and keeps the
// accumulators in registers; the wavefronts split the tile WGM x WGN ways.  BK-wide slices of
// both operands go from global memory straight into LDS (global_load_lds, 16 bytes per lane, no
// trip through registers), two slices deep: the next slice is in flight while the current one
// is multiplied.  Such a load writes the wavefront's 64 pieces to consecutive LDS addresses,
// so LDS rows cannot be padded; instead the 16-byte piece at position c of row r holds piece
// c ^ swz(r) of that row's slice (the lanes fetch their global pieces in that order), which
// spreads the MFMA operand reads of 16 consecutive rows over all banks.
// The contraction may also be split over `splits` workgroups per tile, each taking K / splits
// consecutive columns and handing its split number to the epilogue.
// K / splits must be a multiple of BK.  Loads of rows beyond M / N are redirected to the last valid row:
// such rows only feed accumulator rows / columns that the epilogue never stores.
// ----------------------------------------------------------------------------------------
struct GemmArgs {
    const bf16_bits* A;
    unsigned int lda;
    const bf16_bits* Bt;
    const bf16_bits* Bt_hi;        // B operand of the tiles whose first row is m_split or beyond
    unsigned int m_split;
    unsigned int ldb;
    unsigned int M, N, K;          // K: columns one workgroup contracts over
    unsigned int tiles_m, tiles_n, splits;
    unsigned int band;             // tiles are numbered band by band: `band` tile columns at a time, rows fastest after that
};

template <int BM, int BN, int BK, int WGM, int WGN, int NSTAGE = 2>
constexpr size_t gemm_lds_bytes() {
    const size_t slices = NSTAGE * (size_t)(BM + BN) * BK * 2;
    // staged epilogues park every wavefront's bf16 tile, rows padded by 16 bytes
    const size_t parked = 4 * (size_t)(BM / WGM) * ((BN / WGN) * 2 + 16);
    return slices > parked ? slices : parked;
}

#define RP_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define RP_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

template <int BM, int BN, int BK, int WGM, int WGN, int NSTAGE = 2, class Epi>
__device__ __forceinline__ void gemm_nt_block(const GemmArgs& p, const Epi& epi, unsigned int block) {
    static_assert(WGM * WGN == 4, "four wavefronts");
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "slices in flight");
    static_assert(BK == 32 || BK == 64, "slice width");
    constexpr int RB = BK * 2;                             // bytes per LDS row
    constexpr int CPR = RB / 16;                           // 16-byte pieces per row
    constexpr int RPI = 64 / CPR;                          // rows one wavefront-wide load covers
    constexpr int A_BYTES = BM * RB, STAGE = (BM + BN) * RB;
    constexpr int GA = BM / RPI / 4, GB = BN / RPI / 4;    // loads per wavefront, slice and operand
    static_assert(GA >= 1 && GB >= 1 && BM % (4 * RPI) == 0 && BN % (4 * RPI) == 0, "loader shape");
    constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;  // 32x32 tiles per wavefront
    static_assert(TM >= 1 && TN >= 1, "wavefront shape");

    extern __shared__ uint4 gemm_smem[];
    unsigned char* smem = reinterpret_cast<unsigned char*>(gemm_smem);

    // Workgroups are dealt to the eight XCDs round-robin; each XCD gets a contiguous range of
    // tile numbers, and tiles are numbered so that such a range is a compact block of the output
    // (bands of `band` tile columns, within a band row by row): the workgroups that share an L2
    // then share as few operand panels as possible, and each panel is fetched by few XCDs.
    const unsigned int per_split = p.tiles_m * p.tiles_n, n_tiles = per_split * p.splits;
    const unsigned int per_xcd = (n_tiles + 7u) / 8u;
    const unsigned int tile_s = (block & 7u) * per_xcd + (block >> 3);
    if (tile_s >= n_tiles) return;
    const unsigned int split = tile_s / per_split, tile = tile_s % per_split;
    const unsigned int band_tiles = p.tiles_m * p.band, band_id = tile / band_tiles, in_band = tile % band_tiles;
    const unsigned int width = min(p.band, p.tiles_n - band_id * p.band);
    const unsigned int m0 = (in_band / width) * BM, n0 = (band_id * p.band + in_band % width) * BN;
    const unsigned int k_base = split * p.K;

    const unsigned int tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const unsigned int wn = wave % WGN, wm = wave / WGN;
    // LDS has 64 four-byte banks: 16 lanes' 16-byte reads are conflict-free when they fall into 16
    // different slots of a 256-byte span.  256 / RB rows share such a span; successive groups of
    // that many rows get their pieces rotated by XOR with the group number.
    auto swz = [](unsigned int r) { return (r / (256u / RB)) & (CPR - 1u); };

    // loader: wavefront w moves row groups w*GA.. of A and w*GB.. of B; a lane's piece lands at
    // LDS position `lane` of the group, so the lane fetches the piece that belongs there
    // A request's address is a wavefront-uniform base (the operand, advanced by the slice's
    // column: scalar registers) plus a per-lane byte offset that never changes (one 32-bit
    // register per request, at most a tile's rows away from row 0 of the operand, which must
    // therefore stay below 4 GiB), and its LDS destination is uniform as well: issuing a request
    // then costs two scalar instructions and the load itself, no vector arithmetic.
    const unsigned int lr = lane / CPR, lc = lane % CPR;
    const unsigned int wave_u = __builtin_amdgcn_readfirstlane(wave);
    unsigned int a_off[GA], b_off[GB];
#pragma unroll
    for (int u = 0; u < GA; ++u) {
        const unsigned int r = (wave * GA + u) * RPI + lr;
        unsigned int gm = m0 + r;
        gm = gm < p.M ? gm : p.M - 1;
        a_off[u] = (gm * p.lda + (lc ^ swz(r)) * 8u) * 2u;
    }
#pragma unroll
    for (int u = 0; u < GB; ++u) {
        const unsigned int r = (wave * GB + u) * RPI + lr;
        unsigned int gn = n0 + r;
        gn = gn < p.N ? gn : p.N - 1;
        b_off[u] = (gn * p.ldb + (lc ^ swz(r)) * 8u) * 2u;
    }
    typedef const __attribute__((address_space(1))) char* gchar;
    const gchar a_base = (gchar)reinterpret_cast<const char*>(p.A + k_base);
    const gchar b_base = (gchar)reinterpret_cast<const char*>((m0 >= p.m_split ? p.Bt_hi : p.Bt) + k_base);
    // request u (0 .. GA + GB - 1) of a slice: one wavefront-wide 16-byte-per-lane load into LDS
    constexpr int L = GA + GB;                              // loads per wavefront and slice
    auto fetch_one = [&](int u, unsigned int buf, unsigned int k0) {
        if (u < GA) {
            unsigned char* sa = smem + buf * STAGE + (wave_u * GA) * 1024u;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a_base + (size_t)k0 * 2u + a_off[u < GA ? u : 0]),
                                             RP_LDS_PTR(sa + u * 1024), 16, 0, 0);
        } else {
            unsigned char* sb = smem + buf * STAGE + A_BYTES + (wave_u * GB) * 1024u;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(b_base + (size_t)k0 * 2u + b_off[u >= GA ? u - GA : 0]),
                                             RP_LDS_PTR(sb + (u - GA) * 1024), 16, 0, 0);
        }
    };
    auto fetch = [&](unsigned int buf, unsigned int k0) {
#pragma unroll
        for (int u = 0; u < L; ++u) fetch_one(u, buf, k0);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const unsigned int a_row = (wm * TM * 32u + (lane & 31u)) * RB;
    const unsigned int b_row = (wn * TN * 32u + (lane & 31u)) * RB;
    const unsigned int sw = swz(lane & 31u), half = lane >> 5;
    // One slice's multiply.  A wavefront issues in order, and it is alone on its SIMD when the
    // workgroup has the compute unit to itself, so everything that has to happen during a
    // slice is interleaved with its MFMAs by hand: the LDS reads of step s + 1 are issued before
    // the MFMAs of step s (two sets of fragment registers), and the global -> LDS requests of a
    // later slice (FETCH) are spread out between the MFMAs, one at a time, instead of being
    // issued in a burst during which no MFMA could start.  The scheduling barriers keep the
    // compiler from regrouping them.
    auto multiply = [&](unsigned int buf, auto fetch_flag, unsigned int fbuf, unsigned int fk0) {
        constexpr bool FETCH = decltype(fetch_flag)::value;
        const unsigned char* as = smem + buf * STAGE + a_row;
        const unsigned char* bs = smem + buf * STAGE + A_BYTES + b_row;
        constexpr int STEPS = BK / 16, NM = STEPS * TM * TN;
        u32x4 a[2][TM], b[2][TN];
        auto request = [&](int s, int set) {
            const unsigned int ko = ((2u * s + half) ^ sw) * 16u;   // where this 16-deep step's piece sits
#pragma unroll
            for (int i = 0; i < TM; ++i) a[set][i] = *reinterpret_cast<const u32x4*>(as + i * 32 * RB + ko);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[set][j] = *reinterpret_cast<const u32x4*>(bs + j * 32 * RB + ko);
        };
        request(0, 0);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            if (s + 1 < STEPS) request(s + 1, (s + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = Epi::kStaged
                                    ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(b[s & 1][j]), as_bf16x8(a[s & 1][i]), acc[i][j], 0, 0, 0)
                                    : __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a[s & 1][i]), as_bf16x8(b[s & 1][j]), acc[i][j], 0, 0, 0);
                    if (FETCH) {
                        const int m = (s * TM + i) * TN + j;          // this MFMA's number within the slice
#pragma unroll
                        for (int u = m * L / NM; u < (m + 1) * L / NM; ++u) fetch_one(u, fbuf, fk0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // NSTAGE slices deep: slice kt is awaited (every wavefront waits for its own loads, the barrier
    // covers the others'); after the barrier nobody reads the buffer of slice kt - 1 any more, so
    // slice kt + NSTAGE - 1 is requested into it and travels while slices kt .. are multiplied.
    // With two workgroups on a compute unit two slices are enough (the other workgroup computes
    // while this one waits); a workgroup that has a compute unit to itself needs its requests
    // further ahead than one slice's multiply time.
    auto wait_vm = [](auto n) {                             // s_waitcnt vmcnt(n), nothing else
        constexpr unsigned int N = decltype(n)::value;
        __builtin_amdgcn_s_waitcnt((N & 0xFu) | ((N >> 4) << 14) | 0x0F70u);
    };
    const unsigned int nk = p.K / BK;
#pragma unroll
    for (unsigned int s0 = 0; s0 + 1 < (unsigned int)NSTAGE; ++s0)
        if (s0 < nk) fetch(s0, s0 * BK);
    // steady state: slices kt + 1 .. kt + NSTAGE - 2 may still be in flight while slice kt is awaited
    // (two loops, so that each has one straight-line body: with both kinds of multiply in one loop
    // the compiler moved all accumulators between register files on every iteration)
    unsigned int kt = 0;
    for (; kt + NSTAGE - 1 < nk; ++kt) {
        wait_vm(std::integral_constant<unsigned int, (NSTAGE - 2) * L>{});
        __syncthreads();
        multiply(kt % NSTAGE, std::true_type{}, (kt + NSTAGE - 1) % NSTAGE, (kt + NSTAGE - 1) * BK);
    }
    // the last NSTAGE - 1 slices: nothing left to request
    for (; kt < nk; ++kt) {
        const unsigned int later = nk - 1u - kt;
        if (NSTAGE >= 4 && later == 2u) wait_vm(std::integral_constant<unsigned int, 2 * L>{});
        else if (NSTAGE >= 3 && later == 1u) wait_vm(std::integral_constant<unsigned int, L>{});
        else wait_vm(std::integral_constant<unsigned int, 0>{});
        __syncthreads();
        multiply(kt % NSTAGE, std::false_type{}, 0u, 0u);
    }

    if constexpr (Epi::kStaged) {
        // The accumulator of tile (i, j) is transposed: element v of a lane is output row
        // lane % 32, column acc_row(v, lane).  Park the wavefront's (TM*32) x (TN*32) tile as
        // bf16 in its own LDS region (the operand slices are no longer needed).
        constexpr int TSTRIDE = TN * 64 + 16;                // bytes per parked row
        constexpr int CR = TN * 4;                           // 16-byte pieces per row
        constexpr int RP = 64 / CR;                          // rows per pass of the wavefront
        static_assert(4 * TM * 32 * TSTRIDE <= (int)gemm_lds_bytes<BM, BN, BK, WGM, WGN, NSTAGE>(), "parked tiles fit");
        __syncthreads();
        unsigned char* park = smem + wave * (TM * 32 * TSTRIDE);
        const unsigned int wm0 = m0 + wm * TM * 32u, wn0 = n0 + wn * TN * 32u;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (unsigned int grp = 0; grp < 4; ++grp) {
                    const unsigned int nl = j * 32u + 8u * grp + 4u * (lane >> 5);
                    bf16_bits h[4];
#pragma unroll
                    for (unsigned int e = 0; e < 4; ++e)
                        h[e] = bf16_bits_rne(epi.pre(m0, wn0 + nl + e, acc[i][j][4 * grp + e]));
                    uint2 pk;
                    pk.x = (unsigned int)h[0] | ((unsigned int)h[1] << 16);
                    pk.y = (unsigned int)h[2] | ((unsigned int)h[3] << 16);
                    *reinterpret_cast<uint2*>(park + (i * 32u + (lane & 31u)) * TSTRIDE + nl * 2u) = pk;
                }
        // same wavefront reads what it wrote: LDS operations of a wavefront complete in order
#pragma unroll
        for (int pass = 0; pass < TM * 32 / RP; ++pass) {
            const unsigned int row = pass * RP + lane / CR, piece = lane % CR;
            const u32x4 v = *reinterpret_cast<const u32x4*>(park + row * TSTRIDE + piece * 16u);
            epi.store(wm0 + row, wn0 + piece * 8u, v);
        }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                epi.tile(m0 + (wm * TM + i) * 32u, n0 + (wn * TN + j) * 32u, acc[i][j], lane, split);
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, int NSTAGE, class Epi>
__global__ __launch_bounds__(kGemmThreads) void gemm_nt_kernel(GemmArgs p, Epi epi) {
    gemm_nt_block<BM, BN, BK, WGM, WGN, NSTAGE>(p, epi, blockIdx.x);
}

// The three weight-gradient products of a step in one launch (each writes K-split partials):
// workgroups [0, n2) take the square layer's, [n2, n2 + n3) the output layer's, the rest the
// first layer's.  n2 and n3 are multiples of 8, which keeps a workgroup's index within its
// product congruent to its XCD.  NARROW3 / NARROW1: the layer's gradient is at most 64 / 32
// columns wide and uses the matching narrow tile.
template <bool NARROW3, bool NARROW1>
__global__ __launch_bounds__(kGemmThreads) void grad_products_kernel(GemmArgs p2, EpiPartial e2, unsigned int n2,
                                                                     GemmArgs p3, EpiPartial e3, unsigned int n3,
                                                                     GemmArgs p1, EpiPartial e1) {
    const unsigned int b = blockIdx.x;
    if (b < n2) {
        gemm_nt_block<128, 128, 64, 2, 2>(p2, e2, b);
    } else if (b < n2 + n3) {
        if constexpr (NARROW3) gemm_nt_block<128, 64, 64, 4, 1>(p3, e3, b - n2);
        else gemm_nt_block<128, 128, 64, 2, 2>(p3, e3, b - n2);
    } else {
        if constexpr (NARROW1) gemm_nt_block<128, 32, 64, 4, 1>(p1, e1, b - n2 - n3);
        else gemm_nt_block<128, 128, 64, 2, 2>(p1, e1, b - n2 - n3);
    }
}

// The dynamic LDS size of each kernel (up to 64 KB) is announced per kernel before the first
// launch (done at trainer creation, outside any stream capture).
template <int BM, int BN, int BK, int WGM, int WGN, class Epi, int NSTAGE = 2>
hipError_t configure_gemm() {
    auto kernel = gemm_nt_kernel<BM, BN, BK, WGM, WGN, NSTAGE, Epi>;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)gemm_lds_bytes<BM, BN, BK, WGM, WGN, NSTAGE>());
}

template <bool NARROW3, bool NARROW1>
hipError_t configure_grad_products() {
    auto kernel = grad_products_kernel<NARROW3, NARROW1>;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)gemm_lds_bytes<128, 128, 64, 2, 2>());
}

// Arguments and workgroup count (a multiple of 8) of one product with BM x BN tiles and BK-wide
// slices; false when the shape does not fit the kernel's assumptions.
template <int BM, int BN, int BK>
bool gemm_args(const bf16_bits* A, unsigned int lda, const bf16_bits* Bt, unsigned int ldb,
               unsigned int M, unsigned int N, unsigned int K, unsigned int splits,
               const bf16_bits* Bt_hi, unsigned int m_split, GemmArgs* a, unsigned int* blocks) {
    if (K == 0 || splits == 0 || K % (splits * BK) != 0 || lda % 8 != 0 || ldb % 8 != 0 || M == 0 || N == 0)
        return false;
    if (Bt_hi && m_split % BM != 0) return false;   // a tile takes one B operand
    a->A = A; a->lda = lda; a->Bt = Bt; a->ldb = ldb; a->M = M; a->N = N; a->K = K / splits;
    a->Bt_hi = Bt_hi ? Bt_hi : Bt;
    a->m_split = Bt_hi ? m_split : 0xFFFFFFFFu;
    a->tiles_m = (M + BM - 1) / BM;
    a->tiles_n = (N + BN - 1) / BN;
    a->splits = splits;
    const unsigned int n_tiles = a->tiles_m * a->tiles_n * splits;
    *blocks = 8u * ((n_tiles + 7u) / 8u);
    // band width: the one for which an XCD's share of the tiles (a block of about per_xcd / band
    // tile rows by `band` tile columns) touches the fewest operand rows
    const unsigned int per_xcd = std::min((n_tiles + 7u) / 8u, a->tiles_m * a->tiles_n);
    unsigned int best = a->tiles_n;
    size_t best_cost = ~(size_t)0;
    // (first among the widths whose bands line up with the XCDs' ranges, so that a range does not
    // straddle two bands; any width if there is none)
    for (int aligned = 1; aligned >= 0 && best_cost == ~(size_t)0; --aligned)
        for (unsigned int w = 1; w <= a->tiles_n; ++w) {
            const unsigned int band_tiles = a->tiles_m * w;
            if (aligned && band_tiles % per_xcd != 0 && per_xcd % band_tiles != 0) continue;
            // a range of per_xcd tile numbers covers whole bands when it is longer than one
            const unsigned int rows = per_xcd >= band_tiles ? a->tiles_m : std::min(a->tiles_m, (per_xcd + w - 1) / w);
            const unsigned int cols = per_xcd >= band_tiles
                                          ? std::min(a->tiles_n, w * ((per_xcd + band_tiles - 1) / band_tiles))
                                          : w;
            const size_t cost = (size_t)rows * BM + (size_t)cols * BN;
            if (cost < best_cost) {
                best_cost = cost;
                best = w;
            }
        }
    a->band = best;
    return true;
}

template <int BM, int BN, int BK, int WGM, int WGN, int NSTAGE = 2, class Epi>
hipError_t launch_gemm(hipStream_t st, const bf16_bits* A, unsigned int lda, const bf16_bits* Bt,
                       unsigned int ldb, unsigned int M, unsigned int N, unsigned int K,
                       const Epi& epi, unsigned int splits = 1, const bf16_bits* Bt_hi = nullptr,
                       unsigned int m_split = 0xFFFFFFFFu) {
    GemmArgs a;
    unsigned int blocks;
    if (!gemm_args<BM, BN, BK>(A, lda, Bt, ldb, M, N, K, splits, Bt_hi, m_split, &a, &blocks))
        return hipErrorInvalidValue;
    constexpr size_t lds = gemm_lds_bytes<BM, BN, BK, WGM, WGN, NSTAGE>();
    hipLaunchKernelGGL((gemm_nt_kernel<BM, BN, BK, WGM, WGN, NSTAGE, Epi>), dim3(blocks),
                       dim3(kGemmThreads), lds, st, a, epi);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------------------
// Skinny product for the output layer, Q = H2 W3 + b3 (a few 32-wide column tiles, many rows):
// one 32x32 output tile per workgroup; the wavefronts split K, each loading its MFMA operands
// straight from global memory (eight 16-deep steps requested before the first multiply), and
// add their accumulators through LDS.  K is a multiple of 16.  Rows beyond M / N read row 0
// instead: they only reach accumulator elements that are not stored.
// ----------------------------------------------------------------------------------------
struct SkinnyArgs {
    const bf16_bits* A;
    unsigned int lda;
    const bf16_bits* Bt;
    unsigned int ldb;
    unsigned int M, N, K;
    const float* bias;   // [N]
    float* out;          // [M x ldo], fp32
    unsigned int ldo;
    // tiles whose first row is m_split (a multiple of 32) or beyond use these (the target network's)
    const bf16_bits* Bt_hi;
    const float* bias_hi;
    unsigned int m_split;
};

template <int NW>
__global__ __launch_bounds__(64 * NW) void skinny_nt_kernel(SkinnyArgs p) {
    __shared__ float red[NW * 16 * 64];
    const unsigned int tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const unsigned int m0 = blockIdx.x * 32u, n0 = blockIdx.y * 32u;
    const unsigned int am = m0 + (lane & 31u), bn = n0 + (lane & 31u);
    const bf16_bits* ap = p.A + (size_t)(am < p.M ? am : 0u) * p.lda + 8u * (lane >> 5);
    const bool hi = m0 >= p.m_split;
    const bf16_bits* bp = (hi ? p.Bt_hi : p.Bt) + (size_t)(bn < p.N ? bn : 0u) * p.ldb + 8u * (lane >> 5);
    const float* bias = hi ? p.bias_hi : p.bias;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (unsigned int kc = wave * 128u; kc < p.K; kc += NW * 128u) {
        u32x4 a[8], b[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const unsigned int k = kc + s * 16u;
            const bool in = k < p.K;
            a[s] = in ? *reinterpret_cast<const u32x4*>(ap + k) : zero4;
            b[s] = in ? *reinterpret_cast<const u32x4*>(bp + k) : zero4;
        }
#pragma unroll
        for (int s = 0; s < 8; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a[s]), as_bf16x8(b[s]), acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[(wave * 16u + v) * 64u + lane] = acc[v];
    __syncthreads();
    for (unsigned int e = tid; e < 1024u; e += 64u * NW) {
        const unsigned int v = e >> 6, l = e & 63u;
        float s = 0.f;
#pragma unroll
        for (unsigned int w = 0; w < (unsigned int)NW; ++w) s += red[(w * 16u + v) * 64u + l];
        const unsigned int m = m0 + acc_row(v, l), n = n0 + (l & 31u);
        if (m < p.M && n < p.N) p.out[(size_t)m * p.ldo + n] = s + bias[n];
    }
}

// ----------------------------------------------------------------------------------------
// TD target, loss and the gradient at the second hidden layer's pre-activation.
// A workgroup owns 64 batch rows x 64 hidden units.  It first repeats, for its 64 rows, the
// per-row part: y_i = r_i + gamma (1 - term_i) max_a Q(s'_i, a), delta_i = y_i - Q(s_i, a_i),
// the loss term and g_i = dL/dQ(s_i, a_i)  (four lanes per row share the max).  Workgroups of
// the first hidden-unit stripe store those and dL/dQ transposed, split into a bf16 high and
// low part so that the output-layer weight gradient keeps fp32 accuracy.  Then
//   dZ2[i][k] = g_i * W3[k][a_i] * 1[H2[i][k] > 0]
// goes out in both orientations (the transposed one through an LDS tile), and so do the
// transposed copies of this tile of H1 and H2 that the weight-gradient products read.
// ----------------------------------------------------------------------------------------
struct TdArgs {
    unsigned int B, Bp, H, A, Ap;
    const float* Q;              // [2B x Ap]
    const int* act;
    const float* rew;
    const unsigned char* term;
    float gamma;
    unsigned int loss_kind;
    float beta1, beta2;
    float *y, *delta, *lossi;
    bf16_bits *dQT_hi, *dQT_lo;  // [Ap x Bp]
    const bf16_bits* W3T;        // [Ap x H]
    const bf16_bits* H1;         // [2B x H]
    const bf16_bits* H2;         // [2B x H]
    bf16_bits* dZ2;              // [B x H]
    bf16_bits* dZ2T;             // [H x Bp]
    bf16_bits *H1T, *H2T;        // [H+1 x Bp]: transposed copies of the first B rows of H1, H2
    TrainCounters* ctr;
};

__global__ __launch_bounds__(256) void td_dz_kernel(TdArgs p) {
    __shared__ float gs[64];
    __shared__ unsigned int as_[64];
    // [k][row] tiles, padded: dZ2, H2 and H1 on their way to the transposed buffers
    __shared__ __attribute__((aligned(16))) bf16_bits tileT[3][64][72];
    const unsigned int tid = threadIdx.x;
    const unsigned int i0 = blockIdx.x * 64u, k0 = blockIdx.y * 64u;
    if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) {
        // (running products beta^t in double precision: no power function on the device)
        const double pw1 = p.ctr->pw1 * (double)p.beta1, pw2 = p.ctr->pw2 * (double)p.beta2;
        p.ctr->adam_t = p.ctr->adam_t + 1;
        p.ctr->pw1 = pw1;
        p.ctr->pw2 = pw2;
        p.ctr->c1 = (float)(1.0 - pw1);
        p.ctr->c2 = (float)(1.0 - pw2);
    }
    {
        const unsigned int r = tid >> 2, part = tid & 3u, i = i0 + r;
        const bool live = i < p.B;
        float best = -INFINITY;
        if (live) {
            const float* qn = p.Q + (size_t)(p.B + i) * p.Ap;
            for (unsigned int a = part; a < p.A; a += 4) best = fmaxf(best, qn[a]);
        }
        best = fmaxf(best, __shfl_xor(best, 1, 64));
        best = fmaxf(best, __shfl_xor(best, 2, 64));
        if (part == 0) {
            float g = 0.f;
            unsigned int ai = 0;
            if (live) {
                ai = (unsigned int)p.act[i];
                if (ai >= p.A) ai = p.A - 1;  // an out-of-range action must not turn into a wild address
                const float q = p.Q[(size_t)i * p.Ap + ai];
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
                g = -slope / (float)p.B;
                if (blockIdx.y == 0) {
                    p.y[i] = y;
                    p.delta[i] = d;
                    p.lossi[i] = li;
                }
            }
            gs[r] = g;
            as_[r] = ai;
        }
    }
    __syncthreads();
    if (blockIdx.y == 0) {
        for (unsigned int e = tid; e < p.Ap * 64u; e += 256u) {
            const unsigned int a = e >> 6, r = e & 63u;
            const float g = (a == as_[r]) ? gs[r] : 0.f;
            const bf16_bits hi = bf16_bits_rne(g);
            const bf16_bits lo = bf16_bits_rne(g - bits_to_float(hi));
            p.dQT_hi[(size_t)a * p.Bp + i0 + r] = hi;
            p.dQT_lo[(size_t)a * p.Bp + i0 + r] = lo;
        }
    }
    {
        // 16 consecutive hidden units of one row per thread
        const unsigned int r = tid >> 2, ks = (tid & 3u) * 16u, i = i0 + r;
        const bool live = i < p.B;
        bf16_bits out[16], h2[16], h1[16];
        if (live) {
            const float g = gs[r];
            const u32x4* hp = reinterpret_cast<const u32x4*>(p.H2 + (size_t)i * p.H + k0 + ks);
            const u32x4* gp = reinterpret_cast<const u32x4*>(p.H1 + (size_t)i * p.H + k0 + ks);
            const u32x4* wp = reinterpret_cast<const u32x4*>(p.W3T + (size_t)as_[r] * p.H + k0 + ks);
            const u32x4 hv0 = hp[0], hv1 = hp[1], gv0 = gp[0], gv1 = gp[1], wv0 = wp[0], wv1 = wp[1];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const unsigned int hw = e < 8 ? hv0[e >> 1] : hv1[(e - 8) >> 1];
                const unsigned int gw = e < 8 ? gv0[e >> 1] : gv1[(e - 8) >> 1];
                const unsigned int ww = e < 8 ? wv0[e >> 1] : wv1[(e - 8) >> 1];
                h2[e] = (bf16_bits)(hw >> (16 * (e & 1)));
                h1[e] = (bf16_bits)(gw >> (16 * (e & 1)));
                const bf16_bits wb = (bf16_bits)(ww >> (16 * (e & 1)));
                const float x = bits_to_float(h2[e]) > 0.f ? g * bits_to_float(wb) : 0.f;
                out[e] = bf16_bits_rne(x);
            }
            u32x4 o0, o1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o0[e] = out[2 * e] | ((unsigned int)out[2 * e + 1] << 16);
                o1[e] = out[8 + 2 * e] | ((unsigned int)out[8 + 2 * e + 1] << 16);
            }
            u32x4* dp = reinterpret_cast<u32x4*>(p.dZ2 + (size_t)i * p.H + k0 + ks);
            dp[0] = o0;
            dp[1] = o1;
        } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) out[e] = h2[e] = h1[e] = 0;
        }
#pragma unroll
        // (the four lanes of a row hold k-ranges 16 apart, whose tile rows start in the same bank:
        // each range gets its columns rotated by a different multiple of 16, undone when read)
        for (int e = 0; e < 16; ++e) {
            tileT[0][ks + e][r ^ ks] = out[e];
            tileT[1][ks + e][r ^ ks] = h2[e];
            tileT[2][ks + e][r ^ ks] = h1[e];
        }
    }
    __syncthreads();
    {
        // 16 consecutive batch rows of one hidden unit per thread
        const unsigned int k = tid >> 2, rs = (tid & 3u) * 16u;
        const size_t at = (size_t)(k0 + k) * p.Bp + i0 + rs;
        bf16_bits* const dst[3] = {p.dZ2T, p.H2T, p.H1T};
#pragma unroll
        for (int w = 0; w < 3; ++w) {
            const u32x4* sp = reinterpret_cast<const u32x4*>(&tileT[w][k][rs ^ (k & 48u)]);
            u32x4* dp = reinterpret_cast<u32x4*>(dst[w] + at);
            dp[0] = sp[0];
            dp[1] = sp[1];
        }
    }
}

// The two narrow layers' update, from the K-split partial products of their gradients:
//   part3[z][m][c]: m <= H (row H = bias), c < 2*Ap; gradient of W3[m][a] = sum_z part3[z][m][a]
//                   + part3[z][m][Ap + a]  (dL/dQ was split into a bf16 high and low part)
//   part1[z][j][d]: j < H, d <= D (column D = bias); gradient of W1[d][j] = sum_z part1[z][j][d]
// One thread per parameter; splits (at most 16) are added in order.  Workgroup 0 also reduces the
// per-sample losses to their mean and advances the sampling step counter.
struct SmallOptArgs {
    OptState o;
    unsigned int splits, H, D, Dp, Dx, Ap, B;
    const float* part3;
    const float* part1;
    size_t oW1, ob1, oW3, ob3;
    bf16_bits* W1T;   // [H x Dp]
    bf16_bits* W3T;   // [Ap x H]
    bf16_bits *W1T_target, *W3T_target;   // the target network's, or null
    TrainCounters* ctr;
    const float* lossi;
    unsigned int out_grad_only;   // dueling head: only store the output layer's gradient
};

__device__ __forceinline__ void small_opt_block(const SmallOptArgs& p, unsigned int block) {
    const unsigned int n3 = (p.H + 1u) * p.Ap, n1 = p.H * (p.D + 1u);
    const unsigned int e = block * 256u + threadIdx.x;
    const OptStep st = opt_step(p.o);
    if (e < n3) {
        const unsigned int m = e / p.Ap, a = e - m * p.Ap;
        const size_t stride = (size_t)(p.H + 1u) * 2u * p.Ap;
        const float* src = p.part3 + (size_t)m * 2u * p.Ap + a;
        float hi[16], lo[16];
#pragma unroll
        for (unsigned int z = 0; z < 16; ++z) {
            hi[z] = z < p.splits ? src[z * stride] : 0.f;
            lo[z] = z < p.splits ? src[z * stride + p.Ap] : 0.f;
        }
        float g = 0.f;
#pragma unroll
        for (unsigned int z = 0; z < 16; ++z) g += hi[z] + lo[z];
        if (p.out_grad_only) {
            p.o.g[m < p.H ? p.oW3 + (size_t)m * p.Ap + a : p.ob3 + a] = g;
        } else if (m < p.H) {
            const bf16_bits h = bf16_bits_rne(opt_update(p.o, p.oW3 + (size_t)m * p.Ap + a, g, st));
            p.W3T[(size_t)a * p.H + m] = h;
            if (st.sync) p.W3T_target[(size_t)a * p.H + m] = h;
        } else {
            opt_update(p.o, p.ob3 + a, g, st);
        }
    } else if (e < n3 + n1) {
        const unsigned int f = e - n3, j = f / (p.D + 1u), d = f - j * (p.D + 1u);
        const size_t stride = (size_t)p.H * p.Dx;
        const float* src = p.part1 + (size_t)j * p.Dx + d;
        float part[16];
#pragma unroll
        for (unsigned int z = 0; z < 16; ++z) part[z] = z < p.splits ? src[z * stride] : 0.f;
        float g = 0.f;
#pragma unroll
        for (unsigned int z = 0; z < 16; ++z) g += part[z];
        if (d < p.D) {
            const bf16_bits h = bf16_bits_rne(opt_update(p.o, p.oW1 + (size_t)d * p.H + j, g, st));
            p.W1T[(size_t)j * p.Dp + d] = h;
            if (st.sync) p.W1T_target[(size_t)j * p.Dp + d] = h;
        } else {
            opt_update(p.o, p.ob1 + j, g, st);
        }
    }
    if (block == 0) {
        __shared__ float wsum[4];
        float acc = 0.f;
        for (unsigned int i = threadIdx.x; i < p.B; i += 256) acc += p.lossi[i];
        acc = wave_sum(acc);
        if ((threadIdx.x & 63u) == 0) wsum[threadIdx.x >> 6] = acc;
        __syncthreads();
        if (threadIdx.x == 0) {
            p.ctr->loss = (wsum[0] + wsum[1] + wsum[2] + wsum[3]) / (float)p.B;
            p.ctr->step += 1;
        }
    }
}

// The square layer's update from the K-split partial products of [dW ; db] (row R = bias):
//   part[z][m][n], m <= R, n < N; the gradient is the sum over z, splits added in order.
// A workgroup owns a kSqRows x 64 tile of W: a thread takes four consecutive columns of a row
// (16-byte accesses to the partials and to the fp32 weight, gradient and moments), writes the
// new weights' bf16 copy in the same orientation and parks it in LDS, from where the
// transposed copy (and the target network's, when a sync is due) leaves as 128-byte runs.
// R and N are multiples of 64.
struct SquareOptArgs {
    OptState o;
    unsigned int R, N, splits;
    const float* part;
    size_t w_off, b_off;
    bf16_bits* wb;              // [R x N]
    bf16_bits* wbT;             // [N x R]
    bf16_bits* wbT_target;      // [N x R] of the target network, or null
};

__device__ __forceinline__ f32x4 opt_update4(const OptState& o, size_t k, const f32x4& g, const OptStep& st) {
    f32x4 w = *reinterpret_cast<const f32x4*>(o.w + k);
    *reinterpret_cast<f32x4*>(o.g + k) = g;
    if (o.opt == RP_SGD) {
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] -= o.lr * g[e];
    } else {
        f32x4 m = *reinterpret_cast<const f32x4*>(o.m + k);
        f32x4 v = *reinterpret_cast<const f32x4*>(o.v + k);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            m[e] = o.beta1 * m[e] + (1.f - o.beta1) * g[e];
            v[e] = o.beta2 * v[e] + (1.f - o.beta2) * g[e] * g[e];
            w[e] -= o.lr * (m[e] / st.c1) / (sqrtf(v[e] / st.c2) + o.eps);
        }
        *reinterpret_cast<f32x4*>(o.m + k) = m;
        *reinterpret_cast<f32x4*>(o.v + k) = v;
    }
    *reinterpret_cast<f32x4*>(o.w + k) = w;
    if (st.sync) *reinterpret_cast<f32x4*>(o.wt + k) = w;
    return w;
}

constexpr unsigned int kSqRows = 32;   // rows of W per workgroup of the square layer's update (columns: 64)

__device__ __forceinline__ void square_opt_block(const SquareOptArgs& p, unsigned int block_x, unsigned int block_y) {
    constexpr unsigned int TS = 68;                       // bf16 per parked row (64 + padding)
    __shared__ bf16_bits tile[kSqRows * TS];
    const unsigned int tid = threadIdx.x, c4 = (tid & 15u) * 4u, r0 = tid >> 4;
    const unsigned int m0 = block_y * kSqRows, n0 = block_x * 64u;
    const OptStep st = opt_step(p.o);
    const size_t zs = (size_t)(p.R + 1u) * p.N;           // one split's partials
    constexpr unsigned int Q = kSqRows / 16u;
    f32x4 g[Q];
#pragma unroll
    for (unsigned int q = 0; q < Q; ++q) {
        const float* src = p.part + (size_t)(m0 + q * 16u + r0) * p.N + n0 + c4;
        g[q] = *reinterpret_cast<const f32x4*>(src);
        for (unsigned int z = 1; z < p.splits; ++z) g[q] += *reinterpret_cast<const f32x4*>(src + z * zs);
    }
#pragma unroll
    for (unsigned int q = 0; q < Q; ++q) {
        const unsigned int r = q * 16u + r0;
        const size_t at = (size_t)(m0 + r) * p.N + n0 + c4;
        const f32x4 w = opt_update4(p.o, p.w_off + at, g[q], st);
        bf16_bits h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = bf16_bits_rne(w[e]);
        uint2 pk;
        pk.x = (unsigned int)h[0] | ((unsigned int)h[1] << 16);
        pk.y = (unsigned int)h[2] | ((unsigned int)h[3] << 16);
        *reinterpret_cast<uint2*>(p.wb + at) = pk;
        *reinterpret_cast<uint2*>(tile + r * TS + c4) = pk;
    }
    if (block_y == 0 && tid < 16) {                        // the bias: row R of the partials
        const float* src = p.part + (size_t)p.R * p.N + n0 + c4;
        f32x4 gb = *reinterpret_cast<const f32x4*>(src);
        for (unsigned int z = 1; z < p.splits; ++z) gb += *reinterpret_cast<const f32x4*>(src + z * zs);
        opt_update4(p.o, p.b_off + n0 + c4, gb, st);
    }
    __syncthreads();
    // transposed copy: kSqRows / 2 lanes write one column of the tile as pairs of rows
    constexpr unsigned int LPC = kSqRows / 2u, CPP = 256u / LPC;   // lanes per column, columns per pass
    const unsigned int mp = (tid % LPC) * 2u;
#pragma unroll
    for (unsigned int pass = 0; pass < 64u / CPP; ++pass) {
        const unsigned int n = pass * CPP + tid / LPC;
        const unsigned int pair = (unsigned int)tile[mp * TS + n] | ((unsigned int)tile[(mp + 1u) * TS + n] << 16);
        const size_t at = (size_t)(n0 + n) * p.R + m0 + mp;
        *reinterpret_cast<unsigned int*>(p.wbT + at) = pair;
        if (st.sync) *reinterpret_cast<unsigned int*>(p.wbT_target + at) = pair;
    }
}

// One launch updates all three layers: the first (N / 64) (R / kSqRows) workgroups take the tiles
// of the square layer, the rest the two narrow layers.
__global__ __launch_bounds__(256) void opt_kernel(SquareOptArgs sq, SmallOptArgs sm) {
    const unsigned int tiles_n = sq.N / 64u, n_square = tiles_n * (sq.R / kSqRows);
    if (blockIdx.x < n_square)
        square_opt_block(sq, blockIdx.x % tiles_n, blockIdx.x / tiles_n);
    else
        small_opt_block(sm, blockIdx.x - n_square);
}

// The same launch with `next_blocks` more workgroups after its `own` ones, which append, sample and
// gather for the NEXT train step (inside a recorded run of steps): nothing the optimizer reads or
// writes is touched by them, and the next step then begins with its first layer.
__global__ __launch_bounds__(256) void opt_ahead_kernel(SquareOptArgs sq, SmallOptArgs sm, AppendGatherArgs next,
                                                        unsigned int own, unsigned int next_blocks) {
    if (blockIdx.x >= own) {
        append_gather_block<2, kDrawUniform>(next, blockIdx.x - own, next_blocks);
        return;
    }
    const unsigned int tiles_n = sq.N / 64u, n_square = tiles_n * (sq.R / kSqRows);
    if (blockIdx.x < n_square)
        square_opt_block(sq, blockIdx.x % tiles_n, blockIdx.x / tiles_n);
    else
        small_opt_block(sm, blockIdx.x - n_square);
}

// What a recorded opt_ahead_kernel node was launched with, apart from the next step's part.
struct OptRecorded {
    SquareOptArgs sq;
    SmallOptArgs sm;
    unsigned int own;
};

// K splits of the narrow layers' gradient products (contraction over the padded batch): as
// many as leave every workgroup at least 256 columns, in whole 64-wide slices, at most 16.
unsigned int batch_splits(unsigned int Bp) {
    unsigned int best = 1;
    for (unsigned int s = 2; s <= 16; ++s)
        if (Bp % (s * 64u) == 0 && Bp / s >= 256u) best = s;
    return best;
}

// K splits of the square layer's gradient product: doubled while its 128 x 128 tiles number
// fewer than the compute units, every split keeps at least 256 columns in whole 64-wide slices.
unsigned int square_splits_for(unsigned int Bp, unsigned int H) {
    const unsigned int tiles = ((H + 1u + 127u) / 128u) * ((H + 127u) / 128u);
    unsigned int s = 1;
    while (tiles * s < 256u && s < 8u && Bp % (2u * s * 64u) == 0 && Bp / (2u * s) >= 256u) s *= 2u;
    return s;
}

bf16_bits host_bf16(float f) {
    unsigned int u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (bf16_bits)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_bits)(u >> 16);
}

}  // namespace

unsigned int square_splits(unsigned int Bp, unsigned int H) { return square_splits_for(Bp, H); }

bool wide_step_supported(const train_config& cfg, const replay* rp_) {
    return cfg.param_dtype == RP_BF16 && rp_->cfg.state_dtype == RP_BF16 &&
           rp_->cfg.layout == RP_PAIR && cfg.hidden % 64 == 0 &&
           (cfg.hidden2 == 0 || cfg.hidden2 == cfg.hidden);   // two hidden layers of one width
}

// Allow the products' LDS sizes and fill the ones rows of the transposed activation buffers
// (once, at creation).
hipError_t wide_init_buffers(trainer* t) {
    hipError_t ec = configure_gemm<128, 128, 32, 2, 2, EpiForward>();
    if (ec == hipSuccess) ec = configure_gemm<128, 128, 64, 2, 2, EpiForward>();
    if (ec == hipSuccess) ec = configure_gemm<128, 64, 64, 2, 2, EpiMask>();
    if (ec == hipSuccess) ec = configure_grad_products<true, true>();
    if (ec == hipSuccess) ec = configure_grad_products<true, false>();
    if (ec == hipSuccess) ec = configure_grad_products<false, true>();
    if (ec == hipSuccess) ec = configure_grad_products<false, false>();
    if (ec != hipSuccess) return ec;
    std::vector<bf16_bits> ones(t->Bp, (bf16_bits)0x3F80u);
    const size_t bytes = (size_t)t->Bp * sizeof(bf16_bits);
    hipError_t e = hipMemcpy(t->wd.H1T + (size_t)t->H * t->Bp, ones.data(), bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(t->wd.H2T + (size_t)t->H * t->Bp, ones.data(), bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(t->wd.XT + (size_t)t->cfg.state_dim * t->Bp, ones.data(), bytes,
                      hipMemcpyHostToDevice);
    return e;
}

// Refresh the bf16 operand copies of the weights from padded fp32 parameters (host array): all
// four of the trained network, or the three forward operands of the target network.
hipError_t wide_set_weights(trainer* t, const float* padded, bool target) {
    const size_t H = t->H, Dp = t->Dp, Ap = t->Ap;
    std::vector<bf16_bits> w1t(H * Dp), w2(H * H), w2t(H * H), w3t(Ap * H);
    for (size_t d = 0; d < Dp; ++d)
        for (size_t j = 0; j < H; ++j) w1t[j * Dp + d] = host_bf16(padded[t->oW1 + d * H + j]);
    for (size_t j = 0; j < H; ++j)
        for (size_t k = 0; k < H; ++k) {
            const bf16_bits h = host_bf16(padded[t->oW2 + j * H + k]);
            w2[j * H + k] = h;
            w2t[k * H + j] = h;
        }
    for (size_t k = 0; k < H; ++k)
        for (size_t a = 0; a < Ap; ++a) w3t[a * H + k] = host_bf16(padded[t->oW3 + k * Ap + a]);
    const WideBuffers& w = t->wd;
    hipError_t e = hipMemcpy(target ? w.W1T_t : w.W1T, w1t.data(), w1t.size() * 2, hipMemcpyHostToDevice);
    if (e == hipSuccess && !target) e = hipMemcpy(w.W2, w2.data(), w2.size() * 2, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(target ? w.W2T_t : w.W2T, w2t.data(), w2t.size() * 2, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(target ? w.W3T_t : w.W3T, w3t.data(), w3t.size() * 2, hipMemcpyHostToDevice);
    return e;
}

// Enqueue every kernel of one executed step after the append.
hipError_t enqueue_wide_step(trainer* t, hipStream_t st, unsigned int* count, bool sample) {
    const unsigned int B = t->B, Bp = t->Bp, H = t->H, Dp = t->Dp, Ap = t->Ap;
    const unsigned int D = t->cfg.state_dim, A = t->cfg.num_actions;
    WideBuffers& w = t->wd;
    bf16_bits* X = static_cast<bf16_bits*>(t->X);
    bf16_bits* H1 = static_cast<bf16_bits*>(t->H1);
    bf16_bits* H2 = static_cast<bf16_bits*>(t->H2);
    bf16_bits* dZ2 = static_cast<bf16_bits*>(t->dZ2);
    unsigned int n = 0;
    OptState o{t->w, t->g, t->m, t->v, t->cfg.opt, t->cfg.lr, t->cfg.beta1, t->cfg.beta2, t->cfg.eps,
               t->ctr, t->wt, t->cfg.target_sync};
    // With a frozen target network the rows of S' (B .. 2B-1) are multiplied by its weights: in
    // the same launch when tiles do not straddle row B, else in a launch of their own.
    const bool tgt = t->wt != nullptr;
    const float *b1t = tgt ? t->wt + t->ob1 : nullptr, *b2t = tgt ? t->wt + t->ob2 : nullptr;
    const float* b3t = tgt ? t->wt + t->ob3 : nullptr;
    const bool one_launch = !tgt || B % 128 == 0;
    const unsigned int rows = one_launch ? 2 * B : B;   // rows of the first forward launch

    // sample B slots and unpack into X = [S ; S'] and the transposed copy of S
    hipError_t e = hipSuccess;
    unsigned int launched = 0;
    if (sample) {
        e = launch_sample_gather(t->rp_->geom, t->rp_->cfg.seed, 0, &t->ctr->step, B, X,
                                 X + (size_t)B * Dp, Dp, t->act, t->rew, t->term, t->idx, st, w.XT, Bp,
                                 0, 0, t->rp_->draw_scratch, &launched);
        if (e != hipSuccess) return e;
        n += launched;
    }
    // forward on the 2B rows
    e = launch_gemm<128, 128, 32, 2, 2>(st, X, Dp, w.W1T, Dp, rows, H, Dp,
                                           EpiForward{t->w + t->ob1, b1t, tgt ? B : ~0u, H1, H, rows, H},
                                           1, tgt && one_launch ? w.W1T_t : nullptr, B);
    if (e != hipSuccess) return e;
    ++n;
    if (!one_launch) {
        e = launch_gemm<128, 128, 32, 2, 2>(st, X + (size_t)B * Dp, Dp, w.W1T_t, Dp, B, H, Dp,
                                               EpiForward{b1t, b1t, ~0u, H1 + (size_t)B * H, H, B, H});
        if (e != hipSuccess) return e;
        ++n;
    }
    e = launch_gemm<128, 128, 64, 2, 2>(st, H1, H, w.W2T, H, rows, H, H,
                                           EpiForward{t->w + t->ob2, b2t, tgt ? B : ~0u, H2, H, rows, H},
                                           1, tgt && one_launch ? w.W2T_t : nullptr, B);
    if (e != hipSuccess) return e;
    ++n;
    if (!one_launch) {
        e = launch_gemm<128, 128, 64, 2, 2>(st, H1 + (size_t)B * H, H, w.W2T_t, H, B, H, H,
                                               EpiForward{b2t, b2t, ~0u, H2 + (size_t)B * H, H, B, H});
        if (e != hipSuccess) return e;
        ++n;
    }
    {
        SkinnyArgs a;
        a.A = H2; a.lda = H; a.Bt = w.W3T; a.ldb = H; a.M = rows; a.N = Ap; a.K = H;
        a.bias = t->w + t->ob3; a.out = t->Q; a.ldo = Ap;
        a.Bt_hi = tgt ? w.W3T_t : w.W3T; a.bias_hi = tgt ? b3t : a.bias; a.m_split = tgt ? B : ~0u;
        hipLaunchKernelGGL(skinny_nt_kernel<8>, dim3((rows + 31) / 32, Ap / 32), dim3(512), 0, st, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        ++n;
        if (!one_launch) {
            a.A = H2 + (size_t)B * H; a.Bt = w.W3T_t; a.bias = b3t; a.out = t->Q + (size_t)B * Ap;
            a.M = B; a.Bt_hi = a.Bt; a.bias_hi = a.bias; a.m_split = ~0u;
            hipLaunchKernelGGL(skinny_nt_kernel<8>, dim3((B + 31) / 32, Ap / 32), dim3(512), 0, st, a);
            e = hipGetLastError();
        }
    }
    if (e != hipSuccess) return e;
    if (!one_launch) ++n;
    // targets, TD errors, loss terms, dL/dQ and dZ2
    {
        TdArgs a;
        a.B = B; a.Bp = Bp; a.H = H; a.A = A; a.Ap = Ap;
        a.Q = t->Q; a.act = t->act; a.rew = t->rew; a.term = t->term;
        a.gamma = t->cfg.gamma; a.loss_kind = t->cfg.loss; a.beta1 = t->cfg.beta1; a.beta2 = t->cfg.beta2;
        a.y = t->y; a.delta = t->delta; a.lossi = t->lossi;
        a.dQT_hi = w.dQT_hi; a.dQT_lo = w.dQT_lo; a.W3T = w.W3T; a.H1 = H1; a.H2 = H2; a.dZ2 = dZ2;
        a.dZ2T = w.dZ2T; a.H1T = w.H1T; a.H2T = w.H2T;
        a.ctr = t->ctr;
        hipLaunchKernelGGL(td_dz_kernel, dim3(Bp / 64, H / 64), dim3(256), 0, st, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        ++n;
    }
    // dZ1^T = (W2 dZ2^T) masked by the first ReLU; uses W2 before its update
    e = launch_gemm<128, 64, 64, 2, 2>(st, w.W2, H, dZ2, H, H, B, H,
                                          EpiMask{w.H1T, w.dZ1T, Bp, H, B});
    if (e != hipSuccess) return e;
    ++n;
    // the three weight-gradient products, K-split partials each, in one launch:
    //   [dW2 ; db2] (row H);  [dW3 ; db3] (row H) with the high and low part of dL/dQ side by
    //   side;  [dW1^T | db1] (column D)
    const unsigned int splits = batch_splits(Bp);
    const unsigned int splits2 = square_splits_for(Bp, H);
    const unsigned int Dx = (D + 1 + 31) / 32 * 32;
    {
        GemmArgs g2, g3, g1;
        unsigned int n2 = 0, n3 = 0, n1 = 0;
        const bool narrow3 = Ap == 32, narrow1 = Dx == 32;
        bool ok = gemm_args<128, 128, 64>(w.H1T, Bp, w.dZ2T, Bp, H + 1, H, Bp, splits2, nullptr, 0, &g2, &n2);
        ok = ok && (narrow3 ? gemm_args<128, 64, 64>(w.H2T, Bp, w.dQT_hi, Bp, H + 1, 2 * Ap, Bp, splits,
                                                     nullptr, 0, &g3, &n3)
                            : gemm_args<128, 128, 64>(w.H2T, Bp, w.dQT_hi, Bp, H + 1, 2 * Ap, Bp, splits,
                                                      nullptr, 0, &g3, &n3));
        ok = ok && (narrow1 ? gemm_args<128, 32, 64>(w.dZ1T, Bp, w.XT, Bp, H, Dx, Bp, splits, nullptr, 0,
                                                     &g1, &n1)
                            : gemm_args<128, 128, 64>(w.dZ1T, Bp, w.XT, Bp, H, Dx, Bp, splits, nullptr, 0,
                                                      &g1, &n1));
        if (!ok) return hipErrorInvalidValue;
        const EpiPartial e2{w.part2, H + 1, H}, e3{w.part3, H + 1, 2 * Ap}, e1{w.part1, H, Dx};
        constexpr size_t lds = gemm_lds_bytes<128, 128, 64, 2, 2>();
        const dim3 grid(n2 + n3 + n1), block(kGemmThreads);
        if (narrow3 && narrow1)
            hipLaunchKernelGGL((grad_products_kernel<true, true>), grid, block, lds, st, g2, e2, n2, g3, e3, n3, g1, e1);
        else if (narrow3)
            hipLaunchKernelGGL((grad_products_kernel<true, false>), grid, block, lds, st, g2, e2, n2, g3, e3, n3, g1, e1);
        else if (narrow1)
            hipLaunchKernelGGL((grad_products_kernel<false, true>), grid, block, lds, st, g2, e2, n2, g3, e3, n3, g1, e1);
        else
            hipLaunchKernelGGL((grad_products_kernel<false, false>), grid, block, lds, st, g2, e2, n2, g3, e3, n3, g1, e1);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        ++n;
    }
    // all three layers' update, mean loss, step counter
    {
        SquareOptArgs q;
        q.o = o; q.R = H; q.N = H; q.splits = splits2; q.part = w.part2;
        q.w_off = t->oW2; q.b_off = t->ob2; q.wb = w.W2; q.wbT = w.W2T; q.wbT_target = w.W2T_t;
        SmallOptArgs a;
        a.o = o; a.splits = splits; a.H = H; a.D = D; a.Dp = Dp; a.Dx = Dx; a.Ap = Ap; a.B = B;
        a.part3 = w.part3; a.part1 = w.part1;
        a.oW1 = t->oW1; a.ob1 = t->ob1; a.oW3 = t->oW3; a.ob3 = t->ob3;
        a.W1T = w.W1T; a.W3T = w.W3T; a.W1T_target = w.W1T_t; a.W3T_target = w.W3T_t;
        a.ctr = t->ctr; a.lossi = t->lossi;
        a.out_grad_only = t->dueling ? 1u : 0u;
        const unsigned int elems = (H + 1) * Ap + H * (D + 1);
        const unsigned int own = (H / 64) * (H / kSqRows) + (elems + 255) / 256;
        if (t->rec_next) {
            // (recording a run of steps: this launch also gathers the next step's batch; the rest of
            // its arguments is kept for the launches that replace the next step's part)
            if (!t->w_args_host[0]) t->w_args_host[0] = malloc(sizeof(OptRecorded));
            if (!t->w_args_host[0]) return hipErrorOutOfMemory;
            const OptRecorded rec{q, a, own};
            memcpy(t->w_args_host[0], &rec, sizeof(rec));
            unsigned int nb = 0;
            size_t lds = 0;
            append_gather_shape(*t->rec_next, &nb, &lds);
            hipLaunchKernelGGL(opt_ahead_kernel, dim3(own + nb), dim3(256), lds, st, q, a, *t->rec_next, own, nb);
        } else {
            hipLaunchKernelGGL(opt_kernel, dim3(own), dim3(256), 0, st, q, a);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        ++n;
        unsigned int nh = 0;
        e = enqueue_head_update(t, st, &nh);
        if (e != hipSuccess) return e;
        n += nh;
    }
    if (count) *count = n;
    return hipGetLastError();
}

void* opt_ahead_func() { return reinterpret_cast<void*>(opt_ahead_kernel); }

hipError_t patch_opt_ahead_node(trainer* t, hipGraphExec_t exec, hipGraphNode_t node,
                                const hipKernelNodeParams& recorded, const AppendGatherArgs& next) {
    OptRecorded rec;
    memcpy(&rec, t->w_args_host[0], sizeof(rec));
    AppendGatherArgs nx = next;
    unsigned int nb = 0;
    size_t lds = 0;
    append_gather_shape(nx, &nb, &lds);
    void* kargs[] = {&rec.sq, &rec.sm, &nx, &rec.own, &nb};
    hipKernelNodeParams np = recorded;
    np.kernelParams = kargs;
    np.extra = nullptr;
    return hipGraphExecKernelNodeSetParams(exec, node, &np);
}

}  // namespace rp
